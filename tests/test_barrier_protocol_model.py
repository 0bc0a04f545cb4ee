"""A model of the give-up handshake inside the one-launch step's grid-wide barrier, checked over
every interleaving (host only, no GPU).

The kernel's claim: a workgroup that ends without writing is always reported.  Two parties share
two words, each operation is an atomic performed at one point in time and a party issues its
next operation only after the previous one has returned:

    last arrival L:   V := verdict        then   read M  -> report incomplete iff M is set
    waiting group A:  (polls ran out)  M := mark   then   read V  -> give up iff V is not there

If A gives up, L must have seen the mark.  The model also shows what the ordering is for: with
either party's two operations swapped, an interleaving exists in which A gives up unreported.
"""
import itertools


def outcomes(l_ops, a_ops):
    """All results of interleaving the two parties' operation lists (each kept in order).
    Returns a set of (a_gave_up, l_reported)."""
    seen = set()
    slots = len(l_ops) + len(a_ops)
    for l_positions in itertools.combinations(range(slots), len(l_ops)):
        order = ["A"] * slots
        for p in l_positions:
            order[p] = "L"
        state = {"V": False, "M": False}
        result = {}
        it = {"L": iter(l_ops), "A": iter(a_ops)}
        for who in order:
            op = next(it[who])
            if op == "write V":
                state["V"] = True
            elif op == "write M":
                state["M"] = True
            elif op == "read M":
                result["l_reported"] = state["M"]
            elif op == "read V":
                result["a_gave_up"] = not state["V"]
        seen.add((result["a_gave_up"], result["l_reported"]))
    return seen


def test_a_group_that_gives_up_is_always_reported():
    seen = outcomes(["write V", "read M"], ["write M", "read V"])
    assert (True, False) not in seen            # gave up, not reported: must never happen
    # the other three outcomes all occur: proceeds unreported (the normal case), gives up and is
    # reported, and the harmless false alarm (marked, then found the verdict after all)
    assert seen == {(False, False), (True, True), (False, True)}


def test_either_party_in_the_other_order_can_lose_a_report():
    assert (True, False) in outcomes(["read M", "write V"], ["write M", "read V"])
    assert (True, False) in outcomes(["write V", "read M"], ["read V", "write M"])
