"""Oracle for the holistic traffic-aware activation swapping planner (Sec. IV-D): the iteration-
time model of Eq. 1-5, the interpolated recomputation cost of Eq. 7-8 and the greedy search of
Algorithm 1, in plain python floats (float64), in
the paper's notation and step order.  TEST INFRASTRUCTURE; shares nothing with the C++ planner.

Readings where the paper is silent:
  * alpha*A_G2M = A_G2M - MEM_avail (Eq. 3) is clamped at 0: activations only spill to the far tier
    once main memory is full.
  * Sizes (A, MEM_avail) are bytes, P is a parameter count (so 2P and 14P are bytes: fp16
    parameters; fp32 parameters + two moments + fp16 gradients), bandwidths bytes/s, FLOP counts
    operations, THP_G operations/s.
  * layer_list is sorted by offloading benefit OB = FLOP_layer / A_layer (Eq. 6), highest first,
    ties keeping the original order; a layer with A = 0 has infinite benefit.
  * Algorithm 1 is read as a rule over the prefixes of the benefit order: a prefix ENDS the search
    when it holds at least A_interBlock bytes (the floor that avoids running out of GPU memory)
    and its T_iter is no better than the best T_iter of any shorter non-empty prefix; the plan is
    the prefix just before the first one that ends the search (all layers if none does).  A prefix
    below the floor never ends the search, however bad its T_iter.
"""
import math


def iter_time(hw: dict, a_g2m: float, flop_r: float) -> float:
    """T_iter = T_f + T_b (Eq. 1) with T_f from Eq. 4 and T_b from Eq. 5."""
    spill = max(0.0, a_g2m - hw["mem_avail"])                       # Eq. 3, clamped
    t_f = max(hw["flop_f"] / hw["thp_g"],                           # T_f^G
              a_g2m / hw["bw_g"],                                   # T_f^G2M
              2.0 * hw["params"] / hw["bw_g"],                      # T_f^M2G
              2.0 * hw["params"] / hw["bw_s2m"] + spill / hw["bw_m2s"])   # T_f^S
    t_b = max((2.0 * hw["flop_f"] + flop_r) / hw["thp_g"],          # T_b^G
              2.0 * hw["params"] / hw["bw_g"],                      # T_b^G2M
              (2.0 * hw["params"] + a_g2m) / hw["bw_g"],            # T_b^M2G
              (14.0 * hw["params"] + spill) / hw["bw_s2m"] + 14.0 * hw["params"] / hw["bw_m2s"])
    return t_f + t_b


def offloading_benefit(flop: float, act_bytes: float) -> float:
    """OB_layer = FLOP_layer / A_layer (Eq. 6)."""
    return math.inf if act_bytes == 0 else flop / act_bytes


def recompute_flops(layers, flop_f: float, a_g2m: float):
    """FLOP_r(A_G2M) of Eq. 7 and its derivative, Eq. 8.  With the layers numbered by decreasing
    OB, find i with sum_{k<=i} A_k <= A_G2M < sum_{k<=i+1} A_k (right-hand piece at a breakpoint);
    beyond the last breakpoint everything is swapped and the derivative is 0."""
    ranked = sorted(layers, key=lambda la: -offloading_benefit(*la))
    i = 0
    while i < len(ranked) and sum(a for _, a in ranked[:i + 1]) <= a_g2m:
        i += 1
    whole = sum(f for f, _ in ranked[:i])
    if i == len(ranked):
        return flop_f - whole, 0.0
    flop_next, a_next = ranked[i]
    covered = sum(a for _, a in ranked[:i])
    flop_r = flop_f - whole - flop_next * (a_g2m - covered) / a_next
    return flop_r, -offloading_benefit(flop_next, a_next)


def plan(layers, hw: dict):
    """Algorithm 1 by its definition over prefixes.  layers: list of (flop, act_bytes).  Returns
    (swap_list as indices into `layers` in swapping order, A_G2M of the swap list, FLOP_r,
    T_iter of the swap list)."""
    order = sorted(range(len(layers)), key=lambda i: -offloading_benefit(*layers[i]))

    def swapped_bytes(k):                    # A_G2M when the first k layers are swapped
        return sum((layers[i][1] for i in order[:k]), 0.0)

    def recompute_left(k):                   # FLOP_r of Eq. 7 at the k-th breakpoint
        return hw["flop_f"] - sum((layers[i][0] for i in order[:k]), 0.0)

    def t_iter(k):
        return iter_time(hw, swapped_bytes(k), recompute_left(k))

    def ends_search(k):
        best_shorter = min((t_iter(j) for j in range(1, k)), default=math.inf)
        return swapped_bytes(k) >= hw["a_interblock"] and t_iter(k) >= best_shorter

    first_end = next((k for k in range(1, len(order) + 1) if ends_search(k)), None)
    count = len(order) if first_end is None else first_end - 1
    return order[:count], swapped_bytes(count), recompute_left(count), t_iter(count)
