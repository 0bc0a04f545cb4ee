"""Activation swapping planner (Sec. IV-D: Eq. 1-6, Algorithm 1).  CPU only.

First the oracle (oracle/swap_planner.py) is pinned against things other than itself: a worked
example evaluated by hand, each of the eight terms of Eq. 4-5 made dominant in turn, the convexity
the paper proves, brute force over all prefixes, and the three cases of Sec. IV-D.  Then the C++
planner in the library is compared with the oracle decision by decision."""
import math

import numpy as np
import pytest

import paper_2403_06504_amd as lohan
from oracle import swap_planner as orc

# Hand example.  THP_G = 100 op/s, BW_G = 10 B/s, BW_S2M = BW_M2S = 5 B/s, P = 0.1, main memory
# never fills, FLOP_f = 600.  Constant terms: 2P/BW_G = 0.02, 2P/BW_S2M = 0.04,
# 14P/BW_S2M + 14P/BW_M2S = 0.56.  Layers (FLOP, A): (300, 10) OB 30; (200, 20) OB 10;
# (100, 100) OB 1 -- given out of order to exercise the sort.
HW = dict(thp_g=100.0, bw_g=10.0, bw_s2m=5.0, bw_m2s=5.0, params=0.1, mem_avail=1e9,
          flop_f=600.0, a_interblock=0.0)
LAYERS = [(100.0, 100.0), (300.0, 10.0), (200.0, 20.0)]


def test_hand_example_iteration_times():
    # +layer OB30: A=10, FLOP_r=300: T_f = max(6, 1, .02, .04) = 6; T_b = max(15, .02, 1.02, .56)
    assert orc.iter_time(HW, 10.0, 300.0) == pytest.approx(6.0 + 15.0, rel=1e-15)
    # +layer OB10: A=30, FLOP_r=100: T_f = max(6, 3) = 6; T_b = max(13, 3.02) = 13
    assert orc.iter_time(HW, 30.0, 100.0) == pytest.approx(6.0 + 13.0, rel=1e-15)
    # +layer OB1: A=130, FLOP_r=0: T_f = max(6, 13) = 13; T_b = max(12, 13.02) = 13.02
    assert orc.iter_time(HW, 130.0, 0.0) == pytest.approx(13.0 + 13.02, rel=1e-15)


def test_hand_example_plan():
    """21 -> 19 -> 26.02: the third layer does not improve, the search stops before it."""
    swap, a, f, t = orc.plan(LAYERS, HW)
    assert swap == [1, 2] and a == 30.0 and f == 100.0 and t == pytest.approx(19.0)
    # with a floor of 200 bytes the non-improving layer is still taken (A = 130 < 200)
    swap, a, f, t = orc.plan(LAYERS, dict(HW, a_interblock=200.0))
    assert swap == [1, 2, 0] and a == 130.0 and f == 0.0 and t == pytest.approx(26.02)
    # with a floor of 120 the third layer brings A to 130 >= 120 and, not improving, ends the
    # search without being appended (Algorithm 1 as printed)
    swap, a, _, _ = orc.plan(LAYERS, dict(HW, a_interblock=120.0))
    assert swap == [1, 2] and a == 30.0


BIG = 1e30


@pytest.mark.parametrize("which,hw_over,a,fr,want", [
    ("T_f^G", dict(), 0.0, 0.0, lambda h: h["flop_f"] / h["thp_g"] + 2 * h["flop_f"] / h["thp_g"]),
    ("T_f^G2M + T_b^M2G", dict(thp_g=BIG), 50.0, 0.0,
     lambda h: 50.0 / h["bw_g"] + (2 * h["params"] + 50.0) / h["bw_g"]),
    ("T_f^M2G + T_b^M2G", dict(thp_g=BIG, bw_s2m=BIG, bw_m2s=BIG), 0.0, 0.0,
     lambda h: 2 * h["params"] / h["bw_g"] * 2),
    ("T_f^S + T_b^S, no spill", dict(thp_g=BIG, bw_g=BIG), 10.0, 0.0,
     lambda h: 2 * h["params"] / h["bw_s2m"] + 14 * h["params"] / h["bw_s2m"]
     + 14 * h["params"] / h["bw_m2s"]),
    ("T_f^S + T_b^S, spill", dict(thp_g=BIG, bw_g=BIG, mem_avail=4.0, bw_m2s=2.0), 10.0, 0.0,
     lambda h: 2 * h["params"] / h["bw_s2m"] + 6.0 / 2.0
     + (14 * h["params"] + 6.0) / h["bw_s2m"] + 14 * h["params"] / 2.0),
    ("T_b^G with recomputation", dict(bw_g=BIG, bw_s2m=BIG, bw_m2s=BIG), 0.0, 250.0,
     lambda h: h["flop_f"] / h["thp_g"] + (2 * h["flop_f"] + 250.0) / h["thp_g"]),
])
def test_each_term_of_the_time_model(which, hw_over, a, fr, want):
    """Catches a wrong factor (2P, 14P, 2 FLOP_f), a swapped bandwidth, a missing spill clamp."""
    hw = dict(HW, **hw_over)
    assert orc.iter_time(hw, a, fr) == pytest.approx(want(hw), rel=1e-12), which


def random_instance(rng, n):
    flop = rng.uniform(1.0, 100.0, n) * 1e9
    act = rng.uniform(1.0, 100.0, n) * 1e6
    hw = dict(thp_g=10 ** rng.uniform(11, 14), bw_g=10 ** rng.uniform(9, 11),
              bw_s2m=10 ** rng.uniform(9, 10.5), bw_m2s=10 ** rng.uniform(9, 10.5),
              params=10 ** rng.uniform(6, 9), mem_avail=float(rng.uniform(0, act.sum())),
              flop_f=float(flop.sum() * rng.uniform(1.0, 1.5)),
              a_interblock=float(rng.choice([0.0, rng.uniform(0, act.sum())])))
    return [(float(f), float(a)) for f, a in zip(flop, act)], hw


def prefix_times(layers, hw):
    order = sorted(range(len(layers)), key=lambda i: -layers[i][0] / layers[i][1])
    a, f, out = 0.0, hw["flop_f"], []
    for i in order:
        a += layers[i][1]
        f -= layers[i][0]
        out.append((a, f, orc.iter_time(hw, a, f)))
    return order, out


def test_iteration_time_is_convex_along_the_benefit_order():
    """Sec. IV-D proves T_iter convex in A_G2M when layers are taken by decreasing OB: slopes
    between consecutive prefixes never decrease.  Fails if the sort order or a term is wrong."""
    rng = np.random.default_rng(0)
    for _ in range(300):
        layers, hw = random_instance(rng, int(rng.integers(2, 30)))
        _, pts = prefix_times(layers, hw)
        pts = [(0.0, hw["flop_f"], orc.iter_time(hw, 0.0, hw["flop_f"]))] + pts
        slopes = [(pts[k + 1][2] - pts[k][2]) / (pts[k + 1][0] - pts[k][0])
                  for k in range(len(pts) - 1)]
        scale = max(abs(s) for s in slopes) + 1e-30
        assert all(slopes[k + 1] >= slopes[k] - 1e-9 * scale for k in range(len(slopes) - 1))


def test_plan_is_the_brute_force_optimum_over_prefixes():
    """Without a floor the greedy stop is the global minimum over all non-empty prefixes."""
    rng = np.random.default_rng(1)
    for _ in range(300):
        layers, hw = random_instance(rng, int(rng.integers(1, 25)))
        hw["a_interblock"] = 0.0
        order, pts = prefix_times(layers, hw)
        swap, a, f, t = orc.plan(layers, hw)
        best = min(p[2] for p in pts)
        assert t <= best * (1 + 1e-12)
        assert swap == order[:len(swap)] and len(swap) >= 1
        assert a == pytest.approx(pts[len(swap) - 1][0]) and f == pytest.approx(pts[len(swap) - 1][1])


def test_three_cases_of_the_time_curve():
    layers = [(50e9, 10e6)] * 8
    base = dict(thp_g=1e12, bw_g=1e10, bw_s2m=1e10, bw_m2s=1e10, params=1e6, mem_avail=1e12,
                flop_f=400e9, a_interblock=25e6)
    # Case 1: PCIe-bound from the start -> only the floor is swapped (A reaches 30 MB >= 25 MB
    # with the third layer, which does not improve and is not appended)
    swap, a, _, _ = orc.plan(layers, dict(base, bw_g=1e6))
    assert swap == [0, 1] and a == 20e6
    # Case 2: GPU-bound throughout -> everything is swapped
    swap, a, f, _ = orc.plan(layers, dict(base, thp_g=1e9))
    assert swap == list(range(8)) and a == 80e6 and f == 0.0
    # Case 3: interior optimum where the transfer term overtakes the compute term
    swap, _, _, t = orc.plan(layers, dict(base, bw_g=3e7, a_interblock=0.0))
    assert 1 <= len(swap) < 8
    _, pts = prefix_times(layers, dict(base, bw_g=3e7, a_interblock=0.0))
    assert t == pytest.approx(min(p[2] for p in pts))


def test_recompute_flops_hand_example():
    """Eq. 7-8 on the hand example: benefit order (300,10) OB 30, (200,20) OB 10, (100,100) OB 1."""
    for a, want_f, want_d in ((0.0, 600.0, -30.0), (5.0, 450.0, -30.0), (10.0, 300.0, -10.0),
                              (20.0, 200.0, -10.0), (30.0, 100.0, -1.0), (80.0, 50.0, -1.0),
                              (130.0, 0.0, 0.0), (200.0, 0.0, 0.0)):
        f, d = orc.recompute_flops(LAYERS, 600.0, a)
        assert f == pytest.approx(want_f, rel=1e-15) and d == want_d, a


def test_recompute_flops_matches_prefixes_differences_and_convexity():
    """At every breakpoint Eq. 7 must give the discrete FLOP_r that Algorithm 1 accumulates; the
    slope of Eq. 8 must be the finite difference inside a piece; and the slopes never decrease
    (the convexity argument of Sec. IV-D)."""
    rng = np.random.default_rng(3)
    for _ in range(200):
        layers, hw = random_instance(rng, int(rng.integers(1, 20)))
        _, pts = prefix_times(layers, hw)
        for a, f, _t in pts:
            got, _ = orc.recompute_flops(layers, hw["flop_f"], a)
            assert got == pytest.approx(f, rel=1e-9, abs=1e-3)
        total = pts[-1][0]
        grid = np.sort(rng.uniform(0, total, 40))
        slopes = []
        for a in grid:
            f0, d0 = orc.recompute_flops(layers, hw["flop_f"], float(a))
            h = total * 1e-9
            f1, d1 = orc.recompute_flops(layers, hw["flop_f"], float(a) + h)
            if d0 == d1:                                      # same piece
                assert (f1 - f0) / h == pytest.approx(d0, rel=1e-3, abs=1e-6 * abs(d0))
            slopes.append(d0)
        assert all(b >= a for a, b in zip(slopes, slopes[1:]))
        assert orc.recompute_flops(layers, hw["flop_f"], total * 2)[1] == 0.0


def test_continuous_iteration_time_is_convex():
    """T_iter(A_G2M) with the interpolated FLOP_r is convex: midpoints lie below chords."""
    rng = np.random.default_rng(4)
    for _ in range(200):
        layers, hw = random_instance(rng, int(rng.integers(2, 20)))
        total = sum(a for _, a in layers)

        def t(a):
            return orc.iter_time(hw, a, orc.recompute_flops(layers, hw["flop_f"], a)[0])

        for _ in range(20):
            a, b = sorted(rng.uniform(0, total, 2))
            mid = t(0.5 * (a + b))
            assert mid <= 0.5 * (t(a) + t(b)) * (1 + 1e-12) + 1e-15


# ----------------------------------------------------------------------------- C++ planner

def test_library_recompute_flops_matches_oracle():
    rng = np.random.default_rng(5)
    for trial in range(300):
        layers, hw = random_instance(rng, int(rng.integers(1, 30)))
        if trial % 5 == 0 and len(layers) > 2:
            layers[1] = (layers[1][0], 0.0)                   # a layer without activation bytes
            layers[2] = layers[0]                             # a tie
        total = sum(a for _, a in layers)
        prefix = np.cumsum([a for _, a in sorted(layers, key=lambda la: -orc.offloading_benefit(*la))])
        for a in list(rng.uniform(0, 1.2 * total, 10)) + [0.0, total] + [float(x) for x in prefix[:3]]:
            got = lohan.lohan_swap_recompute_flops(layers, hw["flop_f"], a)
            want = orc.recompute_flops(layers, hw["flop_f"], a)
            assert got[0] == pytest.approx(want[0], rel=1e-12, abs=1e-3), (trial, a)
            # FLOP_r is continuous; the slope jumps at a breakpoint, where the last bit of a sum
            # decides the side, so it is compared away from breakpoints only
            if np.min(np.abs(prefix - a)) > 1e-9 * total:
                assert got[1] == pytest.approx(want[1], rel=1e-14), (trial, a)
    assert lohan.lohan_swap_recompute_flops([], 7.0, 3.0) == (7.0, 0.0)
    for bad in ((LAYERS, -1.0, 0.0), (LAYERS, 1.0, -1.0), (LAYERS, math.nan, 0.0),
                (LAYERS, 1.0, math.inf), ([(1.0, -2.0)], 1.0, 0.0)):
        with pytest.raises(lohan.LohanError) as e:
            lohan.lohan_swap_recompute_flops(*bad)
        assert e.value.status == 3


def test_library_planner_matches_oracle_on_random_instances():
    rng = np.random.default_rng(2)
    for trial in range(500):
        n = int(rng.integers(0, 40))
        layers, hw = random_instance(rng, max(n, 1))
        layers = layers[:n]
        if trial % 7 == 0 and n > 3:                      # ties in OB and zero-size activations
            layers[1] = layers[0]
            layers[2] = (layers[2][0], 0.0)
        want = orc.plan(layers, hw)
        got = lohan.lohan_plan_activation_swapping(layers, hw)
        assert got[0] == want[0], (trial, got[0], want[0])
        for g, w in zip(got[1:], want[1:]):
            assert g == pytest.approx(w, rel=1e-12, abs=1e-6)
        a = float(rng.uniform(0, 1e9))
        f = float(rng.uniform(0, 1e12))
        assert lohan.lohan_swap_iter_time(hw, a, f) == pytest.approx(orc.iter_time(hw, a, f),
                                                                     rel=1e-14)


def test_library_planner_hand_example_and_edges():
    assert lohan.lohan_plan_activation_swapping(LAYERS, HW)[0] == [1, 2]
    assert lohan.lohan_plan_activation_swapping(LAYERS, dict(HW, a_interblock=200.0))[0] == [1, 2, 0]
    swap, a, f, t = lohan.lohan_plan_activation_swapping([], HW)
    assert swap == [] and a == 0.0 and f == HW["flop_f"]
    assert t == pytest.approx(orc.iter_time(HW, 0.0, HW["flop_f"]))
    assert lohan.lohan_plan_activation_swapping([(5.0, 1.0)], HW)[0] == [0]
    for bad in (dict(thp_g=0.0), dict(bw_g=-1.0), dict(bw_s2m=math.nan), dict(bw_m2s=math.inf),
                dict(params=-1.0), dict(mem_avail=math.nan), dict(flop_f=-5.0),
                dict(a_interblock=-1.0)):
        with pytest.raises(lohan.LohanError) as e:
            lohan.lohan_plan_activation_swapping(LAYERS, dict(HW, **bad))
        assert e.value.status == 3
    for bad_layer in ((-1.0, 1.0), (1.0, -1.0), (math.nan, 1.0), (1.0, math.inf)):
        with pytest.raises(lohan.LohanError):
            lohan.lohan_plan_activation_swapping([bad_layer], HW)
    assert math.isnan(lohan.lohan_swap_iter_time(dict(HW, bw_g=0.0), 1.0, 1.0))
