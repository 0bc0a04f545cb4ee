"""GPU parity of the out-of-place block step with the overflow test fused in (one 28 B/element
pass; same tensors and skip rule as the in-place step, Sec. IV-C and Table II).  The oracle is the
same in-place function run on host copies: on a clean block the GPU's output arrays must equal the
oracle's updated state while the GPU's input arrays stay as they were; on an overflowing block the
flag must be 1 and the inputs bit-identical (the outputs are unspecified and not compared)."""
import sys

import numpy as np
import pytest
import torch

import paper_2403_06504_amd as lohan
from paper_2403_06504_amd import synthetic_inputs as synth

from gpu_util import DeviceBlock, assert_state_parity, oracle_steps

pytestmark = pytest.mark.gpu

DEV = "cuda"
SIZES = list(range(0, 10)) + [255, 256, 257, 1023, 1025, 4099, 65537, 1_000_003]


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def small_workload(n):
    return synth.Workload(name=f"n{n}", n=n, step=100, loss_scale=65536.0, zero_moments=False)


class TwoSets:
    """A block with two sets of p, m, v and of the 16-bit copy; `cur` names the live set."""

    def __init__(self, tensors):
        self.n = tensors["p"].numel()
        self.g = tensors["g"]
        self.sets = [{k: tensors[k] for k in ("p", "m", "v", "p16")},
                     {k: torch.full_like(tensors[k], -7.0) for k in ("p", "m", "v", "p16")}]
        self.cur = 0
        self.flag = torch.full((1,), 9, dtype=torch.int32, device=DEV)        # stale on purpose

    def step(self, hy, flags=0, stream=None):
        a, b = self.sets[self.cur], self.sets[1 - self.cur]
        lohan.lohan_adam_block_step_out_of_place(
            a["p"], a["m"], a["v"], self.g, b["p"], b["m"], b["v"], b["p16"], self.n,
            hy["lr"], hy["beta1"], hy["beta2"], hy["eps"], hy["weight_decay"], hy["step"],
            hy["loss_scale"], self.flag, flags, stream=stream)
        torch.cuda.synchronize()
        f = int(self.flag.cpu().item())
        if f == 0:
            self.cur = 1 - self.cur                  # commit: the outputs become the state
        return f

    def host(self, which=None):
        s = self.sets[self.cur if which is None else which]
        out = {k: synth.to_numpy_bits(s[k]) for k in ("p", "m", "v", "p16")}
        out["g"] = synth.to_numpy_bits(self.g)
        return out


@pytest.mark.parametrize("flags", [0, lohan.LOHAN_FLAG_L2_MODE, lohan.LOHAN_FLAG_P16_FP16,
                                   lohan.LOHAN_FLAG_L2_MODE | lohan.LOHAN_FLAG_P16_FP16])
def test_chained_steps_with_pointer_swap(oracle, flags):
    l2 = bool(flags & lohan.LOHAN_FLAG_L2_MODE)
    half = bool(flags & lohan.LOHAN_FLAG_P16_FP16)
    for n in SIZES:
        say(f"[oop] n={n} flags={flags}")
        wl = small_workload(n)
        hy = wl.hyper()
        blk = TwoSets(synth.make_block(wl, seed=100 + n, device=DEV))
        host = blk.host()
        for k in range(4):
            h = dict(hy, step=hy["step"] + k)
            before = blk.host()
            live = blk.cur
            assert blk.step(h, flags) == 0
            after_inputs = blk.host(which=live)
            for name in ("p", "m", "v"):        # the inputs are never written
                assert np.array_equal(after_inputs[name].view(np.uint8),
                                      before[name].view(np.uint8)), (n, k, name)
            f = oracle.adam_block_step(host["p"], host["m"], host["v"], host["g"], host["p16"],
                                       nthreads=4, l2_mode=l2, half_out=half, **h)
            assert f == 0
            worst = assert_state_parity(blk.host(), host, what=f"out of place n={n} step {k}")
            assert worst == {"p": 0, "m": 0, "v": 0, "p16": 0}, (n, k, worst)


@pytest.mark.parametrize("n", [1, 7, 9, 4099, 1_000_003])
def test_overflow_raises_the_flag_and_the_inputs_survive(oracle, n):
    wl = small_workload(n)
    hy = wl.hyper()
    base = synth.make_block(wl, seed=3, device=DEV)
    positions = sorted({0, n - 1, n // 2, max(0, n - 2), (n // 4) * 4 % n})
    for pat in synth.NONFINITE_FP16 + (0x7BFF, 0xFBFF):
        for pos in positions:
            blk = TwoSets({k: t.clone() for k, t in base.items()})
            blk.g.view(torch.int16)[pos] = pat if pat < 0x8000 else pat - 0x10000
            before = blk.host()
            want = oracle.grad_overflow_check(before["g"])
            assert want == (0 if pat in (0x7BFF, 0xFBFF) else 1)
            assert blk.step(hy) == want, (n, hex(pat), pos)
            if want:
                assert blk.cur == 0
                after = blk.host()
                for k in ("p", "m", "v", "p16", "g"):
                    assert np.array_equal(after[k].view(np.uint8), before[k].view(np.uint8)), k
                # the flag is rewritten by every call: a clean gradient afterwards clears it
                blk.g.view(torch.int16)[pos] = 0x3C00
                assert blk.step(hy) == 0
            else:
                host = before
                oracle_steps(oracle, host, hy, 1, nthreads=2)
                worst = assert_state_parity(blk.host(), host, what="largest finite gradients")
                assert worst == {"p": 0, "m": 0, "v": 0, "p16": 0}


def test_every_gradient_non_finite(oracle):
    """The usual way to overflow: all of a block's gradients are inf or NaN, so every wavefront
    raises the flag.  Flag 1, inputs bit-identical; a clean step afterwards is taken."""
    n = 5_000_011
    wl = small_workload(n)
    hy = wl.hyper()
    blk = TwoSets(synth.make_block(wl, seed=9, device=DEV))
    clean_g = blk.g.clone()
    pattern = torch.tensor([0x7C00, -0x400, 0x7E00, 0x7FFF], dtype=torch.int16, device=DEV)
    blk.g.view(torch.int16).copy_(pattern.repeat((n + 3) // 4)[:n])
    before = blk.host()
    assert oracle.grad_overflow_check(before["g"]) == 1
    assert blk.step(hy) == 1
    after = blk.host()
    for k in ("p", "m", "v"):
        assert np.array_equal(after[k].view(np.uint32), before[k].view(np.uint32)), k
    blk.g.copy_(clean_g)
    host = blk.host()
    assert blk.step(hy) == 0
    assert oracle_steps(oracle, host, hy, 1, nthreads=8) == [0]
    worst = assert_state_parity(blk.host(), host, what="clean step after an all-NaN one")
    assert worst == {"p": 0, "m": 0, "v": 0, "p16": 0}


def test_every_kernel_variant_out_of_place(oracle):
    n = 1_000_003
    wl = small_workload(n)
    ref = synth.make_block(wl, seed=1, device=DEV)
    host = DeviceBlock({k: t.clone() for k, t in ref.items()}).host()
    hy = wl.hyper()
    oracle_steps(oracle, host, hy, 1, nthreads=16)
    variants = [wg | (u << 2) | (pol << 4) for pol in range(3) for u in range(2) for wg in range(3)]
    try:
        for variant in variants:
            for wgs, waves in ((0, 0), (1, 8), (0, 2)):
                say(f"[oop variant] variant={variant} wgs_per_cu={wgs} waves_per_cu={waves}")
                lohan.lohan_tuning_set_launch_config(variant, wgs, waves, 0)
                blk = TwoSets({k: t.clone() for k, t in ref.items()})
                assert blk.step(hy) == 0
                worst = assert_state_parity(blk.host(), host, what=f"oop variant={variant}")
                assert worst == {"p": 0, "m": 0, "v": 0, "p16": 0}
                # and with a non-finite value in the very last (ragged) element
                blk2 = TwoSets({k: t.clone() for k, t in ref.items()})
                blk2.g.view(torch.int16)[n - 1] = 0x7C00
                assert blk2.step(hy) == 1
    finally:
        lohan.lohan_tuning_set_launch_config()


def test_empty_block_out_of_place():
    flag = torch.full((1,), 5, dtype=torch.int32, device=DEV)
    lohan.lohan_adam_block_step_out_of_place(None, None, None, None, None, None, None, None, 0,
                                             1e-4, 0.9, 0.999, 1e-8, 0.01, 1, 1024.0, flag, 0)
    torch.cuda.synchronize()
    assert int(flag.cpu().item()) == 0


def test_13b_block_full_size_out_of_place(oracle):
    """The benchmark's block at full size in the automatic launch configuration: a clean step
    compared over all elements, then the same block with one non-finite gradient in the last
    tile."""
    wl = synth.WORKLOADS["gpt13b"]
    say(f"[oop 13b] n={wl.n} generating")
    blk = TwoSets(synth.make_block(wl, seed=0, device=DEV))
    host = blk.host()
    hy = wl.hyper()
    say("[oop 13b] gpu step")
    assert blk.step(hy) == 0
    say("[oop 13b] oracle step")
    assert oracle_steps(oracle, host, hy, 1) == [0]
    worst = assert_state_parity(blk.host(), host, what="13B out of place")
    assert worst == {"p": 0, "m": 0, "v": 0, "p16": 0}
    say(f"[oop 13b] worst ulp {worst}")
    del host
    live = blk.cur
    snap = {k: blk.sets[live][k].clone() for k in ("p", "m", "v")}
    blk.g.view(torch.int16)[wl.n - 3] = -1                 # 0xFFFF: a NaN
    assert blk.step(dict(hy, step=hy["step"] + 1)) == 1
    assert blk.cur == live
    for k in ("p", "m", "v"):
        assert torch.equal(blk.sets[live][k].view(torch.int32), snap[k].view(torch.int32)), k


def test_175b_block_out_of_place_sampled(oracle):
    """n = 12*12288^2 with a second set of state (54 GB resident, byte offsets beyond 2^32):
    sampled ranges -- head, end, seeded interior, ranges whose fp32 byte offsets cross 2^32 --
    against the oracle, whole-buffer properties for the rest, then one NaN in the last element."""
    wl = synth.WORKLOADS["gpt175b"]
    say(f"[oop 175b] n={wl.n} generating")
    blk = TwoSets(synth.make_block(wl, seed=0, device=DEV))
    span = 1 << 21
    rng = np.random.default_rng(14)
    starts = [0, wl.n - span] + [int(x) for x in rng.integers(span, wl.n - 2 * span, size=4)]
    starts += [(1 << 30) - 3, wl.n // 2 + 1]
    src = blk.sets[0]

    def sample(s, which):
        st = blk.sets[which]
        out = {k: synth.to_numpy_bits(st[k][s:s + span]) for k in ("p", "m", "v", "p16")}
        out["g"] = synth.to_numpy_bits(blk.g[s:s + span])
        return out

    before = {s: sample(s, 0) for s in starts}
    hy = wl.hyper()
    assert blk.step(hy) == 0 and blk.cur == 1
    for s in starts:
        host = before[s]
        assert oracle_steps(oracle, host, hy, 1, nthreads=8) == [0]
        worst = assert_state_parity(sample(s, 1), host, what=f"175B out of place, range {s}")
        assert worst == {"p": 0, "m": 0, "v": 0, "p16": 0}, (s, worst)
    out = blk.sets[1]
    assert bool(torch.all(out["v"] >= 0))
    assert torch.equal(out["p16"].view(torch.int16), out["p"].to(torch.bfloat16).view(torch.int16))
    # m' = beta1 m + (1 - beta1) g everywhere (a whole-buffer check of the first moment in
    # float64: one fp32 rounding per operation keeps it within a few ulp)
    g = blk.g[:1 << 26].double() / hy["loss_scale"]
    want_m = hy["beta1"] * src["m"][:1 << 26].double() + (1.0 - hy["beta1"]) * g
    err = (out["m"][:1 << 26].double() - want_m).abs()
    scale = torch.maximum(src["m"][:1 << 26].abs().double(), g.abs()) * 2.0 ** -22 + 1e-30
    assert bool(torch.all(err <= scale))
    blk.g.view(torch.int16)[wl.n - 1] = 0x7E00
    assert blk.step(dict(hy, step=hy["step"] + 1)) == 1 and blk.cur == 1


@pytest.mark.parametrize("n,S,max_norm", [(1_000_003, 65536.0, 0.5), (70_001, 3000.0, 0.05),
                                          (5_000, 1024.0, 100.0), (7, 65536.0, 1e-3)])
def test_clipped_single_pass_form(oracle, n, S, max_norm):
    """lohan_grad_sqnorm + lohan_adam_block_step_out_of_place_clipped: per-block clipping resolved
    on the device, the update out of place with the overflow test fused in.  Bit-identical to the
    in-place clipped step given the same squared norm; against the oracle, the effective scale is
    within one fp32 ulp of the oracle's own and the oracle stepped with the HIP path's scale
    reproduces the outputs bit for bit.  An overflowing block raises the flag and leaves the
    inputs untouched."""
    from gpu_util import assert_scale_within_one_ulp
    wl = synth.Workload(name=f"n{n}", n=n, step=100, loss_scale=S, zero_moments=False)
    hy = wl.hyper()
    base = synth.make_block(wl, seed=300 + n % 89, device=DEV)
    blk = TwoSets({k: t.clone() for k, t in base.items()})
    inplace = DeviceBlock({k: t.clone() for k, t in base.items()})
    host = blk.host()
    sqnorm = torch.zeros(1, dtype=torch.float64, device=DEV)
    ws = lohan.new_workspace(DEV)

    def clipped_step(b):
        a, o = b.sets[b.cur], b.sets[1 - b.cur]
        lohan.lohan_grad_sqnorm(b.g, n, S, sqnorm, None, ws)
        lohan.lohan_adam_block_step_out_of_place_clipped(
            a["p"], a["m"], a["v"], b.g, o["p"], o["m"], o["v"], o["p16"], n, hy["lr"],
            hy["beta1"], hy["beta2"], hy["eps"], hy["weight_decay"], hy["step"], S, sqnorm,
            max_norm, b.flag, 0, ws)
        torch.cuda.synchronize()
        return int(b.flag.cpu().item())

    assert clipped_step(blk) == 0
    got = blk.host(which=1)
    inputs_after = blk.host(which=0)
    for k in ("p", "m", "v"):
        assert np.array_equal(inputs_after[k].view(np.uint8), host[k].view(np.uint8)), k

    inplace.norm(S)
    lohan.lohan_adam_block_step_clipped(inplace.p, inplace.m, inplace.v, inplace.g, inplace.p16,
                                        n, hy["lr"], hy["beta1"], hy["beta2"], hy["eps"],
                                        hy["weight_decay"], hy["step"], S, inplace.sqnorm,
                                        max_norm, inplace.flag, 0, inplace.ws)
    torch.cuda.synchronize()
    assert float(inplace.sqnorm.cpu().item()) == float(sqnorm.cpu().item())
    same = inplace.host()
    for k in ("p", "m", "v", "p16"):
        assert np.array_equal(got[k].view(np.uint8), same[k].view(np.uint8)), k

    sq_gpu = float(sqnorm.cpu().item())
    sq_orc = oracle.grad_sqnorm(host["g"], S)
    assert abs(sq_gpu - sq_orc) <= 1e-5 * sq_orc
    s_eff_gpu = lohan.lohan_clip_loss_scale(sq_gpu, S, max_norm)
    assert_scale_within_one_ulp(s_eff_gpu, float(oracle.clip_loss_scale(sq_orc, S, max_norm)))
    assert (s_eff_gpu == S) == (max_norm >= 100.0)
    oracle_steps(oracle, host, dict(hy, loss_scale=s_eff_gpu), 1, nthreads=4)
    worst = assert_state_parity(got, host, what="clipped out-of-place step")
    assert worst == {"p": 0, "m": 0, "v": 0, "p16": 0}, worst

    bad = TwoSets({k: t.clone() for k, t in base.items()})
    bad.g.view(torch.int16)[n // 2] = 0x7E00
    before = bad.host(which=0)
    assert clipped_step(bad) == 1
    after = bad.host(which=0)
    for k in ("p", "m", "v", "p16"):
        assert np.array_equal(after[k].view(np.uint8), before[k].view(np.uint8)), k
