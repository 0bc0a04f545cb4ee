"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
bits.  Every test needs an MI355X and the built in-tree library (no fallback exists)."""
import sys

import numpy as np
import pytest
import torch

import paper_2403_06504_amd as lohan
from paper_2403_06504_amd import synthetic_inputs as synth

from gpu_util import (RTOL_SQNORM, DeviceBlock, assert_scale_within_one_ulp, assert_state_parity,
                      gpu_steps, oracle_steps)

pytestmark = pytest.mark.gpu

DEV = "cuda"


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def _library_is_native():
    assert torch.cuda.is_available(), "these tests need a GPU"
    lohan.load_library()            # raises if the HIP library was not built
    lohan.lohan_tuning_set_launch_config()         # built-in defaults, the shape bench.py times
    yield


def small_workload(n, step=100, S=65536.0, zero=False):
    return synth.Workload(name=f"n{n}", n=n, step=step, loss_scale=S, zero_moments=zero)


SMALL_N = list(range(0, 18)) + [255, 256, 257, 1023, 1024, 1025, 2047, 2048, 2049, 4095, 4096,
                                4097, 8191, 8193, 65537, 1_000_003]


@pytest.mark.parametrize("l2_mode", [False, True])
def test_ten_chained_steps_small_sizes(oracle, l2_mode):
    """All tail residues of the 4-wide vectors and of the workgroup tiles, 10 chained steps."""
    worst_all = {"p": 0, "m": 0, "v": 0, "p16": 0}
    for n in SMALL_N:
        wl = small_workload(n)
        say(f"[small] n={n} l2={l2_mode}")
        blk = DeviceBlock(synth.make_block(wl, seed=n, device=DEV))
        host = blk.host()
        hy = wl.hyper()
        gflags = gpu_steps(blk, hy, 10, l2_mode=l2_mode)
        oflags = oracle_steps(oracle, host, hy, 10, l2_mode=l2_mode, nthreads=4)
        assert gflags == oflags == [0] * 10
        worst = assert_state_parity(blk.host(), host, what=f"n={n}")
        for k in worst:
            worst_all[k] = max(worst_all[k], worst[k])
    say(f"[small] worst ulp over all sizes: {worst_all}")


def all_variants():
    return [wg | (u << 2) | (pol << 4) for pol in range(3) for u in range(2) for wg in range(3)]


def test_every_kernel_variant_matches(oracle):
    """Every compiled launch shape (workgroup size x unroll x cache policy), with and without a
    grid cap and an occupancy throttle, at a ragged size."""
    n = 1_000_003
    wl = small_workload(n)
    ref_blk = synth.make_block(wl, seed=1, device=DEV)
    host = DeviceBlock({k: t.clone() for k, t in ref_blk.items()}).host()
    hy = wl.hyper()
    oracle_steps(oracle, host, hy, 2, nthreads=16)
    try:
        for variant in all_variants():
            for wgs, waves in ((0, 0), (1, 8), (8, 4), (0, 2)):
                say(f"[variant] variant={variant} wgs_per_cu={wgs} waves_per_cu={waves}")
                lohan.lohan_tuning_set_launch_config(variant, wgs, waves, 0)
                blk = DeviceBlock({k: t.clone() for k, t in ref_blk.items()})
                assert gpu_steps(blk, hy, 2) == [0, 0]
                assert_state_parity(blk.host(), host, what=f"variant={variant}")
    finally:
        lohan.lohan_tuning_set_launch_config()


def test_bf16_copy_rounding_all_upper_halves(oracle):
    """The hardware fp32->bf16 conversion against the oracle's round-to-nearest-even on crafted
    parameters: every bf16 value's tie, just-below-tie and just-above-tie neighbour (lr = 0 and
    wd = 0 make the step leave p unchanged, so p16 is the rounding of the crafted p)."""
    hi = torch.arange(0, 1 << 16, dtype=torch.int64)
    hi = hi[((hi >> 7) & 0xFF) != 0xFF]                       # finite bf16 values only
    lows = torch.tensor([0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF], dtype=torch.int64)
    bits = ((hi[:, None] << 16) | lows[None, :]).reshape(-1)
    bits = bits[((bits >> 23) & 0xFF) != 0xFF]                # keep fp32 finite
    n = bits.numel()
    p = (bits.to(torch.int64) - ((bits >> 31) << 32)).to(torch.int32).view(torch.float32).to(DEV)
    wl = small_workload(n)
    t = synth.make_block(wl, seed=0, device=DEV)
    t["p"] = p.contiguous()
    t["g"].zero_()
    blk = DeviceBlock(t)
    host = blk.host()
    hy = dict(wl.hyper(), lr=0.0, weight_decay=0.0)
    assert gpu_steps(blk, hy, 1) == [0]
    oracle_steps(oracle, host, hy, 1, nthreads=4)
    got = blk.host()
    assert np.array_equal(got["p"].view(np.uint32), host["p"].view(np.uint32))
    assert np.array_equal(got["p16"], host["p16"])


def test_fp16_working_copy_option(oracle):
    """LOHAN_FLAG_P16_FP16: the 16-bit copy is IEEE binary16 (RNE, overflow to infinity, gradual
    underflow); p, m, v are unaffected.  Crafted parameters cover the overflow threshold, ties
    and the subnormal range of binary16; lr = wd = 0 keeps p fixed so the copy is its rounding."""
    halves = torch.arange(0, 0x7C00, dtype=torch.int32).to(torch.int16).view(torch.float16)
    base = halves.float().view(torch.int32)
    crafted = torch.cat([base | 0x1000, (base | 0x1000) - 1, (base | 0x1000) + 1, base,
                         base | 0x0FFF]).view(torch.float32)
    extra = torch.tensor([65504.0, 65519.996, 65520.0, 70000.0, -70000.0, 2.0 ** -25,
                          2.0 ** -25 * 1.0000001, 2.0 ** -24, 1e-30, 0.0, -0.0], dtype=torch.float32)
    pvals = torch.cat([crafted, -crafted, extra])
    n = pvals.numel()
    wl = small_workload(n)
    t = synth.make_block(wl, seed=0, device=DEV)
    t["p"] = pvals.to(DEV).contiguous()
    t["g"].zero_()
    t["p16"] = torch.full((n,), -3.0, dtype=torch.float16, device=DEV)
    blk = DeviceBlock(t)
    host = blk.host()
    hy = dict(wl.hyper(), lr=0.0, weight_decay=0.0)
    blk.step(hy, flags=lohan.LOHAN_FLAG_P16_FP16)
    torch.cuda.synchronize()
    assert blk.flag_value() == 0
    assert oracle.adam_block_step(host["p"], host["m"], host["v"], host["g"], host["p16"],
                                  half_out=True, nthreads=4, **hy) == 0
    got = blk.host()
    assert np.array_equal(got["p"].view(np.uint32), host["p"].view(np.uint32))
    assert np.array_equal(got["p16"], host["p16"])
    # and on ordinary data, chained with L2 mode, every variant of the flag combination
    n2 = 300_007
    wl2 = small_workload(n2)
    for flags, l2 in ((lohan.LOHAN_FLAG_P16_FP16, False),
                      (lohan.LOHAN_FLAG_P16_FP16 | lohan.LOHAN_FLAG_L2_MODE, True)):
        t2 = synth.make_block(wl2, seed=3, device=DEV)
        t2["p16"] = torch.zeros(n2, dtype=torch.float16, device=DEV)
        b2 = DeviceBlock(t2)
        h2 = b2.host()
        for k in range(3):
            b2.step(dict(wl2.hyper(), step=100 + k), flags=flags)
            oracle.adam_block_step(h2["p"], h2["m"], h2["v"], h2["g"], h2["p16"], l2_mode=l2,
                                   half_out=True, nthreads=8, **dict(wl2.hyper(), step=100 + k))
        torch.cuda.synchronize()
        worst = assert_state_parity(b2.host(), h2, what=f"fp16 copy flags={flags}")
        assert worst == {"p": 0, "m": 0, "v": 0, "p16": 0}


def test_l2_mode_at_13b_scale(oracle):
    """The L2-regularisation variant on the full 13B-shaped block."""
    wl = synth.WORKLOADS["gpt13b"]
    blk = DeviceBlock(synth.make_block(wl, seed=1, device=DEV))
    host = blk.host()
    hy = wl.hyper()
    assert gpu_steps(blk, hy, 2, l2_mode=True) == [0, 0]
    assert oracle_steps(oracle, host, hy, 2, l2_mode=True) == [0, 0]
    worst = assert_state_parity(blk.host(), host, what="13B block, L2 mode")
    say(f"[l2@13b] worst ulp {worst}")
    # a third step that also emits the 16-bit copy as binary16
    h3 = dict(hy, step=hy["step"] + 2)
    blk.step(h3, flags=lohan.LOHAN_FLAG_L2_MODE | lohan.LOHAN_FLAG_P16_FP16)
    torch.cuda.synchronize()
    assert blk.flag_value() == 0
    assert oracle.adam_block_step(host["p"], host["m"], host["v"], host["g"], host["p16"],
                                  l2_mode=True, half_out=True, nthreads=16, **h3) == 0
    worst = assert_state_parity(blk.host(), host, what="13B block, L2 mode + fp16 copy")
    say(f"[l2+fp16@13b] worst ulp {worst}")
    assert worst == {"p": 0, "m": 0, "v": 0, "p16": 0}


def test_config1_h768_block_ten_steps(oracle):
    wl = synth.WORKLOADS["gpt_h768"]
    say(f"[cfg1] n={wl.n}")
    blk = DeviceBlock(synth.make_block(wl, seed=0, device=DEV))
    host = blk.host()
    hy = wl.hyper()
    assert gpu_steps(blk, hy, 10) == [0] * 10
    assert oracle_steps(oracle, host, hy, 10) == [0] * 10
    worst = assert_state_parity(blk.host(), host, what="config 1")
    say(f"[cfg1] worst ulp {worst}")
    # first step closed form also holds on the GPU result after step 1 (fresh block)
    blk1 = DeviceBlock(synth.make_block(wl, seed=0, device=DEV))
    p0 = blk1.p.clone()
    gpu_steps(blk1, hy, 1)
    g = blk1.g.float() / wl.loss_scale
    dp = (blk1.p.double() - p0.double() * (1.0 - wl.lr * wl.weight_decay))
    big = g.abs() > 1e-5
    assert torch.all((dp[big].abs() - wl.lr).abs() <= 2e-3 * wl.lr + 1e-8)
    assert torch.all(torch.sign(dp[big]) == -torch.sign(g[big].double()))


def test_config2_13b_block_full_size(oracle):
    """The benchmark's workload at full size and in its launch configuration: one step compared
    over all 314,572,800 elements, then ten chained steps."""
    wl = synth.WORKLOADS["gpt13b"]
    say(f"[cfg2] n={wl.n} generating")
    blk = DeviceBlock(synth.make_block(wl, seed=0, device=DEV))
    host = blk.host()
    hy = wl.hyper()
    say("[cfg2] step 1 gpu")
    assert gpu_steps(blk, hy, 1) == [0]
    say("[cfg2] step 1 oracle")
    assert oracle_steps(oracle, host, hy, 1) == [0]
    worst = assert_state_parity(blk.host(), host, what="config 2, 1 step")
    say(f"[cfg2] 1 step worst ulp {worst}")
    hy2 = dict(hy, step=hy["step"] + 1)
    assert gpu_steps(blk, hy2, 9) == [0] * 9
    say("[cfg2] 9 more oracle steps")
    assert oracle_steps(oracle, host, hy2, 9) == [0] * 9
    worst = assert_state_parity(blk.host(), host, what="config 2, 10 steps")
    say(f"[cfg2] 10 steps worst ulp {worst}")


def test_config4_175b_block_sampled(oracle):
    """n = 12*12288^2 (29 GB resident, byte offsets beyond 2^32): the elements are independent, so
    the oracle is run on sampled ranges -- the head, the end, and seeded unaligned interior
    ranges -- of the same buffers."""
    wl = synth.WORKLOADS["gpt175b"]
    say(f"[cfg4] n={wl.n} generating")
    blk = DeviceBlock(synth.make_block(wl, seed=0, device=DEV))
    span = 1 << 21
    rng = np.random.default_rng(4)
    starts = [0, wl.n - span] + [int(x) for x in rng.integers(span, wl.n - 2 * span, size=6)]
    starts += [(1 << 30) - 3, (1 << 30) + (1 << 29) + 1, wl.n // 2 + 1]   # fp32 byte offsets cross 2^32
    before = {s: blk.host(s, s + span) for s in starts}
    hy = wl.hyper()
    say("[cfg4] 3 gpu steps")
    assert gpu_steps(blk, hy, 3) == [0, 0, 0]
    for s in starts:
        host = before[s]
        assert oracle_steps(oracle, host, hy, 3, nthreads=8) == [0, 0, 0]
        worst = assert_state_parity(blk.host(s, s + span), host, what=f"config 4 range {s}")
        say(f"[cfg4] range start {s}: worst ulp {worst}")
    # sampled check and whole-buffer properties
    blk.check()
    torch.cuda.synchronize()
    assert blk.flag_value() == 0
    assert bool(torch.all(blk.v >= 0))
    assert torch.equal(blk.p16.view(torch.int16), blk.p.to(torch.bfloat16).view(torch.int16))


def test_every_evaluation_model_block_shape_sampled(oracle):
    """One block of every model shape the paper evaluates (Table IV: 12*h^2, h = 4096..16384;
    Table VI DiT: 18*h^2, h = 1152..7168), up to 3.2e9 elements (above 2^31).  Sampled ranges
    -- head, end, seeded interior -- against the oracle, plus whole-buffer properties."""
    rng = np.random.default_rng(6)
    span = 1 << 19
    for wl in synth.shape_workloads():
        say(f"[shapes] {wl.name} n={wl.n}")
        blk = DeviceBlock(synth.make_block(wl, seed=0, device=DEV))
        starts = [0, wl.n - span] + [int(x) for x in rng.integers(span, wl.n - 2 * span, size=3)]
        before = {s: blk.host(s, s + span) for s in starts}
        hy = wl.hyper()
        assert gpu_steps(blk, hy, 1) == [0]
        for s in starts:
            host = before[s]
            assert oracle_steps(oracle, host, hy, 1, nthreads=8) == [0]
            worst = assert_state_parity(blk.host(s, s + span), host, what=f"{wl.name} @ {s}")
            assert worst == {"p": 0, "m": 0, "v": 0, "p16": 0}
        assert torch.equal(blk.p16.view(torch.int16), blk.p.to(torch.bfloat16).view(torch.int16))
        blk.norm(wl.loss_scale)
        torch.cuda.synchronize()
        sq = float(blk.sqnorm.cpu().item())
        assert blk.flag_value() == 0 and abs(sq - wl.n * 1e-6) < 0.01 * wl.n * 1e-6
        del blk, before
        torch.cuda.empty_cache()


def test_element_count_beyond_32_bits(oracle):
    """n = 2^32 + 4099 elements (68.7 GB resident, ragged): every index, offset and trip count
    in the kernels must be 64-bit.  Sampled ranges around the 2^32-element boundary, at the
    ragged end and at the head; a non-finite gradient in the very last element must raise the
    flag and skip the step."""
    n = (1 << 32) + 4099
    wl = small_workload(n)
    say(f"[2^32] n={n} generating")
    blk = DeviceBlock(synth.make_block(wl, seed=0, device=DEV))
    span = 1 << 19
    starts = [0, (1 << 32) - span // 2, (1 << 32) - 3, n - span, (1 << 31) - 7, 3 * (1 << 30) + 11]
    before = {s: blk.host(s, min(n, s + span)) for s in starts}
    hy = wl.hyper()
    blk.g.view(torch.int16)[n - 1] = 0x7C00                   # +inf in the last element
    p_tail = blk.p[n - 8:].clone()
    assert gpu_steps(blk, hy, 1) == [1]
    assert torch.equal(blk.p[n - 8:].view(torch.int32), p_tail.view(torch.int32))
    assert torch.equal(blk.p[:span].view(torch.int32),
                       torch.from_numpy(before[0]["p"]).to(DEV).view(torch.int32))
    blk.g.view(torch.int16)[n - 1] = int(before[n - span]["g"][-1]) - (
        0x10000 if before[n - span]["g"][-1] >= 0x8000 else 0)  # restore the original value
    say("[2^32] step")
    assert gpu_steps(blk, hy, 1) == [0]
    for s in starts:
        host = before[s]
        assert oracle_steps(oracle, host, hy, 1, nthreads=8) == [0]
        worst = assert_state_parity(blk.host(s, min(n, s + span)), host, what=f"2^32 range {s}")
        assert worst == {"p": 0, "m": 0, "v": 0, "p16": 0}
    blk.norm(wl.loss_scale)
    torch.cuda.synchronize()
    sq = float(blk.sqnorm.cpu().item())
    assert blk.flag_value() == 0 and abs(sq - n * 1e-6) < 0.01 * n * 1e-6
    # nothing left unwritten anywhere: the sentinel of the bf16 buffer is gone
    assert torch.equal(blk.p16.view(torch.int16), blk.p.to(torch.bfloat16).view(torch.int16))


def test_config5_ragged_overflow_skip_and_clipping(oracle):
    """Ragged 13B block (n = 12*5120^2 + 1).  With 0.01 % of the gradients set to inf/NaN the
    flag is 1 and p, m, v, p16 stay bit-identical; without them a clipping run (max-norm 1.0)
    goes through lohan_grad_sqnorm and matches the oracle."""
    wl = synth.WORKLOADS["gpt13b_ragged"]
    hy = wl.hyper()
    for seed in (0, 1):
        say(f"[cfg5] overflow run seed={seed}")
        blk = DeviceBlock(synth.make_block(wl, seed=seed, device=DEV))
        pos = synth.plant_nonfinite(blk.g, 1e-4, seed, always=(0, wl.n - 1) if seed == 0 else ())
        assert pos.numel() > 30000
        keep = {k: getattr(blk, k).clone() for k in ("p", "m", "v", "p16")}
        assert gpu_steps(blk, hy, 1) == [1]
        for k, t in keep.items():
            a, b = getattr(blk, k), t
            if a.dtype == torch.bfloat16:
                a, b = a.view(torch.int16), b.view(torch.int16)
            else:
                a, b = a.view(torch.int32), b.view(torch.int32)
            assert torch.equal(a, b), f"{k} changed on a skipped step"
        assert oracle.grad_overflow_check(synth.to_numpy_bits(blk.g)) == 1
        blk.norm(wl.loss_scale)
        torch.cuda.synchronize()
        assert blk.flag_value() == 1
        del blk, keep
    # a single non-finite value in the ragged last element is enough
    say("[cfg5] single nan at n-1")
    blk = DeviceBlock(synth.make_block(wl, seed=2, device=DEV))
    blk.g.view(torch.int16)[wl.n - 1] = 0x7E00
    p_before = blk.p.clone()
    assert gpu_steps(blk, hy, 1) == [1]
    assert torch.equal(blk.p.view(torch.int32), p_before.view(torch.int32))
    blk.g.view(torch.int16)[wl.n - 1] = 0x7BFF                # largest finite value: no overflow
    del p_before

    say("[cfg5] clipping run")
    host = blk.host()
    blk.norm(wl.loss_scale)
    torch.cuda.synchronize()
    assert blk.flag_value() == 0
    sq_gpu = float(blk.sqnorm.cpu().item())
    sq_orc = oracle.grad_sqnorm(host["g"], wl.loss_scale)
    assert abs(sq_gpu - sq_orc) <= RTOL_SQNORM * sq_orc
    assert 0.9 * wl.n * 1e-6 < sq_gpu < 1.1 * wl.n * 1e-6     # ||g||^2 ~ n * std^2, norm ~ 17.7
    s_eff_gpu = lohan.lohan_clip_loss_scale(sq_gpu, wl.loss_scale, 1.0)
    s_eff_orc = float(oracle.clip_loss_scale(sq_orc, wl.loss_scale, 1.0))
    assert abs(s_eff_gpu - s_eff_orc) <= 1e-5 * s_eff_orc
    # the step itself is compared with both sides using the oracle's effective scale, so that a
    # last-digit difference of the two norms does not leak into a bit-level comparison
    hy_clip = dict(hy, loss_scale=s_eff_orc)
    blk.step(hy_clip, flags=lohan.LOHAN_FLAG_PRECHECKED)
    torch.cuda.synchronize()
    assert oracle_steps(oracle, host, hy_clip, 1) == [0]
    worst = assert_state_parity(blk.host(), host, what="config 5 clipping run")
    say(f"[cfg5] clipping run worst ulp {worst}, sqnorm rel err {abs(sq_gpu - sq_orc) / sq_orc:.2e}")


@pytest.mark.parametrize("n", [1, 7, 8, 9, 4099, 1_000_003])
def test_overflow_patterns_and_positions(oracle, n):
    wl = small_workload(n)
    hy = wl.hyper()
    base = synth.make_block(wl, seed=3, device=DEV)
    positions = sorted({0, n - 1, n // 2, max(0, n - 2), (n // 8) * 8 % n})
    for pat in synth.NONFINITE_FP16 + (0x7BFF, 0xFBFF):
        for pos in positions:
            blk = DeviceBlock({k: t.clone() for k, t in base.items()})
            blk.g.view(torch.int16)[pos] = pat if pat < 0x8000 else pat - 0x10000
            host = blk.host()
            want = oracle.grad_overflow_check(host["g"])
            assert want == (0 if pat in (0x7BFF, 0xFBFF) else 1)
            blk.check()
            torch.cuda.synchronize()
            assert blk.flag_value() == want
            blk.flag.fill_(5)
            blk.norm(wl.loss_scale)
            torch.cuda.synchronize()
            assert blk.flag_value() == want
            blk.flag.fill_(5)
            assert gpu_steps(blk, hy, 1) == [want]
            oracle_steps(oracle, host, hy, 1, nthreads=1)
            after = blk.host()
            for k in ("p", "m", "v", "p16"):
                assert np.array_equal(after[k].view(np.uint8), host[k].view(np.uint8)), (k, pat, pos)


def test_prechecked_flag_is_honoured(oracle):
    n = 70_001
    wl = small_workload(n)
    hy = wl.hyper()
    blk = DeviceBlock(synth.make_block(wl, seed=5, device=DEV))
    host = blk.host()
    before = blk.host()
    blk.flag.fill_(1)                     # caller says: overflow
    blk.step(hy, flags=lohan.LOHAN_FLAG_PRECHECKED)
    torch.cuda.synchronize()
    after = blk.host()
    for k in ("p", "m", "v", "p16"):
        assert np.array_equal(after[k], before[k])
    assert blk.flag_value() == 1          # read-only in this mode
    blk.flag.fill_(0)
    blk.step(hy, flags=lohan.LOHAN_FLAG_PRECHECKED, stream=None)
    torch.cuda.synchronize()
    oracle_steps(oracle, host, hy, 1)
    assert_state_parity(blk.host(), host, what="prechecked")
    # prechecked calls need no workspace at all
    lohan.lohan_adam_block_step(blk.p, blk.m, blk.v, blk.g, blk.p16, n, hy["lr"], hy["beta1"],
                                hy["beta2"], hy["eps"], hy["weight_decay"], hy["step"] + 1,
                                hy["loss_scale"], blk.flag, lohan.LOHAN_FLAG_PRECHECKED, None)
    torch.cuda.synchronize()
    oracle_steps(oracle, host, dict(hy, step=hy["step"] + 1), 1)
    assert_state_parity(blk.host(), host, what="prechecked, no workspace")


@pytest.mark.parametrize("n,S,max_norm", [(1_000_003, 65536.0, 1.0), (300_007, 1024.0, 0.05),
                                          (70_001, 3000.0, 0.1), (5_000, 65536.0, 100.0),
                                          (257, 1.0, 1e-3)])
def test_device_side_clipping(oracle, n, S, max_norm):
    """lohan_adam_block_step_clipped resolves the clip coefficient on the device.  It must be
    bit-identical to the host route through lohan_clip_loss_scale (same formula, same norm).
    Against the oracle the bar has two halves: the effective loss scale each side derives from
    its own squared norm agrees to one fp32 ulp, and the oracle stepped with the HIP path's
    effective scale gives the HIP path's state bit for bit (0 ulp)."""
    wl = small_workload(n, S=S)
    hy = wl.hyper()
    base = synth.make_block(wl, seed=11, device=DEV)
    dev_route = DeviceBlock({k: t.clone() for k, t in base.items()})
    host_route = DeviceBlock({k: t.clone() for k, t in base.items()})
    host = dev_route.host()

    dev_route.norm(S)
    lohan.lohan_adam_block_step_clipped(
        dev_route.p, dev_route.m, dev_route.v, dev_route.g, dev_route.p16, n, hy["lr"],
        hy["beta1"], hy["beta2"], hy["eps"], hy["weight_decay"], hy["step"], S, dev_route.sqnorm,
        max_norm, dev_route.flag, 0, dev_route.ws)
    torch.cuda.synchronize()
    assert dev_route.flag_value() == 0

    host_route.norm(S)
    torch.cuda.synchronize()
    sq_gpu = float(host_route.sqnorm.cpu().item())
    s_eff_gpu = lohan.lohan_clip_loss_scale(sq_gpu, S, max_norm)
    host_route.step(dict(hy, loss_scale=s_eff_gpu), flags=lohan.LOHAN_FLAG_PRECHECKED)
    torch.cuda.synchronize()
    a, b = dev_route.host(), host_route.host()
    for k in ("p", "m", "v", "p16"):
        assert np.array_equal(a[k].view(np.uint8), b[k].view(np.uint8)), k

    sq_orc = oracle.grad_sqnorm(host["g"], S)
    assert abs(sq_gpu - sq_orc) <= RTOL_SQNORM * sq_orc
    s_eff_orc = float(oracle.clip_loss_scale(sq_orc, S, max_norm))
    if max_norm >= 100.0:
        assert s_eff_orc == S                                  # norm below the threshold
    else:
        assert s_eff_orc > S                                   # really clipped
    assert_scale_within_one_ulp(s_eff_gpu, s_eff_orc, what="device-side clipping")
    oracle_steps(oracle, host, dict(hy, loss_scale=s_eff_gpu), 1, nthreads=4)
    worst = assert_state_parity(a, host, what="device-side clipping")
    assert worst == {"p": 0, "m": 0, "v": 0, "p16": 0}, worst

    # an overflowing block is skipped whatever the norm holds
    skip = DeviceBlock({k: t.clone() for k, t in base.items()})
    skip.g.view(torch.int16)[n // 2] = 0x7C00
    before = skip.host()
    skip.norm(S)
    lohan.lohan_adam_block_step_clipped(
        skip.p, skip.m, skip.v, skip.g, skip.p16, n, hy["lr"], hy["beta1"], hy["beta2"],
        hy["eps"], hy["weight_decay"], hy["step"], S, skip.sqnorm, max_norm, skip.flag,
        lohan.LOHAN_FLAG_L2_MODE, skip.ws)
    torch.cuda.synchronize()
    assert skip.flag_value() == 1
    after = skip.host()
    for k in ("p", "m", "v", "p16"):
        assert np.array_equal(after[k].view(np.uint8), before[k].view(np.uint8)), k


@pytest.mark.parametrize("S", [65536.0, 1024.0, 3000.0, 1.0])
def test_sqnorm_parity_and_determinism(oracle, S):
    # 4096 elements per workgroup: 131072 / 135168 elements are 32 / 33 workgroups, the sizes at
    # which the ticket goes from one level to two; 4_190_209 makes 1023 + a ragged last group
    for n in (0, 1, 5, 8, 2047, 8192, 8193, 65537, 131_072, 131_073, 135_168, 262_149,
              3_000_001, 4_190_209, 40_000_003):
        wl = small_workload(n, S=S)
        blk = DeviceBlock(synth.make_block(wl, seed=n % 97, device=DEV))
        blk.norm(S)
        torch.cuda.synchronize()
        got = float(blk.sqnorm.cpu().item())
        want = oracle.grad_sqnorm(synth.to_numpy_bits(blk.g), S)
        assert abs(got - want) <= RTOL_SQNORM * want, (n, got, want)
        assert blk.flag_value() == 0
        blk.sqnorm.fill_(-1.0)
        blk.norm(S, want_flag=False)
        torch.cuda.synchronize()
        assert float(blk.sqnorm.cpu().item()) == got          # fixed-order reduction
    # all-subnormal gradients are not flushed: n * (2^-24)^2 / S^2
    n = 10_000
    blk = DeviceBlock(synth.make_block(small_workload(n, S=S), seed=0, device=DEV))
    blk.g.view(torch.int16).fill_(1)
    blk.norm(S)
    torch.cuda.synchronize()
    want = oracle.grad_sqnorm(synth.to_numpy_bits(blk.g), S)
    assert want > 0 and abs(float(blk.sqnorm.cpu().item()) - want) <= RTOL_SQNORM * want


def test_denormals_and_extremes_bit_exact(oracle):
    """Hand-placed extreme values: subnormal gradients, moments and parameters, the largest fp16
    value, signed zeros -- the regions where flush-to-zero or an approximate divide would show."""
    n = 4096 + 3
    wl = small_workload(n)
    t = synth.make_block(wl, seed=9, device=DEV)
    edge32 = torch.tensor([0.0, -0.0, 1e-38, -1e-38, 1.4e-45, 3e-39, 1e-30, 1e-20, 1.0, -1.0,
                           123.456, -7.5e3, 2.0 ** -126, 2.0 ** -127, 1e10, 3e-41],
                          dtype=torch.float32, device=DEV)
    edge16 = torch.tensor([0x0000, 0x0001, -0x7FFF, 0x03FF, 0x0400, 0x7BFF, -0x0401, 0x3C00,
                           -0x4400, 0x3555, 0x0200, 0x6400, -0x8000, 0x0002, 0x7BFE, 0x1234],
                          dtype=torch.int16, device=DEV)
    k = edge32.numel()
    for rep in range(0, n - 4 * k, 4 * k):
        t["p"][rep:rep + k] = edge32
        t["m"][rep + k:rep + 2 * k] = edge32 * 1e-3
        t["v"][rep + 2 * k:rep + 3 * k] = edge32.abs()
        t["g"].view(torch.int16)[rep + (rep // 7) % k:rep + (rep // 7) % k + k] = edge16
    for l2_mode in (False, True):
        blk = DeviceBlock({kk: x.clone() for kk, x in t.items()})
        host = blk.host()
        hy = wl.hyper()
        assert gpu_steps(blk, hy, 10, l2_mode=l2_mode) == [0] * 10
        oracle_steps(oracle, host, hy, 10, l2_mode=l2_mode, nthreads=1)
        got = blk.host()
        for kk in ("p", "m", "v", "p16"):
            assert np.array_equal(got[kk].view(np.uint8), host[kk].view(np.uint8)), (kk, l2_mode)


def test_other_hyperparameters(oracle):
    n = 300_007
    cases = [
        dict(lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, step=1, loss_scale=1024.0),
        dict(lr=3e-3, beta1=0.8, beta2=0.95, eps=1e-6, weight_decay=0.1, step=7, loss_scale=3000.0),
        dict(lr=1e-4, beta1=0.0, beta2=0.5, eps=1e-3, weight_decay=0.01, step=3, loss_scale=1.0),
        dict(lr=0.0, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.5, step=12345678,
             loss_scale=2346.2798),
    ]
    for i, hy in enumerate(cases):
        hy = {k: (float(np.float32(v)) if k != "step" else v) for k, v in hy.items()}
        for l2_mode in (False, True):
            wl = small_workload(n, S=hy["loss_scale"])
            blk = DeviceBlock(synth.make_block(wl, seed=i, device=DEV))
            host = blk.host()
            assert gpu_steps(blk, hy, 3, l2_mode=l2_mode) == [0, 0, 0]
            oracle_steps(oracle, host, hy, 3, l2_mode=l2_mode)
            assert_state_parity(blk.host(), host, what=f"hyper case {i} l2={l2_mode}")


def test_empty_block_defines_outputs():
    blk = DeviceBlock(synth.make_block(small_workload(0), seed=0, device=DEV))
    blk.check()
    torch.cuda.synchronize()
    assert blk.flag_value() == 0
    blk.flag.fill_(9)
    blk.norm(1024.0)
    torch.cuda.synchronize()
    assert blk.flag_value() == 0 and float(blk.sqnorm.cpu().item()) == 0.0
    blk.flag.fill_(9)
    blk.step(small_workload(0).hyper())
    torch.cuda.synchronize()
    assert blk.flag_value() == 0


def test_blocks_on_two_side_streams_behind_gemms(oracle):
    """The streaming pattern of active gradient offloading: blocks arrive with decreasing index
    while backward GEMMs run on the main stream; each block step is issued on one of two side
    streams behind the event of its GEMM.  Every block must match the oracle."""
    nblocks, n = 12, 2_000_003
    wl = small_workload(n)
    hy = wl.hyper()
    blocks = [DeviceBlock(synth.make_block(wl, seed=100 + i, device=DEV)) for i in range(nblocks)]
    hosts = [b.host() for b in blocks]
    side = [torch.cuda.Stream(), torch.cuda.Stream()]
    a = torch.randn(1024, 2048, device=DEV, dtype=torch.bfloat16)
    b = torch.randn(2048, 4096, device=DEV, dtype=torch.bfloat16)
    main = torch.cuda.current_stream()
    for i in reversed(range(nblocks)):
        torch.matmul(a, b)
        ev = torch.cuda.Event()
        ev.record(main)
        s = side[i % 2]
        s.wait_event(ev)
        blocks[i].step(hy, stream=s)
    for s in side:
        s.synchronize()
    torch.cuda.synchronize()
    for i in range(nblocks):
        assert blocks[i].flag_value() == 0
        oracle_steps(oracle, hosts[i], hy, 1)
        assert_state_parity(blocks[i].host(), hosts[i], what=f"block {i}")


def test_same_input_same_bits():
    n = 5_000_011
    wl = small_workload(n)
    outs = []
    for _ in range(2):
        blk = DeviceBlock(synth.make_block(wl, seed=42, device=DEV))
        gpu_steps(blk, wl.hyper(), 2)
        blk.norm(wl.loss_scale)
        torch.cuda.synchronize()
        outs.append((blk.host(), float(blk.sqnorm.cpu().item())))
    for k in ("p", "m", "v", "p16"):
        assert np.array_equal(outs[0][0][k], outs[1][0][k])
    assert outs[0][1] == outs[1][1]


def test_step_can_be_captured_in_a_hip_graph(oracle):
    """The entry points allocate nothing, never synchronise and issue no memsets, so a caller may
    capture norm + step into a HIP graph and replay it.  Three replays with eager work and
    synchronisations between them; every replay is checked against the oracle (the step index is
    baked into the captured launch, so each replay repeats step 100 on the evolving state)."""
    n = 1_000_003
    wl = small_workload(n)
    hy = wl.hyper()
    blk = DeviceBlock(synth.make_block(wl, seed=8, device=DEV))
    host = blk.host()
    # warm-up outside capture (first-use initialisation must not happen while capturing)
    warm = DeviceBlock(synth.make_block(small_workload(4096), seed=1, device=DEV))
    warm.norm(wl.loss_scale)
    warm.step(wl.hyper(), flags=lohan.LOHAN_FLAG_PRECHECKED)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            blk.norm(wl.loss_scale, stream=side)
            blk.step(hy, flags=lohan.LOHAN_FLAG_PRECHECKED, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    # capture itself executes nothing
    assert np.array_equal(blk.host()["p"].view(np.uint32), host["p"].view(np.uint32))

    scratch = torch.zeros(1 << 20, device=DEV)
    for r in range(3):
        graph.replay()
        torch.cuda.synchronize()
        assert oracle_steps(oracle, host, hy, 1, nthreads=8) == [0]
        worst = assert_state_parity(blk.host(), host, what=f"graph replay {r}")
        assert worst == {"p": 0, "m": 0, "v": 0, "p16": 0}
        want = oracle.grad_sqnorm(host["g"], wl.loss_scale)
        assert abs(float(blk.sqnorm.cpu().item()) - want) <= RTOL_SQNORM * want
        scratch.add_(1.0)                       # eager work between replays
        warm.norm(wl.loss_scale)
        torch.cuda.synchronize()
    assert float(scratch[0].cpu()) == 3.0


def test_13b_blocks_in_the_library_placement(oracle):
    """The layout bench.py times: a full group of 13B-shaped blocks inside one slab at the offsets
    lohan_model_placement gives (fp32 arrays in three lanes, 4 GiB + 8 MiB and 8 GiB + 9 MiB from
    the first).  All
    blocks are stepped; block 0 is compared with the oracle over every element, the others on
    sampled ranges -- an overlap between any two arrays would corrupt one of them."""
    wl = synth.WORKLOADS["gpt13b"]
    n = wl.n
    offsets, slab_bytes, align, group = lohan.lohan_model_placement(n)
    assert group == 3
    slab = torch.empty(slab_bytes + align, dtype=torch.uint8, device=DEV)
    start = (-slab.data_ptr()) % align
    fields = {"p": "param_fp32", "m": "exp_avg", "v": "exp_avg_sq", "g": "grad_fp16",
              "p16": "param_bf16"}
    blocks = []
    for b in range(group):
        src = synth.make_block(wl, seed=40 + b, device=DEV)
        placed = {}
        for k, field in fields.items():
            off = start + offsets[b][field]
            placed[k] = slab[off: off + n * src[k].element_size()].view(src[k].dtype)
            placed[k].copy_(src[k])
        blocks.append(DeviceBlock(placed))
        del src
    assert blocks[0].m.data_ptr() - blocks[0].p.data_ptr() == (4 << 30) + (8 << 20)
    assert blocks[0].v.data_ptr() - blocks[0].p.data_ptr() == (8 << 30) + (9 << 20)
    span = 1 << 21
    rng = np.random.default_rng(17)
    starts = [0, n - span] + [int(x) for x in rng.integers(span, n - 2 * span, size=2)]
    full0 = blocks[0].host()
    before = [None] + [{s: blk.host(s, s + span) for s in starts} for blk in blocks[1:]]
    hy = wl.hyper()
    for blk in blocks:
        assert gpu_steps(blk, hy, 2) == [0, 0]
    say("[placement] oracle on block 0")
    assert oracle_steps(oracle, full0, hy, 2) == [0, 0]
    worst = assert_state_parity(blocks[0].host(), full0, what="library placement, block 0")
    assert worst == {"p": 0, "m": 0, "v": 0, "p16": 0}
    for b in (1, 2):
        for s in starts:
            host = before[b][s]
            assert oracle_steps(oracle, host, hy, 2, nthreads=8) == [0, 0]
            worst = assert_state_parity(blocks[b].host(s, s + span), host,
                                        what=f"library placement, block {b} range {s}")
            assert worst == {"p": 0, "m": 0, "v": 0, "p16": 0}


def nan_aware_equal(got: np.ndarray, want: np.ndarray, nan_mask_fn) -> bool:
    """Bit equality, except that a NaN on one side only has to be a NaN on the other (payload and
    sign of a NaN are not part of the contract)."""
    gn, wn = nan_mask_fn(got), nan_mask_fn(want)
    return bool(np.array_equal(gn, wn) and np.array_equal(got[~gn], want[~wn]))


def test_random_bit_patterns_and_hyperparameters(oracle):
    """Seeded differential test far outside the training regime: p and m are arbitrary finite
    float32 bit patterns, v arbitrary non-negative ones, g arbitrary finite binary16 patterns, the
    hyper-parameters log-uniform over many decades -- so squares overflow, sums cancel, quotients
    underflow and inf - inf appears.  In place and out of place; every non-NaN result must match
    the oracle bit for bit, and NaNs must appear in the same places."""
    rng = np.random.default_rng(2403)
    n = 50_003

    def finite32(count):
        bits = rng.integers(0, 1 << 32, size=count, dtype=np.uint64).astype(np.uint32)
        bits = np.where((bits & 0x7F800000) == 0x7F800000, bits & 0xBFFFFFFF, bits)
        return bits

    f32nan = lambda a: np.isnan(a.view(np.float32))
    bf16nan = lambda a: ((a & 0x7F80) == 0x7F80) & ((a & 0x007F) != 0)
    f16nan = lambda a: ((a & 0x7C00) == 0x7C00) & ((a & 0x03FF) != 0)
    for case in range(24):
        p = finite32(n)
        m = finite32(n)
        v = finite32(n) & 0x7FFFFFFF
        g = rng.integers(0, 1 << 16, size=n, dtype=np.uint32).astype(np.uint16)
        g = np.where((g & 0x7C00) == 0x7C00, g & 0xBFFF, g).astype(np.uint16)
        hy = dict(lr=float(np.float32(10 ** rng.uniform(-6, -1))),
                  beta1=float(np.float32(rng.uniform(0, 0.999))),
                  beta2=float(np.float32(rng.uniform(0.5, 0.9999))),
                  eps=float(np.float32(10 ** rng.uniform(-10, -3))),
                  weight_decay=float(np.float32(rng.uniform(0, 0.3))),
                  step=int(rng.integers(1, 1_000_000)),
                  loss_scale=float(np.float32(2.0 ** rng.integers(0, 17) if case % 2 else
                                              10 ** rng.uniform(0, 5))))
        l2, half = bool(case & 1), bool(case & 2)
        flags = (lohan.LOHAN_FLAG_L2_MODE if l2 else 0) | (lohan.LOHAN_FLAG_P16_FP16 if half else 0)
        host = {"p": p.view(np.float32).copy(), "m": m.view(np.float32).copy(),
                "v": v.view(np.float32).copy(), "g": g.copy(),
                "p16": np.zeros(n, dtype=np.uint16)}
        dev = {k: torch.from_numpy(host[k].copy()).to(DEV) for k in ("p", "m", "v")}
        dev["g"] = torch.from_numpy(g.view(np.int16).copy()).to(DEV).view(torch.float16)
        dev["p16"] = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
        out = {k: torch.empty_like(dev[k]) for k in ("p", "m", "v", "p16")}
        flag = torch.full((1,), 3, dtype=torch.int32, device=DEV)
        lohan.lohan_adam_block_step_out_of_place(
            dev["p"], dev["m"], dev["v"], dev["g"], out["p"], out["m"], out["v"], out["p16"], n,
            hy["lr"], hy["beta1"], hy["beta2"], hy["eps"], hy["weight_decay"], hy["step"],
            hy["loss_scale"], flag, flags)
        blk = DeviceBlock(dev)
        blk.step(hy, flags=flags)
        torch.cuda.synchronize()
        assert blk.flag_value() == 0 and int(flag.cpu().item()) == 0
        assert oracle.adam_block_step(host["p"], host["m"], host["v"], host["g"], host["p16"],
                                      nthreads=4, l2_mode=l2, half_out=half, **hy) == 0
        in_place = blk.host()
        oop = {k: synth.to_numpy_bits(out[k]) for k in ("p", "m", "v", "p16")}
        nan16 = f16nan if half else bf16nan
        for name, got in (("in place", in_place), ("out of place", oop)):
            for k in ("p", "m", "v"):
                assert nan_aware_equal(got[k].view(np.uint32), host[k].view(np.uint32),
                                       f32nan), (case, name, k, hy)
            assert nan_aware_equal(got["p16"], host["p16"], nan16), (case, name, "p16", hy)
        # a second step in place on the state the first one left (now holding infinities):
        # inf / inf and inf - inf turn up, and must turn up in the same elements
        hy2 = dict(hy, step=hy["step"] + 1)
        blk.step(hy2, flags=flags)
        torch.cuda.synchronize()
        assert oracle.adam_block_step(host["p"], host["m"], host["v"], host["g"], host["p16"],
                                      nthreads=4, l2_mode=l2, half_out=half, **hy2) == 0
        got = blk.host()
        for k in ("p", "m", "v"):
            assert nan_aware_equal(got[k].view(np.uint32), host[k].view(np.uint32),
                                   f32nan), (case, "second step", k, hy)
        assert nan_aware_equal(got["p16"], host["p16"], nan16), (case, "second step", "p16", hy)
        say(f"[random] case {case}: {int(np.isnan(host['p']).sum())} NaN, "
            f"{int(np.isinf(host['p']).sum())} inf of {n} parameters after two steps")


def test_unprepared_workspace_fails_on_the_safe_side(oracle):
    """A workspace that lohan_workspace_init never saw (here: filled with a byte pattern, so its
    ticket counters hold garbage) must not leave a stale flag behind: the reducing calls report
    flag 1 and a NaN norm, and the self-checking step writes nothing.  Once prepared, the same
    memory works."""
    n = 300_007
    wl = small_workload(n)
    hy = wl.hyper()
    blk = DeviceBlock(synth.make_block(wl, seed=3, device=DEV))
    before = blk.host()
    for fill in (0xA5, 0x00, 0xFF):
        raw = torch.full((lohan.lohan_workspace_bytes(),), fill, dtype=torch.uint8, device=DEV)
        blk.flag.fill_(0)
        blk.sqnorm.fill_(0.0)
        lohan.lohan_grad_sqnorm(blk.g, n, wl.loss_scale, blk.sqnorm, blk.flag, raw)
        torch.cuda.synchronize()
        assert blk.flag_value() == 1 and np.isnan(float(blk.sqnorm.cpu().item())), fill
        blk.flag.fill_(0)
        lohan.lohan_grad_overflow_check(blk.g, n, blk.flag, raw)
        torch.cuda.synchronize()
        assert blk.flag_value() == 1, fill
        blk.flag.fill_(0)
        lohan.lohan_adam_block_step(blk.p, blk.m, blk.v, blk.g, blk.p16, n, hy["lr"], hy["beta1"],
                                    hy["beta2"], hy["eps"], hy["weight_decay"], hy["step"],
                                    hy["loss_scale"], blk.flag, 0, raw)
        torch.cuda.synchronize()
        assert blk.flag_value() == 1
        after = blk.host()
        for k in ("p", "m", "v", "p16"):
            assert np.array_equal(after[k].view(np.uint8), before[k].view(np.uint8)), (fill, k)
    lohan.lohan_workspace_init(raw)
    lohan.lohan_adam_block_step(blk.p, blk.m, blk.v, blk.g, blk.p16, n, hy["lr"], hy["beta1"],
                                hy["beta2"], hy["eps"], hy["weight_decay"], hy["step"],
                                hy["loss_scale"], blk.flag, 0, raw)
    torch.cuda.synchronize()
    assert blk.flag_value() == 0
    assert oracle_steps(oracle, before, hy, 1, nthreads=4) == [0]
    worst = assert_state_parity(blk.host(), before, what="after preparing the workspace")
    assert worst == {"p": 0, "m": 0, "v": 0, "p16": 0}
