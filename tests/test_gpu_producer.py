"""GPU parity of lohan_grad_produce_fp16: the gradient producer with the block's overflow flag and
squared norm in its epilogue (fp32 accumulator -> the G16 tensor of Table II), and of the 28
B/element step that follows it with LOHAN_FLAG_PRECHECKED."""
import numpy as np
import pytest
import torch

import paper_2403_06504_amd as lohan
from paper_2403_06504_amd import synthetic_inputs as synth

from gpu_util import RTOL_SQNORM, DeviceBlock, assert_state_parity, oracle_steps

pytestmark = pytest.mark.gpu
DEV = "cuda"
SIZES = list(range(0, 10)) + [255, 256, 257, 2047, 2048, 2049, 8191, 65537, 1_000_003, 5_000_001]


def accumulator(n, seed, S):
    """fp32 gradients as backward leaves them: N(0, 1e-3) times the loss scale."""
    gen = torch.Generator(device=DEV)
    gen.manual_seed(1000 + seed)
    x = torch.randn(max(n, 1), generator=gen, device=DEV, dtype=torch.float32)[:n]
    return (x * (1e-3 * S)).contiguous()


def produce(src, mul, S, want_norm=True):
    n = src.numel()
    out = torch.full((n,), -3.0, dtype=torch.float16, device=DEV)
    flag = torch.full((1,), 7, dtype=torch.int32, device=DEV)
    sq = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
    ws = lohan.new_workspace(DEV)
    lohan.lohan_grad_produce_fp16(src, n, mul, out, S, sq if want_norm else None, flag, ws)
    torch.cuda.synchronize()
    return out, int(flag.cpu().item()), float(sq.cpu().item())


@pytest.mark.parametrize("mul,S", [(1.0, 65536.0), (0.25, 65536.0), (1.0 / 3.0, 1024.0)])
def test_producer_output_flag_and_norm(oracle, mul, S):
    for n in SIZES:
        src = accumulator(n, n % 89, S)
        if n > 4:                                  # subnormal, tie and near-overflow products
            src[1], src[2], src[3] = 3e-8 / mul, 65519.0 / mul, (1.0 + 2.0 ** -11) / mul
        out, flag, sq = produce(src, mul, S)
        want = oracle.grad_produce(src.cpu().numpy(), mul)
        got = synth.to_numpy_bits(out)
        assert np.array_equal(got, want), (n, mul)
        assert flag == oracle.grad_overflow_check(want) == 0, n
        ref = oracle.grad_sqnorm(want, S)
        assert abs(sq - ref) <= RTOL_SQNORM * ref, (n, sq, ref)
        _, flag2, sq2 = produce(src, mul, S)
        assert (flag2, sq2) == (flag, sq)          # fixed-order reduction: same bits again
        _, flag3, _ = produce(src, mul, S, want_norm=False)
        assert flag3 == 0


def test_producer_overflow_comes_from_the_cast_or_from_the_input(oracle):
    n = 300_007
    for where in (0, 1, n // 2, n - 2, n - 1):
        for value in (70000.0, -1e30, float("inf"), float("nan")):
            src = accumulator(n, 5, 65536.0)
            src[where] = value
            out, flag, _ = produce(src, 1.0, 65536.0)
            want = oracle.grad_produce(src.cpu().numpy(), 1.0)
            got = synth.to_numpy_bits(out)
            finite = ~np.isnan(want.view(np.float16))
            assert np.array_equal(got[finite], want[finite])
            assert (got[where] & 0x7C00) == 0x7C00
            assert flag == oracle.grad_overflow_check(want) == 1, (where, value)
    src = accumulator(n, 6, 65536.0)
    src[7] = 65504.0                               # the largest finite binary16: not an overflow
    assert produce(src, 1.0, 65536.0)[1] == 0


def test_step_after_the_producer_needs_no_check_pass(oracle):
    """producer -> lohan_adam_block_step(PRECHECKED): the whole step without the 2 B/element
    pass, against the oracle run on the oracle's own G16; and an overflowing accumulator leaves
    the state untouched."""
    n, S, mul = 1_000_003, 65536.0, 0.5
    wl = synth.Workload(name="p", n=n, step=100, loss_scale=S, zero_moments=False)
    hy = wl.hyper()
    for overflow in (False, True):
        blk = DeviceBlock(synth.make_block(wl, seed=12, device=DEV))
        src = accumulator(n, 9, S) * 2.0
        if overflow:
            src[n - 1] = 1e9
        host = blk.host()
        before = {k: host[k].copy() for k in ("p", "m", "v", "p16")}
        lohan.lohan_grad_produce_fp16(src, n, mul, blk.g, S, blk.sqnorm, blk.flag, blk.ws)
        lohan.lohan_adam_block_step(blk.p, blk.m, blk.v, blk.g, blk.p16, n, hy["lr"], hy["beta1"],
                                    hy["beta2"], hy["eps"], hy["weight_decay"], hy["step"], S,
                                    blk.flag, lohan.LOHAN_FLAG_PRECHECKED, None)
        torch.cuda.synchronize()
        host["g"] = oracle.grad_produce(src.cpu().numpy(), mul)
        assert oracle_steps(oracle, host, hy, 1, nthreads=4) == [int(overflow)]
        assert blk.flag_value() == int(overflow)
        got = blk.host()
        assert np.array_equal(got["g"], host["g"]) or overflow
        if overflow:
            for k in ("p", "m", "v", "p16"):
                assert np.array_equal(got[k].view(np.uint8), before[k].view(np.uint8)), k
        else:
            worst = assert_state_parity(got, host, what="step after the producer")
            assert worst == {"p": 0, "m": 0, "v": 0, "p16": 0}, worst


def test_producer_on_the_13b_block_shape(oracle):
    """The bench's block shape in the bench's launch configuration: whole-array flag and norm,
    output bits on sampled ranges (first, last, seeded interior)."""
    wl = synth.WORKLOADS["gpt13b"]
    n, S = wl.n, wl.loss_scale
    src = accumulator(n, 3, S)
    out, flag, sq = produce(src, 0.5, S)
    assert flag == 0
    span = 1 << 21
    rng = np.random.default_rng(5)
    for lo in [0, n - span] + [int(x) for x in rng.integers(span, n - 2 * span, size=3)]:
        want = oracle.grad_produce(src[lo:lo + span].cpu().numpy(), 0.5)
        assert np.array_equal(synth.to_numpy_bits(out[lo:lo + span]), want), lo
    ref = oracle.grad_sqnorm(synth.to_numpy_bits(out), S)
    assert abs(sq - ref) <= RTOL_SQNORM * ref, (sq, ref)
    src[n - 3] = 1e9
    assert produce(src, 0.5, S)[1] == 1
