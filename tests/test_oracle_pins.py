"""Pins for the CPU oracle (oracle/lohan_oracle.c) -- none of these touch the HIP path.

The paper (Sec. IV-C "CPU Compute" step; Table II tensors; Adam per Sec. II) prints no numbers for
the step, so the oracle is pinned against: hand examples (tests/golden), an exact-rational
re-evaluation, the closed form of the first Adam step, a float64 evaluation of the textbook
formula, a library AdamW/Adam, library number-format conversions, brute force over all fp16 bit
patterns, and invariants.  Each pin is aimed at a class of plausible mistakes (named in its
docstring).
"""
import json
import os
import struct

import numpy as np
import pytest
import torch

from oracle import exact, textbook_f64

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_examples.json")

HY = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)


def f32(x):
    return np.float32(x)


def bits32(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def hexlist(a):
    return [f"0x{int(x):08X}" for x in a]


def ulp_diff(a, b):
    """Distance in units in the last place between two float32 arrays (monotone integer map)."""
    ia = bits32(a).astype(np.int64)
    ib = bits32(b).astype(np.int64)
    ia = np.where(ia & 0x80000000, 0x80000000 - ia, ia)
    ib = np.where(ib & 0x80000000, 0x80000000 - ib, ib)
    return np.abs(ia - ib)


def rand_block(n, seed, S=65536.0, zero_moments=False, g_std=1e-3):
    rng = np.random.default_rng(seed)
    p = (rng.standard_normal(n) * 0.02).astype(np.float32)
    g = (rng.standard_normal(n) * g_std * S).astype(np.float16).view(np.uint16).copy()
    if zero_moments:
        m = np.zeros(n, np.float32)
        v = np.zeros(n, np.float32)
    else:
        m = (rng.standard_normal(n) * 1e-4).astype(np.float32)
        v = np.abs(rng.standard_normal(n) * 1e-7).astype(np.float32)
    return p, m, v, g


def run_oracle(oracle, p, m, v, g, **hy):
    p, m, v = p.copy(), m.copy(), v.copy()
    h = np.full(p.size, 0xDEAD, dtype=np.uint16)
    flag = oracle.adam_block_step(p, m, v, g, h, **hy)
    return flag, p, m, v, h


# ------------------------------------------------------------------------------ golden examples

def _golden():
    with open(GOLDEN) as f:
        return json.load(f)


@pytest.mark.parametrize("idx", [0, 1, 2])
def test_hand_examples_bit_exact(oracle, idx):
    """Catches: any wrong term, sign, operand order, rounding point, decay placement, L2 vs
    decoupled mix-up -- the stored bits were derived by hand, independently of the C code."""
    ex = _golden()["examples"][idx]
    hy = dict(ex["hyper"])
    p = np.array(ex["p"], np.float32)
    m = np.array(ex["m"], np.float32)
    v = np.array(ex["v"], np.float32)
    g = np.array([int(x, 16) for x in ex["g16"]], np.uint16)
    flag, p2, m2, v2, h = run_oracle(oracle, p, m, v, g, **hy)
    assert flag == 0
    assert hexlist(bits32(p2)) == [x.upper().replace("0X", "0x") for x in ex["p_out"]]
    assert hexlist(bits32(m2)) == [x.upper().replace("0X", "0x") for x in ex["m_out"]]
    assert hexlist(bits32(v2)) == [x.upper().replace("0X", "0x") for x in ex["v_out"]]
    assert [f"0x{int(x):04X}" for x in h] == ex["bf16_out"]
    if "p_out_f64" in ex:
        np.testing.assert_allclose(p2.astype(np.float64), ex["p_out_f64"], rtol=2e-7, atol=1e-12)


@pytest.mark.parametrize("idx", [0, 1])
def test_hand_scalars(oracle, idx):
    """Catches: bias correction with the wrong exponent/base, bc computed in fp32 instead of
    float64-then-round, a missing sqrt on bc2, lr*bc1 instead of lr/bc1, decay = lr*wd."""
    ex = _golden()["examples"][idx]
    hy = ex["hyper"]
    sc = oracle.step_scalars(hy["lr"], hy["beta1"], hy["beta2"], hy["weight_decay"], hy["step"],
                             hy["loss_scale"])
    for k, want in ex["scalars"].items():
        got = struct.unpack("<I", struct.pack("<f", float(sc[k])))[0]
        assert got == int(want, 16), (k, hex(got), want)


def test_bf16_golden_samples(oracle):
    for s in _golden()["bf16_rne_samples"]:
        x = np.array([int(s["f32"], 16)], np.uint32).view(np.float32)[0]
        assert oracle.float_to_bf16_bits(x) == int(s["bf16"], 16), s["note"]


def test_fp16_golden_encodings(oracle):
    for text, enc in _golden()["fp16_encodings"].items():
        got = float(oracle.half_bits_to_float(int(enc, 16)))
        if text == "nan":
            assert np.isnan(got)
        else:
            assert got == float(text)


def test_clipping_golden(oracle):
    c = _golden()["clipping"]
    g = np.array(c["g"], np.float64) * c["loss_scale"]
    g16 = g.astype(np.float16).view(np.uint16).copy()
    sq = oracle.grad_sqnorm(g16, c["loss_scale"])
    assert sq == c["sqnorm"]
    s_eff = oracle.clip_loss_scale(sq, c["loss_scale"], c["max_norm"])
    assert abs(float(s_eff) - c["loss_scale_eff"]) < 2e-3
    assert abs(np.sqrt(sq) - c["norm"]) < 1e-6
    # below the threshold nothing is clipped
    assert float(oracle.clip_loss_scale(0.25, 1024.0, 1.0)) == 1024.0


# ----------------------------------------------------------------------- exact rational evaluation

EDGE_F32 = [0.0, 1.0, -1.0, 1e-38, -1e-38, 1.4e-45, 3.0e-39, 1e-20, 0.02, -0.02, 1e-4, 123.456,
            -7.5e3, 2.0 ** -126, 2.0 ** -127]
EDGE_F16 = [0x0000, 0x0001, 0x8001, 0x03FF, 0x0400, 0x7BFF, 0xFBFF, 0x3C00, 0xBC00, 0x3555,
            0x0200, 0x6400]


@pytest.mark.parametrize("l2_mode", [False, True])
@pytest.mark.parametrize("case", [
    dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, step=100, loss_scale=65536.0),
    dict(lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, step=1, loss_scale=1024.0),
    dict(lr=3e-3, beta1=0.8, beta2=0.95, eps=1e-6, weight_decay=0.1, step=7, loss_scale=3000.0),
    dict(lr=1e-4, beta1=0.0, beta2=0.5, eps=1e-3, weight_decay=0.01, step=3, loss_scale=1.0),
    dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, step=1000,
         loss_scale=2346.2798),
])
def test_matches_exact_rational_arithmetic(oracle, case, l2_mode):
    """Catches: compiler contraction into FMA, double-precision intermediates, wrong fp16
    decoding, flush-to-zero, a bf16 rounding that truncates or rounds half away."""
    n = 160
    seed = hash((case["step"], l2_mode)) % 1000
    p, m, v, g = rand_block(n, seed, S=case["loss_scale"])
    rng = np.random.default_rng(seed + 1)
    k = len(EDGE_F32)
    p[:k] = np.array(EDGE_F32, np.float32)
    m[k:2 * k] = np.array(EDGE_F32, np.float32) * np.float32(1e-3)
    v[2 * k:3 * k] = np.abs(np.array(EDGE_F32, np.float32))
    g[:len(EDGE_F16)] = np.array(EDGE_F16, np.uint16)
    g[3 * k:3 * k + len(EDGE_F16)] = np.array(EDGE_F16, np.uint16)
    perm = rng.permutation(n)
    g = g[perm].copy()
    hy = dict(case, l2_mode=l2_mode, half_out=(case["step"] % 2 == 1))
    flag, p2, m2, v2, h = run_oracle(oracle, p, m, v, g, **hy)
    assert flag == 0
    ep, em, ev, eh = exact.adam_block_step_exact(
        [int(x) for x in bits32(p)], [int(x) for x in bits32(m)], [int(x) for x in bits32(v)],
        [int(x) for x in g], **hy)

    def same(got_bits, want_bits, width_mask):
        got = np.asarray(got_bits, dtype=np.uint64)
        want = np.asarray(want_bits, dtype=np.uint64)
        # the rational evaluator has no signed zero: +-0 compare equal
        gz = (got & width_mask) == 0
        wz = (want & width_mask) == 0
        return bool(np.all((got == want) | (gz & wz)))

    assert same(bits32(p2), ep, 0x7FFFFFFF)
    assert same(bits32(m2), em, 0x7FFFFFFF)
    assert same(bits32(v2), ev, 0x7FFFFFFF)
    assert same(h, eh, 0x7FFF)


def test_exact_evaluator_bias_correction_is_unambiguous():
    """The rational evaluator rounds the exact 1-beta^t to fp32; the oracle rounds the float64
    value of it.  Show that both roundings coincide for the (beta, t) pairs used in the tests
    (they could only differ if the exact value sat within ~2^-51 of an fp32 rounding boundary)."""
    from fractions import Fraction
    for beta in (0.9, 0.999, 0.8, 0.95, 0.5, 0.0):
        b32 = float(np.float32(beta))
        b = exact.float_to_frac(beta)
        for t in list(range(1, 120)) + [1000, 1001, 1009]:
            via_f64 = exact.rn32(Fraction(1.0 - b32 ** t))
            assert via_f64 == exact.rn32(Fraction(1) - b ** t), (beta, t)


# ------------------------------------------------------------------------------------ closed form

def test_first_step_closed_form(oracle):
    """t=1, m=v=0, wd=0, p=0: p' = -lr*sign(g) for |g| >> eps, 0 for g=0; m'=(1-b1)g,
    v'=(1-b2)g^2.  Catches: missing bias correction, eps inside the sqrt, wrong sign of the
    update, a missing unscale."""
    n = 4096
    S = 1024.0
    rng = np.random.default_rng(3)
    gf = rng.standard_normal(n) * 1e-3
    gf[:8] = 0.0
    g16 = (gf * S).astype(np.float16)
    g = g16.view(np.uint16).copy()
    gval = g16.astype(np.float64) / S
    p0 = np.zeros(n, np.float32)
    z = np.zeros(n, np.float32)
    lr = 1e-2
    flag, p, m, v, h = run_oracle(oracle, p0, z, z, g, lr=lr, beta1=0.9, beta2=0.999, eps=1e-8,
                                  weight_decay=0.0, step=1, loss_scale=S)
    assert flag == 0
    big = np.abs(gval) > 1e-5            # eps/|g| < 1e-3
    expect = -np.float64(f32(lr)) * gval / (np.abs(gval) + 1e-8)
    np.testing.assert_allclose(p[big].astype(np.float64), expect[big], rtol=1e-6)
    assert np.all(np.abs(np.abs(p[big].astype(np.float64)) - lr) <= 1.1e-3 * lr)
    assert np.all(ulp_diff(np.abs(p[np.abs(gval) > 1e-2]), np.full((np.abs(gval) > 1e-2).sum(),
                                                                     f32(lr))) <= 64)
    assert np.all(p[gval == 0] == 0) and np.all(m[gval == 0] == 0) and np.all(v[gval == 0] == 0)
    np.testing.assert_allclose(m.astype(np.float64), (1 - np.float64(f32(0.9))) * gval, rtol=1e-6)
    np.testing.assert_allclose(v.astype(np.float64), (1 - np.float64(f32(0.999))) * gval ** 2,
                               rtol=1e-6)
    assert np.all(np.sign(p[big]) == -np.sign(gval[big]))


# --------------------------------------------------------------------- float64 textbook formula

@pytest.mark.parametrize("l2_mode", [False, True])
@pytest.mark.parametrize("step,S,zero", [(1, 1024.0, True), (100, 65536.0, False),
                                         (1000, 65536.0, False)])
def test_against_float64_textbook(oracle, step, S, zero, l2_mode):
    """Catches: dropped/extra terms, beta1/beta2 swapped, 1-beta on the wrong operand, decay
    applied to the new p, transposed m/v, step off by one."""
    n = 50_000
    p, m, v, g = rand_block(n, 11 + step, S=S, zero_moments=zero)
    hy = dict(HY, step=step, loss_scale=S, l2_mode=l2_mode)
    flag, p2, m2, v2, _ = run_oracle(oracle, p, m, v, g, **hy)
    assert flag == 0
    tp, tm, tv = textbook_f64.adam_step_f64(p, m, v, g, **hy)
    # Error bounds are relative to the magnitudes that enter each sum (in L2 mode g + wd*p can
    # cancel, so the bound is on the operands, not on the result).
    g0 = np.abs(textbook_f64.half_bits_to_f64(g)) / S
    gmag = g0 + (hy["weight_decay"] * np.abs(p.astype(np.float64)) if l2_mode else 0.0)
    m_mag = 0.9 * np.abs(m.astype(np.float64)) + 0.1 * gmag
    v_mag = 0.999 * v.astype(np.float64) + 0.001 * gmag ** 2
    assert np.all(np.abs(m2.astype(np.float64) - tm) <= 3e-7 * m_mag + 1e-45)
    assert np.all(np.abs(v2.astype(np.float64) - tv) <= 5e-7 * v_mag + 1e-45)
    dp_true = tp - p.astype(np.float64)
    err = np.abs(p2.astype(np.float64) - tp)
    # two roundings happen at the magnitude of p (p*decay, then the subtraction): allow half a
    # unit in the last place of each, taken at the larger of |p| and |p'|, plus 1e-6 of the
    # step, plus the rounding of the fp32 decay factor 1 - lr*wd itself (half an ulp of 1.0
    # relative to |p|).  Elements whose L2 gradient cancelled badly are left to the m/v bounds.
    ulp = np.maximum(np.spacing(np.abs(p2)), np.spacing(np.abs(p))).astype(np.float64)
    mild = np.abs(tm) >= 0.25 * m_mag
    assert mild.mean() > 0.7
    bound = ulp + 1e-6 * np.abs(dp_true) + np.abs(p) * 2.0 ** -24
    assert np.all(err[mild] <= bound[mild])


# ------------------------------------------------------------------------------- library AdamW

@pytest.mark.parametrize("l2_mode", [False, True])
def test_against_library_adam(oracle, l2_mode):
    """Five chained steps from zero moments against torch.optim.AdamW / Adam on the CPU (a
    different operation order, so only ~1e-6 relative agreement is expected).  Catches: a
    misreading of Adam itself shared by the oracle and the float64 formula."""
    n = 20_000
    S = 1024.0
    p, _, _, _ = rand_block(n, 5, S=S, zero_moments=True)
    hy = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
    tparam = torch.nn.Parameter(torch.from_numpy(p.copy()))
    # the C ABI carries the hyper-parameters as fp32, so the library gets the fp32-rounded
    # values too (fp32(0.999) differs from 0.999 by 1.3e-5 relative in 1-beta2)
    lib = {k: float(np.float32(x)) for k, x in hy.items()}
    cls = torch.optim.Adam if l2_mode else torch.optim.AdamW
    opt = cls([tparam], lr=lib["lr"], betas=(lib["beta1"], lib["beta2"]), eps=lib["eps"],
              weight_decay=lib["weight_decay"])
    po = p.copy()
    mo = np.zeros(n, np.float32)
    vo = np.zeros(n, np.float32)
    h = np.zeros(n, np.uint16)
    for t in range(1, 6):
        _, _, _, g = rand_block(n, 100 + t, S=S)
        tparam.grad = torch.from_numpy(g.view(np.float16).astype(np.float32) / np.float32(S))
        opt.step()
        flag = oracle.adam_block_step(po, mo, vo, g, h, step=t, loss_scale=S, l2_mode=l2_mode,
                                      **hy)
        assert flag == 0
    lib_p = tparam.detach().numpy()
    st = opt.state[tparam]
    np.testing.assert_allclose(mo, st["exp_avg"].numpy(), rtol=2e-6, atol=2e-9)   # |g| ~ 1e-3
    np.testing.assert_allclose(vo, st["exp_avg_sq"].numpy(), rtol=2e-6, atol=1e-14)
    dp_lib = lib_p.astype(np.float64) - p.astype(np.float64)
    dp_orc = po.astype(np.float64) - p.astype(np.float64)
    big = np.maximum(np.abs(p), np.maximum(np.abs(lib_p), np.float32(5e-3)))   # five steps of ~lr
    assert np.all(np.abs(dp_lib - dp_orc) <= 2e-5 * np.abs(dp_lib) + 8 * np.spacing(big))
    assert np.max(np.abs(dp_lib)) > 1e-3          # the five steps really moved the parameters


# ------------------------------------------------------------------------------ number formats

def test_fp16_decode_all_patterns(oracle):
    """All 65536 binary16 patterns against numpy's float16 (library conversion)."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.half_bits_to_float(int(b)) for b in bits], np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_bf16_encode_against_library(oracle):
    """Random, tie, subnormal and extreme fp32 values against torch's bfloat16 conversion."""
    rng = np.random.default_rng(9)
    raw = rng.integers(0, 2 ** 32, size=20000, dtype=np.uint64).astype(np.uint32)
    ties = (rng.integers(0, 2 ** 16, size=2000, dtype=np.uint64).astype(np.uint32) << 16) | 0x8000
    near = ties + rng.integers(-2, 3, size=2000).astype(np.uint32)
    allb = np.concatenate([raw, ties, near, np.array([0, 1, 0x7F7FFFFF, 0x7F800000, 0xFF800000,
                                                      0x80000000, 0x00008000, 0x00018000],
                                                     np.uint32)])
    x = allb.view(np.float32)
    finite_or_inf = ~np.isnan(x)
    t = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.float_to_bf16_bits(v) for v in x], np.uint16)
    assert np.array_equal(got[finite_or_inf], t[finite_or_inf])
    nan_out = got[~finite_or_inf]
    assert np.all((nan_out & 0x7F80) == 0x7F80) and np.all((nan_out & 0x007F) != 0)


def test_fp16_encode_against_library(oracle):
    """The optional binary16 working copy: random bit patterns, the half range, ties, the
    overflow threshold (65520), the subnormal range and its rounding-to-zero threshold (2^-25)
    against numpy's float16 conversion."""
    rng = np.random.default_rng(13)
    raw = rng.integers(0, 2 ** 32, size=20000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    mid = (rng.standard_normal(20000) * 1e-2).astype(np.float32)
    tiny = (rng.standard_normal(20000) * 3e-7).astype(np.float32)
    halves = np.arange(0, 0x7C00, 7, dtype=np.uint32).astype(np.uint16).view(np.float16).astype(np.float32)
    ties = (halves.view(np.uint32) | 0x1000).view(np.float32)             # exactly between halves
    edge = np.array([65504, 65519.996, 65520, 65535, 65536, 1e30, -65520, 2.0 ** -14,
                     2.0 ** -14 - 2.0 ** -26, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0000001,
                     1.5 * 2.0 ** -24, 2.5 * 2.0 ** -24, 0.0, -0.0, np.inf, -np.inf], np.float32)
    x = np.concatenate([raw, mid, tiny, halves, ties, np.nextafter(ties, np.float32(0)),
                        np.nextafter(ties, np.float32(1e9)), edge, -ties])
    x = x[~np.isnan(x)]
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = np.array([oracle.float_to_half_bits(v) for v in x], np.uint16)
    assert np.array_equal(got, want)
    assert (oracle.float_to_half_bits(np.float32(np.nan)) & 0x7FFF) > 0x7C00


def test_grad_produce_against_library(oracle):
    """The gradient producer (fp32 accumulator -> G16): one fp32 multiplication, then the
    binary16 rounding, against numpy doing the same two operations; the flag and norm of the
    produced tensor are the pinned functions applied to it.  Includes products that overflow
    binary16 (they must become infinities and raise the flag), ties, subnormal results, and a
    multiplier that is not a power of two (so that the product's own rounding matters)."""
    rng = np.random.default_rng(17)
    halves = np.arange(1, 0x7C00, 3, dtype=np.uint32).astype(np.uint16).view(np.float16).astype(np.float32)
    ties = (halves.view(np.uint32) | 0x1000).view(np.float32)
    for mul in (1.0, 0.125, 1.0 / 3.0, 0.7, 3.0):
        m32 = np.float32(mul)
        x = np.concatenate([(rng.standard_normal(50000) * 65.5).astype(np.float32),
                            (rng.standard_normal(5000) * 3e-7).astype(np.float32),
                            ties / m32, -ties / m32, halves / m32,
                            np.array([0.0, -0.0, 65504.0, 65520.0, -65520.0, 70000.0, 2.0 ** -25,
                                      1e30, -1e30], np.float32) / m32])
        with np.errstate(over="ignore"):
            want = (x * m32).astype(np.float16).view(np.uint16)
        got = oracle.grad_produce(x, mul)
        assert np.array_equal(got, want), mul
        assert oracle.grad_overflow_check(got) == int(np.any(~np.isfinite(want.view(np.float16))))
    clean = (rng.standard_normal(4096) * 65.5).astype(np.float32)
    assert oracle.grad_overflow_check(oracle.grad_produce(clean, 0.5)) == 0
    assert np.array_equal(oracle.grad_produce(np.array([np.nan], np.float32), 1.0) & 0x7C00,
                          np.array([0x7C00], np.uint16))


def test_fp16_copy_option_only_changes_the_copy(oracle):
    n = 5000
    p, m, v, g = rand_block(n, 41)
    p[:8] = np.array([70000.0, -70000.0, 65519.0, 65520.0, 1e-7, -3e-8, 2.0 ** -25, 0.0], np.float32)
    hy = dict(HY, step=100, loss_scale=65536.0)
    a = run_oracle(oracle, p, m, v, g, **hy)
    b = run_oracle(oracle, p, m, v, g, half_out=True, **hy)
    for x, y in zip(a[1:4], b[1:4]):
        assert np.array_equal(bits32(x), bits32(y))
    with np.errstate(over="ignore"):
        assert np.array_equal(b[4], b[1].astype(np.float16).view(np.uint16))
    assert not np.array_equal(a[4], b[4])


# ------------------------------------------------------------------------------ overflow / skip

def test_overflow_flag_brute_force_all_patterns(oracle):
    """Every fp16 pattern alone in a vector of zeros: flagged iff numpy says it is not finite."""
    for b in range(0, 65536, 1):
        if (b & 0x7C00) != 0x7C00 and b % 97:     # all non-finite patterns + a sample of finite
            continue
        g = np.zeros(5, np.uint16)
        g[3] = b
        finite = np.isfinite(g.view(np.float16)[3])
        assert oracle.grad_overflow_check(g) == (0 if finite else 1), hex(b)
    for b in (0x7BFF, 0xFBFF, 0x0001, 0x8000, 0x3C00):
        assert oracle.grad_overflow_check(np.full(9, b, np.uint16)) == 0


@pytest.mark.parametrize("pos", ["first", "last", "middle"])
@pytest.mark.parametrize("pattern", [0x7C00, 0xFC00, 0x7E00, 0xFFFF, 0x7C01])
def test_overflow_skips_and_leaves_state_untouched(oracle, pos, pattern):
    n = 1001
    p, m, v, g = rand_block(n, 21)
    idx = {"first": 0, "last": n - 1, "middle": 500}[pos]
    g[idx] = pattern
    hy = dict(HY, step=100, loss_scale=65536.0)
    flag, p2, m2, v2, h = run_oracle(oracle, p, m, v, g, **hy)
    assert flag == 1
    assert np.array_equal(bits32(p2), bits32(p)) and np.array_equal(bits32(m2), bits32(m))
    assert np.array_equal(bits32(v2), bits32(v)) and np.all(h == 0xDEAD)
    assert oracle.grad_overflow_check(g) == 1
    g[idx] = 0x7BFF                      # largest finite value is not an overflow
    assert oracle.grad_overflow_check(g) == 0
    assert oracle.grad_overflow_check(np.zeros(0, np.uint16)) == 0


# ----------------------------------------------------------------------------------- invariants

def test_invariants(oracle):
    n = 30_000
    p, m, v, g = rand_block(n, 33)
    hy = dict(HY, step=100, loss_scale=65536.0)
    flag, p2, m2, v2, h = run_oracle(oracle, p, m, v, g, **hy)
    assert flag == 0
    assert np.all(v2 >= 0)
    assert np.all(v2 >= f32(0.999) * v)                      # beta2*v plus a non-negative term
    # the 16-bit copy is the rounding of the new fp32 parameters (synchronous update)
    want16 = torch.from_numpy(p2.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(h, want16)
    # m' lies between beta1*m and g-dominated value with the sign of the convex combination
    gval = g.view(np.float16).astype(np.float64) / 65536.0
    comb = 0.9 * m.astype(np.float64) + 0.1 * gval
    sure = np.abs(comb) > 1e-9
    assert np.all(np.sign(m2[sure]) == np.sign(comb[sure]))
    # elementwise independence: permuting inputs permutes outputs
    perm = np.random.default_rng(0).permutation(n)
    _, pp, mp, vp, hp = run_oracle(oracle, p[perm].copy(), m[perm].copy(), v[perm].copy(),
                                   g[perm].copy(), **hy)
    assert np.array_equal(bits32(pp), bits32(p2[perm])) and np.array_equal(hp, h[perm])
    assert np.array_equal(bits32(mp), bits32(m2[perm])) and np.array_equal(bits32(vp), bits32(v2[perm]))
    # splitting a block into two calls gives the same result
    k = 12_345
    _, pa, ma, va, ha = run_oracle(oracle, p[:k].copy(), m[:k].copy(), v[:k].copy(), g[:k].copy(), **hy)
    _, pb, mb, vb, hb = run_oracle(oracle, p[k:].copy(), m[k:].copy(), v[k:].copy(), g[k:].copy(), **hy)
    assert np.array_equal(bits32(np.concatenate([pa, pb])), bits32(p2))
    assert np.array_equal(np.concatenate([ha, hb]), h)
    # threaded evaluation is bit-identical to the serial loop
    p3, m3, v3 = p.copy(), m.copy(), v.copy()
    h3 = np.zeros(n, np.uint16)
    oracle.adam_block_step(p3, m3, v3, g, h3, nthreads=4, **hy)
    assert np.array_equal(bits32(p3), bits32(p2)) and np.array_equal(h3, h)
    assert np.array_equal(bits32(m3), bits32(m2)) and np.array_equal(bits32(v3), bits32(v2))


def test_zero_gradient_zero_moments_no_decay_is_identity(oracle):
    n = 257
    p, _, _, _ = rand_block(n, 1)
    z = np.zeros(n, np.float32)
    g = np.zeros(n, np.uint16)
    g[::2] = 0x8000                                           # negative zero is still zero
    flag, p2, m2, v2, _ = run_oracle(oracle, p, z, z, g, lr=1e-3, beta1=0.9, beta2=0.999,
                                     eps=1e-8, weight_decay=0.0, step=5, loss_scale=128.0)
    assert flag == 0 and np.array_equal(p2, p) and np.all(m2 == 0) and np.all(v2 == 0)
    # with decoupled decay the parameter only shrinks by (1 - lr*wd)
    _, p3, _, _, _ = run_oracle(oracle, p, z, z, g, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8,
                                weight_decay=0.5, step=5, loss_scale=128.0)
    assert np.array_equal(p3, p * (f32(1) - f32(1e-3) * f32(0.5)))


def test_wd_zero_makes_both_modes_identical(oracle):
    n = 999
    p, m, v, g = rand_block(n, 77)
    hy = dict(HY, weight_decay=0.0, step=100, loss_scale=65536.0)
    a = run_oracle(oracle, p, m, v, g, l2_mode=False, **hy)
    b = run_oracle(oracle, p, m, v, g, l2_mode=True, **hy)
    for x, y in zip(a[1:], b[1:]):
        assert np.array_equal(x.view(np.uint8), y.view(np.uint8))


def test_tiny_gradients_keep_gradual_underflow(oracle):
    """g16 = smallest fp16 subnormal with S=65536 gives g = 2^-40; v' = (1-b2)*2^-80 is tiny but
    normal; nothing may flush to zero."""
    g = np.full(4, 0x0001, np.uint16)
    z = np.zeros(4, np.float32)
    flag, p, m, v, _ = run_oracle(oracle, z, z, z, g, lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8,
                                  weight_decay=0.0, step=1, loss_scale=65536.0)
    assert flag == 0
    assert np.all(m == f32(1 - f32(0.9)) * f32(2.0 ** -40))
    assert np.all(v > 0)
    np.testing.assert_allclose(v.astype(np.float64), (1 - np.float64(f32(0.999))) * 2.0 ** -80,
                               rtol=1e-6)
    # and a subnormal result: v starts at the smallest subnormal, g = 0 -> beta2*v rounds to it
    v0 = np.full(4, 1.4e-45, np.float32)
    _, _, _, v2, _ = run_oracle(oracle, z, z, v0, np.zeros(4, np.uint16), lr=1e-4, beta1=0.9,
                                beta2=0.999, eps=1e-8, weight_decay=0.0, step=1, loss_scale=1.0)
    assert np.all(bits32(v2) == 1)


# --------------------------------------------------------------------------------------- sqnorm

def test_sqnorm_closed_form_and_library(oracle):
    """Catches: a missing unscale, scale applied once instead of squared, fp32 accumulation."""
    n = 100_003
    c = np.float16(3.0)
    g = np.full(n, c).view(np.uint16).copy()
    assert oracle.grad_sqnorm(g, 2.0) == n * 2.25                     # n * (3/2)^2, exact
    assert oracle.grad_sqnorm(np.zeros(0, np.uint16), 2.0) == 0.0
    _, _, _, g2 = rand_block(n, 8)
    want = textbook_f64.sqnorm_f64(g2, 65536.0)
    got = oracle.grad_sqnorm(g2, 65536.0)
    assert abs(got - want) <= 1e-12 * want
    assert abs(got - n * 1e-6) < 0.02 * n * 1e-6                      # ||g||^2 ~ n * std^2
    # a non-power-of-two scale
    want3 = textbook_f64.sqnorm_f64(g2, 3000.0)
    assert abs(oracle.grad_sqnorm(g2, 3000.0) - want3) <= 1e-12 * want3
