"""Are the oracle's pins sharp?  Each case below plants one plausible mistake in a COPY of the
oracle's C source (never in the oracle itself, and nowhere near the GPU), builds it, and runs the
pin tests of test_oracle_pins.py against the broken build: at least one pin must fail.  A mutant
that survived would mean a mistake of that kind could hide in the real oracle."""
import ctypes
import os
import subprocess

import pytest

import test_oracle_pins as pins
from oracle import build as oracle_build
from oracle import reference

MUTANTS = [
    ("moments swapped in the update", "float u = m_new / den;", "float u = v_new / den;"),
    ("beta1 and beta2 swapped", "float b1m = beta1 * (*m);", "float b1m = beta2 * (*m);"),
    ("1-beta1 on the wrong operand", "float o1g = s->omb1 * g;", "float o1g = s->omb2 * g;"),
    ("gradient not squared", "float gg = g * g;", "float gg = g;"),
    ("no unscale", "float g = half_bits_to_float(g16) * s->inv;",
     "float g = half_bits_to_float(g16);"),
    ("eps inside the square root", "float root = sqrtf(v_new);", "float root = sqrtf(v_new + eps);"),
    ("eps dropped", "float den = root_hat + eps;", "float den = root_hat;"),
    ("no bias correction of v", "float root_hat = root / s->sbc2;", "float root_hat = root;"),
    ("no bias correction of m", "s.ss = lr / s.bc1;", "s.ss = lr;"),
    ("bias correction multiplied instead of divided", "s.ss = lr / s.bc1;", "s.ss = lr * s.bc1;"),
    ("step off by one", "s.bc2 = (float)(1.0 - pow((double)beta2, (double)t));",
     "s.bc2 = (float)(1.0 - pow((double)beta2, (double)(t + 1)));"),
    ("update added instead of subtracted", "float p_new = pp - su;", "float p_new = pp + su;"),
    ("decay factor is lr*wd", "s.decay = 1.0f - lrwd;", "s.decay = lrwd;"),
    ("decay applied in L2 mode too", "float pp = l2_mode ? (*p) : (*p) * s->decay;",
     "float pp = (*p) * s->decay;"),
    ("L2 term missing", "g = g + wp;", "g = g;"),
    ("fused multiply-add in the first moment", "float m_new = b1m + o1g;",
     "float m_new = fmaf(beta1, *m, o1g);"),
    ("double-precision second moment", "float v_new = b2v + o2gg;",
     "float v_new = (float)((double)beta2 * (double)(*v) + (double)s->omb2 * (double)gg);"),
    ("bf16 by truncation", "b += 0x7FFFu + lsb;", "b += 0u;"),
    ("bf16 rounds half up", "b += 0x7FFFu + lsb;", "b += 0x8000u;"),
    ("16-bit copy taken from the old p", "*p = p_new;\n", "*p = p_new; p_new = pp;\n"),
    ("overflow test misses NaN", "if ((grad_fp16[i] & 0x7C00u) == 0x7C00u) flag = 1;",
     "if ((grad_fp16[i] & 0x7FFFu) == 0x7C00u) flag = 1;"),
    ("overflow test skips the last element", "for (uint64_t i = 0; i < n; ++i) {\n        if ((grad",
     "for (uint64_t i = 0; i + 1 < n; ++i) {\n        if ((grad"),
    ("state written despite overflow",
     "if (lohan_oracle_grad_overflow_check(grad_fp16, n)) return 1;",
     "int ovf = lohan_oracle_grad_overflow_check(grad_fp16, n); if (ovf && n > 1) n = n / 2;"),
    ("fp16 subnormals flushed", "mag = ldexpf((float)frac, -24);", "mag = 0.0f;"),
    ("fp16 exponent bias off by one", "(int)expo - 25", "(int)expo - 24"),
    ("norm scaled once instead of squared", "acc += g * g;", "acc += g * g * s;"),
    ("norm accumulated in fp32", "double acc = 0.0;\n    double s = (double)loss_scale;",
     "float acc = 0.0f;\n    double s = (double)loss_scale;"),
    ("fp16 copy truncates", "if (rest > 0x1000u || (rest == 0x1000u && (h & 1u))) h += 1u;",
     "if (0) h += 1u;"),
    ("fp16 copy overflow threshold wrong", "if (a >= 0x47800000u) return (uint16_t)(sign | 0x7C00u);",
     "if (a >= 0x47000000u) return (uint16_t)(sign | 0x7C00u);"),
    ("producer forgets the multiplier", "float scaled = grad_fp32[i] * multiplier;",
     "float scaled = grad_fp32[i];"),
    ("producer divides instead of multiplying", "float scaled = grad_fp32[i] * multiplier;",
     "float scaled = grad_fp32[i] / multiplier;"),
    ("producer flushes subnormal results", "float scaled = grad_fp32[i] * multiplier;",
     "float scaled = grad_fp32[i] * multiplier; if (fabsf(scaled) < 6.1035156e-05f) scaled = 0.0f;"),
]

# The pins that take the `oracle` fixture, with the parameter sets they are collected with.
PIN_CALLS = [
    (pins.test_hand_examples_bit_exact, [dict(idx=i) for i in range(3)]),
    (pins.test_hand_scalars, [dict(idx=0), dict(idx=1)]),
    (pins.test_bf16_golden_samples, [dict()]),
    (pins.test_fp16_golden_encodings, [dict()]),
    (pins.test_clipping_golden, [dict()]),
    (pins.test_first_step_closed_form, [dict()]),
    (pins.test_against_float64_textbook,
     [dict(step=s, S=S, zero=z, l2_mode=l2) for (s, S, z) in ((1, 1024.0, True), (100, 65536.0, False))
      for l2 in (False, True)]),
    (pins.test_against_library_adam, [dict(l2_mode=False), dict(l2_mode=True)]),
    (pins.test_matches_exact_rational_arithmetic,
     [dict(case=dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, step=100,
                     loss_scale=65536.0), l2_mode=False),
      dict(case=dict(lr=3e-3, beta1=0.8, beta2=0.95, eps=1e-6, weight_decay=0.1, step=7,
                     loss_scale=3000.0), l2_mode=True)]),
    (pins.test_fp16_decode_all_patterns, [dict()]),
    (pins.test_bf16_encode_against_library, [dict()]),
    (pins.test_fp16_encode_against_library, [dict()]),
    (pins.test_grad_produce_against_library, [dict()]),
    (pins.test_fp16_copy_option_only_changes_the_copy, [dict()]),
    (pins.test_overflow_flag_brute_force_all_patterns, [dict()]),
    (pins.test_overflow_skips_and_leaves_state_untouched,
     [dict(pos=p, pattern=pat) for p in ("first", "last", "middle") for pat in (0x7C00, 0x7E00)]),
    (pins.test_invariants, [dict()]),
    (pins.test_zero_gradient_zero_moments_no_decay_is_identity, [dict()]),
    (pins.test_tiny_gradients_keep_gradual_underflow, [dict()]),
    (pins.test_sqnorm_closed_form_and_library, [dict()]),
]


class _OracleView:
    """reference.py's functions bound to another shared object."""

    def __init__(self, lib_path):
        self._saved = None
        self._path = lib_path

    def __enter__(self):
        self._saved = (reference._LIB, oracle_build.LIB)
        reference._LIB = None
        oracle_build.LIB = self._path
        reference._lib()                     # load and set the prototypes on the mutant
        return reference

    def __exit__(self, *exc):
        reference._LIB, oracle_build.LIB = self._saved
        return False


def first_failing_pin(oracle_like):
    for fn, param_sets in PIN_CALLS:
        for kw in param_sets:
            try:
                fn(oracle_like, **kw)
            except AssertionError:
                return f"{fn.__name__}{kw}"
            except OverflowError:            # the exact evaluator refuses non-finite values
                return f"{fn.__name__}{kw} (non-finite)"
    return None


def test_the_pins_pass_on_the_real_oracle(oracle):
    assert first_failing_pin(oracle) is None


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_is_caught(tmp_path, name, old, new):
    src = open(oracle_build.SRC).read()
    assert src.count(old) >= 1, f"mutation site for '{name}' not found in the oracle source"
    mutated = src.replace(old, new, 1)
    assert mutated != src
    c_path = tmp_path / "mutant.c"
    so_path = tmp_path / "libmutant.so"
    c_path.write_text(mutated)
    flags = [f for f in oracle_build.CFLAGS if f not in ("-Wall", "-Wextra")]
    subprocess.run(["gcc", *flags, "-o", str(so_path), str(c_path), "-lm"], check=True)
    with _OracleView(str(so_path)) as broken:
        caught = first_failing_pin(broken)
    assert caught is not None, f"no pin noticed: {name}"
