"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares, and
its host-side logic (validation order, status strings, clipping helper, launch-config knob)
behaves as documented.  No kernel is launched: every call here returns from validation, which
runs before the library touches the HIP runtime."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

import paper_2403_06504_amd as lohan
from paper_2403_06504_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PRODUCT_HEADERS = [os.path.join(ROOT, "include", "lohan_adam.h"),
                   os.path.join(ROOT, "include", "lohan_swap_planner.h")]
TUNING_HEADER = os.path.join(ROOT, "include", "lohan_adam_tuning.h")      # bench-only
HEADERS = PRODUCT_HEADERS + [TUNING_HEADER]


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(lohan.library_path()):
        from paper_2403_06504_amd import build
        build.build(force=True)
    return lohan.load_library()


def declared_functions(headers=None):
    text = "".join(open(h).read() for h in (HEADERS if headers is None else headers))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lohan_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_three_named_entry_points():
    names = declared_functions()
    for must in ("lohan_adam_block_step", "lohan_grad_overflow_check", "lohan_grad_sqnorm"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    names = declared_functions()
    assert len(names) >= 9
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in the header but not exported"
    assert sorted(binding.EXPORTS) == names


def test_workspace_bytes_and_status_strings(lib):
    ws = lohan.lohan_workspace_bytes()
    assert 0 < ws <= (1 << 20) and ws % 16 == 0
    seen = set()
    for code in range(0, 7):
        s = lohan.lohan_status_string(code)
        assert s and s not in seen
        seen.add(s)
    assert lohan.lohan_status_string(0) == "ok"
    assert "unknown" in lohan.lohan_status_string(99)


GOOD = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, step=1,
            loss_scale=1024.0)
A = 0x1000   # a fake, aligned, never dereferenced device address


def step_status(lib, *, p=A, m=A * 2, v=A * 3, g=A * 4, h=A * 5, n=16, flag=A * 6, flags=0,
                ws=A * 7, ws_bytes=None, **hy):
    args = dict(GOOD, **hy)
    if ws_bytes is None:
        ws_bytes = lib.lohan_workspace_bytes()
    return lib.lohan_adam_block_step(p, m, v, g, h, n, args["lr"], args["beta1"], args["beta2"],
                                     args["eps"], args["weight_decay"], args["step"],
                                     args["loss_scale"], flag, flags, ws, ws_bytes, None)


def test_step_validation_returns_before_any_launch(lib):
    assert step_status(lib, flag=None) == 1                       # LOHAN_ERR_NULL
    for name in ("p", "m", "v", "g", "h"):
        assert step_status(lib, **{name: None}) == 1
    for name in ("p", "m", "v", "g", "h"):
        assert step_status(lib, **{name: A + 4}) == 2             # LOHAN_ERR_ALIGN
    assert step_status(lib, flag=A + 2) == 2
    assert step_status(lib, step=0) == 3                          # LOHAN_ERR_ARG
    assert step_status(lib, step=-5) == 3
    for bad in (0.0, -1.0, math.inf, math.nan):
        assert step_status(lib, loss_scale=bad) == 3
    for name in ("lr", "eps", "weight_decay"):
        for bad in (-1e-3, math.inf, math.nan):
            assert step_status(lib, **{name: bad}) == 3
    for name in ("beta1", "beta2"):
        for bad in (1.0, 1.5, -0.1, math.nan):
            assert step_status(lib, **{name: bad}) == 3
    assert step_status(lib, flags=8) == 3                         # unknown flag bit
    assert step_status(lib, ws=None) == 1
    assert step_status(lib, ws=A + 8) == 2
    assert step_status(lib, ws_bytes=16) == 4                     # LOHAN_ERR_WORKSPACE


def test_reduction_validation_returns_before_any_launch(lib):
    ws_bytes = lib.lohan_workspace_bytes()
    assert lib.lohan_grad_overflow_check(A, 8, None, A * 2, ws_bytes, None) == 1
    assert lib.lohan_grad_overflow_check(None, 8, A, A * 2, ws_bytes, None) == 1
    assert lib.lohan_grad_overflow_check(A + 2, 8, A, A * 2, ws_bytes, None) == 2
    assert lib.lohan_grad_overflow_check(A, 8, A * 3, None, ws_bytes, None) == 1
    assert lib.lohan_grad_overflow_check(A, 8, A * 3, A * 2, ws_bytes - 1, None) == 4
    f = ctypes.c_float
    assert lib.lohan_grad_sqnorm(A, 8, f(1.0), None, A * 3, A * 2, ws_bytes, None) == 1
    assert lib.lohan_grad_sqnorm(A, 8, f(1.0), A * 4 + 4, A * 3, A * 2, ws_bytes, None) == 2
    for bad in (0.0, -2.0, math.inf, math.nan):
        assert lib.lohan_grad_sqnorm(A, 8, f(bad), A * 4, A * 3, A * 2, ws_bytes, None) == 3
    assert lib.lohan_grad_sqnorm(A, 8, f(1.0), A * 4, None, A * 2, 8, None) == 4


def test_grad_produce_validation_returns_before_any_launch(lib):
    ws_bytes = lib.lohan_workspace_bytes()
    f = ctypes.c_float

    def status(src=A, out=A * 2, mul=1.0, S=1024.0, sq=A * 3, flag=A * 4, ws=A * 5, wsb=ws_bytes):
        return lib.lohan_grad_produce_fp16(src, 64, f(mul), out, f(S), sq, flag, ws, wsb, None)

    assert status(src=None) == 1 and status(out=None) == 1 and status(flag=None) == 1
    assert status(ws=None) == 1
    assert status(src=A + 4) == 2 and status(out=A * 2 + 8) == 2 and status(sq=A * 3 + 4) == 2
    assert status(flag=A * 4 + 2) == 2 and status(ws=A * 5 + 8) == 2
    for bad in (math.inf, math.nan):
        assert status(mul=bad) == 3
    for bad in (0.0, -1.0, math.inf, math.nan):
        assert status(S=bad) == 3
    assert status(wsb=ws_bytes - 1) == 4


def test_static_sqnorm_validation_returns_before_any_launch(lib):
    f = ctypes.c_float
    assert lib.lohan_grad_sqnorm_static(A, 8, f(1.0), None, A * 3, None) == 1
    assert lib.lohan_grad_sqnorm_static(None, 8, f(1.0), A * 4, A * 3, None) == 1
    assert lib.lohan_grad_sqnorm_static(A + 2, 8, f(1.0), A * 4, A * 3, None) == 2
    assert lib.lohan_grad_sqnorm_static(A, 8, f(1.0), A * 4 + 4, A * 3, None) == 2
    for bad in (0.0, -2.0, math.inf, math.nan):
        assert lib.lohan_grad_sqnorm_static(A, 8, f(bad), A * 4, A * 3, None) == 3
    assert lib.lohan_grad_sqnorm_static(A, (1 << 40) + 1, f(1.0), A * 4, A * 3, None) == 6
    assert "maximum" in lohan.lohan_status_string(6)


def test_clipped_step_validation_returns_before_any_launch(lib):
    ws_bytes = lib.lohan_workspace_bytes()

    def status(sqnorm=A * 8, max_norm=1.0, flag=A * 6, ws=A * 7, wsb=ws_bytes, flags=0, step=1):
        return lib.lohan_adam_block_step_clipped(
            A, A * 2, A * 3, A * 4, A * 5, 16, GOOD["lr"], GOOD["beta1"], GOOD["beta2"],
            GOOD["eps"], GOOD["weight_decay"], step, GOOD["loss_scale"], sqnorm, max_norm, flag,
            flags, ws, wsb, None)

    assert status(sqnorm=None) == 1
    assert status(flag=None) == 1
    assert status(sqnorm=A * 8 + 4) == 2
    for bad in (0.0, -1.0, math.inf, math.nan):
        assert status(max_norm=bad) == 3
    assert status(step=0) == 3
    assert status(flags=8) == 3
    assert status(ws=None) == 1
    assert status(wsb=ws_bytes - 1) == 4


def test_small_block_step_validation_returns_before_any_launch(lib):
    ws_bytes = lib.lohan_workspace_bytes()

    def status(p=A, m=A * 2, v=A * 3, g=A * 4, p16=A * 5, sqnorm=A * 8, flag=A * 6, ws=A * 7,
               wsb=ws_bytes, flags=0, step=1, loss_scale=1024.0, **over):
        h = dict(GOOD, **over)
        return lib.lohan_adam_small_block_step(
            p, m, v, g, p16, 16, h["lr"], h["beta1"], h["beta2"], h["eps"], h["weight_decay"],
            step, loss_scale, sqnorm, flag, flags, ws, wsb, None)

    for name in ("p", "m", "v", "g", "p16", "flag", "ws"):
        assert status(**{name: None}) == 1, name
    for name in ("p", "m", "v", "g", "p16", "ws"):
        assert status(**{name: A * 10 + 8}) == 2, name
    assert status(flag=A * 6 + 2) == 2 and status(sqnorm=A * 8 + 4) == 2
    assert status(flags=2) == 3                  # a known flag belongs to the two-call step
    assert status(flags=8) == 3 and status(step=0) == 3
    for bad in (0.0, -1.0, math.inf, math.nan):
        assert status(loss_scale=bad) == 3
    assert status(beta1=1.0) == 3 and status(lr=-1.0) == 3 and status(eps=math.nan) == 3
    assert status(wsb=ws_bytes - 1) == 4
    assert lib.lohan_adam_small_block_max_n(None) == 1
    assert lib.lohan_tuning_set_wait_limit(1 << 32) == 3
    assert lib.lohan_tuning_set_wait_limit(-1) == 0


def test_out_of_place_step_validation_returns_before_any_launch(lib):
    def status(pi=A, mi=A * 2, vi=A * 3, g=A * 4, po=A * 5, mo=A * 6, vo=A * 7, p16=A * 8, n=16,
               step=1, loss_scale=1024.0, flag=A * 9, flags=0, **over):
        h = dict(GOOD, **over)
        return lib.lohan_adam_block_step_out_of_place(
            pi, mi, vi, g, po, mo, vo, p16, n, h["lr"], h["beta1"], h["beta2"], h["eps"],
            h["weight_decay"], step, loss_scale, flag, flags, None)

    for name in ("pi", "mi", "vi", "g", "po", "mo", "vo", "p16", "flag"):
        assert status(**{name: None}) == 1, name
    for name in ("pi", "mi", "vi", "g", "po", "mo", "vo", "p16"):
        assert status(**{name: A * 10 + 8}) == 2, name
    assert status(flag=A * 9 + 2) == 2
    assert status(po=A) == 3 and status(mo=A * 2) == 3 and status(vo=A * 3) == 3   # in == out
    assert status(flags=2) == 3                  # a prechecked flag belongs to the in-place step
    assert status(flags=8) == 3
    assert status(step=0) == 3
    for bad in (0.0, -1.0, math.inf, math.nan):
        assert status(loss_scale=bad) == 3
    assert status(beta1=1.0) == 3 and status(beta2=-0.1) == 3 and status(lr=-1.0) == 3
    assert status(eps=math.nan) == 3 and status(weight_decay=math.inf) == 3


def test_multi_block_step_validation_returns_before_any_launch(lib):
    ws_bytes = lib.lohan_workspace_bytes()

    def status(blocks=((A, A * 2, A * 3, A * 4, A * 5, 16), (A * 6, A * 7, A * 8, A * 9, A * 10, 0)),
               count=None, step=1, loss_scale=1024.0, max_norm=0.0, flags_dev=A * 11,
               norms=A * 12, flags=0, ws=A * 13, wsb=ws_bytes, **over):
        h = dict(GOOD, **over)
        arr = (binding.LohanBlock * max(1, len(blocks)))(*[binding.LohanBlock(*b) for b in blocks])
        return lib.lohan_adam_multi_block_step(
            arr if blocks is not None else None, len(blocks) if count is None else count,
            h["lr"], h["beta1"], h["beta2"], h["eps"], h["weight_decay"], step, loss_scale,
            max_norm, flags_dev, norms, flags, ws, wsb, None)

    assert lib.lohan_adam_multi_block_step(None, 0, 1e-4, 0.9, 0.999, 1e-8, 0.0, 1, 1.0, 0.0, None,
                                           None, 0, None, 0, None) == 0      # nothing to do
    assert lib.lohan_adam_multi_block_step(None, 2, 1e-4, 0.9, 0.999, 1e-8, 0.0, 1, 1.0, 0.0,
                                           A, None, 0, A, ws_bytes, None) == 1
    assert status(flags_dev=None) == 1
    for field in range(5):                       # a NULL or misaligned array in the second block
        blk = [A * 6, A * 7, A * 8, A * 9, A * 10, 16]
        blk[field] = None
        assert status(blocks=((A, A * 2, A * 3, A * 4, A * 5, 16), tuple(blk))) == 1, field
        blk[field] = A * 20 + 4
        assert status(blocks=((A, A * 2, A * 3, A * 4, A * 5, 16), tuple(blk))) == 2, field
    assert status(norms=A * 12 + 4) == 2
    assert status(norms=None, ws=None) == 1
    assert status(ws=A * 13 + 8) == 2
    assert status(wsb=ws_bytes - 1) == 4
    assert status(step=0) == 3 and status(flags=8) == 3 and status(loss_scale=0.0) == 3
    for bad in (-1.0, math.inf, math.nan):
        assert status(max_norm=bad) == 3
    assert status(beta1=1.0) == 3 and status(lr=math.nan) == 3


def test_model_placement_properties(lib):
    """No two arrays overlap, every array starts on a 1 MiB boundary inside the slab, and for
    blocks whose fp32 arrays fit a 4 GiB (else a 12 GiB) period and are not below 256 MiB the
    three fp32 arrays of a block sit at the same offset in consecutive lanes (whose starts are
    skewed by a few MiB against the period); longer arrays are packed an odd number of MiB apart."""
    gib, mib = 1 << 30, 1 << 20
    cases = [(12 * 5120 ** 2, 40), (12 * 5120 ** 2, 4), (12 * 4096 ** 2, 7), (12 * 7168 ** 2, 2),
             (12 * 8192 ** 2, 1), (12 * 11264 ** 2, 3), (12 * 12288 ** 2, 2), (12 * 14336 ** 2, 2),
             (12 * 16384 ** 2, 2), (18 * 1536 ** 2, 30), (7, 3), (0, 2), (1 << 26, 5),
             ((1 << 26) - 1, 5), ((1 << 30) - (1 << 19), 2), ((1 << 30), 2),
             (3 * (1 << 30) - (1 << 19), 2), (3 * (1 << 30), 2)]
    for n, nb in cases:
        offs, total, align, per_group = lohan.lohan_model_placement(n, nb)
        assert align == 2 * mib and len(offs) == nb
        spans = []
        for o in offs:
            for key, width in (("param_fp32", 4), ("exp_avg", 4), ("exp_avg_sq", 4),
                               ("grad_fp16", 2), ("param_bf16", 2)):
                assert o[key] % mib == 0
                assert o[key] + n * width <= total
                spans.append((o[key], o[key] + n * width))
        spans.sort()
        for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
            assert a1 <= b0, (n, nb, a0, a1, b0, b1)
        wide = (4 * n + 2 * mib - 1) // (2 * mib) * (2 * mib)
        narrow = (2 * n + 2 * mib - 1) // (2 * mib) * (2 * mib)
        period = 0
        if wide >= 256 * mib:
            period = 4 * gib if wide <= 4 * gib - 2 * mib else \
                12 * gib if wide <= 12 * gib - 2 * mib else 0
        # arrays too long for any lane are packed with an odd number of MiB between p, m, v;
        # arrays below 256 MiB are packed plainly
        skew = mib if (not period and wide >= 256 * mib) else 0
        # lanes 1 and 2: at the period + 8 MiB and twice the period + 9 MiB for the 4 GiB period,
        # + 1 and + 2 MiB for the 12 GiB period
        lane1, lane2 = {4 * gib: (4 * gib + 8 * mib, 8 * gib + 9 * mib),
                        12 * gib: (12 * gib + mib, 24 * gib + 2 * mib),
                        0: (wide + skew, 2 * (wide + skew))}[period]
        for o in offs:
            assert o["exp_avg"] - o["param_fp32"] == lane1
            assert o["exp_avg_sq"] - o["param_fp32"] == lane2
            if period or skew:                   # m and v an odd number of MiB apart
                assert ((lane2 - lane1) // mib) % 2 == 1
        if period:
            assert per_group == (period - 2 * mib) // wide >= 1
            first = offs[0]["param_fp32"]
            for j, o in enumerate(offs[:per_group]):          # block j at j arrays into lane 0
                assert o["param_fp32"] - first == j * wide
        else:
            assert per_group == 1 and total == nb * (3 * wide + 2 * narrow + 4 * skew)
    # the documented price of full groups
    for n, worst in ((12 * 4096 ** 2, 1.04), (12 * 5120 ** 2, 1.07), (12 * 7168 ** 2, 1.13),
                     (12 * 8192 ** 2, 1.17), (12 * 11264 ** 2, 1.05), (12 * 12288 ** 2, 1.14),
                     (12 * 14336 ** 2, 1.16)):
        offs, total, _, per_group = lohan.lohan_model_placement(n)
        assert len(offs) == per_group
        assert 1.0 <= total / (16 * n * per_group) <= worst, (n, total / (16 * n * per_group))
    assert lohan.lohan_model_placement(5, 0)[1] == 0
    total, align = ctypes.c_size_t(), ctypes.c_size_t()
    assert lib.lohan_model_placement(8, 1, None, ctypes.byref(total), ctypes.byref(align),
                                     None) == 1
    one = (binding.LohanBlockOffsets * 1)()
    assert lib.lohan_model_placement(8, 1, one, None, ctypes.byref(align), None) == 1
    assert lib.lohan_model_placement(8, 1, one, ctypes.byref(total), None, None) == 1
    assert lib.lohan_model_placement((1 << 40) + 1, 1, one, ctypes.byref(total),
                                     ctypes.byref(align), None) == 3


def test_ring_validation_returns_before_any_device_call(lib):
    need = lib.lohan_ring_bytes(4, 1)
    assert need >= 5 * 40 + 2 * 4 * 8 + 2 * 4 * 4 + 4 + 4 * 4 and need % 16 == 0
    assert lib.lohan_ring_bytes(40, 1) > need and lib.lohan_ring_bytes(4, 3) > need

    def slots(lengths):
        return (binding.LohanRingSlot * len(lengths))(*[
            binding.LohanRingSlot(A * (4 * i + 1), A * (4 * i + 2), A * (4 * i + 3),
                                  A * (4 * i + 4), n) for i, n in enumerate(lengths)])

    good = slots([16] * 5)
    assert lib.lohan_ring_init(None, need, good, 4, 1) == 1
    assert lib.lohan_ring_init(A, need, None, 4, 1) == 1
    assert lib.lohan_ring_init(A + 8, need, good, 4, 1) == 2
    assert lib.lohan_ring_init(A, need, good, 0, 1) == 3
    assert lib.lohan_ring_init(A, need, good, 4, 0) == 3            # at least one spare
    assert lib.lohan_ring_init(A, need, good, 2, 3) == 3            # more spares than blocks
    assert lib.lohan_ring_init(A, need - 1, good, 4, 1) == 4
    for field in ("param_fp32", "exp_avg", "exp_avg_sq", "param_16"):
        bad = slots([16] * 5)
        setattr(bad[4], field, None)                             # the spare slot counts too
        assert lib.lohan_ring_init(A, need, bad, 4, 1) == 1, field
        setattr(bad[4], field, A * 50 + 4)
        assert lib.lohan_ring_init(A, need, bad, 4, 1) == 2, field
    # unequal lengths: every block needs a spare of exactly its length, spares must be distinct
    need2 = lib.lohan_ring_bytes(4, 2)
    assert lib.lohan_ring_init(A, need2, slots([16, 8, 16, 8, 16, 9]), 4, 2) == 3
    assert lib.lohan_ring_init(A, need2, slots([16, 8, 16, 8, 16, 16]), 4, 2) == 3
    assert lib.lohan_ring_init(A, need2, slots([16, 8, 16, 7, 16, 8]), 4, 2) == 3

    def step(ring=A, nb=4, ns=1, block=1, g=A * 2, n=16, step=1, loss_scale=1024.0, flags=0,
             **over):
        h = dict(GOOD, **over)
        return lib.lohan_ring_adam_block_step(ring, nb, ns, block, g, n, h["lr"], h["beta1"],
                                              h["beta2"], h["eps"], h["weight_decay"], step,
                                              loss_scale, flags, None)

    assert step(ring=None) == 1 and step(g=None) == 1
    assert step(ring=A + 4) == 2 and step(g=A * 2 + 2) == 2
    assert step(block=4) == 3 and step(nb=0) == 3 and step(ns=0) == 3 and step(ns=5) == 3
    assert step(flags=2) == 3 and step(flags=8) == 3            # no prechecked form
    assert step(step=0) == 3 and step(loss_scale=math.nan) == 3 and step(beta2=1.0) == 3

    def clipped(sqnorm=A * 9, max_norm=1.0, **kw):
        return lib.lohan_ring_adam_block_step_clipped(
            kw.get("ring", A), 4, 1, kw.get("block", 1), A * 2, 16, GOOD["lr"], GOOD["beta1"],
            GOOD["beta2"], GOOD["eps"], GOOD["weight_decay"], 1, GOOD["loss_scale"], sqnorm,
            max_norm, 0, None)

    assert clipped(sqnorm=None) == 1 and clipped(sqnorm=A * 9 + 4) == 2
    for bad in (0.0, -1.0, math.inf, math.nan):
        assert clipped(max_norm=bad) == 3
    assert lib.lohan_ring_read(None, 4, 1, None, None, None, None) == 1
    assert lib.lohan_ring_read(A + 4, 4, 1, None, None, None, None) == 2
    assert lib.lohan_ring_read(A, 0, 1, None, None, None, None) == 3


def test_out_of_place_clipped_validation(lib):
    ws_bytes = lib.lohan_workspace_bytes()

    def status(sqnorm=A * 20, max_norm=1.0, ws=A * 21, wsb=ws_bytes, flags=0, po=A * 11):
        return lib.lohan_adam_block_step_out_of_place_clipped(
            A, A * 2, A * 3, A * 4, po, A * 12, A * 13, A * 5, 16, GOOD["lr"], GOOD["beta1"],
            GOOD["beta2"], GOOD["eps"], GOOD["weight_decay"], 1, GOOD["loss_scale"], sqnorm,
            max_norm, A * 6, flags, ws, wsb, None)

    assert status(sqnorm=None) == 1 and status(ws=None) == 1
    assert status(sqnorm=A * 20 + 4) == 2 and status(ws=A * 21 + 8) == 2
    assert status(max_norm=0.0) == 3 and status(max_norm=math.nan) == 3
    assert status(flags=lohan.LOHAN_FLAG_PRECHECKED) == 3
    assert status(po=A) == 3                                   # output must differ from input
    assert status(wsb=16) == 4


def test_compact_placement_properties(lib):
    mib = 1 << 20
    for n, blocks in ((12 * 5120 ** 2, 5), (12 * 12288 ** 2, 2), (12 * 768 ** 2, 12), (1000, 3),
                      (0, 2)):
        offsets, total, align = lohan.lohan_model_placement_compact(n, blocks)
        assert align == 2 * mib
        spans = []
        for o in offsets:
            assert (o["exp_avg"] - o["param_fp32"]) % (2 * mib) == mib      # odd MiB apart
            assert (o["exp_avg_sq"] - o["exp_avg"]) % (2 * mib) == mib
            for field, width in (("param_fp32", 4), ("exp_avg", 4), ("exp_avg_sq", 4),
                                 ("grad_fp16", 2), ("param_bf16", 2)):
                assert o[field] % mib == 0 and o[field] + n * width <= total
                spans.append((o[field], o[field] + n * width))
        spans = sorted(s for s in spans if s[1] > s[0])
        assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))
        assert total <= 16 * n * blocks + blocks * 14 * mib
    _, total, _ = lohan.lohan_model_placement_compact(12 * 5120 ** 2, 40)
    assert total <= 1.002 * 16 * 12 * 5120 ** 2 * 40
    total_c, align_c = ctypes.c_size_t(), ctypes.c_size_t()
    assert lib.lohan_model_placement_compact(8, 1, None, ctypes.byref(total_c),
                                             ctypes.byref(align_c)) == 1
    one = (binding.LohanBlockOffsets * 1)()
    assert lib.lohan_model_placement_compact((1 << 40) + 1, 1, one, ctypes.byref(total_c),
                                             ctypes.byref(align_c)) == 3


def test_tensor_placement_properties(lib):
    """Per-tensor placement: inside the slab, aligned, disjoint, p/m/v of one tensor at the same
    offset within the three lanes, and equal to the equal-block placement when the lengths are
    equal."""
    mib, gib = 1 << 20, 1 << 30
    h = 5120
    one_layer = [3 * h * h, 3 * h, h * h, h, 4 * h * h, 4 * h, 4 * h * h, h, h, h, h, h]
    cases = [one_layer * 40, [12 * 1024 * 1024] * 3, [7, 0, 300, 5_000_000],
             [12 * 12288 * 12288, 12 * 5120 * 5120, 1000], [1 << 26] * 9, [3 * (1 << 30) + 5] * 2]
    for lengths in cases:
        offsets, total, align = lohan.lohan_tensor_placement(lengths)
        assert align == 2 * mib and len(offsets) == len(lengths)
        spans = []
        for n, o in zip(lengths, offsets):
            for field, width in (("param_fp32", 4), ("exp_avg", 4), ("exp_avg_sq", 4),
                                 ("grad_fp16", 2), ("param_bf16", 2)):
                assert o[field] % 4096 == 0 and o[field] + n * width <= total
                if n * width >= 2 * mib:
                    assert o[field] % mib == 0
                spans.append((o[field], o[field] + n * width))
        spans = sorted(s for s in spans if s[1] > s[0])
        assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:])), "arrays overlap"
        widest = max(lengths) * 4
        if 256 * mib <= widest <= 12 * gib - 2 * mib:
            period = 4 * gib if widest <= 4 * gib - 2 * mib else 12 * gib
            lane1, lane2 = ((period + 8 * mib, 2 * period + 9 * mib) if period == 4 * gib
                            else (period + mib, 2 * period + 2 * mib))
            for o in offsets:
                assert o["exp_avg"] - o["param_fp32"] == lane1
                assert o["exp_avg_sq"] - o["param_fp32"] == lane2
        payload = 16 * sum(lengths)
        assert total >= payload
    # equal lengths of 2^26 elements and more: the same offsets as lohan_model_placement
    for n, count in ((12 * 5120 * 5120, 7), (12 * 12288 * 12288, 3), (1 << 26, 20)):
        a, total_a, _, _ = lohan.lohan_model_placement(n, count)
        b, total_b, _ = lohan.lohan_tensor_placement([n] * count)
        assert a == b and total_a == total_b
    # a 13B model tensor by tensor: the short vectors cost little
    offsets, total, _ = lohan.lohan_tensor_placement(one_layer * 40)
    equal, total_equal, _, _ = lohan.lohan_model_placement(12 * h * h, 40)
    assert total <= 1.02 * total_equal
    with pytest.raises(lohan.LohanError) as e:
        lohan.lohan_tensor_placement([1, (1 << 40) + 1])
    assert e.value.status == 3


def test_offload_create_validation_touches_no_device(lib):
    handle = ctypes.c_void_p()
    need = lib.lohan_offload_slab_bytes(1000, 3)
    assert need >= 3 * (3 * 4000 + lib.lohan_workspace_bytes()) and need % 256 == 0
    assert lib.lohan_offload_slab_bytes(1000, 0) == 0
    assert lib.lohan_offload_create(None, A * 16, need, 1000, 3, 1) == 1
    assert lib.lohan_offload_create(ctypes.byref(handle), None, need, 1000, 3, 1) == 1
    assert lib.lohan_offload_create(ctypes.byref(handle), A * 16 + 64, need, 1000, 3, 1) == 2
    for bad in ((0, 3, 1), (1000, 0, 1), (1000, 17, 1), (1000, 3, 2), (1000, 3, -1)):
        assert lib.lohan_offload_create(ctypes.byref(handle), A * 16, need, *bad) == 3
    assert lib.lohan_offload_create(ctypes.byref(handle), A * 16, need - 1, 1000, 3, 1) == 4
    assert handle.value is None
    assert lib.lohan_offload_drain(None) == 1 and lib.lohan_offload_destroy(None) == 1
    assert lib.lohan_offload_wait_last_step(None, None) == 1
    assert lib.lohan_offload_submit(None, None, 0, 0, 0, 0, 0, 1, 1, 0, 0, None) == 1


def test_plain_c_client_builds_and_runs(lib, tmp_path):
    """Both headers compile as C11 with -Wall -Wextra -Werror, and a C program linked against the
    library gets the documented answers from the host-only entry points."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    exe = tmp_path / "c_abi_client"
    libdir = os.path.dirname(lohan.library_path())
    subprocess.run(["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-D__HIP_PLATFORM_AMD__",
                    "-I/opt/rocm/include", "-I" + os.path.join(ROOT, "include"), "-o", str(exe),
                    os.path.join(ROOT, "tests", "c_abi_client.c"), "-L" + libdir,
                    "-l:" + os.path.basename(lohan.library_path()), "-Wl,-rpath," + libdir,
                    "-Wl,-rpath,/opt/rocm/lib", "-lm"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    lines = dict(line.split(" ", 1) for line in out.strip().splitlines())
    assert int(lines["workspace_bytes"]) == lohan.lohan_workspace_bytes()
    assert lines["status_3"] == lohan.lohan_status_string(3)
    assert lines["clip"] == "2346.2798"
    assert lines["placement"] == f"0 group 3 lane {(4 << 30) + (8 << 20)} align {2 << 20}"
    assert lines["null_step"] == "1"
    assert lines["plan"] == "0 n 2 first 1 a 30.0 f 100.0 t 19.00"
    assert lines["flops"] == "0 200.0 -10.0"


def test_host_code_under_address_and_undefined_sanitizers(lib, tmp_path):
    """The host side of the library (C ABI layer, offload handle, planner) rebuilt with
    AddressSanitizer + UBSan (host code only; the kernels come from the regular library), driven
    by a C client through many planner instances, placements and validation paths."""
    import shutil
    import subprocess
    from paper_2403_06504_amd import build
    clang = "/opt/rocm/llvm/bin/clang"
    if not (os.path.exists(build.HIPCC) and os.path.exists(clang)):
        pytest.skip("no ROCm toolchain")
    libdir = os.path.dirname(lohan.library_path())
    san = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]
    host_san = [x for flag in san for x in ("-Xarch_host", flag)]
    sources = [f for f in build.SOURCES if not f.endswith("lohan_kernels.hip")]
    so = tmp_path / "liblohan_hostsan.so"
    subprocess.run([build.HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC",
                    "-shared", *host_san, "-I", os.path.join(ROOT, "include"), "-I", build.CSRC,
                    "-o", str(so), *sources, "-L" + libdir,
                    "-l:" + os.path.basename(lohan.library_path()), "-Wl,-rpath," + libdir],
                   check=True, capture_output=True)
    exe = tmp_path / "stress"
    subprocess.run([clang, "-std=c11", "-g", "-Wall", "-Wextra", "-Werror", *san,
                    "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
                    "-I" + os.path.join(ROOT, "include"), "-o", str(exe),
                    os.path.join(ROOT, "tests", "c_abi_host_stress.c"), "-L" + str(tmp_path),
                    "-l:" + so.name, "-Wl,-rpath," + str(tmp_path), "-Wl,-rpath,/opt/rocm/lib",
                    "-Wl,-rpath," + libdir, "-lm"], check=True, capture_output=True)
    run = subprocess.run([str(exe)], capture_output=True, text=True)
    assert run.returncode == 0 and run.stdout.startswith("ok "), (run.stdout, run.stderr[-2000:])


def test_binding_raises_with_status(lib):
    with pytest.raises(lohan.LohanError) as e:
        lohan.lohan_adam_block_step(A, A * 2, A * 3, A * 4, A * 5, 16, 1e-4, 0.9, 0.999, 1e-8,
                                    0.01, 0, 1024.0, A * 6, 0, A * 7,
                                    lohan.lohan_workspace_bytes(), stream=0)
    assert e.value.status == 3


def test_clip_loss_scale_matches_oracle(lib, oracle):
    rng = np.random.default_rng(0)
    for _ in range(200):
        sq = float(10 ** rng.uniform(-8, 6))
        S = float(np.float32(2.0 ** rng.integers(0, 17)))
        mx = float(np.float32(10 ** rng.uniform(-2, 1)))
        got = np.float32(lohan.lohan_clip_loss_scale(sq, S, mx))
        want = oracle.clip_loss_scale(sq, S, mx)
        assert got == want, (sq, S, mx)
    assert lohan.lohan_clip_loss_scale(0.0, 1024.0, 1.0) == 1024.0
    assert abs(lohan.lohan_clip_loss_scale(5.25, 1024.0, 1.0) - 2346.2798) < 2e-3
    for bad in ((-1.0, 1.0, 1.0), (math.nan, 1.0, 1.0), (math.inf, 1.0, 1.0), (1.0, 0.0, 1.0),
                (1.0, 1.0, 0.0), (1.0, 1.0, -1.0)):
        assert math.isnan(lohan.lohan_clip_loss_scale(*bad))


def test_launch_config_knob(lib):
    before = lohan.lohan_tuning_get_launch_config()
    try:
        lohan.lohan_tuning_set_launch_config(2 | (1 << 2) | (1 << 4), 16, 12, 4, 1)
        assert lohan.lohan_tuning_get_launch_config() == (2 | (1 << 2) | (1 << 4), 16, 12, 4, 1)
        lohan.lohan_tuning_set_launch_config()                       # all defaults
        v, a, w, r, pol = lohan.lohan_tuning_get_launch_config()
        assert v == -1 and a >= 0 and w >= 0 and r > 0 and pol == -1   # -1: chosen per call
        lohan.lohan_tuning_set_launch_config(0, 0, 0, 0, 0)
        assert lohan.lohan_tuning_get_launch_config()[:3] == (0, 0, 0)
        assert lohan.lohan_tuning_get_launch_config()[4] == 0
        for bad in (3, 2 << 2, 3 << 4, 1 << 6, 1000):
            with pytest.raises(lohan.LohanError):
                lohan.lohan_tuning_set_launch_config(bad, 0, 0, 0)
        for bad in ((0, 100000, 0, 0), (0, 0, 33, 0), (0, 0, 0, 17), (0, 0, 0, 0, 2)):
            with pytest.raises(lohan.LohanError):
                lohan.lohan_tuning_set_launch_config(*bad)
    finally:
        lohan.lohan_tuning_set_launch_config(*before)


def test_launch_override_is_per_thread_and_not_in_the_product_header(lib):
    """The product headers expose no process-wide mutable setting: the launch-shape override
    lives in the bench-only header and only affects the thread that set it."""
    import threading
    product = declared_functions(PRODUCT_HEADERS)
    assert not [n for n in product if "launch_config" in n or n.startswith("lohan_tuning_")]
    assert not [n for n in product if re.search(r"(^|_)set_", n)]
    tuning = declared_functions([TUNING_HEADER])
    assert "lohan_tuning_set_launch_config" in tuning
    assert all(n.startswith("lohan_tuning_") for n in tuning)
    before = lohan.lohan_tuning_get_launch_config()
    seen = {}

    def other_thread():
        seen["initial"] = lohan.lohan_tuning_get_launch_config()
        lohan.lohan_tuning_set_launch_config(1, 8, 16, 2, 0)
        seen["after_own_set"] = lohan.lohan_tuning_get_launch_config()

    try:
        lohan.lohan_tuning_set_launch_config(2, 4, 8, 3, 1)
        t = threading.Thread(target=other_thread)
        t.start()
        t.join()
        assert seen["initial"][0] == -1 and seen["initial"][4] == -1      # built-in defaults
        assert seen["after_own_set"] == (1, 8, 16, 2, 0)
        assert lohan.lohan_tuning_get_launch_config() == (2, 4, 8, 3, 1)   # untouched by it
    finally:
        lohan.lohan_tuning_set_launch_config(*before)


def test_workspace_init_validation(lib):
    ws_bytes = lib.lohan_workspace_bytes()
    assert lib.lohan_workspace_init(None, ws_bytes, None) == 1
    assert lib.lohan_workspace_init(A + 8, ws_bytes, None) == 2
    assert lib.lohan_workspace_init(A, ws_bytes - 1, None) == 4


def test_probe_validation_returns_before_any_launch(lib):
    def probe(pattern, a=A, b=A * 2, c=A * 3, g=A * 4, h=A * 5, n=1024, waves=0):
        return lib.lohan_tuning_probe(pattern, a, b, c, g, h, n, waves, None)
    assert probe(-1) == 3 and probe(5) == 3 and probe(0, waves=33) == 3 and probe(0, waves=-1) == 3
    assert probe(lohan.LOHAN_PROBE_READ, a=None) == 1
    assert probe(lohan.LOHAN_PROBE_WRITE, b=None) == 1
    assert probe(lohan.LOHAN_PROBE_COPY, b=None) == 1
    for name in ("a", "b", "c", "g", "h"):
        assert probe(lohan.LOHAN_PROBE_FIVE_STREAM, **{name: None}) == 1
        assert probe(lohan.LOHAN_PROBE_FIVE_STREAM, **{name: A + 8}) == 2
    assert probe(lohan.LOHAN_PROBE_FIVE_STREAM, n=(1 << 31) * 256) == 3
    assert probe(lohan.LOHAN_PROBE_FIVE_STREAM, n=255) == 0          # no whole tile: nothing to do


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_LIB", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.lohan_workspace_bytes()
