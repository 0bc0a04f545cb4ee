"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI, run the oracle on
host copies of the same bits, and compare in units in the last place."""
import numpy as np
import torch

import paper_2403_06504_amd as lohan
from paper_2403_06504_amd import synthetic_inputs as synth

# Parity bar: overflow flag and skipped state bit-exact; p/m/v within 2 fp32 ulp after 10 chained
# steps; bf16 copy within 1 bf16 ulp; squared norm within 1e-5 relative.
ULP_F32 = 2
ULP_BF16 = 1
RTOL_SQNORM = 1e-5


def ordered_int(bits: np.ndarray, width: int) -> np.ndarray:
    """Map sign-magnitude float bit patterns to integers whose order is the numeric order."""
    sign = 1 << (width - 1)
    b = bits.astype(np.int64)
    return np.where(b & sign, sign - b, b)


def max_ulp(got_bits: np.ndarray, want_bits: np.ndarray, width: int) -> int:
    """Largest distance in units in the last place; 0 fast path when the bits are equal."""
    if got_bits.size == 0 or np.array_equal(got_bits, want_bits):
        return 0
    idx = np.nonzero(got_bits != want_bits)[0]
    d = np.abs(ordered_int(got_bits[idx], width) - ordered_int(want_bits[idx], width))
    return int(d.max())


class DeviceBlock:
    """One block's buffers on the GPU plus the per-call scratch the ABI needs."""

    def __init__(self, tensors: dict, device="cuda"):
        self.p, self.m, self.v = tensors["p"], tensors["m"], tensors["v"]
        self.g, self.p16 = tensors["g"], tensors["p16"]
        self.n = self.p.numel()
        self.flag = torch.full((1,), 7, dtype=torch.int32, device=device)     # stale on purpose
        self.sqnorm = torch.full((1,), -1.0, dtype=torch.float64, device=device)
        # Garbage everywhere, then the documented one-time preparation.
        self.ws = torch.full((lohan.lohan_workspace_bytes(),), 0xA5, dtype=torch.uint8,
                             device=device)
        lohan.lohan_workspace_init(self.ws)
        torch.cuda.current_stream().synchronize()      # usable from side streams from here on

    def step(self, hy: dict, flags: int = 0, stream=None):
        lohan.lohan_adam_block_step(self.p, self.m, self.v, self.g, self.p16, self.n,
                                    hy["lr"], hy["beta1"], hy["beta2"], hy["eps"],
                                    hy["weight_decay"], hy["step"], hy["loss_scale"],
                                    self.flag, flags, self.ws, stream=stream)

    def check(self, stream=None):
        lohan.lohan_grad_overflow_check(self.g, self.n, self.flag, self.ws, stream=stream)

    def norm(self, loss_scale, want_flag=True, stream=None):
        lohan.lohan_grad_sqnorm(self.g, self.n, loss_scale, self.sqnorm,
                                self.flag if want_flag else None, self.ws, stream=stream)

    def host(self, lo=0, hi=None) -> dict:
        """Host copies (numpy; 16-bit floats as uint16 bit patterns) of [lo, hi)."""
        hi = self.n if hi is None else hi
        return {k: synth.to_numpy_bits(getattr(self, k)[lo:hi]) for k in ("p", "m", "v", "g", "p16")}

    def flag_value(self) -> int:
        return int(self.flag.cpu().item())


def oracle_steps(oracle, host: dict, hy: dict, steps: int, l2_mode=False, nthreads=16):
    """Chain `steps` oracle steps in place on host copies, advancing the step index; returns the
    flags of every step."""
    flags = []
    for k in range(steps):
        f = oracle.adam_block_step(host["p"], host["m"], host["v"], host["g"], host["p16"],
                                   lr=hy["lr"], beta1=hy["beta1"], beta2=hy["beta2"],
                                   eps=hy["eps"], weight_decay=hy["weight_decay"],
                                   step=hy["step"] + k, loss_scale=hy["loss_scale"],
                                   l2_mode=l2_mode, nthreads=nthreads)
        flags.append(f)
    return flags


def gpu_steps(blk: DeviceBlock, hy: dict, steps: int, l2_mode=False, stream=None):
    flags = []
    for k in range(steps):
        h = dict(hy, step=hy["step"] + k)
        blk.step(h, flags=lohan.LOHAN_FLAG_L2_MODE if l2_mode else 0, stream=stream)
        torch.cuda.synchronize()
        flags.append(blk.flag_value())
    return flags


def assert_state_parity(got: dict, want: dict, what=""):
    """got/want: host dicts with p, m, v (float32) and p16 (uint16 bits)."""
    worst = {}
    for k in ("p", "m", "v"):
        worst[k] = max_ulp(got[k].view(np.uint32), want[k].view(np.uint32), 32)
    worst["p16"] = max_ulp(got["p16"], want["p16"], 16)
    for k in ("p", "m", "v"):
        assert worst[k] <= ULP_F32, f"{what}: {k} differs by {worst[k]} ulp (bar {ULP_F32})"
    assert worst["p16"] <= ULP_BF16, f"{what}: p16 differs by {worst['p16']} ulp (bar {ULP_BF16})"
    return worst


def assert_scale_within_one_ulp(s_eff_gpu, s_eff_orc, what=""):
    """Clipped route, first half of the bar: the effective loss scale fp32(S / coef) that the HIP
    path derives from ITS squared norm and the one the oracle derives from its own may differ by
    at most one fp32 unit in the last place (the two norms agree to 1e-5 relative or far better,
    and the scale is rounded once to fp32).  The second half -- the oracle stepped with the HIP
    path's own effective scale equals the HIP result bit for bit -- is assert_state_parity with
    an all-zero worst case, at the call site."""
    a = int(np.float32(s_eff_gpu).view(np.uint32))
    b = int(np.float32(s_eff_orc).view(np.uint32))
    assert abs(a - b) <= 1, (what, float(np.float32(s_eff_gpu)), float(np.float32(s_eff_orc)))
