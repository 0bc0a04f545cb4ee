"""ctypes front end of the C oracle (oracle/lohan_oracle.c).

TEST INFRASTRUCTURE: imported only by tests/, __graft_entry__.smoke() and bench.py's cpu_baseline
leg.  Nothing here touches the HIP library.  Arrays are numpy, host memory, modified in place.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        path = _build.LIB
        if not os.path.exists(path):
            path = _build.build(force=True)
        lib = ctypes.CDLL(path)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f32p = ctypes.POINTER(ctypes.c_float)
        lib.lohan_oracle_grad_overflow_check.argtypes = [u16p, ctypes.c_uint64]
        lib.lohan_oracle_grad_overflow_check.restype = ctypes.c_int
        lib.lohan_oracle_grad_sqnorm.argtypes = [u16p, ctypes.c_uint64, ctypes.c_float]
        lib.lohan_oracle_grad_sqnorm.restype = ctypes.c_double
        lib.lohan_oracle_grad_produce.argtypes = [f32p, ctypes.c_uint64, ctypes.c_float, u16p]
        lib.lohan_oracle_grad_produce.restype = None
        lib.lohan_oracle_step_scalars.argtypes = [ctypes.c_float] * 4 + [ctypes.c_int64,
                                                                         ctypes.c_float, f32p]
        lib.lohan_oracle_step_scalars.restype = None
        lib.lohan_oracle_adam_block_step.argtypes = [
            f32p, f32p, f32p, u16p, u16p, ctypes.c_uint64,
            ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_float,
            ctypes.c_int64, ctypes.c_float, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.lohan_oracle_adam_block_step.restype = ctypes.c_int
        lib.lohan_oracle_max_threads.argtypes = []
        lib.lohan_oracle_max_threads.restype = ctypes.c_int
        lib.lohan_oracle_half_bits_to_float.argtypes = [ctypes.c_uint16]
        lib.lohan_oracle_half_bits_to_float.restype = ctypes.c_float
        lib.lohan_oracle_float_to_bf16_bits.argtypes = [ctypes.c_float]
        lib.lohan_oracle_float_to_bf16_bits.restype = ctypes.c_uint16
        lib.lohan_oracle_float_to_half_bits.argtypes = [ctypes.c_float]
        lib.lohan_oracle_float_to_half_bits.restype = ctypes.c_uint16
        _LIB = lib
    return _LIB


def _ptr(a, dtype, ctype):
    if not isinstance(a, np.ndarray) or a.dtype != dtype or not a.flags.c_contiguous:
        raise TypeError(f"expected a C-contiguous numpy array of {dtype}, got {type(a)} "
                        f"{getattr(a, 'dtype', None)}")
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def grad_overflow_check(grad_fp16_bits: np.ndarray) -> int:
    """Overflow flag of a block: 1 if any fp16 gradient has an all-ones exponent field."""
    g = _ptr(grad_fp16_bits, np.uint16, ctypes.c_uint16)
    return int(_lib().lohan_oracle_grad_overflow_check(g, grad_fp16_bits.size))


def grad_sqnorm(grad_fp16_bits: np.ndarray, loss_scale: float) -> float:
    """sum_i (g16_i / loss_scale)^2 in float64, index order."""
    g = _ptr(grad_fp16_bits, np.uint16, ctypes.c_uint16)
    return float(_lib().lohan_oracle_grad_sqnorm(g, grad_fp16_bits.size, loss_scale))


def grad_produce(grad_fp32: np.ndarray, multiplier: float) -> np.ndarray:
    """binary16 bit patterns of fl(grad_fp32 * multiplier), round to nearest even."""
    out = np.empty(grad_fp32.size, dtype=np.uint16)
    _lib().lohan_oracle_grad_produce(_ptr(grad_fp32, np.float32, ctypes.c_float), grad_fp32.size,
                                     float(multiplier), _ptr(out, np.uint16, ctypes.c_uint16))
    return out


def step_scalars(lr, beta1, beta2, weight_decay, step, loss_scale) -> dict:
    """The per-call fp32 scalars, as a dict of numpy float32."""
    out = np.zeros(8, dtype=np.float32)
    _lib().lohan_oracle_step_scalars(lr, beta1, beta2, weight_decay, int(step), loss_scale,
                                     _ptr(out, np.float32, ctypes.c_float))
    names = ["inv", "omb1", "omb2", "bc1", "bc2", "sbc2", "ss", "decay"]
    return {k: out[i] for i, k in enumerate(names)}


def adam_block_step(param_fp32, exp_avg, exp_avg_sq, grad_fp16_bits, param_bf16_bits, *,
                    lr, beta1, beta2, eps, weight_decay, step, loss_scale, l2_mode=False,
                    half_out=False, nthreads=1) -> int:
    """One block step in place on numpy arrays; returns the overflow flag (1 = nothing written).
    half_out=True emits the 16-bit copy as IEEE binary16 instead of bfloat16."""
    n = param_fp32.size
    for a in (exp_avg, exp_avg_sq, grad_fp16_bits, param_bf16_bits):
        if a.size != n:
            raise ValueError("all block buffers must have the same element count")
    return int(_lib().lohan_oracle_adam_block_step(
        _ptr(param_fp32, np.float32, ctypes.c_float),
        _ptr(exp_avg, np.float32, ctypes.c_float),
        _ptr(exp_avg_sq, np.float32, ctypes.c_float),
        _ptr(grad_fp16_bits, np.uint16, ctypes.c_uint16),
        _ptr(param_bf16_bits, np.uint16, ctypes.c_uint16),
        n, lr, beta1, beta2, eps, weight_decay, int(step), loss_scale, int(bool(l2_mode)),
        int(bool(half_out)), int(nthreads)))


def max_threads() -> int:
    return int(_lib().lohan_oracle_max_threads())


def half_bits_to_float(h: int) -> np.float32:
    return np.float32(_lib().lohan_oracle_half_bits_to_float(int(h)))


def float_to_bf16_bits(x) -> int:
    return int(_lib().lohan_oracle_float_to_bf16_bits(np.float32(x)))


def float_to_half_bits(x) -> int:
    return int(_lib().lohan_oracle_float_to_half_bits(np.float32(x)))


def clip_loss_scale(sqnorm: float, loss_scale: float, max_norm: float) -> np.float32:
    """Effective loss scale that folds per-block norm clipping into the unscale multiply:
    coef = min(1, max_norm / (sqrt(sqnorm) + 1e-6)); S_eff = fl32(S / coef), in float64 until
    the final rounding."""
    coef = min(1.0, float(max_norm) / (float(np.sqrt(np.float64(sqnorm))) + 1e-6))
    return np.float32(np.float64(loss_scale) / np.float64(coef))
