"""ctypes binding of liblohan_adam.so -- argument marshalling only.

Each function has the name and argument order of the C entry point it calls
(include/lohan_adam.h).  Device buffers may be given as torch tensors (their data_ptr() is taken;
dtype, contiguity and length are checked against n) or as raw integer device addresses; `stream`
may be a torch.cuda.Stream, a raw hipStream_t integer, or None for torch's current stream.
Nothing is computed here, and nothing falls back to the host: without the built library every
call raises.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liblohan_adam.so")
_LIB = None

LOHAN_OK = 0
LOHAN_FLAG_L2_MODE = 1
LOHAN_FLAG_PRECHECKED = 2
LOHAN_FLAG_P16_FP16 = 4

EXPORTS = (
    "lohan_workspace_bytes", "lohan_status_string", "lohan_grad_overflow_check",
    "lohan_grad_sqnorm", "lohan_grad_sqnorm_static", "lohan_grad_produce_fp16",
    "lohan_adam_block_step", "lohan_adam_block_step_clipped",
    "lohan_adam_small_block_max_n", "lohan_adam_small_block_step",
    "lohan_adam_block_step_out_of_place", "lohan_adam_block_step_out_of_place_clipped",
    "lohan_adam_multi_block_step", "lohan_model_placement", "lohan_model_placement_compact",
    "lohan_tensor_placement",
    "lohan_ring_bytes", "lohan_ring_init", "lohan_ring_adam_block_step",
    "lohan_ring_adam_block_step_clipped", "lohan_ring_read",
    "lohan_clip_loss_scale", "lohan_workspace_init",
    "lohan_tuning_set_launch_config", "lohan_tuning_get_launch_config",
    "lohan_tuning_set_wait_limit",
    "lohan_tuning_device_info", "lohan_tuning_probe", "lohan_tuning_offload_inject_failure",
    "lohan_tuning_offload_slot_times",
    "lohan_offload_slab_bytes", "lohan_offload_create", "lohan_offload_submit",
    "lohan_offload_wait_last_step", "lohan_offload_drain", "lohan_offload_destroy",
    "lohan_swap_iter_time", "lohan_swap_recompute_flops", "lohan_plan_activation_swapping",
)

LOHAN_OFFLOAD_SERIALIZED = 0
LOHAN_OFFLOAD_OVERLAPPED = 1


class LohanLayer(ctypes.Structure):
    """Mirror of lohan_layer_t."""
    _fields_ = [("flop", ctypes.c_double), ("act_bytes", ctypes.c_double)]


class LohanSwapHw(ctypes.Structure):
    """Mirror of lohan_swap_hw_t."""
    _fields_ = [(k, ctypes.c_double) for k in ("thp_g", "bw_g", "bw_s2m", "bw_m2s", "params",
                                               "mem_avail", "flop_f", "a_interblock")]


class LohanOffloadBlock(ctypes.Structure):
    """Mirror of lohan_offload_block_t."""
    _fields_ = [("host_param_fp32", ctypes.c_void_p), ("host_exp_avg", ctypes.c_void_p),
                ("host_exp_avg_sq", ctypes.c_void_p), ("grad_fp16", ctypes.c_void_p),
                ("param_bf16_out", ctypes.c_void_p), ("n", ctypes.c_uint64),
                ("overflow_flag", ctypes.c_void_p), ("sqnorm", ctypes.c_void_p)]


class LohanBlock(ctypes.Structure):
    """Mirror of lohan_block_t."""
    _fields_ = [("param_fp32", ctypes.c_void_p), ("exp_avg", ctypes.c_void_p),
                ("exp_avg_sq", ctypes.c_void_p), ("grad_fp16", ctypes.c_void_p),
                ("param_bf16_out", ctypes.c_void_p), ("n", ctypes.c_uint64)]


class LohanRingSlot(ctypes.Structure):
    """Mirror of lohan_ring_slot_t."""
    _fields_ = [("param_fp32", ctypes.c_void_p), ("exp_avg", ctypes.c_void_p),
                ("exp_avg_sq", ctypes.c_void_p), ("param_16", ctypes.c_void_p),
                ("n", ctypes.c_uint64)]


class LohanBlockOffsets(ctypes.Structure):
    """Mirror of lohan_block_offsets_t."""
    _fields_ = [(k, ctypes.c_size_t) for k in ("param_fp32", "exp_avg", "exp_avg_sq", "grad_fp16",
                                               "param_bf16")]


class LohanError(RuntimeError):
    """A C entry point returned a status other than LOHAN_OK."""

    def __init__(self, status: int, message: str):
        super().__init__(f"lohan status {status}: {message}")
        self.status = status


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the in-tree shared library (built by paper_2403_06504_amd/build.py)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: build it first (python -m paper_2403_06504_amd.build, or "
            "__graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, u64, f32, sz = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_float, ctypes.c_size_t
    lib.lohan_workspace_bytes.argtypes = []
    lib.lohan_workspace_bytes.restype = sz
    lib.lohan_status_string.argtypes = [ctypes.c_int]
    lib.lohan_status_string.restype = ctypes.c_char_p
    lib.lohan_grad_overflow_check.argtypes = [vp, u64, vp, vp, sz, vp]
    lib.lohan_grad_overflow_check.restype = ctypes.c_int
    lib.lohan_grad_sqnorm.argtypes = [vp, u64, f32, vp, vp, vp, sz, vp]
    lib.lohan_grad_sqnorm.restype = ctypes.c_int
    lib.lohan_grad_sqnorm_static.argtypes = [vp, u64, f32, vp, vp, vp]
    lib.lohan_grad_sqnorm_static.restype = ctypes.c_int
    lib.lohan_grad_produce_fp16.argtypes = [vp, u64, f32, vp, f32, vp, vp, vp, sz, vp]
    lib.lohan_grad_produce_fp16.restype = ctypes.c_int
    lib.lohan_adam_block_step.argtypes = [vp, vp, vp, vp, vp, u64, f32, f32, f32, f32, f32,
                                          ctypes.c_int64, f32, vp, ctypes.c_uint32, vp, sz, vp]
    lib.lohan_adam_block_step.restype = ctypes.c_int
    lib.lohan_adam_block_step_clipped.argtypes = [vp, vp, vp, vp, vp, u64, f32, f32, f32, f32,
                                                  f32, ctypes.c_int64, f32, vp, f32, vp,
                                                  ctypes.c_uint32, vp, sz, vp]
    lib.lohan_adam_block_step_clipped.restype = ctypes.c_int
    lib.lohan_adam_small_block_max_n.argtypes = [ctypes.POINTER(u64)]
    lib.lohan_adam_small_block_max_n.restype = ctypes.c_int
    lib.lohan_adam_small_block_step.argtypes = [vp, vp, vp, vp, vp, u64, f32, f32, f32, f32, f32,
                                                ctypes.c_int64, f32, vp, vp, ctypes.c_uint32, vp,
                                                sz, vp]
    lib.lohan_adam_small_block_step.restype = ctypes.c_int
    lib.lohan_tuning_set_wait_limit.argtypes = [ctypes.c_int64]
    lib.lohan_tuning_set_wait_limit.restype = ctypes.c_int
    lib.lohan_adam_block_step_out_of_place.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, u64, f32,
                                                       f32, f32, f32, f32, ctypes.c_int64, f32,
                                                       vp, ctypes.c_uint32, vp]
    lib.lohan_adam_block_step_out_of_place.restype = ctypes.c_int
    lib.lohan_adam_multi_block_step.argtypes = [ctypes.POINTER(LohanBlock), ctypes.c_uint32, f32,
                                                f32, f32, f32, f32, ctypes.c_int64, f32, f32, vp,
                                                vp, ctypes.c_uint32, vp, sz, vp]
    lib.lohan_adam_multi_block_step.restype = ctypes.c_int
    lib.lohan_adam_block_step_out_of_place_clipped.argtypes = [
        vp, vp, vp, vp, vp, vp, vp, vp, u64, f32, f32, f32, f32, f32, ctypes.c_int64, f32, vp, f32,
        vp, ctypes.c_uint32, vp, sz, vp]
    lib.lohan_adam_block_step_out_of_place_clipped.restype = ctypes.c_int
    u32 = ctypes.c_uint32
    lib.lohan_ring_bytes.argtypes = [u32, u32]
    lib.lohan_ring_bytes.restype = sz
    lib.lohan_ring_init.argtypes = [vp, sz, ctypes.POINTER(LohanRingSlot), u32, u32]
    lib.lohan_ring_init.restype = ctypes.c_int
    lib.lohan_ring_adam_block_step.argtypes = [vp, u32, u32, u32, vp, u64, f32, f32, f32, f32, f32,
                                               ctypes.c_int64, f32, u32, vp]
    lib.lohan_ring_adam_block_step.restype = ctypes.c_int
    lib.lohan_ring_adam_block_step_clipped.argtypes = [vp, u32, u32, u32, vp, u64, f32, f32, f32,
                                                       f32, f32, ctypes.c_int64, f32, vp, f32,
                                                       u32, vp]
    lib.lohan_ring_adam_block_step_clipped.restype = ctypes.c_int
    lib.lohan_ring_read.argtypes = [vp, u32, u32, ctypes.POINTER(u32), ctypes.POINTER(u32),
                                    ctypes.POINTER(u32), vp]
    lib.lohan_ring_read.restype = ctypes.c_int
    lib.lohan_model_placement_compact.argtypes = [u64, u32, ctypes.POINTER(LohanBlockOffsets),
                                                  ctypes.POINTER(sz), ctypes.POINTER(sz)]
    lib.lohan_model_placement_compact.restype = ctypes.c_int
    lib.lohan_tensor_placement.argtypes = [ctypes.POINTER(u64), u32,
                                           ctypes.POINTER(LohanBlockOffsets), ctypes.POINTER(sz),
                                           ctypes.POINTER(sz)]
    lib.lohan_tensor_placement.restype = ctypes.c_int
    lib.lohan_model_placement.argtypes = [u64, ctypes.c_uint32, ctypes.POINTER(LohanBlockOffsets),
                                          ctypes.POINTER(sz), ctypes.POINTER(sz),
                                          ctypes.POINTER(ctypes.c_uint32)]
    lib.lohan_model_placement.restype = ctypes.c_int
    lib.lohan_clip_loss_scale.argtypes = [ctypes.c_double, f32, f32]
    lib.lohan_clip_loss_scale.restype = f32
    lib.lohan_workspace_init.argtypes = [vp, sz, vp]
    lib.lohan_workspace_init.restype = ctypes.c_int
    lib.lohan_tuning_set_launch_config.argtypes = [ctypes.c_int] * 5
    lib.lohan_tuning_set_launch_config.restype = ctypes.c_int
    lib.lohan_tuning_get_launch_config.argtypes = [ctypes.POINTER(ctypes.c_int)] * 5
    lib.lohan_tuning_get_launch_config.restype = None
    lib.lohan_tuning_device_info.argtypes = [ctypes.POINTER(ctypes.c_int), ctypes.POINTER(sz)]
    lib.lohan_tuning_device_info.restype = ctypes.c_int
    lib.lohan_tuning_probe.argtypes = [ctypes.c_int, vp, vp, vp, vp, vp, u64, ctypes.c_int, vp]
    lib.lohan_tuning_probe.restype = ctypes.c_int
    lib.lohan_tuning_offload_inject_failure.argtypes = [vp, ctypes.c_int]
    lib.lohan_tuning_offload_inject_failure.restype = ctypes.c_int
    fp = ctypes.POINTER(ctypes.c_float)
    lib.lohan_tuning_offload_slot_times.argtypes = [vp, ctypes.c_int, fp, fp, fp]
    lib.lohan_tuning_offload_slot_times.restype = ctypes.c_int
    lib.lohan_offload_slab_bytes.argtypes = [u64, ctypes.c_int]
    lib.lohan_offload_slab_bytes.restype = sz
    lib.lohan_offload_create.argtypes = [ctypes.POINTER(vp), vp, sz, u64, ctypes.c_int,
                                         ctypes.c_int]
    lib.lohan_offload_create.restype = ctypes.c_int
    lib.lohan_offload_submit.argtypes = [vp, ctypes.POINTER(LohanOffloadBlock), f32, f32, f32,
                                         f32, f32, ctypes.c_int64, f32, f32, ctypes.c_uint32, vp]
    lib.lohan_offload_submit.restype = ctypes.c_int
    lib.lohan_offload_wait_last_step.argtypes = [vp, vp]
    lib.lohan_offload_wait_last_step.restype = ctypes.c_int
    lib.lohan_offload_drain.argtypes = [vp]
    lib.lohan_offload_drain.restype = ctypes.c_int
    lib.lohan_offload_destroy.argtypes = [vp]
    lib.lohan_offload_destroy.restype = ctypes.c_int
    lib.lohan_swap_iter_time.argtypes = [ctypes.POINTER(LohanSwapHw), ctypes.c_double,
                                         ctypes.c_double]
    lib.lohan_swap_iter_time.restype = ctypes.c_double
    lib.lohan_swap_recompute_flops.argtypes = [ctypes.POINTER(LohanLayer), sz, ctypes.c_double,
                                               ctypes.c_double, ctypes.POINTER(ctypes.c_double),
                                               ctypes.POINTER(ctypes.c_double)]
    lib.lohan_swap_recompute_flops.restype = ctypes.c_int
    lib.lohan_plan_activation_swapping.argtypes = [
        ctypes.POINTER(LohanLayer), sz, ctypes.POINTER(LohanSwapHw),
        ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(sz), ctypes.POINTER(ctypes.c_double),
        ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.lohan_plan_activation_swapping.restype = ctypes.c_int
    _LIB = lib
    return lib


def _check(status: int):
    if status != LOHAN_OK:
        raise LohanError(status, lohan_status_string(status))


def _addr(buf, n=None, dtype_name=None, what="buffer"):
    """Device address of a torch tensor or pass-through of an integer address / None."""
    if buf is None:
        return None
    if isinstance(buf, int):
        return buf
    if hasattr(buf, "data_ptr"):
        if not buf.is_contiguous():
            raise TypeError(f"{what}: tensor must be contiguous")
        if dtype_name is not None and str(buf.dtype) not in dtype_name:
            raise TypeError(f"{what}: expected dtype in {dtype_name}, got {buf.dtype}")
        if n is not None and buf.numel() < n:
            raise ValueError(f"{what}: tensor holds {buf.numel()} elements, need {n}")
        return buf.data_ptr()
    raise TypeError(f"{what}: expected a torch tensor, an integer device address or None")


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    if hasattr(stream, "cuda_stream"):
        return stream.cuda_stream
    raise TypeError("stream: expected torch.cuda.Stream, an integer hipStream_t or None")


def _workspace(workspace, workspace_bytes):
    if workspace is None:
        return None, 0
    if isinstance(workspace, int):
        if workspace_bytes is None:
            raise ValueError("workspace_bytes is required with a raw workspace address")
        return workspace, int(workspace_bytes)
    nbytes = workspace.numel() * workspace.element_size()
    return _addr(workspace, what="workspace"), nbytes if workspace_bytes is None else int(
        workspace_bytes)


_F16 = ("torch.float16", "torch.int16", "torch.uint16")
_BF16 = ("torch.bfloat16", "torch.float16", "torch.int16", "torch.uint16")
_F32 = ("torch.float32",)
_U32 = ("torch.int32", "torch.uint32")
_F64 = ("torch.float64",)


def lohan_workspace_bytes() -> int:
    return int(load_library().lohan_workspace_bytes())


def lohan_status_string(status: int) -> str:
    return load_library().lohan_status_string(int(status)).decode()


def lohan_workspace_init(workspace, workspace_bytes=None, stream=None):
    ws, ws_bytes = _workspace(workspace, workspace_bytes)
    _check(load_library().lohan_workspace_init(ws, ws_bytes, _stream(stream)))


def new_workspace(device, stream=None):
    """A torch uint8 tensor of lohan_workspace_bytes() on `device`, prepared with
    lohan_workspace_init on `stream` and ready for use on ANY stream when this returns (the
    preparation is waited for; torch supplies the memory, the library the contents)."""
    import torch
    ws = torch.empty(lohan_workspace_bytes(), dtype=torch.uint8, device=device)
    lohan_workspace_init(ws, stream=stream)
    torch.cuda.synchronize()
    return ws


def lohan_grad_overflow_check(grad_fp16, n, overflow_flag, workspace, workspace_bytes=None,
                              stream=None):
    ws, ws_bytes = _workspace(workspace, workspace_bytes)
    _check(load_library().lohan_grad_overflow_check(
        _addr(grad_fp16, n, _F16, "grad_fp16"), int(n),
        _addr(overflow_flag, 1, _U32, "overflow_flag"), ws, ws_bytes, _stream(stream)))


def lohan_grad_sqnorm(grad_fp16, n, loss_scale, sqnorm, overflow_flag, workspace,
                      workspace_bytes=None, stream=None):
    ws, ws_bytes = _workspace(workspace, workspace_bytes)
    _check(load_library().lohan_grad_sqnorm(
        _addr(grad_fp16, n, _F16, "grad_fp16"), int(n), float(loss_scale),
        _addr(sqnorm, 1, _F64, "sqnorm"), _addr(overflow_flag, 1, _U32, "overflow_flag"),
        ws, ws_bytes, _stream(stream)))


def lohan_grad_produce_fp16(grad_fp32, n, multiplier, grad_fp16_out, loss_scale, sqnorm,
                            overflow_flag, workspace, workspace_bytes=None, stream=None):
    ws, ws_bytes = _workspace(workspace, workspace_bytes)
    _check(load_library().lohan_grad_produce_fp16(
        _addr(grad_fp32, n, _F32, "grad_fp32"), int(n), float(multiplier),
        _addr(grad_fp16_out, n, _F16, "grad_fp16_out"), float(loss_scale),
        _addr(sqnorm, 1, _F64, "sqnorm"), _addr(overflow_flag, 1, _U32, "overflow_flag"),
        ws, ws_bytes, _stream(stream)))


def lohan_grad_sqnorm_static(grad_fp16, n, loss_scale, sqnorm, overflow_flag, stream=None):
    _check(load_library().lohan_grad_sqnorm_static(
        _addr(grad_fp16, n, _F16, "grad_fp16"), int(n), float(loss_scale),
        _addr(sqnorm, 1, _F64, "sqnorm"), _addr(overflow_flag, 1, _U32, "overflow_flag"),
        _stream(stream)))


def lohan_adam_block_step(param_fp32, exp_avg, exp_avg_sq, grad_fp16, param_bf16_out, n,
                          lr, beta1, beta2, eps, weight_decay, step, loss_scale,
                          overflow_flag, flags, workspace, workspace_bytes=None, stream=None):
    ws, ws_bytes = _workspace(workspace, workspace_bytes)
    _check(load_library().lohan_adam_block_step(
        _addr(param_fp32, n, _F32, "param_fp32"), _addr(exp_avg, n, _F32, "exp_avg"),
        _addr(exp_avg_sq, n, _F32, "exp_avg_sq"), _addr(grad_fp16, n, _F16, "grad_fp16"),
        _addr(param_bf16_out, n, _BF16, "param_bf16_out"), int(n),
        float(lr), float(beta1), float(beta2), float(eps), float(weight_decay), int(step),
        float(loss_scale), _addr(overflow_flag, 1, _U32, "overflow_flag"), int(flags),
        ws, ws_bytes, _stream(stream)))


def lohan_adam_block_step_clipped(param_fp32, exp_avg, exp_avg_sq, grad_fp16, param_bf16_out, n,
                                  lr, beta1, beta2, eps, weight_decay, step, loss_scale,
                                  sqnorm, max_norm, overflow_flag, flags, workspace,
                                  workspace_bytes=None, stream=None):
    ws, ws_bytes = _workspace(workspace, workspace_bytes)
    _check(load_library().lohan_adam_block_step_clipped(
        _addr(param_fp32, n, _F32, "param_fp32"), _addr(exp_avg, n, _F32, "exp_avg"),
        _addr(exp_avg_sq, n, _F32, "exp_avg_sq"), _addr(grad_fp16, n, _F16, "grad_fp16"),
        _addr(param_bf16_out, n, _BF16, "param_bf16_out"), int(n),
        float(lr), float(beta1), float(beta2), float(eps), float(weight_decay), int(step),
        float(loss_scale), _addr(sqnorm, 1, _F64, "sqnorm"), float(max_norm),
        _addr(overflow_flag, 1, _U32, "overflow_flag"), int(flags), ws, ws_bytes,
        _stream(stream)))


LOHAN_OVERFLOW_INCOMPLETE = 0x80000000


def lohan_adam_small_block_max_n() -> int:
    out = ctypes.c_uint64()
    _check(load_library().lohan_adam_small_block_max_n(ctypes.byref(out)))
    return out.value


def lohan_adam_small_block_step(param_fp32, exp_avg, exp_avg_sq, grad_fp16, param_bf16_out, n,
                                lr, beta1, beta2, eps, weight_decay, step, loss_scale, sqnorm,
                                overflow_flag, flags, workspace, workspace_bytes=None,
                                stream=None):
    ws, ws_bytes = _workspace(workspace, workspace_bytes)
    _check(load_library().lohan_adam_small_block_step(
        _addr(param_fp32, n, _F32, "param_fp32"), _addr(exp_avg, n, _F32, "exp_avg"),
        _addr(exp_avg_sq, n, _F32, "exp_avg_sq"), _addr(grad_fp16, n, _F16, "grad_fp16"),
        _addr(param_bf16_out, n, _BF16, "param_bf16_out"), int(n),
        float(lr), float(beta1), float(beta2), float(eps), float(weight_decay), int(step),
        float(loss_scale), None if sqnorm is None else _addr(sqnorm, 1, _F64, "sqnorm"),
        _addr(overflow_flag, 1, _U32, "overflow_flag"), int(flags), ws, ws_bytes,
        _stream(stream)))


def lohan_adam_block_step_out_of_place(param_fp32_in, exp_avg_in, exp_avg_sq_in, grad_fp16,
                                       param_fp32_out, exp_avg_out, exp_avg_sq_out,
                                       param_bf16_out, n, lr, beta1, beta2, eps, weight_decay,
                                       step, loss_scale, overflow_flag, flags=0, stream=None):
    _check(load_library().lohan_adam_block_step_out_of_place(
        _addr(param_fp32_in, n, _F32, "param_fp32_in"), _addr(exp_avg_in, n, _F32, "exp_avg_in"),
        _addr(exp_avg_sq_in, n, _F32, "exp_avg_sq_in"), _addr(grad_fp16, n, _F16, "grad_fp16"),
        _addr(param_fp32_out, n, _F32, "param_fp32_out"),
        _addr(exp_avg_out, n, _F32, "exp_avg_out"),
        _addr(exp_avg_sq_out, n, _F32, "exp_avg_sq_out"),
        _addr(param_bf16_out, n, _BF16, "param_bf16_out"), int(n),
        float(lr), float(beta1), float(beta2), float(eps), float(weight_decay), int(step),
        float(loss_scale), _addr(overflow_flag, 1, _U32, "overflow_flag"), int(flags),
        _stream(stream)))


def make_block_array(blocks):
    """ctypes array of lohan_block_t from a sequence of (param_fp32, exp_avg, exp_avg_sq,
    grad_fp16, param_bf16_out, n) tuples of tensors / addresses.  Build it once and pass it to
    lohan_adam_multi_block_step on every step: the addresses do not change."""
    arr = (LohanBlock * max(1, len(blocks)))()
    for i, (p, m, v, g, h, n) in enumerate(blocks):
        arr[i] = LohanBlock(_addr(p, n, _F32, "param_fp32"), _addr(m, n, _F32, "exp_avg"),
                            _addr(v, n, _F32, "exp_avg_sq"), _addr(g, n, _F16, "grad_fp16"),
                            _addr(h, n, _BF16, "param_bf16_out"), int(n))
    return arr


def lohan_adam_multi_block_step(blocks, lr, beta1, beta2, eps, weight_decay, step, loss_scale,
                                max_norm, overflow_flags, sqnorms, flags, workspace,
                                workspace_bytes=None, stream=None, num_blocks=None):
    """`blocks`: a sequence of tuples (see make_block_array) or an array it returned (then pass
    num_blocks)."""
    if isinstance(blocks, (list, tuple)):
        num_blocks = len(blocks)
        blocks = make_block_array(blocks)
    elif num_blocks is None:
        num_blocks = len(blocks)
    ws, ws_bytes = _workspace(workspace, workspace_bytes)
    _check(load_library().lohan_adam_multi_block_step(
        blocks, int(num_blocks), float(lr), float(beta1), float(beta2), float(eps),
        float(weight_decay), int(step), float(loss_scale), float(max_norm),
        _addr(overflow_flags, num_blocks, _U32, "overflow_flags"),
        _addr(sqnorms, num_blocks, _F64, "sqnorms"), int(flags), ws, ws_bytes, _stream(stream)))


def lohan_adam_block_step_out_of_place_clipped(param_fp32_in, exp_avg_in, exp_avg_sq_in,
                                               grad_fp16, param_fp32_out, exp_avg_out,
                                               exp_avg_sq_out, param_bf16_out, n, lr, beta1,
                                               beta2, eps, weight_decay, step, loss_scale, sqnorm,
                                               max_norm, overflow_flag, flags, workspace,
                                               workspace_bytes=None, stream=None):
    ws, ws_bytes = _workspace(workspace, workspace_bytes)
    _check(load_library().lohan_adam_block_step_out_of_place_clipped(
        _addr(param_fp32_in, n, _F32, "param_fp32_in"), _addr(exp_avg_in, n, _F32, "exp_avg_in"),
        _addr(exp_avg_sq_in, n, _F32, "exp_avg_sq_in"), _addr(grad_fp16, n, _F16, "grad_fp16"),
        _addr(param_fp32_out, n, _F32, "param_fp32_out"),
        _addr(exp_avg_out, n, _F32, "exp_avg_out"),
        _addr(exp_avg_sq_out, n, _F32, "exp_avg_sq_out"),
        _addr(param_bf16_out, n, _BF16, "param_bf16_out"), int(n),
        float(lr), float(beta1), float(beta2), float(eps), float(weight_decay), int(step),
        float(loss_scale), _addr(sqnorm, 1, _F64, "sqnorm"), float(max_norm),
        _addr(overflow_flag, 1, _U32, "overflow_flag"), int(flags), ws, ws_bytes,
        _stream(stream)))


def lohan_ring_bytes(num_blocks, num_spares=1) -> int:
    return int(load_library().lohan_ring_bytes(int(num_blocks), int(num_spares)))


def lohan_ring_init(ring, slots, num_blocks, ring_bytes=None):
    """slots: sequence of tuples (param_fp32, exp_avg, exp_avg_sq, param_16, n) of tensors /
    addresses: first the num_blocks block slots, then one spare per distinct length; `ring`:
    uint8 device tensor or address."""
    num_spares = len(slots) - num_blocks
    arr = (LohanRingSlot * len(slots))()
    for i, (p, m, v, h, n) in enumerate(slots):
        arr[i] = LohanRingSlot(_addr(p, n, _F32, "param_fp32"), _addr(m, n, _F32, "exp_avg"),
                               _addr(v, n, _F32, "exp_avg_sq"), _addr(h, n, _BF16, "param_16"),
                               int(n))
    if ring_bytes is None:
        ring_bytes = ring.numel() * ring.element_size() if hasattr(ring, "numel") else 0
    _check(load_library().lohan_ring_init(_addr(ring, what="ring"), int(ring_bytes), arr,
                                          int(num_blocks), int(num_spares)))


def lohan_ring_adam_block_step(ring, num_blocks, num_spares, block, grad_fp16, n, lr, beta1,
                               beta2, eps, weight_decay, step, loss_scale, flags=0, stream=None):
    _check(load_library().lohan_ring_adam_block_step(
        _addr(ring, what="ring"), int(num_blocks), int(num_spares), int(block),
        _addr(grad_fp16, n, _F16, "grad_fp16"), int(n), float(lr), float(beta1), float(beta2),
        float(eps), float(weight_decay), int(step), float(loss_scale), int(flags),
        _stream(stream)))


def lohan_ring_adam_block_step_clipped(ring, num_blocks, num_spares, block, grad_fp16, n, lr,
                                       beta1, beta2, eps, weight_decay, step, loss_scale, sqnorm,
                                       max_norm, flags=0, stream=None):
    _check(load_library().lohan_ring_adam_block_step_clipped(
        _addr(ring, what="ring"), int(num_blocks), int(num_spares), int(block),
        _addr(grad_fp16, n, _F16, "grad_fp16"), int(n), float(lr), float(beta1), float(beta2),
        float(eps), float(weight_decay), int(step), float(loss_scale),
        _addr(sqnorm, 1, _F64, "sqnorm"), float(max_norm), int(flags), _stream(stream)))


def lohan_ring_read(ring, num_blocks, num_spares=1, stream=None):
    """Synchronises the stream.  Returns (slot_of list, spares list, skipped list of 0/1)."""
    slot_of = (ctypes.c_uint32 * num_blocks)()
    last = (ctypes.c_uint32 * num_blocks)()
    spares = (ctypes.c_uint32 * num_spares)()
    _check(load_library().lohan_ring_read(_addr(ring, what="ring"), int(num_blocks),
                                          int(num_spares), slot_of, spares, last,
                                          _stream(stream)))
    return list(slot_of), list(spares), list(last)


def lohan_model_placement_compact(n, num_blocks=1):
    """Returns (offsets, slab_bytes, slab_alignment); offsets as lohan_model_placement's."""
    arr = (LohanBlockOffsets * max(1, num_blocks))()
    total, align = ctypes.c_size_t(), ctypes.c_size_t()
    _check(load_library().lohan_model_placement_compact(int(n), int(num_blocks), arr,
                                                        ctypes.byref(total), ctypes.byref(align)))
    fields = [f for f, _ in LohanBlockOffsets._fields_]
    return ([{f: getattr(arr[b], f) for f in fields} for b in range(num_blocks)], total.value,
            align.value)


def lohan_tensor_placement(lengths):
    """Returns (offsets, slab_bytes, slab_alignment); offsets as lohan_model_placement's."""
    count = len(lengths)
    arr = (ctypes.c_uint64 * max(1, count))(*[int(x) for x in lengths])
    out = (LohanBlockOffsets * max(1, count))()
    total, align = ctypes.c_size_t(), ctypes.c_size_t()
    _check(load_library().lohan_tensor_placement(arr, count, out, ctypes.byref(total),
                                                 ctypes.byref(align)))
    fields = [f for f, _ in LohanBlockOffsets._fields_]
    return ([{f: getattr(out[b], f) for f in fields} for b in range(count)], total.value,
            align.value)


def lohan_model_placement(n, num_blocks=None):
    """Returns (offsets, slab_bytes, slab_alignment, blocks_per_group); offsets is a list of dicts
    with the byte offsets of param_fp32, exp_avg, exp_avg_sq, grad_fp16, param_bf16 for each
    block.  num_blocks=None lays out exactly one full group."""
    lib = load_library()
    group = ctypes.c_uint32()
    total, align = ctypes.c_size_t(), ctypes.c_size_t()
    if num_blocks is None:
        _check(lib.lohan_model_placement(int(n), 0, None, ctypes.byref(total),
                                         ctypes.byref(align), ctypes.byref(group)))
        num_blocks = group.value
    arr = (LohanBlockOffsets * max(1, num_blocks))()
    _check(lib.lohan_model_placement(int(n), int(num_blocks), arr, ctypes.byref(total),
                                     ctypes.byref(align), ctypes.byref(group)))
    fields = [f for f, _ in LohanBlockOffsets._fields_]
    return ([{f: getattr(arr[b], f) for f in fields} for b in range(num_blocks)], total.value,
            align.value, group.value)


def lohan_clip_loss_scale(sqnorm, loss_scale, max_norm) -> float:
    return float(load_library().lohan_clip_loss_scale(float(sqnorm), float(loss_scale),
                                                      float(max_norm)))


def lohan_tuning_set_launch_config(adam_variant=-1, adam_workgroups_per_cu=-1,
                                   adam_waves_per_cu=-1, reduce_workgroups_per_cu=0,
                                   reduce_policy=-1):
    """Bench-only (include/lohan_adam_tuning.h); affects the calling thread's later calls.
    Negative (for reduce_workgroups_per_cu: non-positive) arguments select the defaults."""
    _check(load_library().lohan_tuning_set_launch_config(
        int(adam_variant), int(adam_workgroups_per_cu), int(adam_waves_per_cu),
        int(reduce_workgroups_per_cu), int(reduce_policy)))


def lohan_tuning_set_wait_limit(polls=-1):
    """Bench/test-only: bound of the grid-wide wait of lohan_adam_small_block_step, in polls, for
    the calling thread's later calls; negative = the built-in bound."""
    _check(load_library().lohan_tuning_set_wait_limit(int(polls)))


def lohan_tuning_get_launch_config():
    vals = [ctypes.c_int() for _ in range(5)]
    load_library().lohan_tuning_get_launch_config(*[ctypes.byref(v) for v in vals])
    return tuple(v.value for v in vals)


def lohan_tuning_device_info():
    """(compute units, LDS bytes per compute unit) as the library read them."""
    cus, lds = ctypes.c_int(), ctypes.c_size_t()
    _check(load_library().lohan_tuning_device_info(ctypes.byref(cus), ctypes.byref(lds)))
    return cus.value, lds.value


LOHAN_PROBE_READ, LOHAN_PROBE_WRITE, LOHAN_PROBE_COPY = 0, 1, 2
LOHAN_PROBE_FIVE_STREAM, LOHAN_PROBE_MEMCPY = 3, 4


def lohan_tuning_probe(pattern, a, b, c, g16, h16, n, waves_per_cu=0, stream=None):
    _check(load_library().lohan_tuning_probe(
        int(pattern), _addr(a, n, _F32, "a"), _addr(b, n, _F32, "b"), _addr(c, n, _F32, "c"),
        _addr(g16, n, _F16, "g16"), _addr(h16, n, _BF16, "h16"), int(n), int(waves_per_cu),
        _stream(stream)))


def lohan_offload_slab_bytes(max_block_elems, num_slots) -> int:
    return int(load_library().lohan_offload_slab_bytes(int(max_block_elems), int(num_slots)))


def lohan_offload_create(device_slab, max_block_elems, num_slots, mode, device_slab_bytes=None):
    """Returns the opaque handle (an integer address) of a new pipeline."""
    slab, nbytes = _workspace(device_slab, device_slab_bytes)
    handle = ctypes.c_void_p()
    _check(load_library().lohan_offload_create(ctypes.byref(handle), slab, nbytes,
                                               int(max_block_elems), int(num_slots), int(mode)))
    return handle.value


def lohan_offload_submit(handle, host_param_fp32, host_exp_avg, host_exp_avg_sq, grad_fp16,
                         param_bf16_out, n, overflow_flag, sqnorm, lr, beta1, beta2, eps,
                         weight_decay, step, loss_scale, max_norm, flags, producer_stream=None):
    """Host arrays: pinned CPU torch tensors (or raw addresses); the rest device tensors."""
    blk = LohanOffloadBlock(
        _addr(host_param_fp32, n, _F32, "host_param_fp32"),
        _addr(host_exp_avg, n, _F32, "host_exp_avg"),
        _addr(host_exp_avg_sq, n, _F32, "host_exp_avg_sq"),
        _addr(grad_fp16, n, _F16, "grad_fp16"),
        _addr(param_bf16_out, n, _BF16, "param_bf16_out"), int(n),
        _addr(overflow_flag, 1, _U32, "overflow_flag"), _addr(sqnorm, 1, _F64, "sqnorm"))
    _check(load_library().lohan_offload_submit(
        handle, ctypes.byref(blk), float(lr), float(beta1), float(beta2), float(eps),
        float(weight_decay), int(step), float(loss_scale), float(max_norm), int(flags),
        _stream(producer_stream)))


def lohan_offload_wait_last_step(handle, stream=None):
    _check(load_library().lohan_offload_wait_last_step(handle, _stream(stream)))


def lohan_offload_drain(handle):
    _check(load_library().lohan_offload_drain(handle))


def lohan_offload_destroy(handle):
    _check(load_library().lohan_offload_destroy(handle))


def lohan_tuning_offload_inject_failure(handle, after_calls):
    _check(load_library().lohan_tuning_offload_inject_failure(handle, int(after_calls)))


def lohan_tuning_offload_slot_times(handle, slot):
    """(h2d_ms, step_ms, d2h_ms) of the block that last used staging slot `slot`."""
    a, b, c = ctypes.c_float(), ctypes.c_float(), ctypes.c_float()
    _check(load_library().lohan_tuning_offload_slot_times(handle, int(slot), ctypes.byref(a),
                                                          ctypes.byref(b), ctypes.byref(c)))
    return a.value, b.value, c.value


def _swap_hw(hw: dict) -> LohanSwapHw:
    return LohanSwapHw(*[float(hw[k]) for k, _ in LohanSwapHw._fields_])


def lohan_swap_iter_time(hw: dict, a_g2m, flop_r) -> float:
    h = _swap_hw(hw)
    return float(load_library().lohan_swap_iter_time(ctypes.byref(h), float(a_g2m), float(flop_r)))


def lohan_swap_recompute_flops(layers, flop_f, a_g2m):
    """layers: sequence of (flop, act_bytes).  Returns (FLOP_r, dFLOP_r/dA_G2M)."""
    n = len(layers)
    arr = (LohanLayer * max(1, n))(*[LohanLayer(float(f), float(a)) for f, a in layers])
    fr, dfr = ctypes.c_double(), ctypes.c_double()
    _check(load_library().lohan_swap_recompute_flops(arr if n else None, n, float(flop_f),
                                                     float(a_g2m), ctypes.byref(fr),
                                                     ctypes.byref(dfr)))
    return fr.value, dfr.value


def lohan_plan_activation_swapping(layers, hw: dict):
    """layers: sequence of (flop, act_bytes).  Returns (swap_list, a_g2m, flop_r, t_iter)."""
    n = len(layers)
    arr = (LohanLayer * max(n, 1))(*[LohanLayer(float(f), float(a)) for f, a in layers])
    out = (ctypes.c_uint32 * max(n, 1))()
    count = ctypes.c_size_t()
    a, f, t = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    h = _swap_hw(hw)
    _check(load_library().lohan_plan_activation_swapping(
        arr, n, ctypes.byref(h), out, ctypes.byref(count), ctypes.byref(a), ctypes.byref(f),
        ctypes.byref(t)))
    return [int(out[i]) for i in range(count.value)], a.value, f.value, t.value
