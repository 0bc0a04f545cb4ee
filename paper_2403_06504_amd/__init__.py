"""MI355X-native per-block fused mixed-precision Adam/AdamW step (LoHan's active gradient
offloading hot path, arxiv 2403.06504 Sec. IV-C).

The product is the C-ABI library declared in include/lohan_adam.h (HIP kernels for gfx950);
`binding` is a thin ctypes layer over it with the same entry-point names.  There is no CPU
fallback: calling an entry point without the built library raises.
"""
from .binding import (  # noqa: F401
    LOHAN_OFFLOAD_OVERLAPPED,
    LOHAN_OFFLOAD_SERIALIZED,
    lohan_offload_create,
    lohan_offload_destroy,
    lohan_offload_drain,
    lohan_offload_slab_bytes,
    lohan_offload_submit,
    lohan_offload_wait_last_step,
    lohan_plan_activation_swapping,
    lohan_swap_iter_time,
    lohan_swap_recompute_flops,
    LOHAN_FLAG_L2_MODE,
    LOHAN_FLAG_P16_FP16,
    LOHAN_FLAG_PRECHECKED,
    LohanError,
    library_path,
    load_library,
    lohan_adam_block_step,
    lohan_adam_block_step_clipped,
    lohan_adam_block_step_out_of_place,
    lohan_adam_multi_block_step,
    lohan_model_placement,
    lohan_ring_adam_block_step,
    lohan_ring_bytes,
    lohan_ring_init,
    lohan_ring_read,
    make_block_array,
    LohanBlock,
    lohan_clip_loss_scale,
    lohan_get_launch_config,
    lohan_grad_overflow_check,
    lohan_grad_sqnorm,
    lohan_set_launch_config,
    lohan_status_string,
    lohan_workspace_bytes,
)
