// C ABI of the per-block fused Adam step: argument validation, host-side scalar precompute,
// launch sizing.  See include/lohan_adam.h for the contract of every entry point.

#include <hip/hip_runtime.h>

#include <atomic>
#include <mutex>
#include <cmath>
#include <cstdint>
#include <limits>
#include <vector>

#include "lohan_adam.h"
#include "lohan_adam_tuning.h"
#include "lohan_kernels.h"

namespace {

// Per-device facts, read once from the device attributes.
constexpr int kMaxDevices = 64;
struct DeviceSlot {
    std::atomic<int> cus{0};
    std::atomic<size_t> lds_per_cu{0};
    std::atomic<int> small_wgs_per_cu[lohan::kSmallVariants];
};
DeviceSlot g_device[kMaxDevices];

// Launch shape.  Automatic variant (-1): 64-lane workgroups, 1 vector per lane; the cache policy
// follows the block's resident size (16 B/element): blocks that fit the memory-side cache keep
// the default policy (measured +5 % there), everything larger streams past the caches.  The
// reduction's loads follow the same rule, so that for a block that fits, the update's read of the
// gradients hits what the reduction left behind.  HIP has no attribute for the size of the
// memory-side cache (hipDeviceAttributeL2CacheSize is the per-XCD L2), so MI355X's 256 MiB is a
// constant here.
constexpr int kAutoAdamVariant = -1;
constexpr int kStreamingVariant = 0 | (0 << 2) | (2 << 4);
constexpr int kCacheResidentVariant = 0 | (0 << 2) | (0 << 4);
constexpr uint64_t kMemorySideCacheBytes = 256ull << 20;
constexpr int kDefaultAdamWgsPerCu = 0;                       // one tile per workgroup
constexpr int kDefaultAdamWavesPerCu = 11;                    // occupancy throttle
constexpr int kDefaultReduceWgsPerCu = 4;
constexpr int kAutoReducePolicy = -1;
// Polls of the grid-wide wait in the one-launch step before a workgroup gives up (a third of a
// second).
constexpr uint32_t kDefaultWaitLimit = 1u << 20;

// Tuning override (lohan_adam_tuning.h): per calling thread, so that a sweep on one thread never
// changes the launch shape under calls made by another.
struct LaunchOverride {
    int adam_variant = kAutoAdamVariant;
    int adam_wgs_per_cu = kDefaultAdamWgsPerCu;
    int adam_waves_per_cu = kDefaultAdamWavesPerCu;
    int reduce_wgs_per_cu = kDefaultReduceWgsPerCu;
    int reduce_policy = kAutoReducePolicy;
    uint32_t wait_limit = kDefaultWaitLimit;
};
thread_local LaunchOverride t_launch;

// Facts about the current device (the device `stream` must belong to).  cus == 0 on error.
lohan::DeviceInfo current_device()
{
    lohan::DeviceInfo info{};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return info;
    const bool cacheable = dev >= 0 && dev < kMaxDevices;
    if (cacheable) {
        info.cus = g_device[dev].cus.load(std::memory_order_acquire);
        info.lds_per_cu = g_device[dev].lds_per_cu.load(std::memory_order_relaxed);
        for (int i = 0; i < lohan::kSmallVariants; ++i)
            info.small_wgs_per_cu[i] =
                g_device[dev].small_wgs_per_cu[i].load(std::memory_order_relaxed);
        if (info.cus > 0 && info.lds_per_cu > 0) return info;
    }
    int cus = 0, lds = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        cus <= 0 ||
        hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) !=
            hipSuccess ||
        lds <= 0)
        return lohan::DeviceInfo{};
    info.cus = cus;
    info.lds_per_cu = (size_t)lds;
    // A device whose occupancy cannot be read simply has no one-launch step (capacity 0).
    if (lohan::small_block_occupancy(info.small_wgs_per_cu) != hipSuccess)
        for (int i = 0; i < lohan::kSmallVariants; ++i) info.small_wgs_per_cu[i] = 0;
    if (cacheable) {
        for (int i = 0; i < lohan::kSmallVariants; ++i)
            g_device[dev].small_wgs_per_cu[i].store(info.small_wgs_per_cu[i],
                                                    std::memory_order_relaxed);
        g_device[dev].lds_per_cu.store(info.lds_per_cu, std::memory_order_relaxed);
        g_device[dev].cus.store(info.cus, std::memory_order_release);
    }
    return info;
}

uint32_t reduce_workgroups(const lohan::DeviceInfo &dev)
{
    return (uint32_t)dev.cus * (uint32_t)t_launch.reduce_wgs_per_cu;
}

// Whether the reduction over a block of n elements streams past the caches.
bool reduce_streams(uint64_t n)
{
    if (t_launch.reduce_policy >= 0) return t_launch.reduce_policy != 0;
    return n * 16 > kMemorySideCacheBytes;
}

inline bool misaligned(const void *ptr, uintptr_t align)
{
    return (reinterpret_cast<uintptr_t>(ptr) & (align - 1)) != 0;
}

inline bool finite_nonneg(float x) { return std::isfinite(x) && x >= 0.0f; }
inline bool finite_pos(float x) { return std::isfinite(x) && x > 0.0f; }
inline bool unit_interval(float x) { return std::isfinite(x) && x >= 0.0f && x < 1.0f; }

lohan_status_t check_workspace(const void *workspace, size_t workspace_bytes)
{
    if (workspace == nullptr) return LOHAN_ERR_NULL;
    if (misaligned(workspace, 16)) return LOHAN_ERR_ALIGN;
    if (workspace_bytes < lohan::kWorkspaceBytes) return LOHAN_ERR_WORKSPACE;
    return LOHAN_OK;
}

}  // namespace

extern "C" {

size_t lohan_workspace_bytes(void) { return lohan::kWorkspaceBytes; }

const char *lohan_status_string(lohan_status_t status)
{
    switch (status) {
    case LOHAN_OK: return "ok";
    case LOHAN_ERR_NULL: return "a required pointer is NULL";
    case LOHAN_ERR_ALIGN: return "a pointer is not sufficiently aligned";
    case LOHAN_ERR_ARG: return "a scalar argument is out of its domain";
    case LOHAN_ERR_WORKSPACE: return "workspace is smaller than lohan_workspace_bytes()";
    case LOHAN_ERR_HIP: return "the HIP runtime reported an error at launch";
    case LOHAN_ERR_TOO_LARGE:
        return "n exceeds the maximum this entry point takes";
    default: return "unknown status";
    }
}

lohan_status_t lohan_grad_overflow_check(const void *grad_fp16, uint64_t n,
                                         uint32_t *overflow_flag, void *workspace,
                                         size_t workspace_bytes, hipStream_t stream)
{
    if (overflow_flag == nullptr || (grad_fp16 == nullptr && n != 0)) return LOHAN_ERR_NULL;
    if (misaligned(grad_fp16, 16) || misaligned(overflow_flag, 4)) return LOHAN_ERR_ALIGN;
    lohan_status_t ws = check_workspace(workspace, workspace_bytes);
    if (ws != LOHAN_OK) return ws;
    const lohan::DeviceInfo dev = current_device();
    if (dev.cus <= 0) return LOHAN_ERR_HIP;
    hipError_t e = lohan::launch_grad_reduce(grad_fp16, n, false, 0.0, nullptr, overflow_flag,
                                             workspace, reduce_workgroups(dev), reduce_streams(n),
                                             stream);
    return e == hipSuccess ? LOHAN_OK : LOHAN_ERR_HIP;
}

lohan_status_t lohan_grad_sqnorm(const void *grad_fp16, uint64_t n, float loss_scale,
                                 double *sqnorm, uint32_t *overflow_flag, void *workspace,
                                 size_t workspace_bytes, hipStream_t stream)
{
    if (sqnorm == nullptr || (grad_fp16 == nullptr && n != 0)) return LOHAN_ERR_NULL;
    if (misaligned(grad_fp16, 16) || misaligned(sqnorm, 8) || misaligned(overflow_flag, 4))
        return LOHAN_ERR_ALIGN;
    if (!finite_pos(loss_scale)) return LOHAN_ERR_ARG;
    lohan_status_t ws = check_workspace(workspace, workspace_bytes);
    if (ws != LOHAN_OK) return ws;
    const lohan::DeviceInfo dev = current_device();
    if (dev.cus <= 0) return LOHAN_ERR_HIP;
    const double inv = 1.0 / (double)loss_scale;
    hipError_t e = lohan::launch_grad_reduce(grad_fp16, n, true, inv * inv, sqnorm, overflow_flag,
                                             workspace, reduce_workgroups(dev), reduce_streams(n),
                                             stream);
    return e == hipSuccess ? LOHAN_OK : LOHAN_ERR_HIP;
}

lohan_status_t lohan_grad_produce_fp16(const float *grad_fp32, uint64_t n, float multiplier,
                                       void *grad_fp16_out, float loss_scale, double *sqnorm,
                                       uint32_t *overflow_flag, void *workspace,
                                       size_t workspace_bytes, hipStream_t stream)
{
    if (overflow_flag == nullptr || (n != 0 && (grad_fp32 == nullptr || grad_fp16_out == nullptr)))
        return LOHAN_ERR_NULL;
    if (misaligned(grad_fp32, 16) || misaligned(grad_fp16_out, 16) || misaligned(sqnorm, 8) ||
        misaligned(overflow_flag, 4))
        return LOHAN_ERR_ALIGN;
    if (!std::isfinite(multiplier) || !finite_pos(loss_scale)) return LOHAN_ERR_ARG;
    lohan_status_t ws = check_workspace(workspace, workspace_bytes);
    if (ws != LOHAN_OK) return ws;
    const lohan::DeviceInfo dev = current_device();
    if (dev.cus <= 0) return LOHAN_ERR_HIP;
    const double inv = 1.0 / (double)loss_scale;
    hipError_t e = lohan::launch_grad_produce(grad_fp32, n, multiplier, grad_fp16_out, inv * inv,
                                              sqnorm, overflow_flag, workspace,
                                              reduce_workgroups(dev), reduce_streams(n), stream);
    return e == hipSuccess ? LOHAN_OK : LOHAN_ERR_HIP;
}

namespace {

lohan_status_t validate_step_args(const float *param_fp32, const float *exp_avg,
                                  const float *exp_avg_sq, const void *grad_fp16,
                                  const void *param_bf16_out, uint64_t n, float lr, float beta1,
                                  float beta2, float eps, float weight_decay, int64_t step,
                                  float loss_scale, const uint32_t *overflow_flag, uint32_t flags)
{
    if (overflow_flag == nullptr) return LOHAN_ERR_NULL;
    if (n != 0 && (param_fp32 == nullptr || exp_avg == nullptr || exp_avg_sq == nullptr ||
                   grad_fp16 == nullptr || param_bf16_out == nullptr))
        return LOHAN_ERR_NULL;
    if (misaligned(param_fp32, 16) || misaligned(exp_avg, 16) || misaligned(exp_avg_sq, 16) ||
        misaligned(grad_fp16, 16) || misaligned(param_bf16_out, 16) ||
        misaligned(overflow_flag, 4))
        return LOHAN_ERR_ALIGN;
    if ((flags & ~(uint32_t)(LOHAN_FLAG_L2_MODE | LOHAN_FLAG_PRECHECKED | LOHAN_FLAG_P16_FP16)) != 0)
        return LOHAN_ERR_ARG;
    if (step < 1 || !finite_pos(loss_scale) || !finite_nonneg(lr) || !finite_nonneg(eps) ||
        !finite_nonneg(weight_decay) || !unit_interval(beta1) || !unit_interval(beta2))
        return LOHAN_ERR_ARG;
    return LOHAN_OK;
}

// Element-independent scalars, each an individually rounded fp32 operation; the bias corrections
// go through float64 and are rounded once.
lohan::StepScalars make_step_scalars(float lr, float beta1, float beta2, float eps,
                                     float weight_decay, int64_t step, float loss_scale)
{
    lohan::StepScalars s;
    s.inv = 1.0f / loss_scale;
    s.beta1 = beta1;
    s.beta2 = beta2;
    s.omb1 = 1.0f - beta1;
    s.omb2 = 1.0f - beta2;
    const float bc1 = (float)(1.0 - std::pow((double)beta1, (double)step));
    const float bc2 = (float)(1.0 - std::pow((double)beta2, (double)step));
    s.sbc2 = std::sqrt(bc2);
    s.ss = lr / bc1;
    const float lr_wd = lr * weight_decay;
    s.decay = 1.0f - lr_wd;
    s.eps = eps;
    s.wd = weight_decay;
    return s;
}

// Kernel mode bits from the ABI flags.
int kernel_mode(uint32_t flags)
{
    return ((flags & LOHAN_FLAG_L2_MODE) ? 1 : 0) | ((flags & LOHAN_FLAG_P16_FP16) ? 2 : 0);
}

lohan::AdamLaunch adam_launch_for(uint64_t n)
{
    int variant = t_launch.adam_variant;
    if (variant < 0)
        variant = n * 16 <= kMemorySideCacheBytes ? kCacheResidentVariant : kStreamingVariant;
    return lohan::AdamLaunch{variant, t_launch.adam_wgs_per_cu, t_launch.adam_waves_per_cu};
}

}  // namespace

lohan_status_t lohan_adam_block_step(float *param_fp32, float *exp_avg, float *exp_avg_sq,
                                     const void *grad_fp16, void *param_bf16_out, uint64_t n,
                                     float lr, float beta1, float beta2, float eps,
                                     float weight_decay, int64_t step, float loss_scale,
                                     uint32_t *overflow_flag, uint32_t flags, void *workspace,
                                     size_t workspace_bytes, hipStream_t stream)
{
    lohan_status_t st = validate_step_args(param_fp32, exp_avg, exp_avg_sq, grad_fp16,
                                           param_bf16_out, n, lr, beta1, beta2, eps, weight_decay,
                                           step, loss_scale, overflow_flag, flags);
    if (st != LOHAN_OK) return st;
    const bool prechecked = (flags & LOHAN_FLAG_PRECHECKED) != 0;
    if (!prechecked) {
        st = check_workspace(workspace, workspace_bytes);
        if (st != LOHAN_OK) return st;
    }
    const lohan::DeviceInfo dev = current_device();
    if (dev.cus <= 0) return LOHAN_ERR_HIP;
    const lohan::StepScalars s =
        make_step_scalars(lr, beta1, beta2, eps, weight_decay, step, loss_scale);
    if (!prechecked) {
        hipError_t e = lohan::launch_grad_reduce(grad_fp16, n, false, 0.0, nullptr, overflow_flag,
                                                 workspace, reduce_workgroups(dev),
                                                 reduce_streams(n), stream);
        if (e != hipSuccess) return LOHAN_ERR_HIP;
    }
    hipError_t e = lohan::launch_adam_block_step(
        param_fp32, exp_avg, exp_avg_sq, grad_fp16, param_bf16_out, n, s,
        kernel_mode(flags), overflow_flag, nullptr, adam_launch_for(n), dev, stream);
    return e == hipSuccess ? LOHAN_OK : LOHAN_ERR_HIP;
}

lohan_status_t lohan_adam_block_step_clipped(float *param_fp32, float *exp_avg, float *exp_avg_sq,
                                             const void *grad_fp16, void *param_bf16_out,
                                             uint64_t n, float lr, float beta1, float beta2,
                                             float eps, float weight_decay, int64_t step,
                                             float loss_scale, const double *sqnorm,
                                             float max_norm, const uint32_t *overflow_flag,
                                             uint32_t flags, void *workspace,
                                             size_t workspace_bytes, hipStream_t stream)
{
    lohan_status_t st = validate_step_args(param_fp32, exp_avg, exp_avg_sq, grad_fp16,
                                           param_bf16_out, n, lr, beta1, beta2, eps, weight_decay,
                                           step, loss_scale, overflow_flag, flags);
    if (st != LOHAN_OK) return st;
    if (sqnorm == nullptr) return LOHAN_ERR_NULL;
    if (misaligned(sqnorm, 8)) return LOHAN_ERR_ALIGN;
    if (!finite_pos(max_norm)) return LOHAN_ERR_ARG;
    st = check_workspace(workspace, workspace_bytes);
    if (st != LOHAN_OK) return st;
    const lohan::DeviceInfo dev = current_device();
    if (dev.cus <= 0) return LOHAN_ERR_HIP;
    if (n == 0) return LOHAN_OK;
    const lohan::StepScalars s =
        make_step_scalars(lr, beta1, beta2, eps, weight_decay, step, loss_scale);
    float *inv_dev = reinterpret_cast<float *>(reinterpret_cast<char *>(workspace) +
                                               lohan::kScalarsOffset);
    hipError_t e = lohan::launch_clip_scale(sqnorm, loss_scale, max_norm, inv_dev, 1, stream);
    if (e != hipSuccess) return LOHAN_ERR_HIP;
    e = lohan::launch_adam_block_step(param_fp32, exp_avg, exp_avg_sq, grad_fp16, param_bf16_out,
                                      n, s, kernel_mode(flags), overflow_flag, inv_dev,
                                      adam_launch_for(n), dev, stream);
    return e == hipSuccess ? LOHAN_OK : LOHAN_ERR_HIP;
}

lohan_status_t lohan_adam_small_block_max_n(uint64_t *max_n)
{
    if (max_n == nullptr) return LOHAN_ERR_NULL;
    const lohan::DeviceInfo dev = current_device();
    if (dev.cus <= 0) return LOHAN_ERR_HIP;
    *max_n = lohan::small_block_max_n(dev);
    return LOHAN_OK;
}

lohan_status_t lohan_adam_small_block_step(float *param_fp32, float *exp_avg, float *exp_avg_sq,
                                           const void *grad_fp16, void *param_bf16_out,
                                           uint64_t n, float lr, float beta1, float beta2,
                                           float eps, float weight_decay, int64_t step,
                                           float loss_scale, double *sqnorm,
                                           uint32_t *overflow_flag, uint32_t flags,
                                           void *workspace, size_t workspace_bytes,
                                           hipStream_t stream)
{
    lohan_status_t st = validate_step_args(param_fp32, exp_avg, exp_avg_sq, grad_fp16,
                                           param_bf16_out, n, lr, beta1, beta2, eps, weight_decay,
                                           step, loss_scale, overflow_flag, flags);
    if (st != LOHAN_OK) return st;
    if ((flags & LOHAN_FLAG_PRECHECKED) != 0) return LOHAN_ERR_ARG;
    if (misaligned(sqnorm, 8)) return LOHAN_ERR_ALIGN;
    st = check_workspace(workspace, workspace_bytes);
    if (st != LOHAN_OK) return st;
    const lohan::DeviceInfo dev = current_device();
    if (dev.cus <= 0) return LOHAN_ERR_HIP;
    if (n > lohan::small_block_max_n(dev)) return LOHAN_ERR_TOO_LARGE;
    const lohan::StepScalars s =
        make_step_scalars(lr, beta1, beta2, eps, weight_decay, step, loss_scale);
    const double inv = 1.0 / (double)loss_scale;
    hipError_t e = lohan::launch_adam_small_block_step(
        param_fp32, exp_avg, exp_avg_sq, grad_fp16, param_bf16_out, n, s, kernel_mode(flags),
        inv * inv, sqnorm, overflow_flag, workspace, t_launch.wait_limit, dev, stream);
    return e == hipSuccess ? LOHAN_OK : LOHAN_ERR_HIP;
}

namespace {

// Shared by the two out-of-place entry points; sqnorm == NULL means no clipping.
lohan_status_t step_out_of_place(const float *param_fp32_in, const float *exp_avg_in,
                                 const float *exp_avg_sq_in, const void *grad_fp16,
                                 float *param_fp32_out, float *exp_avg_out, float *exp_avg_sq_out,
                                 void *param_bf16_out, uint64_t n, float lr, float beta1,
                                 float beta2, float eps, float weight_decay, int64_t step,
                                 float loss_scale, const double *sqnorm, float max_norm,
                                 uint32_t *overflow_flag, uint32_t flags, void *workspace,
                                 size_t workspace_bytes, hipStream_t stream)
{
    if ((flags & LOHAN_FLAG_PRECHECKED) != 0) return LOHAN_ERR_ARG;
    lohan_status_t st = validate_step_args(param_fp32_in, exp_avg_in, exp_avg_sq_in, grad_fp16,
                                           param_bf16_out, n, lr, beta1, beta2, eps, weight_decay,
                                           step, loss_scale, overflow_flag, flags);
    if (st != LOHAN_OK) return st;
    if (n != 0 &&
        (param_fp32_out == nullptr || exp_avg_out == nullptr || exp_avg_sq_out == nullptr))
        return LOHAN_ERR_NULL;
    if (misaligned(param_fp32_out, 16) || misaligned(exp_avg_out, 16) ||
        misaligned(exp_avg_sq_out, 16))
        return LOHAN_ERR_ALIGN;
    if (n != 0 && (param_fp32_out == param_fp32_in || exp_avg_out == exp_avg_in ||
                   exp_avg_sq_out == exp_avg_sq_in))
        return LOHAN_ERR_ARG;
    float *inv_dev = nullptr;
    if (sqnorm != nullptr) {
        if (misaligned(sqnorm, 8)) return LOHAN_ERR_ALIGN;
        if (!finite_pos(max_norm)) return LOHAN_ERR_ARG;
        st = check_workspace(workspace, workspace_bytes);
        if (st != LOHAN_OK) return st;
        inv_dev = reinterpret_cast<float *>(reinterpret_cast<char *>(workspace) +
                                            lohan::kScalarsOffset);
    }
    const lohan::DeviceInfo dev = current_device();
    if (dev.cus <= 0) return LOHAN_ERR_HIP;
    const lohan::StepScalars s =
        make_step_scalars(lr, beta1, beta2, eps, weight_decay, step, loss_scale);
    if (inv_dev != nullptr && n != 0 &&
        lohan::launch_clip_scale(sqnorm, loss_scale, max_norm, inv_dev, 1, stream) != hipSuccess)
        return LOHAN_ERR_HIP;
    hipError_t e = lohan::launch_adam_block_step_oop(
        param_fp32_in, exp_avg_in, exp_avg_sq_in, grad_fp16, param_fp32_out, exp_avg_out,
        exp_avg_sq_out, param_bf16_out, n, s, kernel_mode(flags), overflow_flag, inv_dev,
        adam_launch_for(n), dev, stream);
    return e == hipSuccess ? LOHAN_OK : LOHAN_ERR_HIP;
}

}  // namespace

lohan_status_t lohan_adam_block_step_out_of_place(
    const float *param_fp32_in, const float *exp_avg_in, const float *exp_avg_sq_in,
    const void *grad_fp16, float *param_fp32_out, float *exp_avg_out, float *exp_avg_sq_out,
    void *param_bf16_out, uint64_t n, float lr, float beta1, float beta2, float eps,
    float weight_decay, int64_t step, float loss_scale, uint32_t *overflow_flag, uint32_t flags,
    hipStream_t stream)
{
    return step_out_of_place(param_fp32_in, exp_avg_in, exp_avg_sq_in, grad_fp16, param_fp32_out,
                             exp_avg_out, exp_avg_sq_out, param_bf16_out, n, lr, beta1, beta2, eps,
                             weight_decay, step, loss_scale, nullptr, 0.0f, overflow_flag, flags,
                             nullptr, 0, stream);
}

lohan_status_t lohan_adam_block_step_out_of_place_clipped(
    const float *param_fp32_in, const float *exp_avg_in, const float *exp_avg_sq_in,
    const void *grad_fp16, float *param_fp32_out, float *exp_avg_out, float *exp_avg_sq_out,
    void *param_bf16_out, uint64_t n, float lr, float beta1, float beta2, float eps,
    float weight_decay, int64_t step, float loss_scale, const double *sqnorm, float max_norm,
    uint32_t *overflow_flag, uint32_t flags, void *workspace, size_t workspace_bytes,
    hipStream_t stream)
{
    if (sqnorm == nullptr) return LOHAN_ERR_NULL;
    return step_out_of_place(param_fp32_in, exp_avg_in, exp_avg_sq_in, grad_fp16, param_fp32_out,
                             exp_avg_out, exp_avg_sq_out, param_bf16_out, n, lr, beta1, beta2, eps,
                             weight_decay, step, loss_scale, sqnorm, max_norm, overflow_flag,
                             flags, workspace, workspace_bytes, stream);
}

lohan_status_t lohan_adam_multi_block_step(const lohan_block_t *blocks, uint32_t num_blocks,
                                           float lr, float beta1, float beta2, float eps,
                                           float weight_decay, int64_t step, float loss_scale,
                                           float max_norm, uint32_t *overflow_flags,
                                           double *sqnorms, uint32_t flags, void *workspace,
                                           size_t workspace_bytes, hipStream_t stream)
{
    if (num_blocks == 0) return LOHAN_OK;
    if (blocks == nullptr) return LOHAN_ERR_NULL;
    for (uint32_t b = 0; b < num_blocks; ++b) {
        const lohan_block_t &blk = blocks[b];
        lohan_status_t st = validate_step_args(blk.param_fp32, blk.exp_avg, blk.exp_avg_sq,
                                               blk.grad_fp16, blk.param_bf16_out, blk.n, lr, beta1,
                                               beta2, eps, weight_decay, step, loss_scale,
                                               overflow_flags, flags);
        if (st != LOHAN_OK) return st;
    }
    if (misaligned(sqnorms, 8)) return LOHAN_ERR_ALIGN;
    const bool clip = max_norm != 0.0f;
    if (clip && !finite_pos(max_norm)) return LOHAN_ERR_ARG;
    lohan_status_t st = check_workspace(workspace, workspace_bytes);
    if (st != LOHAN_OK) return st;
    const lohan::DeviceInfo dev = current_device();
    if (dev.cus <= 0) return LOHAN_ERR_HIP;

    const bool prechecked = (flags & LOHAN_FLAG_PRECHECKED) != 0;
    const bool want_norm = clip || sqnorms != nullptr;
    const lohan::StepScalars s =
        make_step_scalars(lr, beta1, beta2, eps, weight_decay, step, loss_scale);
    const uint32_t red_wgs = reduce_workgroups(dev);
    const double inv = 1.0 / (double)loss_scale;
    char *ws = reinterpret_cast<char *>(workspace);
    float *inv_dev = reinterpret_cast<float *>(ws + lohan::kScalarsOffset);
    double *norms_ws = reinterpret_cast<double *>(ws + lohan::kNormsOffset);

    // One launch covers a run of consecutive blocks: at most kMultiMaxBlocks of them, and of
    // similar enough length that the grid, sized for the longest, holds few empty workgroups.
    uint32_t first = 0;
    while (first < num_blocks) {
        lohan::MultiArgs args;
        uint32_t count = 0;
        uint64_t longest = 0, total = 0;
        while (first + count < num_blocks && count < lohan::kMultiMaxBlocks) {
            const uint64_t n = blocks[first + count].n;
            const uint64_t new_longest = n > longest ? n : longest;
            const double covered = (double)new_longest * (double)(count + 1);
            const double used = (double)(total + n);
            if (count > 0 && covered - used > 0.5 * used + 1048576.0) break;
            const lohan_block_t &blk = blocks[first + count];
            lohan::MultiDesc &d = args.d[count];
            d.p = blk.param_fp32;
            d.m = blk.exp_avg;
            d.v = blk.exp_avg_sq;
            d.g = reinterpret_cast<const uint16_t *>(blk.grad_fp16);
            d.p16 = reinterpret_cast<uint16_t *>(blk.param_bf16_out);
            d.n = n;
            longest = new_longest;
            total += n;
            ++count;
        }
        for (uint32_t b = count; b < lohan::kMultiMaxBlocks; ++b) args.d[b] = lohan::MultiDesc{};

        uint32_t *flags_dev = overflow_flags + first;
        double *norms_dev = sqnorms != nullptr ? sqnorms + first : norms_ws;
        if (!prechecked || want_norm) {
            hipError_t e = lohan::launch_multi_grad_reduce(
                args, count, want_norm, inv * inv, want_norm ? norms_dev : nullptr,
                prechecked ? nullptr : flags_dev, workspace, red_wgs, reduce_streams(total),
                stream);
            if (e != hipSuccess) return LOHAN_ERR_HIP;
        }
        if (clip) {
            hipError_t e = lohan::launch_clip_scale(norms_dev, loss_scale, max_norm, inv_dev,
                                                    count, stream);
            if (e != hipSuccess) return LOHAN_ERR_HIP;
        }
        hipError_t e = lohan::launch_adam_multi_block_step(
            args, count, s, kernel_mode(flags), flags_dev, clip ? inv_dev : nullptr,
            adam_launch_for(total), dev, stream);
        if (e != hipSuccess) return LOHAN_ERR_HIP;
        first += count;
    }
    return LOHAN_OK;
}

namespace {

constexpr uint32_t kRingMaxBlocks = 1u << 20;

bool ring_counts_ok(uint32_t num_blocks, uint32_t num_spares)
{
    return num_blocks != 0 && num_blocks <= kRingMaxBlocks && num_spares != 0 &&
           num_spares <= num_blocks;
}

lohan_status_t ring_step(void *ring, uint32_t num_blocks, uint32_t num_spares, uint32_t block,
                         const void *grad_fp16, uint64_t n, float lr, float beta1, float beta2,
                         float eps, float weight_decay, int64_t step, float loss_scale,
                         const double *sqnorm, float max_norm, uint32_t flags, hipStream_t stream)
{
    if (ring == nullptr || (grad_fp16 == nullptr && n != 0)) return LOHAN_ERR_NULL;
    if (misaligned(ring, 16) || misaligned(grad_fp16, 16) || misaligned(sqnorm, 8))
        return LOHAN_ERR_ALIGN;
    if (!ring_counts_ok(num_blocks, num_spares) || block >= num_blocks) return LOHAN_ERR_ARG;
    if ((flags & ~(uint32_t)(LOHAN_FLAG_L2_MODE | LOHAN_FLAG_P16_FP16)) != 0) return LOHAN_ERR_ARG;
    if (step < 1 || !finite_pos(loss_scale) || !finite_nonneg(lr) || !finite_nonneg(eps) ||
        !finite_nonneg(weight_decay) || !unit_interval(beta1) || !unit_interval(beta2))
        return LOHAN_ERR_ARG;
    if (sqnorm != nullptr && !finite_pos(max_norm)) return LOHAN_ERR_ARG;
    const lohan::DeviceInfo dev = current_device();
    if (dev.cus <= 0) return LOHAN_ERR_HIP;
    const lohan::StepScalars s =
        make_step_scalars(lr, beta1, beta2, eps, weight_decay, step, loss_scale);
    const lohan::RingView view = lohan::ring_view(ring, num_blocks, num_spares);
    float *inv_dev = nullptr;
    if (sqnorm != nullptr && n != 0) {
        inv_dev = view.clip_inv + block;
        if (lohan::launch_clip_scale(sqnorm, loss_scale, max_norm, inv_dev, 1, stream) !=
            hipSuccess)
            return LOHAN_ERR_HIP;
    }
    hipError_t e = lohan::launch_adam_ring_step(view, block, grad_fp16, n, s, kernel_mode(flags),
                                                inv_dev, adam_launch_for(n), dev, stream);
    return e == hipSuccess ? LOHAN_OK : LOHAN_ERR_HIP;
}

}  // namespace

size_t lohan_ring_bytes(uint32_t num_blocks, uint32_t num_spares)
{
    return lohan::ring_bytes(num_blocks, num_spares);
}

lohan_status_t lohan_ring_init(void *ring, size_t ring_bytes, const lohan_ring_slot_t *slots,
                               uint32_t num_blocks, uint32_t num_spares)
{
    if (ring == nullptr || slots == nullptr) return LOHAN_ERR_NULL;
    if (misaligned(ring, 16)) return LOHAN_ERR_ALIGN;
    if (!ring_counts_ok(num_blocks, num_spares)) return LOHAN_ERR_ARG;
    if (ring_bytes < lohan::ring_bytes(num_blocks, num_spares)) return LOHAN_ERR_WORKSPACE;
    const uint32_t total = num_blocks + num_spares;
    for (uint32_t i = 0; i < total; ++i) {
        const lohan_ring_slot_t &slot = slots[i];
        if (slot.n == 0) continue;                      // an empty slot needs no memory
        if (slot.param_fp32 == nullptr || slot.exp_avg == nullptr || slot.exp_avg_sq == nullptr ||
            slot.param_16 == nullptr)
            return LOHAN_ERR_NULL;
        if (misaligned(slot.param_fp32, 16) || misaligned(slot.exp_avg, 16) ||
            misaligned(slot.exp_avg_sq, 16) || misaligned(slot.param_16, 16))
            return LOHAN_ERR_ALIGN;
    }
    // Host image of the table: block b starts in slot b; spare j (slot num_blocks + j) founds
    // class j, and a block belongs to the class whose spare has exactly its length.
    const size_t bytes = lohan::ring_bytes(num_blocks, num_spares);
    std::vector<char> image(bytes, 0);
    lohan::RingView view = lohan::ring_view(image.data(), num_blocks, num_spares);
    for (uint32_t i = 0; i < total; ++i)
        view.slots[i] = lohan::RingSlot{slots[i].param_fp32, slots[i].exp_avg,
                                        slots[i].exp_avg_sq,
                                        reinterpret_cast<uint16_t *>(slots[i].param_16),
                                        slots[i].n};
    for (uint32_t j = 0; j < num_spares; ++j) {
        for (uint32_t k = 0; k < j; ++k)
            if (slots[num_blocks + k].n == slots[num_blocks + j].n) return LOHAN_ERR_ARG;
        view.spare_of_class[j] = num_blocks + j;
    }
    for (uint32_t b = 0; b < num_blocks; ++b) {
        uint32_t cls = num_spares;
        for (uint32_t j = 0; j < num_spares; ++j)
            if (slots[num_blocks + j].n == slots[b].n) cls = j;
        if (cls == num_spares) return LOHAN_ERR_ARG;    // no spare of this block's length
        view.slot_of[b] = b;
        view.class_of[b] = cls;
    }
    return hipMemcpy(ring, image.data(), bytes, hipMemcpyHostToDevice) == hipSuccess
               ? LOHAN_OK
               : LOHAN_ERR_HIP;
}

lohan_status_t lohan_ring_read(const void *ring, uint32_t num_blocks, uint32_t num_spares,
                               uint32_t *slot_of, uint32_t *spares, uint32_t *skipped,
                               hipStream_t stream)
{
    if (ring == nullptr) return LOHAN_ERR_NULL;
    if (misaligned(ring, 16)) return LOHAN_ERR_ALIGN;
    if (!ring_counts_ok(num_blocks, num_spares)) return LOHAN_ERR_ARG;
    if (hipStreamSynchronize(stream) != hipSuccess) return LOHAN_ERR_HIP;
    const lohan::RingView view =
        lohan::ring_view(const_cast<void *>(ring), num_blocks, num_spares);
    if (slot_of != nullptr &&
        hipMemcpy(slot_of, view.slot_of, sizeof(uint32_t) * num_blocks, hipMemcpyDeviceToHost) !=
            hipSuccess)
        return LOHAN_ERR_HIP;
    if (spares != nullptr &&
        hipMemcpy(spares, view.spare_of_class, sizeof(uint32_t) * num_spares,
                  hipMemcpyDeviceToHost) != hipSuccess)
        return LOHAN_ERR_HIP;
    if (skipped != nullptr) {
        // The two counter arrays are adjacent in the ring: one copy brings both.
        std::vector<uint64_t> counters(2 * lohan::ring_pad16(sizeof(uint64_t) * num_blocks) / 8);
        if (hipMemcpy(counters.data(), view.attempts, counters.size() * sizeof(uint64_t),
                      hipMemcpyDeviceToHost) != hipSuccess)
            return LOHAN_ERR_HIP;
        const uint64_t *attempts = counters.data();
        const uint64_t *overflow_attempt = counters.data() + counters.size() / 2;
        for (uint32_t b = 0; b < num_blocks; ++b)
            skipped[b] = attempts[b] != 0 && overflow_attempt[b] == attempts[b] ? 1u : 0u;
    }
    return LOHAN_OK;
}

lohan_status_t lohan_ring_adam_block_step(void *ring, uint32_t num_blocks, uint32_t num_spares,
                                          uint32_t block, const void *grad_fp16, uint64_t n,
                                          float lr, float beta1, float beta2, float eps,
                                          float weight_decay, int64_t step, float loss_scale,
                                          uint32_t flags, hipStream_t stream)
{
    return ring_step(ring, num_blocks, num_spares, block, grad_fp16, n, lr, beta1, beta2, eps,
                     weight_decay, step, loss_scale, nullptr, 0.0f, flags, stream);
}

lohan_status_t lohan_ring_adam_block_step_clipped(void *ring, uint32_t num_blocks,
                                                  uint32_t num_spares, uint32_t block,
                                                  const void *grad_fp16, uint64_t n, float lr,
                                                  float beta1, float beta2, float eps,
                                                  float weight_decay, int64_t step,
                                                  float loss_scale, const double *sqnorm,
                                                  float max_norm, uint32_t flags,
                                                  hipStream_t stream)
{
    if (sqnorm == nullptr) return LOHAN_ERR_NULL;
    return ring_step(ring, num_blocks, num_spares, block, grad_fp16, n, lr, beta1, beta2, eps,
                     weight_decay, step, loss_scale, sqnorm, max_norm, flags, stream);
}

}  // extern "C"

namespace {

// Where lanes 1 and 2 start relative to lane 0, for the two lane periods.  Measured on every
// block shape of the evaluation models, all layouts in turn in one process: with the 4 GiB
// period, m at the period + 8 MiB and v at twice the period + 9 MiB beat + 1 / + 2 MiB by
// 0.4-0.7 % (0.863-0.865 of peak against 0.856-0.860); what counts is that m and v are an odd
// number of MiB apart and that no two of the three sit at the same offset modulo 16 MiB.  With
// the 12 GiB period + 1 / + 2 MiB stayed the best of the candidates.
struct LaneStarts {
    size_t lane1, lane2;
};
LaneStarts lane_starts(size_t period)
{
    constexpr size_t kMiB = 1ull << 20;
    if (period == (4ull << 30)) return LaneStarts{period + 8 * kMiB, 2 * period + 9 * kMiB};
    return LaneStarts{period + kMiB, 2 * period + 2 * kMiB};
}

}  // namespace

extern "C" {

lohan_status_t lohan_model_placement(uint64_t n, uint32_t num_blocks,
                                     lohan_block_offsets_t *offsets, size_t *slab_bytes,
                                     size_t *slab_alignment, uint32_t *blocks_per_group)
{
    constexpr size_t kGranule = 2ull << 20;       // array sizes are rounded up to this
    constexpr size_t kSkew = 1ull << 20;          // packed long arrays: this much between them
    constexpr size_t kSmallest = 256ull << 20;    // below this the placement gains under 1 %
    // Lane periods that measured well; a block uses the first one its fp32 arrays fit into.
    constexpr size_t kPeriods[2] = {4ull << 30, 12ull << 30};
    if (slab_bytes == nullptr || slab_alignment == nullptr ||
        (offsets == nullptr && num_blocks != 0))
        return LOHAN_ERR_NULL;
    if (n > (1ull << 40)) return LOHAN_ERR_ARG;
    auto round_up = [](size_t x, size_t a) { return (x + a - 1) / a * a; };
    const size_t wide = round_up((size_t)n * 4, kGranule);      // one fp32 array
    const size_t narrow = round_up((size_t)n * 2, kGranule);    // one 16-bit array
    *slab_alignment = kGranule;

    size_t period = 0;
    if (wide >= kSmallest)
        for (size_t candidate : kPeriods)
            if (period == 0 && wide <= candidate - kGranule) period = candidate;

    if (period == 0) {
        // Block-major packing.  Arrays too long for any lane still get the odd number of MiB
        // between p, m and v (an array of exactly 12 GiB would otherwise put all three at the
        // same offset modulo 4 GiB, the worst case measured); short ones are packed plainly.
        const size_t skew = wide >= kSmallest ? kSkew : 0;
        const size_t block_bytes = 3 * (wide + skew) + 2 * narrow + skew;
        for (uint32_t b = 0; b < num_blocks; ++b) {
            const size_t base = (size_t)b * block_bytes;
            const size_t after = base + 3 * (wide + skew);
            offsets[b] = lohan_block_offsets_t{base, base + wide + skew, base + 2 * (wide + skew),
                                               after, after + narrow};
        }
        *slab_bytes = (size_t)num_blocks * block_bytes;
        if (blocks_per_group != nullptr) *blocks_per_group = 1;
        return LOHAN_OK;
    }

    const size_t per_group = (period - kGranule) / wide;
    if (blocks_per_group != nullptr) *blocks_per_group = (uint32_t)per_group;
    size_t group_base = 0;
    for (uint32_t first = 0; first < num_blocks; first += (uint32_t)per_group) {
        const size_t count = num_blocks - first < per_group ? num_blocks - first : per_group;
        const size_t lane_used = count * wide;
        const LaneStarts starts = lane_starts(period);
        const size_t lane[3] = {0, starts.lane1, starts.lane2};
        // Free room behind the fp32 arrays of lanes 0 and 1 (up to the next lane's start) takes
        // 16-bit arrays; whatever does not fit follows lane 2.
        size_t room_at[3] = {lane[0] + lane_used, lane[1] + lane_used, lane[2] + lane_used};
        const size_t room_end[2] = {lane[1], lane[2]};
        size_t which = 0;
        auto take_narrow = [&]() {
            while (which < 2 && room_at[which] + narrow > room_end[which]) ++which;
            const size_t at = room_at[which];
            room_at[which] += narrow;
            return at;
        };
        for (size_t j = 0; j < count; ++j) {
            lohan_block_offsets_t &o = offsets[first + j];
            o.param_fp32 = group_base + lane[0] + j * wide;
            o.exp_avg = group_base + lane[1] + j * wide;
            o.exp_avg_sq = group_base + lane[2] + j * wide;
            o.grad_fp16 = group_base + take_narrow();
            o.param_bf16 = group_base + take_narrow();
        }
        group_base += round_up(room_at[2], kGranule);   // lane 2 and what follows it end the group
    }
    *slab_bytes = group_base;
    return LOHAN_OK;
}

lohan_status_t lohan_model_placement_compact(uint64_t n, uint32_t num_blocks,
                                             lohan_block_offsets_t *offsets, size_t *slab_bytes,
                                             size_t *slab_alignment)
{
    constexpr size_t kGranule = 2ull << 20;
    constexpr size_t kSkew = 1ull << 20;
    if (slab_bytes == nullptr || slab_alignment == nullptr ||
        (offsets == nullptr && num_blocks != 0))
        return LOHAN_ERR_NULL;
    if (n > (1ull << 40)) return LOHAN_ERR_ARG;
    auto round_up = [](size_t x, size_t a) { return (x + a - 1) / a * a; };
    const size_t wide = round_up((size_t)n * 4, kGranule);
    const size_t narrow = round_up((size_t)n * 2, kGranule);
    // p, m, v an odd number of MiB apart; the block as a whole a multiple of 2 MiB long.
    const size_t block_bytes = 3 * (wide + kSkew) + 2 * narrow + kSkew;
    for (uint32_t b = 0; b < num_blocks; ++b) {
        const size_t base = (size_t)b * block_bytes;
        lohan_block_offsets_t &o = offsets[b];
        o.param_fp32 = base;
        o.exp_avg = base + wide + kSkew;
        o.exp_avg_sq = base + 2 * (wide + kSkew);
        o.grad_fp16 = base + 3 * (wide + kSkew);
        o.param_bf16 = o.grad_fp16 + narrow;
    }
    *slab_bytes = (size_t)num_blocks * block_bytes;
    *slab_alignment = kGranule;
    return LOHAN_OK;
}

lohan_status_t lohan_tensor_placement(const uint64_t *lengths, uint32_t count,
                                      lohan_block_offsets_t *offsets, size_t *slab_bytes,
                                      size_t *slab_alignment)
{
    constexpr size_t kBig = 2ull << 20;           // arrays of this size and more: 2 MiB granule
    constexpr size_t kSmall = 4096;               // smaller ones: 4 KiB granule
    constexpr size_t kSkew = 1ull << 20;          // long arrays start on multiples of this
    constexpr size_t kSmallest = 256ull << 20;    // below this the placement gains under 1 %
    constexpr size_t kPeriods[2] = {4ull << 30, 12ull << 30};
    if (slab_bytes == nullptr || slab_alignment == nullptr ||
        (count != 0 && (lengths == nullptr || offsets == nullptr)))
        return LOHAN_ERR_NULL;
    for (uint32_t i = 0; i < count; ++i)
        if (lengths[i] > (1ull << 40)) return LOHAN_ERR_ARG;
    auto rounded = [&](size_t bytes) {
        const size_t g = bytes >= kBig ? kBig : kSmall;
        return (bytes + g - 1) / g * g;
    };
    *slab_alignment = kBig;
    size_t largest = 0;
    for (uint32_t i = 0; i < count; ++i)
        if (rounded((size_t)lengths[i] * 4) > largest) largest = rounded((size_t)lengths[i] * 4);
    size_t period = 0;
    if (largest >= kSmallest)
        for (size_t candidate : kPeriods)
            if (period == 0 && largest <= candidate - kBig) period = candidate;

    // Where an array of `bytes` may start at or after `at` (relative to a 2 MiB-aligned origin):
    // long arrays on 1 MiB boundaries (the lanes themselves are skewed by 1 MiB), short ones on
    // 4 KiB boundaries.
    auto aligned = [&](size_t at, size_t bytes) {
        const size_t a = bytes >= kBig ? kSkew : kSmall;
        return (at + a - 1) / a * a;
    };
    if (period == 0) {                            // plain tensor-major packing
        size_t at = 0;
        auto take = [&](size_t bytes) {
            const size_t start = aligned(at, bytes);
            at = start + bytes;
            return start;
        };
        for (uint32_t i = 0; i < count; ++i) {
            const size_t wide = rounded((size_t)lengths[i] * 4);
            const size_t narrow = rounded((size_t)lengths[i] * 2);
            lohan_block_offsets_t &o = offsets[i];
            o.param_fp32 = take(wide);
            o.exp_avg = take(wide);
            o.exp_avg_sq = take(wide);
            o.grad_fp16 = take(narrow);
            o.param_bf16 = take(narrow);
        }
        *slab_bytes = at;
        return LOHAN_OK;
    }

    const LaneStarts starts = lane_starts(period);
    const size_t lane[3] = {0, starts.lane1, starts.lane2};
    size_t group_base = 0;
    uint32_t first = 0;
    while (first < count) {
        // A group: consecutive tensors whose fp32 arrays fit one lane together.
        uint32_t end = first;
        size_t lane_used = 0;
        while (end < count) {
            const size_t wide = rounded((size_t)lengths[end] * 4);
            const size_t at = aligned(lane_used, wide);
            if (at + wide > period - kBig) break;
            lane_used = at + wide;
            ++end;
        }
        // Free room behind the fp32 arrays of lanes 0 and 1 (up to the next lane's start) takes
        // 16-bit arrays, first fit; whatever does not fit follows lane 2.
        size_t room_at[3] = {lane[0] + lane_used, lane[1] + lane_used, lane[2] + lane_used};
        const size_t room_end[2] = {lane[1], lane[2]};
        auto take_narrow = [&](size_t bytes) {
            for (int w = 0; w < 2; ++w) {
                const size_t at = aligned(room_at[w], bytes);
                if (at + bytes <= room_end[w]) {
                    room_at[w] = at + bytes;
                    return at;
                }
            }
            const size_t at = aligned(room_at[2], bytes);
            room_at[2] = at + bytes;
            return at;
        };
        size_t within = 0;
        for (uint32_t i = first; i < end; ++i) {
            const size_t wide = rounded((size_t)lengths[i] * 4);
            const size_t narrow = rounded((size_t)lengths[i] * 2);
            within = aligned(within, wide);
            lohan_block_offsets_t &o = offsets[i];
            o.param_fp32 = group_base + lane[0] + within;
            o.exp_avg = group_base + lane[1] + within;
            o.exp_avg_sq = group_base + lane[2] + within;
            o.grad_fp16 = group_base + take_narrow(narrow);
            o.param_bf16 = group_base + take_narrow(narrow);
            within += wide;
        }
        group_base += (room_at[2] + kBig - 1) / kBig * kBig;
        first = end;
    }
    *slab_bytes = group_base;
    return LOHAN_OK;
}

float lohan_clip_loss_scale(double sqnorm, float loss_scale, float max_norm)
{
    if (!(sqnorm >= 0.0) || !std::isfinite(sqnorm) || !finite_pos(loss_scale) ||
        !finite_pos(max_norm))
        return std::numeric_limits<float>::quiet_NaN();
    const double norm = std::sqrt(sqnorm);
    double coef = (double)max_norm / (norm + 1e-6);
    if (coef > 1.0) coef = 1.0;
    return (float)((double)loss_scale / coef);
}

// ------------------------------------------------------------------------------------------------
// lohan_grad_sqnorm for callers that cannot allocate: the workspace is a static device array.
// ------------------------------------------------------------------------------------------------

}  // extern "C"

// One copy of this array exists on every GPU the library runs on, at that GPU's own address, and
// stays there until the process ends.  Its name is only a host-side handle for
// hipGetSymbolAddress: kernels and copies are given the resolved per-device address, never the
// name.  The loader zero-fills it, which is the state the ticket counters need.
static __device__ __align__(256) unsigned char scratch[lohan::kWorkspaceBytes];

namespace {

std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// Address of `scratch` on the current device; resolved once per device, with that device
// current.  The first call on a device also enqueues the counter fill on `stream`, ahead of the
// caller's reduction.  NULL on error.
void *scratch_on_current_device(hipStream_t stream)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] != nullptr) return g_scratch_ptr[dev];
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr)
        return nullptr;
    if (lohan::launch_workspace_init(ptr, stream) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = ptr;
    return ptr;
}

}  // namespace

extern "C" {

lohan_status_t lohan_grad_sqnorm_static(const void *grad_fp16, uint64_t n, float loss_scale,
                                        double *sqnorm, uint32_t *overflow_flag,
                                        hipStream_t stream)
{
    if (sqnorm == nullptr || (grad_fp16 == nullptr && n != 0)) return LOHAN_ERR_NULL;
    if (misaligned(grad_fp16, 16) || misaligned(sqnorm, 8) || misaligned(overflow_flag, 4))
        return LOHAN_ERR_ALIGN;
    if (!finite_pos(loss_scale)) return LOHAN_ERR_ARG;
    if (n > LOHAN_GRAD_SQNORM_STATIC_MAX_N) return LOHAN_ERR_TOO_LARGE;
    const lohan::DeviceInfo dev = current_device();
    if (dev.cus <= 0) return LOHAN_ERR_HIP;
    void *workspace = scratch_on_current_device(stream);
    if (workspace == nullptr) return LOHAN_ERR_HIP;
    const double inv = 1.0 / (double)loss_scale;
    hipError_t e = lohan::launch_grad_reduce(grad_fp16, n, true, inv * inv, sqnorm, overflow_flag,
                                             workspace, reduce_workgroups(dev), reduce_streams(n),
                                             stream);
    return e == hipSuccess ? LOHAN_OK : LOHAN_ERR_HIP;
}

lohan_status_t lohan_workspace_init(void *workspace, size_t workspace_bytes, hipStream_t stream)
{
    lohan_status_t ws = check_workspace(workspace, workspace_bytes);
    if (ws != LOHAN_OK) return ws;
    return lohan::launch_workspace_init(workspace, stream) == hipSuccess ? LOHAN_OK
                                                                         : LOHAN_ERR_HIP;
}

lohan_status_t lohan_tuning_set_launch_config(int adam_variant, int adam_workgroups_per_cu,
                                              int adam_waves_per_cu, int reduce_workgroups_per_cu,
                                              int reduce_policy)
{
    if (adam_variant < 0) adam_variant = kAutoAdamVariant;
    else if (!lohan::adam_variant_valid(adam_variant)) return LOHAN_ERR_ARG;
    if (adam_workgroups_per_cu > 4096 || adam_waves_per_cu > 32 || reduce_workgroups_per_cu > 16 ||
        reduce_policy > 1)
        return LOHAN_ERR_ARG;
    t_launch.adam_variant = adam_variant;
    t_launch.adam_wgs_per_cu = adam_workgroups_per_cu < 0 ? kDefaultAdamWgsPerCu
                                                          : adam_workgroups_per_cu;
    t_launch.adam_waves_per_cu = adam_waves_per_cu < 0 ? kDefaultAdamWavesPerCu
                                                       : adam_waves_per_cu;
    t_launch.reduce_wgs_per_cu = reduce_workgroups_per_cu <= 0 ? kDefaultReduceWgsPerCu
                                                               : reduce_workgroups_per_cu;
    t_launch.reduce_policy = reduce_policy < 0 ? kAutoReducePolicy : reduce_policy;
    return LOHAN_OK;
}

lohan_status_t lohan_tuning_set_wait_limit(int64_t polls)
{
    if (polls > (int64_t)0xFFFFFFFFll) return LOHAN_ERR_ARG;
    t_launch.wait_limit = polls < 0 ? kDefaultWaitLimit : (uint32_t)polls;
    return LOHAN_OK;
}

lohan_status_t lohan_tuning_device_info(int *compute_units, size_t *lds_bytes_per_cu)
{
    const lohan::DeviceInfo dev = current_device();
    if (dev.cus <= 0) return LOHAN_ERR_HIP;
    if (compute_units) *compute_units = dev.cus;
    if (lds_bytes_per_cu) *lds_bytes_per_cu = dev.lds_per_cu;
    return LOHAN_OK;
}

void lohan_tuning_get_launch_config(int *adam_variant, int *adam_workgroups_per_cu,
                                    int *adam_waves_per_cu, int *reduce_workgroups_per_cu,
                                    int *reduce_policy)
{
    if (adam_variant) *adam_variant = t_launch.adam_variant;
    if (adam_workgroups_per_cu) *adam_workgroups_per_cu = t_launch.adam_wgs_per_cu;
    if (adam_waves_per_cu) *adam_waves_per_cu = t_launch.adam_waves_per_cu;
    if (reduce_workgroups_per_cu) *reduce_workgroups_per_cu = t_launch.reduce_wgs_per_cu;
    if (reduce_policy) *reduce_policy = t_launch.reduce_policy;
}

}  // extern "C"
