// Internal interface between the C ABI layer (lohan_api.hip) and the kernels (lohan_kernels.hip).
#ifndef LOHAN_KERNELS_H
#define LOHAN_KERNELS_H

#include <hip/hip_runtime_api.h>
#include <stddef.h>
#include <stdint.h>

namespace lohan {

// Per-call fp32 scalars, computed once on the host and passed by value (they live in SGPRs).
struct StepScalars {
    float inv;    // fl(1 / loss_scale)
    float beta1;
    float omb1;   // fl(1 - beta1)
    float beta2;
    float omb2;   // fl(1 - beta2)
    float sbc2;   // fl(sqrt(bc2)), bc2 = fp32 rounding of the float64 value 1 - beta2^step
    float eps;
    float ss;     // fl(lr / bc1),  bc1 = fp32 rounding of the float64 value 1 - beta1^step
    float decay;  // fl(1 - fl(lr * wd))
    float wd;
};

// Blocks of a multi-block launch travel by value in the kernel arguments (no table in device
// memory, nothing to upload): kMultiMaxBlocks descriptors of 48 bytes stay under the 4 KB limit.
constexpr uint32_t kMultiMaxBlocks = 64;
struct MultiDesc {
    float *p, *m, *v;
    const uint16_t *g;
    uint16_t *p16;
    uint64_t n;
};
struct MultiArgs {
    MultiDesc d[kMultiMaxBlocks];
};

// Ring of slots (see k_adam_ring_step).  Device memory layout of a ring for B blocks and S spare
// slots (one per distinct block length), all parts 16-byte aligned: B + S RingSlot entries, then B
// uint64 attempt counters, then B uint64 "attempt that last overflowed" values, then B uint32 slot
// indices (slot_of), then B uint32 class indices (class_of), then S uint32 slot indices (the
// spare of each class), then B floats (the unscale factor of a clipped step, one per block).
struct RingSlot {
    float *p, *m, *v;
    uint16_t *p16;
    uint64_t n;
};
struct RingView {
    RingSlot *slots;
    uint64_t *attempts;
    uint64_t *overflow_attempt;
    uint32_t *slot_of;
    uint32_t *class_of;
    uint32_t *spare_of_class;
    float *clip_inv;
};
inline size_t ring_pad16(size_t x) { return (x + 15) / 16 * 16; }
inline size_t ring_bytes(uint32_t num_blocks, uint32_t num_spares)
{
    const size_t b = num_blocks, s = num_spares;
    return ring_pad16(sizeof(RingSlot) * (b + s)) + 2 * ring_pad16(sizeof(uint64_t) * b) +
           2 * ring_pad16(sizeof(uint32_t) * b) + ring_pad16(sizeof(uint32_t) * s) +
           ring_pad16(sizeof(float) * b);
}
inline RingView ring_view(void *ring, uint32_t num_blocks, uint32_t num_spares)
{
    const size_t b = num_blocks, s = num_spares;
    char *base = reinterpret_cast<char *>(ring);
    RingView view;
    view.slots = reinterpret_cast<RingSlot *>(base);
    base += ring_pad16(sizeof(RingSlot) * (b + s));
    view.attempts = reinterpret_cast<uint64_t *>(base);
    base += ring_pad16(sizeof(uint64_t) * b);
    view.overflow_attempt = reinterpret_cast<uint64_t *>(base);
    base += ring_pad16(sizeof(uint64_t) * b);
    view.slot_of = reinterpret_cast<uint32_t *>(base);
    base += ring_pad16(sizeof(uint32_t) * b);
    view.class_of = reinterpret_cast<uint32_t *>(base);
    base += ring_pad16(sizeof(uint32_t) * b);
    view.spare_of_class = reinterpret_cast<uint32_t *>(base);
    base += ring_pad16(sizeof(uint32_t) * s);
    view.clip_inv = reinterpret_cast<float *>(base);
    return view;
}

// Workspace layout: kMaxPartials doubles, then kMaxPartials uint32 flags, then the per-call
// scalars: kMultiMaxBlocks unscale factors (float; a single-block clipped step uses the first),
// then kMultiMaxBlocks squared norms (double) for multi-block calls whose caller wants none,
// then kMultiMaxBlocks uint32 ticket counters of the gradient reduction (a single-block call uses
// the first), then a 64-bit word that holds kWorkspaceMagic once the workspace has been prepared,
// then kGroupLines lines of kLineBytes each: word 0 of a line is the ticket counter of one group
// of kGroupSize workgroups (the first level of the two-level ticket), word kVerdictWord of a line
// receives the verdict of the one-launch step's grid-wide barrier for that group, and the last
// line holds that step's call counter (word 0) and its "somebody gave up waiting" mark (word 1).
// Invariants: all ticket counters are zero between calls (launch_workspace_init sets them up,
// every call restores them); the magic word lets the kernels tell a workspace that was never
// prepared, whose counters may hold anything.
constexpr uint32_t kMaxPartials = 4096;
constexpr size_t kScalarsOffset = (size_t)kMaxPartials * (sizeof(double) + sizeof(uint32_t));
constexpr size_t kNormsOffset = kScalarsOffset + 256;
constexpr size_t kCountersOffset = kNormsOffset + kMultiMaxBlocks * sizeof(double);
constexpr size_t kMagicOffset = kCountersOffset + kMultiMaxBlocks * sizeof(uint32_t);
constexpr uint32_t kGroupSize = 32;
constexpr uint32_t kLineBytes = 128;
constexpr uint32_t kLineWords = kLineBytes / sizeof(uint32_t);
constexpr uint32_t kVerdictWord = 16;
constexpr uint32_t kGroupLines = 256;
constexpr uint32_t kCallLine = kGroupLines - 1;
constexpr size_t kLinesOffset = (kMagicOffset + 16 + kLineBytes - 1) / kLineBytes * kLineBytes;
constexpr size_t kWorkspaceBytes = kLinesOffset + (size_t)kGroupLines * kLineBytes;
constexpr uint64_t kWorkspaceMagic = 0x4C6F48616E57531Full;
// A single-block call has at most kMaxPartials / kGroupSize groups; a multi-block call at most
// that plus one partly filled group per block; the last line is not a group's.
static_assert(kMaxPartials / kGroupSize + kMultiMaxBlocks < kCallLine, "group lines");
static_assert(kMultiMaxBlocks * sizeof(float) <= 256, "unscale factors must fit their area");

// The one-launch step for small blocks holds the block in registers: kSmallDepths[i] tiles of
// kSmallTile elements per workgroup, one kernel instantiation per depth (deeper = more registers
// per lane, fewer workgroups resident per compute unit).
constexpr int kSmallVariants = 3;
constexpr int kSmallDepths[kSmallVariants] = {3, 7, 15};
constexpr uint64_t kSmallTile = 1024;
// Bit of the overflow flag that reports a grid-wide wait that was given up (state unspecified).
constexpr uint32_t kFlagIncomplete = 0x80000000u;

// What the launchers need to know about the device the stream belongs to.
struct DeviceInfo {
    int cus;             // compute units
    size_t lds_per_cu;   // bytes of LDS per compute unit (sizes the occupancy throttle)
    int small_wgs_per_cu[kSmallVariants];  // resident workgroups per CU of each small-block depth
};

// Fills small_wgs_per_cu from the occupancy the runtime reports for the kernels (the lowest over
// the modes of a depth).
hipError_t small_block_occupancy(int wgs_per_cu[kSmallVariants]);

// Largest n the one-launch step takes on this device (0 if none of the kernels fits).
uint64_t small_block_max_n(const DeviceInfo &dev);

// Zero the ticket counters of a workspace and set its magic word (a one-workgroup fill kernel).
hipError_t launch_workspace_init(void *workspace, hipStream_t stream);

// stream_past_caches: nontemporal loads (blocks far larger than the memory-side cache) instead
// of the default policy (blocks that fit it, so that the update's read of the gradients hits).
hipError_t launch_grad_reduce(const void *grad_fp16, uint64_t n, bool with_norm, double inv2,
                              double *sqnorm, uint32_t *flag, void *workspace, uint32_t max_wgs,
                              bool stream_past_caches, hipStream_t stream);

// Gradient producer with the flag / norm in its epilogue: out[i] = binary16(grad_fp32[i] *
// multiplier); sqnorm (may be NULL) and flag describe the values written.
hipError_t launch_grad_produce(const float *grad_fp32, uint64_t n, float multiplier,
                               void *grad_fp16_out, double inv2, double *sqnorm, uint32_t *flag,
                               void *workspace, uint32_t max_wgs, bool stream_past_caches,
                               hipStream_t stream);

// Launch shape of the Adam kernel.
struct AdamLaunch {
    int variant;         // see adam_variant_valid
    int max_wgs_per_cu;  // <= 0: one tile per workgroup (grid = number of tiles)
    int waves_per_cu;    // <= 0 or >= 32: no occupancy throttle
};

bool adam_variant_valid(int variant);

// mode bits of launch_adam_block_step: 1 = L2 regularisation, 2 = binary16 output copy.

hipError_t launch_adam_block_step(float *p, float *m, float *v, const void *grad_fp16,
                                  void *p16, uint64_t n, const StepScalars &s, int mode,
                                  const uint32_t *flag, const float *inv_override,
                                  const AdamLaunch &cfg, const DeviceInfo &dev, hipStream_t stream);

// Out-of-place form with the overflow test fused in (clears *flag, then one 28 B/element pass).
hipError_t launch_adam_block_step_oop(const float *p_in, const float *m_in, const float *v_in,
                                      const void *grad_fp16, float *p_out, float *m_out,
                                      float *v_out, void *p16, uint64_t n, const StepScalars &s,
                                      int mode, uint32_t *flag, const float *inv_override,
                                      const AdamLaunch &cfg, const DeviceInfo &dev,
                                      hipStream_t stream);

// Ring form: the step of `block` from its current slot into the spare, then the commit.
hipError_t launch_adam_ring_step(const RingView &ring, uint32_t block, const void *grad_fp16,
                                 uint64_t n, const StepScalars &s, int mode,
                                 const float *inv_override, const AdamLaunch &cfg,
                                 const DeviceInfo &dev, hipStream_t stream);

// One-launch step for a block of at most small_block_max_n(dev) elements (hipErrorInvalidValue
// beyond): flag, squared norm (sqnorm may be NULL) and update.  spin_limit bounds the grid-wide
// wait in polls.
hipError_t launch_adam_small_block_step(float *p, float *m, float *v, const void *grad_fp16,
                                        void *p16, uint64_t n, const StepScalars &s, int mode,
                                        double inv2, double *sqnorm, uint32_t *flag,
                                        void *workspace, uint32_t spin_limit,
                                        const DeviceInfo &dev, hipStream_t stream);

// sqnorm[0..count) -> inv_out[0..count)
hipError_t launch_clip_scale(const double *sqnorm, float loss_scale, float max_norm,
                             float *inv_out, uint32_t count, hipStream_t stream);

// Multi-block forms: num_blocks in [1, kMultiMaxBlocks]; flags / sqnorms / inv_override are
// arrays indexed by block.
hipError_t launch_multi_grad_reduce(const MultiArgs &args, uint32_t num_blocks, bool with_norm,
                                    double inv2, double *sqnorms, uint32_t *flags,
                                    void *workspace, uint32_t max_wgs, bool stream_past_caches,
                                    hipStream_t stream);
hipError_t launch_adam_multi_block_step(const MultiArgs &args, uint32_t num_blocks,
                                        const StepScalars &s, int mode, const uint32_t *flags,
                                        const float *inv_override, const AdamLaunch &cfg,
                                        const DeviceInfo &dev, hipStream_t stream);

}  // namespace lohan

#endif
