/*
 * lohan_adam.h -- C ABI of the per-block fused mixed-precision Adam/AdamW step for MI355X (gfx950).
 *
 * The operation is the "CPU Compute" step of LoHan's active gradient offloading (arxiv 2403.06504,
 * Sec. IV-C, "Naive Active Gradient Offloading"): when the gradients of tensor/block i appear
 * during backward, the model states of that block are updated and a 16-bit parameter copy is
 * produced.  The tensors are those of Table II: P32 (fp32 parameters, 4 B/param), OS32 (the two
 * fp32 Adam moments, 8 B/param), G16 (fp16 gradients, 2 B/param) and P16 (16-bit working copy,
 * 2 B/param, here bfloat16).  The optimizer is Adam (Sec. II, "LLM Training Stages"), run in
 * mixed precision (Sec. V-A, "Workloads"), synchronously: the P16 copy always equals the rounding
 * of the P32 written by the same step (Sec. IV-C, footnote on staleness).  Here the step runs on
 * the GPU out of HBM instead of on the host.
 *
 * Conventions common to all entry points
 *   - Every data pointer is DEVICE memory owned by the caller, valid on `stream`'s device, and
 *     16-byte aligned (4 KiB or better for full bandwidth: bases aligned only to 256 bytes cost
 *     about 4 % on MI355X).  Buffers of one call must not overlap each other.
 *   - The library allocates no device memory, keeps no per-call state, and does not synchronise:
 *     kernels are enqueued on `stream` and the call returns.  Results (state, flag, squared norm)
 *     are valid once the work enqueued on `stream` has completed.  The exceptions say so in their
 *     own comments: lohan_ring_init and lohan_ring_read (synchronous copies), the lohan_offload_*
 *     handle (owns streams and events) and the host-only helpers (no device involved at all).
 *   - `workspace` is device scratch of at least lohan_workspace_bytes() bytes, 16-byte aligned,
 *     private to the call until its kernels complete (calls that may run concurrently on different
 *     streams need different workspaces).  It must have been prepared ONCE with
 *     lohan_workspace_init before its first use; every call leaves it ready for the next one, so
 *     nothing needs clearing between calls.
 *   - n is the element count of the flat block; any n >= 0 is accepted (n == 0: flag = 0,
 *     squared norm = 0, nothing else is touched).
 *   - Errors are reported by return code only.  For codes LOHAN_ERR_NULL .. LOHAN_ERR_WORKSPACE no
 *     kernel was launched and no memory was modified.  After LOHAN_ERR_HIP (a launch failed)
 *     buffer contents are unspecified.
 */
#ifndef LOHAN_ADAM_H
#define LOHAN_ADAM_H

#include <stddef.h>
#include <stdint.h>

#include <hip/hip_runtime_api.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LOHAN_OK = 0,
    LOHAN_ERR_NULL = 1,       /* a required pointer is NULL */
    LOHAN_ERR_ALIGN = 2,      /* a data pointer or the workspace is not 16-byte aligned */
    LOHAN_ERR_ARG = 3,        /* a scalar argument is out of its domain (see each call) */
    LOHAN_ERR_WORKSPACE = 4,  /* workspace_bytes < lohan_workspace_bytes() */
    LOHAN_ERR_HIP = 5,        /* the HIP runtime reported an error at launch */
    LOHAN_ERR_TOO_LARGE = 6   /* n exceeds the maximum of an entry point that has one */
} lohan_status_t;

enum {
    /* Adam with L2 regularisation (g += wd * p) instead of decoupled decay (AdamW, the default). */
    LOHAN_FLAG_L2_MODE = 1u,
    /* *overflow_flag already holds this block's flag on `stream` (from lohan_grad_overflow_check
     * or lohan_grad_sqnorm): lohan_adam_block_step then skips its own 2 B/element check pass. */
    LOHAN_FLAG_PRECHECKED = 2u,
    /* Emit the 16-bit working copy as IEEE binary16 (round to nearest even, overflow to infinity)
     * instead of bfloat16; param_bf16_out then receives n binary16 values. */
    LOHAN_FLAG_P16_FP16 = 4u
};

/* Device scratch bytes one call needs (a constant of the build; about 81 KiB). */
size_t lohan_workspace_bytes(void);

/*
 * Prepare a freshly allocated workspace: the gradient reduction finishes inside its one launch
 * (the workgroup that publishes the last partial result combines them all), which needs a few
 * ticket counters in the workspace to read zero when a call starts.  This enqueues a small fill
 * kernel on `stream` that zeroes them; every later call puts them back to zero itself.  Call it
 * once per workspace (and again after an LOHAN_ERR_HIP, when the contents are unspecified).  It
 * also writes a marker by which the kernels recognise a prepared workspace: a call that is
 * handed one without the marker reduces nothing and reports the block as overflowing
 * (*overflow_flag = 1, *sqnorm = NaN), so the step that follows is skipped -- wrong use fails
 * visibly and on the safe side.  Errors: LOHAN_ERR_NULL / _ALIGN / _WORKSPACE as for any
 * workspace argument.
 */
lohan_status_t lohan_workspace_init(void *workspace, size_t workspace_bytes, hipStream_t stream);

/* Static text for a status code (host memory owned by the library). */
const char *lohan_status_string(lohan_status_t status);

/*
 * Overflow flag of one block's fp16 gradients (G16 of Table II): *overflow_flag = 1 if any of the
 * n stored values is +-inf or NaN (fp16 exponent field all ones, tested on the raw bits before
 * any unscaling), else 0.  The flag is always written (never left stale).
 *   grad_fp16      device, in : n IEEE binary16 values, contiguous
 *   overflow_flag  device, out: one uint32, 4-byte aligned
 */
lohan_status_t lohan_grad_overflow_check(const void *grad_fp16, uint64_t n,
                                         uint32_t *overflow_flag,
                                         void *workspace, size_t workspace_bytes,
                                         hipStream_t stream);

/*
 * Squared l2 norm of one block's unscaled gradients, *sqnorm = sum_i (g16_i / loss_scale)^2,
 * accumulated in float64 in a fixed order (same input -> same bits), for per-block gradient
 * clipping; the same single read of G16 also yields the overflow flag when overflow_flag is not
 * NULL.  When the flag is 1 the value of *sqnorm is unspecified (it may be inf or NaN).
 *   sqnorm         device, out: one double, 8-byte aligned
 *   overflow_flag  device, out: one uint32 or NULL
 *   loss_scale     finite and > 0, else LOHAN_ERR_ARG
 */
lohan_status_t lohan_grad_sqnorm(const void *grad_fp16, uint64_t n, float loss_scale,
                                 double *sqnorm, uint32_t *overflow_flag,
                                 void *workspace, size_t workspace_bytes, hipStream_t stream);

/*
 * A gradient producer with the block's overflow flag and squared norm computed in its epilogue,
 * so that the block step needs no separate 2-byte pass over G16: fp32 gradients (as accumulated
 * over micro-batches by backward, still multiplied by the loss scale) are turned into the G16
 * tensor of Table II -- the form in which Sec. IV-C's handler receives the gradients of block i --
 *     grad_fp16_out[i] = binary16, round to nearest even, of (grad_fp32[i] * multiplier)
 * (one fp32 multiplication, e.g. by 1 / accumulation steps; a product too large for binary16
 * becomes +-inf, which is how fp16 gradients overflow), and *overflow_flag and *sqnorm are those
 * lohan_grad_sqnorm would compute from grad_fp16_out (flag bit-identical; norm accumulated in
 * float64 in a fixed order of its own, same input -> same bits).  The step then runs with
 * LOHAN_FLAG_PRECHECKED (or lohan_adam_block_step_clipped): 28 bytes per element in place.
 *   grad_fp32      device, in : n floats
 *   grad_fp16_out  device, out: n binary16 values (must not overlap grad_fp32)
 *   multiplier     finite, else LOHAN_ERR_ARG
 *   loss_scale     finite and > 0 (only scales the norm), else LOHAN_ERR_ARG
 *   sqnorm         device, out: one double or NULL
 *   overflow_flag  device, out: one uint32, always written
 * Moves 6 bytes per element (4 read, 2 written).  Errors as lohan_grad_sqnorm.
 */
lohan_status_t lohan_grad_produce_fp16(const float *grad_fp32, uint64_t n, float multiplier,
                                       void *grad_fp16_out, float loss_scale, double *sqnorm,
                                       uint32_t *overflow_flag, void *workspace,
                                       size_t workspace_bytes, hipStream_t stream);

/*
 * lohan_grad_sqnorm for callers that cannot allocate device memory or carry a workspace around:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and kernels as lohan_grad_sqnorm, minus the workspace: the partial results
 * and the ticket counter live in a static device array of the library (lohan_workspace_bytes()
 * = about 81 KiB, present on every GPU the library runs on until the process ends).  The call
 * allocates nothing, frees nothing and never synchronises.  Its first call on a device resolves
 * that device's copy of the array and enqueues a small fill kernel ahead of the reduction.
 *   n   at most LOHAN_GRAD_SQNORM_STATIC_MAX_N elements, else LOHAN_ERR_TOO_LARGE
 * All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU (two
 * streams, two threads) race and give unspecified results -- order them, or use
 * lohan_grad_sqnorm with separate workspaces.  Other errors as lohan_grad_sqnorm.
 */
#define LOHAN_GRAD_SQNORM_STATIC_MAX_N (1ull << 40)
lohan_status_t lohan_grad_sqnorm_static(const void *grad_fp16, uint64_t n, float loss_scale,
                                        double *sqnorm, uint32_t *overflow_flag,
                                        hipStream_t stream);

/*
 * One block step (Sec. IV-C "CPU Compute": update the model states of block i and emit its 16-bit
 * parameter copy; tensors of Table II; Adam per Sec. II with bias correction).
 *
 * Unless LOHAN_FLAG_PRECHECKED is given, pass 1 computes *overflow_flag as
 * lohan_grad_overflow_check does.  Pass 2 reads the flag on the device; if it is non-zero the
 * step is skipped and param_fp32, exp_avg, exp_avg_sq and param_bf16_out stay bit-identical.
 * Otherwise, per element, in fp32 with every operation rounded to nearest-even and none fused:
 *     g   = float(g16) * (1 / loss_scale)              [L2 mode: g = g + wd * p]
 *     m'  = beta1 * m + (1 - beta1) * g
 *     v'  = beta2 * v + (1 - beta2) * (g * g)
 *     den = sqrt(v') / sqrt(1 - beta2^step) + eps
 *     p'  = p * (1 - lr * wd) - (lr / (1 - beta1^step)) * (m' / den)     [L2 mode: no p factor]
 *     p16 = bfloat16 round-to-nearest-even of p'        [LOHAN_FLAG_P16_FP16: binary16 instead]
 * and p', m', v' overwrite p, m, v (1 - beta^step is evaluated in float64 and rounded once).
 *
 *   param_fp32, exp_avg, exp_avg_sq   device, in/out: n floats each
 *   grad_fp16                          device, in    : n binary16 values
 *   param_bf16_out                     device, out   : n bfloat16 values
 *   step        1-based index of the step being taken; the caller advances it only when the
 *               flag came back 0.  step < 1 -> LOHAN_ERR_ARG
 *   loss_scale  finite and > 0.  Gradient clipping is folded in by the caller passing
 *               loss_scale / coef (see lohan_clip_loss_scale)
 *   lr, eps, weight_decay  finite and >= 0; beta1, beta2 in [0, 1); else LOHAN_ERR_ARG
 *   overflow_flag  device, in/out: one uint32 (written by pass 1, or read-only when prechecked)
 *   flags       OR of LOHAN_FLAG_*; unknown bits -> LOHAN_ERR_ARG
 * Moves 28 bytes per element (14 read, 14 written), plus 2 read by pass 1 when it runs.
 * "device" above means device-accessible: pinned host memory (hipHostMalloc or equivalent) is
 * accepted for any of the arrays, and the kernel then reads and writes it over the host link
 * (the zero-copy form of the offloaded step of Sec. IV-C; no staging buffer is needed).
 */
lohan_status_t lohan_adam_block_step(float *param_fp32, float *exp_avg, float *exp_avg_sq,
                                     const void *grad_fp16, void *param_bf16_out, uint64_t n,
                                     float lr, float beta1, float beta2, float eps,
                                     float weight_decay, int64_t step, float loss_scale,
                                     uint32_t *overflow_flag, uint32_t flags,
                                     void *workspace, size_t workspace_bytes, hipStream_t stream);

/*
 * The same block step with per-block gradient-norm clipping resolved on the device, so that a
 * clipping run needs no host round trip between lohan_grad_sqnorm and the update: the unscale
 * factor is 1 / fp32(loss_scale / coef) with coef = min(1, max_norm / (sqrt(*sqnorm) + 1e-6)),
 * evaluated in float64 by a one-lane kernel ahead of the update (same formula as
 * lohan_clip_loss_scale).  *sqnorm and *overflow_flag must already hold this block's results of
 * lohan_grad_sqnorm on `stream` (the flag is read-only here, as with LOHAN_FLAG_PRECHECKED; a set
 * flag skips the step whatever *sqnorm holds).
 *   sqnorm      device, in: one double, 8-byte aligned
 *   max_norm    finite and > 0, else LOHAN_ERR_ARG
 *   flags       LOHAN_FLAG_L2_MODE and/or LOHAN_FLAG_P16_FP16 (LOHAN_FLAG_PRECHECKED is implied
 *               and may be given)
 *   workspace   required (holds the device-side scalar); may be the one lohan_grad_sqnorm used
 * Everything else as lohan_adam_block_step.
 */
lohan_status_t lohan_adam_block_step_clipped(float *param_fp32, float *exp_avg, float *exp_avg_sq,
                                             const void *grad_fp16, void *param_bf16_out,
                                             uint64_t n, float lr, float beta1, float beta2,
                                             float eps, float weight_decay, int64_t step,
                                             float loss_scale, const double *sqnorm,
                                             float max_norm, const uint32_t *overflow_flag,
                                             uint32_t flags, void *workspace,
                                             size_t workspace_bytes, hipStream_t stream);

/*
 * The whole step of a SMALL block in one launch (Sec. IV-C: flag, then the update of block i's
 * model states; tensors of Table II): *overflow_flag and *sqnorm as lohan_grad_sqnorm computes
 * them, and the update of lohan_adam_block_step under the same skip rule, without the separate
 * 2-byte pass and without a second launch.  The grid is sized so that all of it is resident on
 * the device at once; every workgroup loads its share of the block into registers, the
 * workgroups meet at a grid-wide barrier whose counter carries the flag, and the update is
 * computed from registers: 28 bytes per element moved, reads and writes in two separate phases.
 * For a block of a few million elements this takes four fifths to nineteen twentieths of the
 * time of lohan_grad_sqnorm + lohan_adam_block_step (30-36 against 37 microseconds per step for
 * 7 million elements on MI355X), which there is a chain of launch and memory latencies; blocks
 * that do not fit the device's registers cannot use it.
 *   n              at most the value lohan_adam_small_block_max_n reports for the device (about
 *                  7.8 million elements on MI355X), else LOHAN_ERR_TOO_LARGE
 *   sqnorm         device, out: one double or NULL; unspecified when the flag is set
 *   overflow_flag  device, out: always written: 0 (step taken), 1 (overflow: state bit-identical)
 *   flags          LOHAN_FLAG_L2_MODE and/or LOHAN_FLAG_P16_FP16; LOHAN_FLAG_PRECHECKED ->
 *                  LOHAN_ERR_ARG (with a known flag lohan_adam_block_step is the one to call)
 *   workspace      required, prepared by lohan_workspace_init
 * State after the call is bit-identical to the two-call sequence; *sqnorm is accumulated in
 * float64 in a fixed order of its own (same input -> same bits; within 1e-5 relative of
 * lohan_grad_sqnorm).
 * The barrier's wait is bounded, so every wavefront exits whatever else runs on the device: the
 * workgroups can only all be resident if the compute units are not held by other kernels for
 * good.  Kernels of other streams that finish by themselves merely delay it; two calls of THIS
 * entry point that may run at the same time on one device (two streams) must have grids that
 * fit the device together (on MI355X: n1 + n2 at most 5 million), or be ordered by the caller:
 * otherwise each holds the compute units the other waits for, and both give up.  If a workgroup
 * does give up waiting (after a third of a second), *overflow_flag has
 * LOHAN_OVERFLOW_INCOMPLETE set and the block's state is unspecified (some workgroups may have
 * written, others not): treat it as a failed step and restore the block from a checkpoint; the
 * workspace itself stays usable.
 * Everything else as lohan_adam_block_step.
 */
#define LOHAN_OVERFLOW_INCOMPLETE 0x80000000u
lohan_status_t lohan_adam_small_block_max_n(uint64_t *max_n);
lohan_status_t lohan_adam_small_block_step(float *param_fp32, float *exp_avg, float *exp_avg_sq,
                                           const void *grad_fp16, void *param_bf16_out,
                                           uint64_t n, float lr, float beta1, float beta2,
                                           float eps, float weight_decay, int64_t step,
                                           float loss_scale, double *sqnorm,
                                           uint32_t *overflow_flag, uint32_t flags,
                                           void *workspace, size_t workspace_bytes,
                                           hipStream_t stream);

/*
 * Out-of-place block step with the overflow test fused into the update: ONE pass of 28 bytes per
 * element instead of the 2-byte flag pass followed by the in-place step (same tensors, same
 * arithmetic and same skip rule of Sec. IV-C / Table II as lohan_adam_block_step; what changes is
 * where the results land).  The kernel reads param_fp32_in, exp_avg_in, exp_avg_sq_in and
 * grad_fp16, writes the updated values to the three *_out arrays and the 16-bit copy, and raises
 * *overflow_flag if any gradient has an all-ones exponent.  The inputs are never written, so the
 * skip costs nothing:
 *     *overflow_flag == 0 : the *_out arrays and param_bf16_out hold the step's results; the
 *                           caller commits by using them as the next step's inputs (pointer swap)
 *     *overflow_flag == 1 : the inputs are the block's state, bit-identical; the contents of the
 *                           *_out arrays and of param_bf16_out are unspecified and to be discarded
 *                           (so param_bf16_out must not be the only live copy of the old P16)
 * The price is a second set of the 12 B/element fp32 state (and of the 16-bit copy).  Clipping by
 * the block's own norm cannot be fused this way (the scale depends on the whole block): use
 * lohan_grad_sqnorm + lohan_adam_block_step_out_of_place_clipped for that.
 *   *_in            device, in : n floats each; must not overlap any output
 *   *_out           device, out: n floats each; each must differ from its input array, else
 *                   LOHAN_ERR_ARG (other overlaps are undefined)
 *   overflow_flag   device, out: always written (0 or 1)
 *   flags           LOHAN_FLAG_L2_MODE and/or LOHAN_FLAG_P16_FP16; LOHAN_FLAG_PRECHECKED ->
 *                   LOHAN_ERR_ARG (with a known flag the in-place step is the one to call)
 * No workspace is needed.  n = 0 writes flag = 0 only.  Everything else as lohan_adam_block_step.
 */
lohan_status_t lohan_adam_block_step_out_of_place(
    const float *param_fp32_in, const float *exp_avg_in, const float *exp_avg_sq_in,
    const void *grad_fp16, float *param_fp32_out, float *exp_avg_out, float *exp_avg_sq_out,
    void *param_bf16_out, uint64_t n, float lr, float beta1, float beta2, float eps,
    float weight_decay, int64_t step, float loss_scale, uint32_t *overflow_flag, uint32_t flags,
    hipStream_t stream);

/*
 * The out-of-place step with per-block gradient-norm clipping resolved on the device: as
 * lohan_adam_block_step_out_of_place, but the unscale factor is 1 / fp32(loss_scale / coef) with
 * coef = min(1, max_norm / (sqrt(*sqnorm) + 1e-6)), computed by a one-lane kernel ahead of the
 * update exactly as in lohan_adam_block_step_clipped.  *sqnorm must already hold this block's
 * result of lohan_grad_sqnorm on `stream`; the clip scale needs the whole block's norm before the
 * first element is updated, so a clipping run keeps that 2-byte pass whatever form the update
 * takes.  The overflow test stays fused into the update (*overflow_flag is written here).
 *   sqnorm      device, in: one double, 8-byte aligned
 *   max_norm    finite and > 0, else LOHAN_ERR_ARG
 *   workspace   required (holds the device-side scalar); may be the one lohan_grad_sqnorm used
 */
lohan_status_t lohan_adam_block_step_out_of_place_clipped(
    const float *param_fp32_in, const float *exp_avg_in, const float *exp_avg_sq_in,
    const void *grad_fp16, float *param_fp32_out, float *exp_avg_out, float *exp_avg_sq_out,
    void *param_bf16_out, uint64_t n, float lr, float beta1, float beta2, float eps,
    float weight_decay, int64_t step, float loss_scale, const double *sqnorm, float max_norm,
    uint32_t *overflow_flag, uint32_t flags, void *workspace, size_t workspace_bytes,
    hipStream_t stream);

/*
 * Ring form of the out-of-place step: single-pass (28 bytes per element) updates for a whole
 * model at the price of ONE spare slot per distinct block length instead of a second copy of
 * everything.  A "block" here is whatever unit the gradient handler of Sec. IV-C fires on: a
 * whole transformer block, or one gradient tensor of it (the attention and MLP weight matrices
 * and the small bias / LayerNorm vectors have different lengths; the same few lengths repeat in
 * every layer).  The B blocks live in B slots, and S further slots are spares, one for each
 * distinct length; a slot holds the P32, the two OS32 moments and the P16 copy of one block
 * (Table II).  The step of block b (the "CPU Compute" step of Sec. IV-C, with
 * lohan_adam_block_step's arithmetic) reads the slot that currently holds b, writes the spare of
 * b's length, and a one-lane kernel then makes that spare b's slot and b's old slot the spare --
 * unless b's gradients held inf/NaN, in which case nothing changes hands and the old slot stays
 * b's state, bit-identical.  Which slot holds which block is a table in DEVICE memory (the ring),
 * read by the kernels themselves, so no host decision and no host synchronisation sits between
 * the blocks of a backward pass.
 *   ring        device memory of lohan_ring_bytes(B, S) bytes, 16-byte aligned, owned by the
 *               caller, initialised once by lohan_ring_init and from then on changed only by the
 *               steps.  All steps of one ring must be enqueued on one stream (or otherwise
 *               ordered).
 *   lohan_ring_init   copies the B + S slot descriptors (HOST array; block b starts in slot b,
 *               slots B .. B+S-1 are the spares) into the ring with a synchronous copy.  Every
 *               block must find a spare of exactly its length and no two spares may have the
 *               same length, else LOHAN_ERR_ARG; also LOHAN_ERR_ARG unless 1 <= S <= B.  Slot
 *               arrays: n elements each, 16-byte aligned, not overlapping (a slot with n == 0
 *               may have NULL arrays); LOHAN_ERR_NULL / _ALIGN per slot, LOHAN_ERR_WORKSPACE if
 *               ring_bytes is too small.
 *   lohan_ring_adam_block_step   enqueues the step of `block` and its commit on `stream`;
 *               allocates nothing, never synchronises.  Arguments as lohan_adam_block_step
 *               (flags: LOHAN_FLAG_L2_MODE, LOHAN_FLAG_P16_FP16); block >= B -> LOHAN_ERR_ARG.
 *               n must be the length the block was registered with: the kernel compares it with
 *               the table and, if it differs, touches nothing and reports the step as skipped.
 *               n == 0 does nothing.
 *   lohan_ring_adam_block_step_clipped   the same with per-block clipping resolved on the device
 *               from *sqnorm (device, this block's result of lohan_grad_sqnorm on `stream`) and
 *               max_norm, as lohan_adam_block_step_clipped; the scalar lives in the ring.
 *   lohan_ring_read   synchronises `stream`, then copies to the host (each output may be NULL):
 *               slot_of[b] = the slot that holds block b, spares[j] = the spare slot of the
 *               length that slot B + j had at init, and skipped[b] = 1 if the most recent step
 *               of block b found inf/NaN gradients (or a wrong n) and was skipped, else 0 -- the
 *               overflow flag of lohan_adam_block_step: the caller does not advance that
 *               block's step count.  The forward pass finds block b's P16 in slot slot_of[b].
 */
typedef struct {
    float *param_fp32, *exp_avg, *exp_avg_sq;   /* device: n floats each */
    void *param_16;                             /* device: n 16-bit values */
    uint64_t n;                                 /* elements this slot holds */
} lohan_ring_slot_t;

size_t lohan_ring_bytes(uint32_t num_blocks, uint32_t num_spares);
lohan_status_t lohan_ring_init(void *ring, size_t ring_bytes, const lohan_ring_slot_t *slots,
                               uint32_t num_blocks, uint32_t num_spares);
lohan_status_t lohan_ring_adam_block_step(void *ring, uint32_t num_blocks, uint32_t num_spares,
                                          uint32_t block, const void *grad_fp16, uint64_t n,
                                          float lr, float beta1, float beta2, float eps,
                                          float weight_decay, int64_t step, float loss_scale,
                                          uint32_t flags, hipStream_t stream);
lohan_status_t lohan_ring_adam_block_step_clipped(void *ring, uint32_t num_blocks,
                                                  uint32_t num_spares, uint32_t block,
                                                  const void *grad_fp16, uint64_t n, float lr,
                                                  float beta1, float beta2, float eps,
                                                  float weight_decay, int64_t step,
                                                  float loss_scale, const double *sqnorm,
                                                  float max_norm, uint32_t flags,
                                                  hipStream_t stream);
lohan_status_t lohan_ring_read(const void *ring, uint32_t num_blocks, uint32_t num_spares,
                               uint32_t *slot_of, uint32_t *spares, uint32_t *skipped,
                               hipStream_t stream);

/*
 * One block of a multi-block call: the tensors of Table II for that block, as the arguments of
 * lohan_adam_block_step (same layout, alignment and aliasing rules).
 */
typedef struct {
    float *param_fp32;       /* device, in/out: n floats */
    float *exp_avg;          /* device, in/out: n floats */
    float *exp_avg_sq;       /* device, in/out: n floats */
    const void *grad_fp16;   /* device, in    : n binary16 values */
    void *param_bf16_out;    /* device, out   : n 16-bit values */
    uint64_t n;              /* may be 0 */
} lohan_block_t;

/*
 * The block step of Sec. IV-C for several blocks whose gradients are all present, in a constant
 * number of launches instead of two or three per block (small blocks -- the DiT shapes of
 * Table VI, the h=768 test block -- are otherwise bound by launch gaps and by the ramp of each
 * short kernel).  Every block keeps its own overflow flag, its own norm and its own skip
 * decision, as if lohan_grad_sqnorm / lohan_adam_block_step[_clipped] had been called on it
 * alone: flags and the state after an unclipped step are bit-identical to those calls.  The
 * squared norm is reduced over a different number of workgroups than in a single-block call, so
 * its float64 value may differ from that call's in the last bits (both are within 1e-5 relative
 * of the exact sum); a clipped step is bit-identical to lohan_adam_block_step_clipped given the
 * same squared norm.
 *   blocks          HOST array of num_blocks descriptors (read during the call only; they travel
 *                   to the device inside the kernel arguments, nothing is uploaded or allocated)
 *   num_blocks      any count; runs of up to 64 consecutive blocks of similar length share one
 *                   launch.  0 -> LOHAN_OK, nothing done
 *   max_norm        0: no clipping.  > 0 and finite: each block is clipped by its own norm,
 *                   resolved on the device as in lohan_adam_block_step_clipped.  Else LOHAN_ERR_ARG
 *   overflow_flags  device, num_blocks uint32: written per block (0 or 1), or read-only with
 *                   LOHAN_FLAG_PRECHECKED
 *   sqnorms         device, num_blocks doubles, 8-byte aligned, or NULL: per-block squared norm
 *                   of the unscaled gradients (unspecified for a block whose flag is 1)
 *   flags           as lohan_adam_block_step
 *   workspace       required, lohan_workspace_bytes() bytes, as for the other entry points
 * Errors as lohan_adam_block_step; all blocks are validated before the first launch.
 */
lohan_status_t lohan_adam_multi_block_step(const lohan_block_t *blocks, uint32_t num_blocks,
                                           float lr, float beta1, float beta2, float eps,
                                           float weight_decay, int64_t step, float loss_scale,
                                           float max_norm, uint32_t *overflow_flags,
                                           double *sqnorms, uint32_t flags, void *workspace,
                                           size_t workspace_bytes, hipStream_t stream);

/*
 * Host-only placement advice (pure arithmetic, touches no device).  Where the fp32 arrays of a
 * block sit relative to each other moves the update kernel by several percent on MI355X: p, m
 * and v advance at the same rate, so their relative position is fixed for a whole launch, and
 * the measured best is "same offset within consecutive periods of 4 GiB (or 12 GiB), shifted by
 * a few MiB" (6.85-6.92 TB/s for a 13B-shaped block); the allocator's placement is a lottery
 * between -4 % and 0 % of that, and all three arrays at the same offset modulo 4 GiB is the worst
 * case.  This function lays out the tensors of Table II for num_blocks equal blocks of n
 * elements inside ONE caller-allocated slab accordingly:
 *   - the period P is 4 GiB if one fp32 array fits into 4 GiB - 2 MiB, else 12 GiB if it fits
 *     into 12 GiB - 2 MiB;
 *   - groups of G = floor((P - 2 MiB) / bytes(p)) consecutive blocks share three "lanes":
 *     lane 0 holds their p arrays back to back, lane 1 their m arrays, lane 2 their v arrays,
 *     block j of the group at the same offset in each lane; lanes 1 and 2 start at P + 8 MiB and
 *     2P + 9 MiB for the 4 GiB period and at P + 1 MiB and 2P + 2 MiB for the 12 GiB period (the
 *     best of the pairs measured: m and v an odd number of MiB apart, no two of the three at the
 *     same offset modulo 16 MiB);
 *   - the 16-bit arrays (which advance at half the rate and may sit anywhere) fill what is left
 *     of lanes 0 and 1 where they fit and otherwise follow lane 2;
 *   - blocks whose fp32 arrays fit neither period (3.2e9 elements and more) are packed block by
 *     block with 1 MiB between p, m, v and the 16-bit arrays, so that p, m and v are an odd
 *     number of MiB apart (arrays of exactly 12 GiB would otherwise all sit at the same offset
 *     modulo 4 GiB); blocks whose fp32 arrays stay below 256 MiB (fewer than 2^26 elements) are
 *     simply packed p, m, v, g, p16 back to back (under 1 % to gain).
 * Every array starts on a 1 MiB boundary relative to the slab base; the base itself needs
 * *slab_alignment (2 MiB).  The price is unused space in lanes 0 and 1: per full group 3 % of the
 * slab for 6B-shaped blocks, 7 % for 13B, 12 % for 30B, 17 % for 70B, 4 % for 135B, 14 % for 175B,
 * 15 % for 276B, and more for a last group that is not full -- compare *slab_bytes with
 * 16 * n * num_blocks and decide.
 *   offsets        host, out: num_blocks entries of byte offsets from the slab base
 *   slab_bytes, slab_alignment   host, out
 *   blocks_per_group   host, out, may be NULL: G (1 when the blocks are packed)
 * LOHAN_ERR_NULL for NULL outputs (offsets may be NULL only if num_blocks == 0), LOHAN_ERR_ARG
 * if n exceeds 2^40.
 */
typedef struct {
    size_t param_fp32, exp_avg, exp_avg_sq, grad_fp16, param_bf16;
} lohan_block_offsets_t;

lohan_status_t lohan_model_placement(uint64_t n, uint32_t num_blocks,
                                     lohan_block_offsets_t *offsets, size_t *slab_bytes,
                                     size_t *slab_alignment, uint32_t *blocks_per_group);

/*
 * The compact alternative: most of lohan_model_placement's gain for almost none of its space.
 * Blocks are packed one after the other (p, m, v, g, p16), every array rounded up to 2 MiB, and
 * the three fp32 arrays of a block start an ODD number of MiB apart (each is followed by 1 MiB
 * of padding).  In an interleaved comparison on one fresh slab (update kernel, of the 8 TB/s
 * peak): 13B-shaped block 0.853 this way, 0.857 in the lanes of lohan_model_placement, 0.840
 * packed with the arrays an even number of MiB apart; 175B-shaped block 0.848 / 0.860 / 0.847.
 * Overhead: 4 MiB per block plus the rounding (0.1 % for a 13B-shaped block) instead of 4-17 %.
 * Arguments and errors as lohan_model_placement (no blocks_per_group).
 */
lohan_status_t lohan_model_placement_compact(uint64_t n, uint32_t num_blocks,
                                             lohan_block_offsets_t *offsets, size_t *slab_bytes,
                                             size_t *slab_alignment);

/*
 * The same placement for units of UNEQUAL length -- the gradient tensors of Sec. IV-C's handler
 * (per layer: the attention and MLP matrices of 3h^2, h^2, 4h^2, 4h^2 elements and the h-sized
 * bias / LayerNorm vectors), or the slots of a ring with its spares.  lengths[i] is the element
 * count of unit i; units keep their order.  The rule is lohan_model_placement's: the period P is
 * chosen for the LONGEST fp32 array (4 GiB, else 12 GiB); maximal runs of consecutive units whose
 * fp32 arrays fit one lane together form a group; within a group all p arrays sit back to back
 * in lane 0, the m arrays at the same offsets in lane 1, the v arrays in lane 2 (lane starts as
 * in lohan_model_placement); the 16-bit arrays fill the room left in lanes 0 and 1, first fit,
 * and otherwise follow lane 2.  Arrays of 2 MiB and more start on 1 MiB boundaries, smaller ones on 4 KiB
 * boundaries (so a model's many short vectors cost little).  If the longest fp32 array is below
 * 256 MiB or fits neither period, the units are packed one after the other (p, m, v, g, p16).
 * For equal lengths of 2^26 elements and more the offsets equal lohan_model_placement's.
 *   lengths, offsets   host: count entries each (both may be NULL only if count == 0)
 * LOHAN_ERR_NULL for NULL outputs, LOHAN_ERR_ARG if a length exceeds 2^40.
 */
lohan_status_t lohan_tensor_placement(const uint64_t *lengths, uint32_t count,
                                      lohan_block_offsets_t *offsets, size_t *slab_bytes,
                                      size_t *slab_alignment);

/*
 * Host-only helper for per-block gradient-norm clipping: returns the loss scale to hand to
 * lohan_adam_block_step so that unscaling and clipping are one multiply,
 *     coef = min(1, max_norm / (sqrt(sqnorm) + 1e-6)),   result = (float)(loss_scale / coef),
 * evaluated in float64.  sqnorm is the host copy of lohan_grad_sqnorm's result.  Returns NaN when
 * an argument is out of domain (sqnorm negative or not finite, loss_scale or max_norm not > 0).
 */
float lohan_clip_loss_scale(double sqnorm, float loss_scale, float max_norm);

/* ---------------------------------------------------------------------------------------------
 * Active gradient offloading pipeline (Sec. IV-C, Fig. 3) for model states kept outside HBM.
 *
 * The paper's handler for gradient tensor i has three steps: bring the model states of block i
 * in from the far tier, run the step, push the updated states back; "naive" active gradient
 * offloading serialises them (Fig. 3a), the "optimized" schedule overlaps the transfers of
 * neighbouring blocks with the compute (Fig. 3b).  Here the far tier is PINNED HOST memory and
 * the compute is the block step above, run in place in a device staging slot:
 *     H2D p,m,v (12 B/element)  ->  flag/norm pass + lohan_adam_block_step  ->  D2H p,m,v
 * on three internal streams chained by events.  Gradients and the bf16 copy stay in HBM.
 * With LOHAN_OFFLOAD_OVERLAPPED and >= 3 slots, H2D(i+1), step(i) and D2H(i-1) run concurrently
 * (PCIe is full duplex); LOHAN_OFFLOAD_SERIALIZED reproduces the naive schedule for comparison.
 * A skipped (overflowing) block is copied back bit-identical.
 *
 * The handle owns three streams and 7 events per slot, nothing else: the staging memory
 * (`device_slab`, lohan_offload_slab_bytes() bytes, 256-byte aligned) is the caller's and must
 * outlive the handle.  A handle is bound to the device that was current at creation and is not
 * thread-safe.  Host state arrays must be pinned (hipHostMalloc or equivalent), otherwise the
 * copies are not asynchronous.
 */
typedef struct lohan_offload lohan_offload_t;

enum { LOHAN_OFFLOAD_SERIALIZED = 0, LOHAN_OFFLOAD_OVERLAPPED = 1 };

typedef struct {
    float *host_param_fp32;   /* pinned host, in/out: n floats */
    float *host_exp_avg;      /* pinned host, in/out: n floats */
    float *host_exp_avg_sq;   /* pinned host, in/out: n floats */
    const void *grad_fp16;    /* device, in : n binary16 values, 16-byte aligned */
    void *param_bf16_out;     /* device, out: n bfloat16 values, 16-byte aligned */
    uint64_t n;               /* 1 <= n <= max_block_elems of the handle */
    uint32_t *overflow_flag;  /* device, out: this block's flag (one uint32 per block) */
    double *sqnorm;           /* device, out: this block's squared norm, or NULL (then only the
                                 flag is computed); required when max_norm > 0 */
} lohan_offload_block_t;

/* Bytes of device staging memory a handle with these parameters needs. 0 if num_slots < 1. */
size_t lohan_offload_slab_bytes(uint64_t max_block_elems, int num_slots);

/* num_slots in [1, 16] (3 gives full overlap); mode is LOHAN_OFFLOAD_*.  LOHAN_ERR_WORKSPACE if
 * the slab is too small, LOHAN_ERR_HIP if streams or events cannot be created. */
lohan_status_t lohan_offload_create(lohan_offload_t **handle, void *device_slab,
                                    size_t device_slab_bytes, uint64_t max_block_elems,
                                    int num_slots, int mode);

/*
 * Enqueue stage-in, step and stage-out of one block and return.  The step waits for the work
 * that `producer_stream` (the stream that writes the gradients) holds at the time of the call.
 * Hyper-parameters as lohan_adam_block_step; max_norm > 0 turns on device-side per-block
 * clipping (lohan_adam_block_step_clipped), 0 turns it off; flags: LOHAN_FLAG_L2_MODE and/or
 * LOHAN_FLAG_P16_FP16.
 * The block's host arrays must not be touched until lohan_offload_drain (or a later
 * synchronisation of the caller's own with the copy-out) and *blk itself is read only during
 * the call.  Validation errors enqueue nothing.  If the HIP runtime fails after part of the
 * block's work has been enqueued, LOHAN_ERR_HIP is returned and the handle is POISONED: its slot
 * bookkeeping no longer describes what is in flight, so every later lohan_offload_submit and
 * lohan_offload_wait_last_step returns LOHAN_ERR_HIP without enqueueing anything;
 * lohan_offload_drain and lohan_offload_destroy still work.  The failed block's host arrays are
 * unspecified.
 */
lohan_status_t lohan_offload_submit(lohan_offload_t *handle, const lohan_offload_block_t *blk,
                                    float lr, float beta1, float beta2, float eps,
                                    float weight_decay, int64_t step, float loss_scale,
                                    float max_norm, uint32_t flags, hipStream_t producer_stream);

/* Make `stream` wait (asynchronously) for the step of the most recently submitted block, i.e.
 * until its bf16 copy, flag and norm are valid.  No-op before the first submit. */
lohan_status_t lohan_offload_wait_last_step(lohan_offload_t *handle, hipStream_t stream);

/* Block the host until everything submitted so far, copy-outs included, has completed. */
lohan_status_t lohan_offload_drain(lohan_offload_t *handle);

/* Drain, then release the streams, events and the handle. */
lohan_status_t lohan_offload_destroy(lohan_offload_t *handle);

#ifdef __cplusplus
}
#endif

#endif /* LOHAN_ADAM_H */
