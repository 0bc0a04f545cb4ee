// Active gradient offloading pipeline around the block step, for model states that live outside
// HBM (Sec. IV-C, Fig. 3).  The paper's handler for gradient tensor i is three steps --
// bring the block's model states in, run the step, push the updated states back -- either
// serialised (naive, Fig. 3a) or with the transfers of neighbouring blocks overlapping the compute
// (optimized, Fig. 3b).  Here the far tier is pinned host memory instead of SSDs and the compute
// is the HIP block step in a device staging slot:
//
//     copy-in stream :  H2D p,m,v of block i      -> slot s
//     compute stream :  flag/norm + Adam step in place in slot s   (waits: H2D(i), gradients ready)
//     copy-out stream:  D2H p,m,v of block i      <- slot s        (waits: step(i))
//
// PCIe is full duplex and the copy engines are independent of the CUs, so with >= 3 slots
// H2D(i+1), step(i) and D2H(i-1) all run at once.  Everything is enqueued asynchronously with
// events; nothing here blocks the host except lohan_offload_drain.  The bf16 working copy and the
// gradients stay in HBM (they are produced / consumed by the GPU's forward and backward).

#include <hip/hip_runtime.h>

#include <cstdint>
#include <new>
#include <vector>

#include "lohan_adam.h"
#include "lohan_adam_tuning.h"
#include "lohan_kernels.h"

struct lohan_offload {
    int mode = LOHAN_OFFLOAD_OVERLAPPED;
    int nslots = 0;
    uint64_t max_elems = 0;
    char *slab = nullptr;
    size_t slot_bytes = 0;
    size_t array_bytes = 0;      // one fp32 array of max_elems, padded to 256 B
    hipStream_t s_in = nullptr, s_compute = nullptr, s_out = nullptr;
    std::vector<hipEvent_t> ev_grad, ev_h2d, ev_step, ev_d2h;
    // Begin markers of the three stages of a slot's latest occupant, for the bench-only timing
    // query (lohan_tuning_offload_slot_times); the end markers are the events above.
    std::vector<hipEvent_t> ev_h2d_begin, ev_step_begin, ev_d2h_begin;
    std::vector<bool> used;
    uint64_t submitted = 0;
    int last_slot = -1;
    // Set when a submit failed after part of its work had been enqueued: the slot bookkeeping no
    // longer describes what is in flight, so the handle only drains and dies from then on.
    bool poisoned = false;
    // Fault injection for tests (lohan_tuning_offload_inject_failure): when positive, counts the
    // HIP runtime calls of submits down; the call that brings it to zero is not issued and
    // reports failure instead.
    int fail_countdown = 0;
};

namespace {

inline size_t pad256(size_t x) { return (x + 255) / 256 * 256; }

size_t slot_bytes_for(uint64_t max_elems)
{
    return 3 * pad256((size_t)max_elems * sizeof(float)) + pad256(lohan::kWorkspaceBytes);
}

void destroy_events(std::vector<hipEvent_t> &v)
{
    for (hipEvent_t e : v)
        if (e != nullptr) (void)hipEventDestroy(e);
    v.clear();
}

bool create_events(std::vector<hipEvent_t> &v, int count)
{
    v.assign((size_t)count, nullptr);
    for (int i = 0; i < count; ++i)
        if (hipEventCreateWithFlags(&v[(size_t)i], hipEventDefault) != hipSuccess) return false;
    return true;
}

void release(lohan_offload *h)
{
    if (h == nullptr) return;
    destroy_events(h->ev_grad);
    destroy_events(h->ev_h2d);
    destroy_events(h->ev_step);
    destroy_events(h->ev_d2h);
    destroy_events(h->ev_h2d_begin);
    destroy_events(h->ev_step_begin);
    destroy_events(h->ev_d2h_begin);
    if (h->s_in) (void)hipStreamDestroy(h->s_in);
    if (h->s_compute) (void)hipStreamDestroy(h->s_compute);
    if (h->s_out) (void)hipStreamDestroy(h->s_out);
    delete h;
}

#define LOHAN_HIP_TRY(expr)                      \
    do {                                         \
        if ((expr) != hipSuccess) return LOHAN_ERR_HIP; \
    } while (0)

// Inside lohan_offload_submit, once enqueueing has begun: a failing runtime call (or an injected
// one) poisons the handle before the error is returned.
inline bool injected_failure(lohan_offload *h)
{
    return h->fail_countdown > 0 && --h->fail_countdown == 0;
}
#define LOHAN_SUBMIT_TRY(h, expr)                                \
    do {                                                         \
        if (injected_failure(h) || (expr) != hipSuccess) {       \
            (h)->poisoned = true;                                \
            return LOHAN_ERR_HIP;                                \
        }                                                        \
    } while (0)

}  // namespace

extern "C" {

size_t lohan_offload_slab_bytes(uint64_t max_block_elems, int num_slots)
{
    if (num_slots < 1) return 0;
    return slot_bytes_for(max_block_elems) * (size_t)num_slots;
}

lohan_status_t lohan_offload_create(lohan_offload_t **handle, void *device_slab,
                                    size_t device_slab_bytes, uint64_t max_block_elems,
                                    int num_slots, int mode)
{
    if (handle == nullptr || device_slab == nullptr) return LOHAN_ERR_NULL;
    *handle = nullptr;
    if ((reinterpret_cast<uintptr_t>(device_slab) & 255u) != 0) return LOHAN_ERR_ALIGN;
    if (max_block_elems == 0 || num_slots < 1 || num_slots > 16 ||
        (mode != LOHAN_OFFLOAD_SERIALIZED && mode != LOHAN_OFFLOAD_OVERLAPPED))
        return LOHAN_ERR_ARG;
    if (device_slab_bytes < lohan_offload_slab_bytes(max_block_elems, num_slots))
        return LOHAN_ERR_WORKSPACE;
    lohan_offload *h = new (std::nothrow) lohan_offload();
    if (h == nullptr) return LOHAN_ERR_HIP;
    h->mode = mode;
    h->nslots = num_slots;
    h->max_elems = max_block_elems;
    h->slab = static_cast<char *>(device_slab);
    h->array_bytes = pad256((size_t)max_block_elems * sizeof(float));
    h->slot_bytes = slot_bytes_for(max_block_elems);
    h->used.assign((size_t)num_slots, false);
    // Default-priority, non-blocking streams (they do not synchronise with the legacy stream).
    bool ok = hipStreamCreateWithFlags(&h->s_in, hipStreamNonBlocking) == hipSuccess &&
              hipStreamCreateWithFlags(&h->s_compute, hipStreamNonBlocking) == hipSuccess &&
              hipStreamCreateWithFlags(&h->s_out, hipStreamNonBlocking) == hipSuccess &&
              create_events(h->ev_grad, num_slots) && create_events(h->ev_h2d, num_slots) &&
              create_events(h->ev_step, num_slots) && create_events(h->ev_d2h, num_slots) &&
              create_events(h->ev_h2d_begin, num_slots) &&
              create_events(h->ev_step_begin, num_slots) &&
              create_events(h->ev_d2h_begin, num_slots);
    // Every slot's workspace starts with its ticket counters at zero.
    for (int i = 0; ok && i < num_slots; ++i)
        ok = lohan_workspace_init(h->slab + h->slot_bytes * (size_t)i + 3 * h->array_bytes,
                                  lohan::kWorkspaceBytes, h->s_compute) == LOHAN_OK;
    if (!ok) {
        release(h);
        return LOHAN_ERR_HIP;
    }
    *handle = h;
    return LOHAN_OK;
}

lohan_status_t lohan_offload_submit(lohan_offload_t *h, const lohan_offload_block_t *blk,
                                    float lr, float beta1, float beta2, float eps,
                                    float weight_decay, int64_t step, float loss_scale,
                                    float max_norm, uint32_t flags, hipStream_t producer_stream)
{
    if (h == nullptr || blk == nullptr) return LOHAN_ERR_NULL;
    if (h->poisoned) return LOHAN_ERR_HIP;
    if (blk->host_param_fp32 == nullptr || blk->host_exp_avg == nullptr ||
        blk->host_exp_avg_sq == nullptr || blk->grad_fp16 == nullptr ||
        blk->param_bf16_out == nullptr || blk->overflow_flag == nullptr)
        return LOHAN_ERR_NULL;
    if (blk->n == 0 || blk->n > h->max_elems) return LOHAN_ERR_ARG;
    if ((flags & ~(uint32_t)(LOHAN_FLAG_L2_MODE | LOHAN_FLAG_P16_FP16)) != 0) return LOHAN_ERR_ARG;
    const bool clip = max_norm > 0.0f;
    if (clip && blk->sqnorm == nullptr) return LOHAN_ERR_NULL;
    if (max_norm != max_norm || max_norm < 0.0f) return LOHAN_ERR_ARG;

    const int slot = (int)(h->submitted % (uint64_t)h->nslots);
    const size_t s = (size_t)slot;
    char *base = h->slab + h->slot_bytes * s;
    float *dp = reinterpret_cast<float *>(base);
    float *dm = reinterpret_cast<float *>(base + h->array_bytes);
    float *dv = reinterpret_cast<float *>(base + 2 * h->array_bytes);
    void *ws = base + 3 * h->array_bytes;
    const size_t bytes = (size_t)blk->n * sizeof(float);

    // Validate the step's scalar arguments before anything is enqueued: a zero-length dry call of
    // the step entry point runs exactly its validation and launches nothing.
    lohan_status_t st = lohan_adam_block_step(dp, dm, dv, blk->grad_fp16, blk->param_bf16_out, 0,
                                              lr, beta1, beta2, eps, weight_decay, step,
                                              loss_scale, blk->overflow_flag,
                                              flags | LOHAN_FLAG_PRECHECKED, nullptr, 0,
                                              h->s_compute);
    if (st != LOHAN_OK) return st;

    // Stage in.  The slot is free once the copy-out of its previous occupant has finished; the
    // serialised mode additionally waits for the copy-out of the previous block, so that no two
    // of the three steps ever overlap.
    if (h->used[s]) LOHAN_SUBMIT_TRY(h, hipStreamWaitEvent(h->s_in, h->ev_d2h[s], 0));
    if (h->mode == LOHAN_OFFLOAD_SERIALIZED && h->last_slot >= 0)
        LOHAN_SUBMIT_TRY(h, hipStreamWaitEvent(h->s_in, h->ev_d2h[(size_t)h->last_slot], 0));
    LOHAN_SUBMIT_TRY(h, hipEventRecord(h->ev_h2d_begin[s], h->s_in));
    LOHAN_SUBMIT_TRY(h, hipMemcpyAsync(dp, blk->host_param_fp32, bytes, hipMemcpyHostToDevice,
                                        h->s_in));
    LOHAN_SUBMIT_TRY(h, hipMemcpyAsync(dm, blk->host_exp_avg, bytes, hipMemcpyHostToDevice,
                                        h->s_in));
    LOHAN_SUBMIT_TRY(h, hipMemcpyAsync(dv, blk->host_exp_avg_sq, bytes, hipMemcpyHostToDevice,
                                        h->s_in));
    LOHAN_SUBMIT_TRY(h, hipEventRecord(h->ev_h2d[s], h->s_in));

    // Step: needs the staged states and the gradients the producer stream has enqueued so far.
    LOHAN_SUBMIT_TRY(h, hipEventRecord(h->ev_grad[s], producer_stream));
    LOHAN_SUBMIT_TRY(h, hipStreamWaitEvent(h->s_compute, h->ev_grad[s], 0));
    LOHAN_SUBMIT_TRY(h, hipStreamWaitEvent(h->s_compute, h->ev_h2d[s], 0));
    LOHAN_SUBMIT_TRY(h, hipEventRecord(h->ev_step_begin[s], h->s_compute));
    if (blk->sqnorm != nullptr)
        st = lohan_grad_sqnorm(blk->grad_fp16, blk->n, loss_scale, blk->sqnorm,
                               blk->overflow_flag, ws, lohan::kWorkspaceBytes, h->s_compute);
    else
        st = lohan_grad_overflow_check(blk->grad_fp16, blk->n, blk->overflow_flag, ws,
                                       lohan::kWorkspaceBytes, h->s_compute);
    if (st != LOHAN_OK) {
        h->poisoned = true;
        return st;
    }
    if (clip)
        st = lohan_adam_block_step_clipped(dp, dm, dv, blk->grad_fp16, blk->param_bf16_out,
                                           blk->n, lr, beta1, beta2, eps, weight_decay, step,
                                           loss_scale, blk->sqnorm, max_norm, blk->overflow_flag,
                                           flags, ws, lohan::kWorkspaceBytes, h->s_compute);
    else
        st = lohan_adam_block_step(dp, dm, dv, blk->grad_fp16, blk->param_bf16_out, blk->n, lr,
                                   beta1, beta2, eps, weight_decay, step, loss_scale,
                                   blk->overflow_flag, flags | LOHAN_FLAG_PRECHECKED, nullptr, 0,
                                   h->s_compute);
    if (st != LOHAN_OK) {
        h->poisoned = true;
        return st;
    }
    LOHAN_SUBMIT_TRY(h, hipEventRecord(h->ev_step[s], h->s_compute));

    // Stage out.  A skipped step left the slot untouched, so the copy writes back the same bits.
    LOHAN_SUBMIT_TRY(h, hipStreamWaitEvent(h->s_out, h->ev_step[s], 0));
    LOHAN_SUBMIT_TRY(h, hipEventRecord(h->ev_d2h_begin[s], h->s_out));
    LOHAN_SUBMIT_TRY(h, hipMemcpyAsync(blk->host_param_fp32, dp, bytes, hipMemcpyDeviceToHost,
                                        h->s_out));
    LOHAN_SUBMIT_TRY(h, hipMemcpyAsync(blk->host_exp_avg, dm, bytes, hipMemcpyDeviceToHost,
                                        h->s_out));
    LOHAN_SUBMIT_TRY(h, hipMemcpyAsync(blk->host_exp_avg_sq, dv, bytes, hipMemcpyDeviceToHost,
                                        h->s_out));
    LOHAN_SUBMIT_TRY(h, hipEventRecord(h->ev_d2h[s], h->s_out));

    h->used[s] = true;
    h->last_slot = slot;
    h->submitted += 1;
    return LOHAN_OK;
}

lohan_status_t lohan_offload_wait_last_step(lohan_offload_t *h, hipStream_t stream)
{
    if (h == nullptr) return LOHAN_ERR_NULL;
    if (h->poisoned) return LOHAN_ERR_HIP;
    if (h->last_slot < 0) return LOHAN_OK;
    LOHAN_HIP_TRY(hipStreamWaitEvent(stream, h->ev_step[(size_t)h->last_slot], 0));
    return LOHAN_OK;
}

lohan_status_t lohan_offload_drain(lohan_offload_t *h)
{
    if (h == nullptr) return LOHAN_ERR_NULL;
    LOHAN_HIP_TRY(hipStreamSynchronize(h->s_in));
    LOHAN_HIP_TRY(hipStreamSynchronize(h->s_compute));
    LOHAN_HIP_TRY(hipStreamSynchronize(h->s_out));
    return LOHAN_OK;
}

lohan_status_t lohan_tuning_offload_inject_failure(lohan_offload_t *h, int after_calls)
{
    if (h == nullptr) return LOHAN_ERR_NULL;
    if (after_calls < 0) return LOHAN_ERR_ARG;
    h->fail_countdown = after_calls + 1;
    return LOHAN_OK;
}

lohan_status_t lohan_tuning_offload_slot_times(lohan_offload_t *h, int slot, float *h2d_ms,
                                               float *step_ms, float *d2h_ms)
{
    if (h == nullptr) return LOHAN_ERR_NULL;
    if (slot < 0 || slot >= h->nslots || !h->used[(size_t)slot]) return LOHAN_ERR_ARG;
    const size_t s = (size_t)slot;
    float a = 0.0f, b = 0.0f, c = 0.0f;
    LOHAN_HIP_TRY(hipEventSynchronize(h->ev_d2h[s]));
    LOHAN_HIP_TRY(hipEventElapsedTime(&a, h->ev_h2d_begin[s], h->ev_h2d[s]));
    LOHAN_HIP_TRY(hipEventElapsedTime(&b, h->ev_step_begin[s], h->ev_step[s]));
    LOHAN_HIP_TRY(hipEventElapsedTime(&c, h->ev_d2h_begin[s], h->ev_d2h[s]));
    if (h2d_ms) *h2d_ms = a;
    if (step_ms) *step_ms = b;
    if (d2h_ms) *d2h_ms = c;
    return LOHAN_OK;
}

lohan_status_t lohan_offload_destroy(lohan_offload_t *h)
{
    if (h == nullptr) return LOHAN_ERR_NULL;
    lohan_status_t st = lohan_offload_drain(h);
    release(h);
    return st;
}

}  // extern "C"
