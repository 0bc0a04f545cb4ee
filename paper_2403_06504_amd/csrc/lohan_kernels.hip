// HIP kernels (gfx950 / CDNA4) for the per-block fused mixed-precision Adam step.
//
// The step is the "CPU Compute" box of LoHan's active gradient offloading (Sec. IV-C): update the
// model states of block i (P32 and the two OS32 moments of Table II) from its G16 gradients and
// emit the P16 working copy, here moved from the host into HBM.  It is an elementwise stream of
// 28 bytes per element with ~1 flop/byte, so there is no MFMA anywhere.  What decides the
// bandwidth on MI355X (all measured): every global access of a wavefront is one contiguous run
// (128-bit per lane for the fp32 streams, 64-bit per lane for the two 16-bit streams); the grid is
// one small tile per workgroup, handed out by the hardware dispatcher in address order, so the
// tiles in flight form a compact sliding window; the number of wavefronts resident per CU is
// bounded well below the hardware limit (more bytes in flight make a mixed read/write HBM stream
// slower); and loads and stores carry streaming cache policies.
//
// Arithmetic contract (must match lohan_adam.h): fp32, one rounding per operation, no contraction
// -- this file is compiled with -ffp-contract=off and with correctly rounded fp32 divide / sqrt
// and denormals kept.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lohan_kernels.h"

namespace lohan {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <bool NT, typename T>
__device__ __forceinline__ T ld(const T *ptr)
{
    if constexpr (NT) return __builtin_nontemporal_load(ptr);
    else return *ptr;
}

template <bool NT, typename T>
__device__ __forceinline__ void st(T *ptr, T val)
{
    if constexpr (NT) __builtin_nontemporal_store(val, ptr);
    else *ptr = val;
}

// 16-bit output formats.
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// fp32 -> bfloat16, round to nearest even; gfx950 converts a pair in one instruction
// (v_cvt_pk_bf16_f32).  lo goes to bits [15:0], hi to bits [31:16].  A NaN stays a quiet NaN.
__device__ __forceinline__ uint32_t bf16_pack_rne(float lo, float hi)
{
    f32x2 x = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

// fp32 -> IEEE binary16, round to nearest even (v_cvt_f16_f32 under the default rounding mode),
// overflow to infinity, gradual underflow.  Same packing as bf16_pack_rne.
__device__ __forceinline__ uint32_t half_pack_rne(float lo, float hi)
{
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
    f32x2 x = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, f16x2));
}

template <bool HALF_OUT>
__device__ __forceinline__ uint32_t pack16(float lo, float hi)
{
    if constexpr (HALF_OUT) return half_pack_rne(lo, hi);
    else return bf16_pack_rne(lo, hi);
}

// ------------------------------------------------------------------------------------------------
// Gradient reduction: overflow flag (integer test on the raw fp16 bits) and, optionally, the sum
// of squares, in ONE launch.  Every workgroup publishes one partial and takes a ticket from a
// counter in the workspace; the workgroup that draws the last ticket combines all partials in a
// fixed order (so the result does not depend on scheduling or on which workgroup came last),
// writes the outputs and puts the counter back to zero for the next call.  Nobody waits for
// anybody: a workgroup that is not last simply ends.
// ------------------------------------------------------------------------------------------------

// Both halves of a packed pair at once: (h & 0x7FFF) + 0x0400 carries into bit 15 exactly when
// the exponent field is all ones (h & 0x7FFF >= 0x7C00); no carry crosses the half boundary.
__device__ __forceinline__ uint32_t overflow_bits(uint32_t packed, uint32_t acc)
{
    uint32_t t = (packed & 0x7FFF7FFFu) + 0x04000400u;
    return (t & 0x80008000u) | acc;
}

// A binary16 value has an 11-bit significand, so its square is exact in fp32; the fp32 running
// sum of a few of them is then folded into a float64 accumulator.
__device__ __forceinline__ float square_pair(uint32_t packed, float acc)
{
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
    f16x2 h = __builtin_bit_cast(f16x2, packed);
    float a = (float)h.x, b = (float)h.y;
    acc = __builtin_fmaf(a, a, acc);
    acc = __builtin_fmaf(b, b, acc);
    return acc;
}

template <bool WITH_NORM>
__device__ __forceinline__ void reduce_vec(u32x4 q, uint32_t &ovf, double &acc)
{
    ovf = overflow_bits(q.x, ovf);
    ovf = overflow_bits(q.y, ovf);
    ovf = overflow_bits(q.z, ovf);
    ovf = overflow_bits(q.w, ovf);
    if constexpr (WITH_NORM) {
        float s = 0.0f;
        s = square_pair(q.x, s);
        s = square_pair(q.y, s);
        s = square_pair(q.z, s);
        s = square_pair(q.w, s);
        acc += (double)s;
    }
}

// kReduceThreads-lane workgroups (one wavefront each: measured best with eight 128-bit loads in
// flight per lane and four such workgroups per CU), persistent over interleaved tiles.
constexpr int kReduceThreads = 64;
constexpr int kReduceUnroll = 8;
constexpr int kReduceWaves = kReduceThreads / 64;

// Accesses to the partials and the ticket counter: they are written by one workgroup and read
// by another within the same launch, possibly on another XCD with its own L2.  All of them are
// device-scope atomics, which are performed at the device's point of coherence, so no cache
// that is private to a CU or an XCD is involved and no cache-wide write-back or invalidation is
// needed (a release/acquire fence per workgroup costs exactly that on this chip, and a thousand
// of them at once tripled the duration of the whole reduction).
template <typename T>
__device__ __forceinline__ T ld_device_scope(const T *ptr)
{
    return __hip_atomic_load(ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ void st_device_scope(T *ptr, T val)
{
    __hip_atomic_store(ptr, val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Publish a value and learn that it has been performed: an exchange returns the old value only
// after the new one is in place.
template <typename T>
__device__ __forceinline__ T publish_device_scope(T *ptr, T val)
{
    return __hip_atomic_exchange(ptr, val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Zero, but computed from a and b as far as the compiler can tell: whatever consumes the result
// is issued after the operations that produced a and b have returned.
__device__ __forceinline__ uint32_t zero_after(uint32_t a, uint32_t b)
{
    uint32_t z = 0;
    asm volatile("" : "+v"(z) : "v"(a), "v"(b));
    return z;
}

// Tickets in two levels.  Atomics on one address are performed one after the other, some 12 ns
// apiece, so a thousand workgroups drawing from one counter spend 12 us queueing -- most of what
// a reduction over a small block costs.  Instead, workgroup wg draws from the counter of its
// group of kGroupSize consecutive workgroups (one 128-byte line per group, so that groups do not
// queue behind each other), and only the workgroup that draws a group's last ticket draws from
// the call's top counter.  Returns true in exactly one workgroup of the nwg: the one after which
// nobody else arrives.  dep: a value the first increment must wait for (pass zero_after(...)).
// base: the workspace; line_base: first group line of this block; top: this block's counter.
__device__ __forceinline__ bool take_ticket(uint32_t wg, uint32_t nwg, void *base,
                                            uint32_t line_base, uint32_t *top, uint32_t dep)
{
    if (nwg <= kGroupSize)                                   // one group: the top counter will do
        return __hip_atomic_fetch_add(top, 1u + dep, __ATOMIC_RELAXED,
                                      __HIP_MEMORY_SCOPE_AGENT) == nwg - 1;
    const uint32_t group = wg / kGroupSize;
    const uint32_t ngroups = (nwg + kGroupSize - 1) / kGroupSize;
    const uint32_t rest = nwg - group * kGroupSize;
    const uint32_t members = rest < kGroupSize ? rest : kGroupSize;
    uint32_t *line = reinterpret_cast<uint32_t *>(reinterpret_cast<char *>(base) + kLinesOffset) +
                     (size_t)(line_base + group) * kLineWords;
    if (__hip_atomic_fetch_add(line, 1u + dep, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) !=
        members - 1)
        return false;
    st_device_scope(line, 0u);                               // nobody else comes to this group
    return __hip_atomic_fetch_add(top, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
           ngroups - 1;
}

// Sum / OR over the workgroup: wavefront butterfly over the 64 lanes (fixed pairing), then LDS
// across the wavefronts in index order.  The totals are valid in thread 0.
template <bool WITH_NORM>
__device__ __forceinline__ void workgroup_combine(uint32_t tid, double &acc, uint32_t &any)
{
    any = __builtin_amdgcn_ballot_w64(any != 0) != 0 ? 1u : 0u;
    if constexpr (WITH_NORM) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    }
    if constexpr (kReduceWaves > 1) {
        __shared__ double s_sum[kReduceWaves];
        __shared__ uint32_t s_flag[kReduceWaves];
        const uint32_t wave = tid >> 6, lane = tid & 63u;
        if (lane == 0) {
            s_sum[wave] = acc;
            s_flag[wave] = any;
        }
        __syncthreads();
        if (tid == 0) {
            acc = 0.0;
            any = 0;
#pragma unroll
            for (int w = 0; w < kReduceWaves; ++w) {
                acc += s_sum[w];
                any |= s_flag[w];
            }
        }
        __syncthreads();
    }
}

// Tail of every reducing kernel: combine the workgroup's lanes, publish the workgroup's partial
// as slot `slot_base + wg`, take a ticket, and -- in the workgroup that draws the last of the nwg
// tickets -- combine all partials into sqnorm_out / flag_out (either may be NULL) and put the
// counter back to zero.  All threads of the workgroup must call it.
template <bool WITH_NORM>
__device__ __forceinline__ void reduce_publish_and_finish(uint32_t tid, double acc, uint32_t ovf,
                                                          uint32_t wg, uint32_t nwg,
                                                          uint32_t slot_base, double *partial_sum,
                                                          uint32_t *partial_flag,
                                                          uint32_t *counter, double inv2,
                                                          double *__restrict__ sqnorm_out,
                                                          uint32_t *__restrict__ flag_out)
{
    constexpr int kThreads = kReduceThreads;
    workgroup_combine<WITH_NORM>(tid, acc, ovf);

    // Publish this workgroup's partial, then take a ticket.  The ticket's increment consumes what
    // the publishing exchanges returned, so it is issued only once the partial is in place: whoever
    // draws a later ticket (of the group, and then of the call) finds it.
    __shared__ uint32_t s_is_last;
    if (tid == 0) {
        uint32_t seen = 0;
        if constexpr (WITH_NORM) {
            const double old = publish_device_scope(partial_sum + slot_base + wg, acc);
            seen = (uint32_t)__builtin_bit_cast(uint64_t, old);
        }
        const uint32_t old_flag = publish_device_scope(partial_flag + slot_base + wg, ovf);
        // partial_sum is the workspace's first byte; block b of a multi-block launch (slot_base =
        // b * nwg) has the b-th run of group lines.
        const uint32_t groups_per_block = (nwg + kGroupSize - 1) / kGroupSize;
        const bool last = take_ticket(wg, nwg, partial_sum, slot_base / nwg * groups_per_block,
                                      counter, zero_after(seen, old_flag));
        s_is_last = last ? 1u : 0u;
    }
    __syncthreads();
    if (s_is_last == 0u) return;

    // Last arrival: every partial has been published.  Combine them in a fixed order (lane l takes
    // partials l, l + kThreads, ... in turn; then the same butterfly as above).
    // The loads of a round are all issued before the first is used: they miss every cache by
    // design, so one round costs one trip to memory instead of kFinalBatch of them.
    constexpr uint32_t kFinalBatch = 16;
    double total = 0.0;
    uint32_t any = 0;
    for (uint32_t first = 0; first < nwg; first += kFinalBatch * kThreads) {
        double part[kFinalBatch];
        uint32_t bits[kFinalBatch];
#pragma unroll
        for (uint32_t j = 0; j < kFinalBatch; ++j) {
            const uint32_t i = first + j * kThreads + tid;
            part[j] = 0.0;
            bits[j] = 0u;
            if (i < nwg) {
                if constexpr (WITH_NORM) part[j] = ld_device_scope(partial_sum + slot_base + i);
                bits[j] = ld_device_scope(partial_flag + slot_base + i);
            }
        }
#pragma unroll
        for (uint32_t j = 0; j < kFinalBatch; ++j) {
            if constexpr (WITH_NORM) total += part[j];     // + 0.0 past the end: no change
            any |= bits[j];
        }
    }
    workgroup_combine<WITH_NORM>(tid, total, any);
    if (tid == 0) {
        if constexpr (WITH_NORM) {
            if (sqnorm_out != nullptr) *sqnorm_out = total * inv2;
        }
        if (flag_out != nullptr) *flag_out = any;
        st_device_scope(counter, 0u);                       // ready for the next call
    }
}

// Workgroup `wg` of `nwg` reduces its interleaved share of g[0, n), publishes partial
// `slot_base + wg`, and -- if it is the last of the nwg to do so -- combines the nwg partials
// into sqnorm_out / flag_out (either may be NULL).  NT: stream the gradients past the caches
// (blocks far larger than the memory-side cache) or leave them cached for the update that
// follows (blocks that fit it).  inv2 = (1/loss_scale)^2 in float64 turns the raw sum of squares
// into the squared norm of the unscaled gradients.
template <bool WITH_NORM, int UNROLL, bool NT>
__device__ __forceinline__ void grad_reduce_body(const uint16_t *__restrict__ g, uint64_t n,
                                                 uint32_t wg, uint32_t nwg, uint32_t slot_base,
                                                 double *partial_sum, uint32_t *partial_flag,
                                                 uint32_t *counter, double inv2,
                                                 double *__restrict__ sqnorm_out,
                                                 uint32_t *__restrict__ flag_out)
{
    constexpr int kThreads = kReduceThreads;
    constexpr uint64_t kVec = 8;                               // halves per 128-bit load
    constexpr uint64_t kTile = (uint64_t)kThreads * kVec * UNROLL;
    const uint32_t tid = threadIdx.x;
    const uint64_t ntiles = n / kTile;

    uint32_t ovf = 0;
    double acc = 0.0;

    for (uint64_t tile = wg; tile < ntiles; tile += nwg) {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(g + tile * kTile) + tid;
        u32x4 q[UNROLL];
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) q[j] = ld<NT>(src + j * kThreads);
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) reduce_vec<WITH_NORM>(q[j], ovf, acc);
    }

    // Ragged end: whole 8-element vectors first, then up to 7 single elements.
    const uint64_t rem_start = ntiles * kTile;
    const uint64_t rem_vecs = (n - rem_start) / kVec;
    for (uint64_t i = (uint64_t)wg * kThreads + tid; i < rem_vecs; i += (uint64_t)nwg * kThreads) {
        u32x4 q = *(reinterpret_cast<const u32x4 *>(g + rem_start) + i);
        reduce_vec<WITH_NORM>(q, ovf, acc);
    }
    const uint64_t tail_start = rem_start + rem_vecs * kVec;
    if (wg == 0 && tail_start + tid < n) {
        uint32_t h = g[tail_start + tid];
        ovf = overflow_bits(h, ovf);
        if constexpr (WITH_NORM) acc += (double)square_pair(h, 0.0f);
    }

    reduce_publish_and_finish<WITH_NORM>(tid, acc, ovf, wg, nwg, slot_base, partial_sum,
                                         partial_flag, counter, inv2, sqnorm_out, flag_out);
}

// A workspace that was never prepared (lohan_workspace_init) may hold anything in its ticket
// counters, and then no workgroup would ever recognise itself as the last one.  Every reducing
// kernel therefore looks at the workspace's magic word first; without it, it reduces nothing
// and reports the block as overflowing (flag 1, norm NaN), which makes the step skip: wrong use
// fails on the safe side and visibly, not with a stale flag.
__device__ __forceinline__ bool workspace_unprepared(const uint64_t *__restrict__ magic,
                                                     double *__restrict__ sqnorm_out,
                                                     uint32_t *__restrict__ flag_out)
{
    if (*magic == kWorkspaceMagic) return false;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (sqnorm_out != nullptr) *sqnorm_out = __builtin_nan("");
        if (flag_out != nullptr) *flag_out = 1u;
    }
    return true;
}

template <bool WITH_NORM, int UNROLL, bool NT>
__global__ __launch_bounds__(kReduceThreads) void k_grad_reduce(const uint16_t *__restrict__ g,
                                                                uint64_t n, double *partial_sum,
                                                                uint32_t *partial_flag,
                                                                uint32_t *counter,
                                                                const uint64_t *__restrict__ magic,
                                                                double inv2,
                                                                double *__restrict__ sqnorm,
                                                                uint32_t *__restrict__ flag)
{
    if (workspace_unprepared(magic, sqnorm, flag)) return;
    grad_reduce_body<WITH_NORM, UNROLL, NT>(g, n, blockIdx.x, gridDim.x, 0u, partial_sum,
                                            partial_flag, counter, inv2, sqnorm, flag);
}

// Several blocks in one launch: grid (workgroups per block, blocks); block b's partials occupy
// slots [b * gridDim.x, (b + 1) * gridDim.x), its ticket counter is counters[b] and its results go
// to sqnorms[b] and flags[b].
template <bool WITH_NORM, int UNROLL, bool NT>
__global__ __launch_bounds__(kReduceThreads) void k_multi_grad_reduce(
    MultiArgs args, double *partial_sum, uint32_t *partial_flag, uint32_t *counters,
    const uint64_t *__restrict__ magic, double inv2, double *__restrict__ sqnorms,
    uint32_t *__restrict__ flags)
{
    const uint32_t b = blockIdx.y;
    if (workspace_unprepared(magic, sqnorms != nullptr ? sqnorms + b : nullptr,
                             flags != nullptr ? flags + b : nullptr))
        return;
    grad_reduce_body<WITH_NORM, UNROLL, NT>(args.d[b].g, args.d[b].n, blockIdx.x, gridDim.x,
                                            b * gridDim.x, partial_sum, partial_flag, counters + b,
                                            inv2, sqnorms != nullptr ? sqnorms + b : nullptr,
                                            flags != nullptr ? flags + b : nullptr);
}

// A gradient producer with the block's flag and norm computed in its epilogue: fp32 gradients
// (accumulated over micro-batches, still multiplied by the loss scale) are scaled by `mul`,
// rounded to binary16 -- the G16 tensor that the block step consumes -- and the overflow flag and
// squared norm of exactly the values written are reduced on the way, so that the step needs no
// separate 2 B/element pass over G16.  A value too large for binary16 becomes +-inf here, which
// is how fp16 gradients overflow in the first place.  Persistent over interleaved tiles of
// 64 lanes x 4 elements x UNROLL rows; the finish is the reduction's.
template <bool WITH_NORM, int UNROLL, bool NT>
__global__ __launch_bounds__(kReduceThreads) void k_grad_produce(
    const float *__restrict__ src, uint64_t n, float mul, uint16_t *__restrict__ out,
    double *partial_sum, uint32_t *partial_flag, uint32_t *counter,
    const uint64_t *__restrict__ magic, double inv2, double *__restrict__ sqnorm_out,
    uint32_t *__restrict__ flag_out)
{
    if (workspace_unprepared(magic, sqnorm_out, flag_out)) return;
    constexpr uint64_t kVec = 4;
    constexpr uint64_t kRow = (uint64_t)kReduceThreads * kVec;
    constexpr uint64_t kTile = kRow * UNROLL;
    const uint32_t tid = threadIdx.x, wg = blockIdx.x, nwg = gridDim.x;
    const uint64_t ntiles = n / kTile;
    uint32_t ovf = 0;
    double acc = 0.0;

    auto emit = [&](f32x4 x) {
        const uint32_t lo = half_pack_rne(x[0] * mul, x[1] * mul);
        const uint32_t hi = half_pack_rne(x[2] * mul, x[3] * mul);
        ovf = overflow_bits(lo, ovf);
        ovf = overflow_bits(hi, ovf);
        if constexpr (WITH_NORM) acc += (double)square_pair(hi, square_pair(lo, 0.0f));
        return u32x2{lo, hi};
    };

    for (uint64_t tile = wg; tile < ntiles; tile += nwg) {
        const uint64_t base = tile * kTile + (uint64_t)tid * kVec;
        f32x4 x[UNROLL];
#pragma unroll
        for (int j = 0; j < UNROLL; ++j)
            x[j] = ld<NT>(reinterpret_cast<const f32x4 *>(src + base + j * kRow));
#pragma unroll
        for (int j = 0; j < UNROLL; ++j)
            st<NT>(reinterpret_cast<u32x2 *>(out + base + j * kRow), emit(x[j]));
    }
    // Ragged end: whole 4-element vectors spread over the grid, then up to 3 single elements.
    const uint64_t rem_start = ntiles * kTile;
    const uint64_t rem_vecs = (n - rem_start) / kVec;
    for (uint64_t i = (uint64_t)wg * kReduceThreads + tid; i < rem_vecs;
         i += (uint64_t)nwg * kReduceThreads) {
        const uint64_t off = rem_start + i * kVec;
        const f32x4 x = *reinterpret_cast<const f32x4 *>(src + off);
        *reinterpret_cast<u32x2 *>(out + off) = emit(x);
    }
    const uint64_t tail = rem_start + rem_vecs * kVec + tid;
    if (wg == 0 && tail < n) {
        const uint32_t h = half_pack_rne(src[tail] * mul, 0.0f) & 0xFFFFu;
        out[tail] = (uint16_t)h;
        ovf = overflow_bits(h, ovf);
        if constexpr (WITH_NORM) acc += (double)square_pair(h, 0.0f);
    }
    reduce_publish_and_finish<WITH_NORM>(tid, acc, ovf, wg, nwg, 0u, partial_sum, partial_flag,
                                         counter, inv2, sqnorm_out, flag_out);
}

// Ticket counters (per block and per group) start at zero; afterwards every call leaves them at
// zero.  The magic word marks the workspace as prepared.
__global__ void k_workspace_init(uint32_t *counters, uint32_t count, uint32_t *lines,
                                 uint32_t line_words, uint64_t *magic)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) counters[i] = 0u;
    if (i < line_words) lines[i] = 0u;
    if (i == 0) *magic = kWorkspaceMagic;
}

// n == 0: nothing to reduce, but the outputs are still defined.
__global__ void k_grad_empty(double *sqnorm, uint32_t *flag)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        if (sqnorm != nullptr) *sqnorm = 0.0;
        if (flag != nullptr) *flag = 0u;
    }
}

// ------------------------------------------------------------------------------------------------
// The 28 B/element stream.
// ------------------------------------------------------------------------------------------------

template <bool L2>
__device__ __forceinline__ void adam_elem(float &p, float &m, float &v, float g_scaled,
                                          const StepScalars &s)
{
    float g = g_scaled * s.inv;
    if constexpr (L2) {
        float wp = s.wd * p;
        g = g + wp;
    }
    float b1m = s.beta1 * m;
    float o1g = s.omb1 * g;
    float m_new = b1m + o1g;
    float gg = g * g;
    float b2v = s.beta2 * v;
    float o2gg = s.omb2 * gg;
    float v_new = b2v + o2gg;
    float root = __builtin_sqrtf(v_new);
    float root_hat = root / s.sbc2;
    float den = root_hat + s.eps;
    float u = m_new / den;
    float pp = L2 ? p : p * s.decay;
    float su = s.ss * u;
    float p_new = pp - su;
    p = p_new;
    m = m_new;
    v = v_new;
}

template <bool L2, bool HALF_OUT>
__device__ __forceinline__ void adam_vec4(f32x4 &p, f32x4 &m, f32x4 &v, f16x4 g,
                                          const StepScalars &s, u32x2 &out16)
{
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float pe = p[k], me = m[k], ve = v[k];
        adam_elem<L2>(pe, me, ve, (float)g[k], s);
        p[k] = pe;
        m[k] = me;
        v[k] = ve;
    }
    out16.x = pack16<HALF_OUT>(p[0], p[1]);
    out16.y = pack16<HALF_OUT>(p[2], p[3]);
}

// Streaming stores with the write-through-to-memory cache policy (sc0 sc1 nt).  The compiler has
// no builtin for this policy on 128-bit vectors, hence the two one-instruction asm wrappers; they
// are ordinary vector stores.  They are issued after all arithmetic of a tile, so that no later
// load of the same wavefront has to wait behind them.  The trailing s_nop covers the two wait
// states gfx940-class hardware needs between a store of more than 64 bits and a VALU write to
// the registers that held its data (the compiler cannot see into the asm to insert them).
__device__ __forceinline__ void st_through(f32x4 *ptr, f32x4 val)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_nop 1" ::"v"(ptr), "v"(val)
                 : "memory");
}
__device__ __forceinline__ void st_through(u32x2 *ptr, u32x2 val)
{
    asm volatile("global_store_dwordx2 %0, %1, off sc0 sc1 nt\n\ts_nop 1" ::"v"(ptr), "v"(val)
                 : "memory");
}

// POLICY: 0 = default cache policy, 1 = nontemporal loads and stores, 2 = nontemporal loads and
// write-through streaming stores.  Nothing is re-read, so nothing should linger in L2 or in the
// memory-side cache.
template <int POLICY, typename T>
__device__ __forceinline__ T ld_stream(const T *ptr)
{
    return ld<(POLICY != 0)>(ptr);
}
template <int POLICY, typename T>
__device__ __forceinline__ void st_stream(T *ptr, T val)
{
    if constexpr (POLICY == 2) st_through(ptr, val);
    else st<(POLICY == 1)>(ptr, val);
}

// One workgroup handles tiles of WG * 4 * UNROLL elements; within a tile every global access of a
// wavefront is one contiguous run (lane l touches elements 4l..4l+3 of its wavefront's row).
// The grid is normally one tile per workgroup, so that the set of tiles in flight is a compact
// window sliding through the buffers in address order (measured: this keeps HBM far busier than
// a persistent grid-stride loop whose workgroups drift apart); the loop only runs more than once
// when the host caps the grid.
// MODE bits: 1 = L2 regularisation instead of decoupled decay, 2 = emit the 16-bit copy as IEEE
// binary16 instead of bfloat16.
template <int WG, int UNROLL, int POLICY, int MODE>
__device__ __forceinline__ void adam_block_body(float *__restrict__ p, float *__restrict__ m,
                                                float *__restrict__ v,
                                                const uint16_t *__restrict__ g,
                                                uint16_t *__restrict__ p16, uint64_t n,
                                                const StepScalars &s)
{
    constexpr bool L2 = (MODE & 1) != 0, HALF_OUT = (MODE & 2) != 0;
    constexpr uint64_t kVec = 4;                                  // elements per lane per access
    constexpr uint64_t kRow = (uint64_t)WG * kVec;                // elements per wg-wide access
    constexpr uint64_t kTile = kRow * UNROLL;
    const uint32_t tid = threadIdx.x;
    const uint64_t ntiles = n / kTile;

    for (uint64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const uint64_t base = tile * kTile + (uint64_t)tid * kVec;
        f16x4 gv[UNROLL];
        f32x4 pv[UNROLL], mv[UNROLL], vv[UNROLL];
        u32x2 hv[UNROLL];
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) {
            const uint64_t off = base + j * kRow;
            gv[j] = ld_stream<POLICY>(reinterpret_cast<const f16x4 *>(g + off));
            pv[j] = ld_stream<POLICY>(reinterpret_cast<const f32x4 *>(p + off));
            mv[j] = ld_stream<POLICY>(reinterpret_cast<const f32x4 *>(m + off));
            vv[j] = ld_stream<POLICY>(reinterpret_cast<const f32x4 *>(v + off));
        }
#pragma unroll
        for (int j = 0; j < UNROLL; ++j)
            adam_vec4<L2, HALF_OUT>(pv[j], mv[j], vv[j], gv[j], s, hv[j]);
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) {
            const uint64_t off = base + j * kRow;
            st_stream<POLICY>(reinterpret_cast<f32x4 *>(p + off), pv[j]);
            st_stream<POLICY>(reinterpret_cast<f32x4 *>(m + off), mv[j]);
            st_stream<POLICY>(reinterpret_cast<f32x4 *>(v + off), vv[j]);
            st_stream<POLICY>(reinterpret_cast<u32x2 *>(p16 + off), hv[j]);
        }
    }

    // Ragged end (fewer than kTile elements): whole 4-element vectors spread over the grid, then
    // up to 3 single elements in workgroup 0.
    const uint64_t rem_start = ntiles * kTile;
    const uint64_t rem_vecs = (n - rem_start) / kVec;
    for (uint64_t i = (uint64_t)blockIdx.x * WG + tid; i < rem_vecs;
         i += (uint64_t)gridDim.x * WG) {
        const uint64_t off = rem_start + i * kVec;
        f16x4 gq = *reinterpret_cast<const f16x4 *>(g + off);
        f32x4 pq = *reinterpret_cast<const f32x4 *>(p + off);
        f32x4 mq = *reinterpret_cast<const f32x4 *>(m + off);
        f32x4 vq = *reinterpret_cast<const f32x4 *>(v + off);
        u32x2 h;
        adam_vec4<L2, HALF_OUT>(pq, mq, vq, gq, s, h);
        *reinterpret_cast<f32x4 *>(p + off) = pq;
        *reinterpret_cast<f32x4 *>(m + off) = mq;
        *reinterpret_cast<f32x4 *>(v + off) = vq;
        *reinterpret_cast<u32x2 *>(p16 + off) = h;
    }
    const uint64_t tail = rem_start + rem_vecs * kVec + tid;
    if (blockIdx.x == 0 && tail < n) {
        _Float16 gh = __builtin_bit_cast(_Float16, g[tail]);
        float pe = p[tail], me = m[tail], ve = v[tail];
        adam_elem<L2>(pe, me, ve, (float)gh, s);
        p[tail] = pe;
        m[tail] = me;
        v[tail] = ve;
        p16[tail] = (uint16_t)pack16<HALF_OUT>(pe, 0.0f);
    }
}

template <int WG, int UNROLL, int POLICY, int MODE>
__global__ __launch_bounds__(WG) void k_adam_block_step(float *__restrict__ p,
                                                        float *__restrict__ m,
                                                        float *__restrict__ v,
                                                        const uint16_t *__restrict__ g,
                                                        uint16_t *__restrict__ p16, uint64_t n,
                                                        StepScalars s,
                                                        const uint32_t *__restrict__ flag,
                                                        const float *__restrict__ inv_override)
{
    // Skip rule: a set overflow flag means nothing at all is written by this kernel.
    if (*flag != 0u) return;
    // Device-side clipping: the unscale factor then comes from k_clip_scale's output.
    if (inv_override != nullptr) s.inv = *inv_override;
    adam_block_body<WG, UNROLL, POLICY, MODE>(p, m, v, g, p16, n, s);
}

// Several blocks in one launch: grid (tiles of the largest block, blocks).  blockIdx.y selects
// the block's descriptor from the kernel arguments; the hardware hands out workgroups with x
// fastest, so the tiles in flight still form a compact window that moves through one block
// after the other.  Each block has its own flag and, when clipping, its own unscale factor.
template <int WG, int UNROLL, int POLICY, int MODE>
__global__ __launch_bounds__(WG) void k_adam_multi_block_step(MultiArgs args, StepScalars s,
                                                              const uint32_t *__restrict__ flags,
                                                              const float *__restrict__ inv_override)
{
    const uint32_t b = blockIdx.y;
    const uint64_t n = args.d[b].n;
    constexpr uint64_t kTile = (uint64_t)WG * 4 * UNROLL;
    // Workgroups beyond this block's tiles have nothing to do, except that the ragged end (fewer
    // than UNROLL * WG vectors) is spread over the first UNROLL workgroups.
    if (blockIdx.x >= UNROLL && (uint64_t)blockIdx.x * kTile >= n) return;
    if (flags[b] != 0u) return;
    if (inv_override != nullptr) s.inv = inv_override[b];
    adam_block_body<WG, UNROLL, POLICY, MODE>(args.d[b].p, args.d[b].m, args.d[b].v, args.d[b].g,
                                              args.d[b].p16, n, s);
}

// Out-of-place form with the overflow test fused in: one pass of 28 B/element instead of the
// 2 B/element flag pass followed by the in-place step.  The inputs are only read, so a block
// whose gradients turn out to hold inf/NaN loses nothing: the kernel raises *flag (cleared by a
// one-lane kernel ahead of it) and the caller discards the outputs.  Each wavefront tests the
// gradient bits it has loaded anyway; only a wavefront that found a non-finite value touches
// *flag, with a plain vector store of 1.
template <int WG, int UNROLL, int POLICY, int MODE>
__device__ __forceinline__ void adam_oop_body(
    const float *__restrict__ pi, const float *__restrict__ mi, const float *__restrict__ vi,
    const uint16_t *__restrict__ g, float *__restrict__ po, float *__restrict__ mo,
    float *__restrict__ vo, uint16_t *__restrict__ p16, uint64_t n, const StepScalars &s,
    uint32_t &ovf)
{
    constexpr bool L2 = (MODE & 1) != 0, HALF_OUT = (MODE & 2) != 0;
    constexpr uint64_t kVec = 4;
    constexpr uint64_t kRow = (uint64_t)WG * kVec;
    constexpr uint64_t kTile = kRow * UNROLL;
    const uint32_t tid = threadIdx.x;
    const uint64_t ntiles = n / kTile;

    for (uint64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const uint64_t base = tile * kTile + (uint64_t)tid * kVec;
        f16x4 gv[UNROLL];
        f32x4 pv[UNROLL], mv[UNROLL], vv[UNROLL];
        u32x2 hv[UNROLL];
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) {
            const uint64_t off = base + j * kRow;
            gv[j] = ld_stream<POLICY>(reinterpret_cast<const f16x4 *>(g + off));
            pv[j] = ld_stream<POLICY>(reinterpret_cast<const f32x4 *>(pi + off));
            mv[j] = ld_stream<POLICY>(reinterpret_cast<const f32x4 *>(mi + off));
            vv[j] = ld_stream<POLICY>(reinterpret_cast<const f32x4 *>(vi + off));
        }
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) {
            const u32x2 bits = __builtin_bit_cast(u32x2, gv[j]);
            ovf = overflow_bits(bits.x, ovf);
            ovf = overflow_bits(bits.y, ovf);
            adam_vec4<L2, HALF_OUT>(pv[j], mv[j], vv[j], gv[j], s, hv[j]);
        }
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) {
            const uint64_t off = base + j * kRow;
            st_stream<POLICY>(reinterpret_cast<f32x4 *>(po + off), pv[j]);
            st_stream<POLICY>(reinterpret_cast<f32x4 *>(mo + off), mv[j]);
            st_stream<POLICY>(reinterpret_cast<f32x4 *>(vo + off), vv[j]);
            st_stream<POLICY>(reinterpret_cast<u32x2 *>(p16 + off), hv[j]);
        }
    }

    const uint64_t rem_start = ntiles * kTile;
    const uint64_t rem_vecs = (n - rem_start) / kVec;
    for (uint64_t i = (uint64_t)blockIdx.x * WG + tid; i < rem_vecs;
         i += (uint64_t)gridDim.x * WG) {
        const uint64_t off = rem_start + i * kVec;
        f16x4 gq = *reinterpret_cast<const f16x4 *>(g + off);
        f32x4 pq = *reinterpret_cast<const f32x4 *>(pi + off);
        f32x4 mq = *reinterpret_cast<const f32x4 *>(mi + off);
        f32x4 vq = *reinterpret_cast<const f32x4 *>(vi + off);
        const u32x2 bits = __builtin_bit_cast(u32x2, gq);
        ovf = overflow_bits(bits.x, ovf);
        ovf = overflow_bits(bits.y, ovf);
        u32x2 h;
        adam_vec4<L2, HALF_OUT>(pq, mq, vq, gq, s, h);
        *reinterpret_cast<f32x4 *>(po + off) = pq;
        *reinterpret_cast<f32x4 *>(mo + off) = mq;
        *reinterpret_cast<f32x4 *>(vo + off) = vq;
        *reinterpret_cast<u32x2 *>(p16 + off) = h;
    }
    const uint64_t tail = rem_start + rem_vecs * kVec + tid;
    if (blockIdx.x == 0 && tail < n) {
        const uint32_t gbits = g[tail];
        ovf = overflow_bits(gbits, ovf);
        _Float16 gh = __builtin_bit_cast(_Float16, (uint16_t)gbits);
        float pe = pi[tail], me = mi[tail], ve = vi[tail];
        adam_elem<L2>(pe, me, ve, (float)gh, s);
        po[tail] = pe;
        mo[tail] = me;
        vo[tail] = ve;
        p16[tail] = (uint16_t)pack16<HALF_OUT>(pe, 0.0f);
    }
}

template <int WG, int UNROLL, int POLICY, int MODE>
__global__ __launch_bounds__(WG) void k_adam_block_step_oop(
    const float *__restrict__ pi, const float *__restrict__ mi, const float *__restrict__ vi,
    const uint16_t *__restrict__ g, float *__restrict__ po, float *__restrict__ mo,
    float *__restrict__ vo, uint16_t *__restrict__ p16, uint64_t n, StepScalars s,
    uint32_t *__restrict__ flag, const float *__restrict__ inv_override)
{
    // Device-side clipping: the unscale factor then comes from k_clip_scale's output.
    if (inv_override != nullptr) s.inv = *inv_override;
    uint32_t ovf = 0;
    adam_oop_body<WG, UNROLL, POLICY, MODE>(pi, mi, vi, g, po, mo, vo, p16, n, s, ovf);
    // Raising the flag is a plain store: the flag was cleared ahead of this launch and every
    // writer writes the same 1, so nothing needs to be atomic -- and a block whose gradients are
    // mostly non-finite (the usual way to overflow) would otherwise queue a million atomics on
    // one address, 12 ns apiece (measured: 12.9 ms instead of 1.3 ms).
    if (__builtin_amdgcn_ballot_w64(ovf != 0) != 0 && (threadIdx.x & 63u) == 0) *flag = 1u;
}

// Ring form of the out-of-place step: the blocks (or single tensors) of a model live in slots
// (each slot holds p, m, v and the 16-bit copy of one block), plus one spare slot per distinct
// length ("class").  The step of block b reads the slot that holds b and writes the spare of b's
// class; k_ring_commit then makes that spare b's slot and b's old slot the class's spare --
// unless the gradients overflowed, in which case nothing changes.  Which slot holds which block
// is a table in device memory, so no host decision (and no host synchronisation) sits between
// the blocks of a backward pass.  Every block counts its attempts (steps enqueued so far); an
// overflowing step records its attempt number (attempt numbers only grow, so the record needs no
// clearing) and so tells "the latest attempt overflowed" from any older one.  A step whose n is
// not the length the block was registered with touches nothing and is recorded like an overflow.
template <int WG, int UNROLL, int POLICY, int MODE>
__global__ __launch_bounds__(WG) void k_adam_ring_step(
    const RingSlot *__restrict__ slots, const uint32_t *__restrict__ slot_of,
    const uint32_t *__restrict__ class_of, const uint32_t *__restrict__ spare_of_class,
    const unsigned long long *__restrict__ attempts,
    unsigned long long *__restrict__ overflow_attempt, uint32_t block,
    const uint16_t *__restrict__ g, uint64_t n, StepScalars s,
    const float *__restrict__ inv_override)
{
    const RingSlot in = slots[slot_of[block]];
    const RingSlot out = slots[spare_of_class[class_of[block]]];
    const unsigned long long attempt = attempts[block] + 1;
    if (in.n != n || out.n != n) {
        if (blockIdx.x == 0 && threadIdx.x == 0) atomicMax(overflow_attempt + block, attempt);
        return;
    }
    if (inv_override != nullptr) s.inv = *inv_override;
    uint32_t ovf = 0;
    adam_oop_body<WG, UNROLL, POLICY, MODE>(in.p, in.m, in.v, g, out.p, out.m, out.v, out.p16, n,
                                            s, ovf);
    // A plain store, as in k_adam_block_step_oop: every writer of this launch writes the same
    // attempt number, and the steps of one block are ordered, so older values are smaller.
    if (__builtin_amdgcn_ballot_w64(ovf != 0) != 0 && (threadIdx.x & 63u) == 0)
        overflow_attempt[block] = attempt;
}

__global__ void k_ring_commit(uint32_t *__restrict__ slot_of,
                              const uint32_t *__restrict__ class_of,
                              uint32_t *__restrict__ spare_of_class,
                              unsigned long long *__restrict__ attempts,
                              const unsigned long long *__restrict__ overflow_attempt,
                              uint32_t block)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const unsigned long long attempt = attempts[block] + 1;
    attempts[block] = attempt;
    if (overflow_attempt[block] == attempt) return;    // skipped: the inputs stay the state
    const uint32_t cls = class_of[block];
    const uint32_t old_slot = slot_of[block];
    slot_of[block] = spare_of_class[cls];
    spare_of_class[cls] = old_slot;
}

// Per-block norm clipping without a host round trip: from the squared norm that
// lohan_grad_sqnorm left in device memory, compute the unscale factor of the clipped step,
//     coef = min(1, max_norm / (sqrt(sqnorm) + 1e-6)),  S_eff = fp32(S / coef),  inv = fl(1 / S_eff),
// in float64 until the two roundings shown -- the same formula as lohan_clip_loss_scale on the
// host.  One lane per block; the result is read by every wavefront of the following update.
__global__ void k_clip_scale(const double *__restrict__ sqnorm, float loss_scale, float max_norm,
                             float *__restrict__ inv_out, uint32_t count)
{
    const uint32_t b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= count) return;
    const double norm = __builtin_sqrt(sqnorm[b]);
    double coef = (double)max_norm / (norm + 1e-6);
    if (coef > 1.0) coef = 1.0;
    const float s_eff = (float)((double)loss_scale / coef);
    inv_out[b] = 1.0f / s_eff;
}

// ------------------------------------------------------------------------------------------------
// Small blocks: flag, norm and update in ONE launch, the block's state held in registers.
//
// For a block of a few million elements the two-launch step is a chain of latencies (a reduction
// of dependent round trips, a launch gap, then 27 thousand one-tile workgroups).  Here the whole
// grid is resident at once.  Every workgroup loads its share of the gradients (K tiles), reduces
// them and arrives at a grid-wide barrier; then it loads its share of p, m, v into registers --
// every load issued before anything is consumed -- and computes the update in registers while
// the barrier completes; then it learns the verdict and stores.  Bytes moved: the 28 per element
// of the update alone, and the chip's reads and writes separate into two phases.
//
// The barrier is the two-level ticket above with the overflow flag folded in: the low half of a
// counter counts arrivals, the high half counts arrivals that saw an overflow, so the one atomic
// a workgroup issues to arrive is also its contribution to the flag.  The workgroup that arrives
// last writes the verdict into every group's line, tagged with the number of this call; the
// others poll their own group's line (32 pollers per address instead of a thousand).  Tags make
// resetting unnecessary: a line left over from an earlier call never matches.
//
// The wait is bounded: a workgroup that does not see the verdict within spin_limit polls marks
// the call as incomplete, looks once more, and otherwise ends without writing; the workgroup
// that arrives last reads that mark after publishing the verdict and reports it in the flag
// (kFlagIncomplete).  Mark-then-look on one side and publish-then-read on the other mean that a
// workgroup which ends without writing is always reported.  Every wavefront exits whatever
// happens.  The host sizes the grid to what the device holds at once, so the wait is over before
// the update has been computed unless other kernels occupy the compute units; those finish by
// themselves.
// ------------------------------------------------------------------------------------------------

constexpr int kFusedThreads = 256;
constexpr int kFusedWaves = kFusedThreads / 64;
constexpr uint64_t kFusedTile = (uint64_t)kFusedThreads * 4;
constexpr uint32_t kArrivedMask = 0xFFFFu;
constexpr uint32_t kOverflowUnit = 0x10000u;
constexpr uint32_t kLastTag = 0x7FFFFFFEu;
static_assert(kMaxPartials <= kArrivedMask, "the arrival count must fit the counter's low half");

// Workgroup barrier that orders LDS traffic only: the global loads in flight stay in flight.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Sum over the workgroup in a fixed order (butterfly within each wavefront, then the wavefronts
// in index order); every lane gets the total.  area: kFusedWaves doubles of LDS, not reused
// before the next barrier.
__device__ __forceinline__ double fused_workgroup_sum(uint32_t tid, double acc, double *area)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if ((tid & 63u) == 0u) area[tid >> 6] = acc;
    lds_barrier();
    double total = 0.0;
#pragma unroll
    for (int w = 0; w < kFusedWaves; ++w) total += area[w];
    return total;
}

// The elements past the last whole tile (fewer than kFusedTile): lane `tid` takes elements
// tail_start + tid, + kFusedThreads, ... one at a time.
__device__ __forceinline__ void fused_tail_reduce(const uint16_t *__restrict__ g,
                                                  uint64_t tail_start, uint64_t n, uint32_t tid,
                                                  uint32_t &ovf, double &acc)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint64_t i = tail_start + (uint64_t)j * kFusedThreads + tid;
        if (i < n) {
            const uint32_t h = g[i];
            ovf = overflow_bits(h, ovf);
            acc += (double)square_pair(h, 0.0f);
        }
    }
}

template <bool L2, bool HALF_OUT>
__device__ __forceinline__ void fused_tail_update(float *__restrict__ p, float *__restrict__ m,
                                                  float *__restrict__ v,
                                                  const uint16_t *__restrict__ g,
                                                  uint16_t *__restrict__ p16, uint64_t tail_start,
                                                  uint64_t n, uint32_t tid, const StepScalars &s)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint64_t i = tail_start + (uint64_t)j * kFusedThreads + tid;
        if (i < n) {
            const _Float16 gh = __builtin_bit_cast(_Float16, g[i]);
            float pe = p[i], me = m[i], ve = v[i];
            adam_elem<L2>(pe, me, ve, (float)gh, s);
            p[i] = pe;
            m[i] = me;
            v[i] = ve;
            p16[i] = (uint16_t)pack16<HALF_OUT>(pe, 0.0f);
        }
    }
}

// What lane 0 of a workgroup knows after arriving.
constexpr uint32_t kOverflowed = 1u, kGaveUp = 2u, kArrivedLast = 4u, kVerdictKnown = 8u;

// Lane 0 of wavefront 0: publish the partial sum, arrive (two levels), and report what is known.
// counters[0] is the call's top counter; lines: the group lines.  any: this workgroup saw an
// overflow; tag: this call's.  Returns kArrivedLast (| kOverflowed) in the workgroup after which
// nobody arrives.
__device__ __forceinline__ uint32_t fused_arrive(uint32_t wg, uint32_t nwg, double part, bool any,
                                                 double *partial_sum, uint32_t *counters,
                                                 uint32_t *lines, uint32_t tag)
{
    // The arrival waits for the partial sum to be in place and for the call's tag to have been
    // read: after the last arrival the call counter moves on.
    const uint64_t old = __builtin_bit_cast(uint64_t, publish_device_scope(partial_sum + wg, part));
    const uint32_t add = 1u + (any ? kOverflowUnit : 0u) +
                         zero_after((uint32_t)old, (uint32_t)(old >> 32)) + zero_after(tag, tag);
    uint32_t now;
    if (nwg <= kGroupSize) {
        now = __hip_atomic_fetch_add(counters, add, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) +
              add;
        if ((now & kArrivedMask) != nwg) return 0u;
    } else {
        const uint32_t group = wg / kGroupSize;
        const uint32_t ngroups = (nwg + kGroupSize - 1) / kGroupSize;
        const uint32_t rest = nwg - group * kGroupSize;
        const uint32_t members = rest < kGroupSize ? rest : kGroupSize;
        uint32_t *line = lines + (size_t)group * kLineWords;
        now = __hip_atomic_fetch_add(line, add, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + add;
        if ((now & kArrivedMask) != members) return 0u;
        st_device_scope(line, 0u);
        const uint32_t add2 = 1u + ((now >> 16) != 0u ? kOverflowUnit : 0u);
        now = __hip_atomic_fetch_add(counters, add2, __ATOMIC_RELAXED,
                                     __HIP_MEMORY_SCOPE_AGENT) + add2;
        if ((now & kArrivedMask) != ngroups) return 0u;
    }
    st_device_scope(counters, 0u);
    return kArrivedLast | kVerdictKnown | ((now >> 16) != 0u ? kOverflowed : 0u);
}

// Scalar registers count against residency too, and the runtime's occupancy query does not see
// it.  Measured: compiled freely the shallowest kernel used 79 SGPRs (85 with VCC and friends),
// the runtime reported 8 workgroups per compute unit, and yet grids of 1,800 and more workgroups
// never completed their barrier while 1,792 = 7 x 256 always did; held to 64 SGPRs, 2,048 are
// resident.  That fits a wavefront being charged 16 more than its own (the trap handler's) in
// granules of 16 out of 800 per SIMD: 85 + 16 -> 112, seven times; 68 + 16 -> 96, eight times.
// The attribute takes no template argument, so the deeper kernels, which need only 4 and 2
// wavefront slots per SIMD, are held to 64 as well; the spills go to lanes of a vector register
// and cost nothing measurable.
template <int K, int MODE>
__global__ __launch_bounds__(kFusedThreads) __attribute__((amdgpu_num_sgpr(64)))
void k_adam_small_block_step(
    float *__restrict__ p, float *__restrict__ m, float *__restrict__ v,
    const uint16_t *__restrict__ g, uint16_t *__restrict__ p16, uint64_t n, StepScalars s,
    double *partial_sum, uint32_t *counters, uint32_t *lines,
    const uint64_t *__restrict__ magic, double inv2, double *__restrict__ sqnorm, uint32_t *flag,
    uint32_t spin_limit)
{
    if (workspace_unprepared(magic, sqnorm, flag)) return;
    constexpr bool L2 = (MODE & 1) != 0, HALF_OUT = (MODE & 2) != 0;
    __shared__ double s_sum[2][kFusedWaves];
    __shared__ uint32_t s_ovf[kFusedWaves];
    __shared__ uint32_t s_verdict;

    const uint32_t tid = threadIdx.x, wg = blockIdx.x, nwg = gridDim.x;
    const uint64_t ntiles = n / kFusedTile;                 // whole tiles; the rest is the tail
    const uint64_t tail_start = ntiles * kFusedTile;
    const uint64_t lane_off = (uint64_t)tid * 4;

    if (ntiles == 0) {
        // Less than one tile: one workgroup does it all and there is nobody to wait for.
        if (wg != 0) return;
        uint32_t ovf = 0;
        double acc = 0.0;
        fused_tail_reduce(g, 0, n, tid, ovf, acc);
        const bool wave_ovf = __builtin_amdgcn_ballot_w64(ovf != 0u) != 0;
        if ((tid & 63u) == 0u) s_ovf[tid >> 6] = wave_ovf ? 1u : 0u;
        const double total = fused_workgroup_sum(tid, acc, s_sum[0]);
        uint32_t any = 0;
#pragma unroll
        for (int w = 0; w < kFusedWaves; ++w) any |= s_ovf[w];
        if (any == 0u) fused_tail_update<L2, HALF_OUT>(p, m, v, g, p16, 0, n, tid, s);
        if (tid == 0) {
            if (sqnorm != nullptr) *sqnorm = total * inv2;
            *flag = any;
        }
        return;
    }

    // The call's tag: one more than the call counter that the previous call left behind.
    uint32_t *call_line = lines + (size_t)kCallLine * kLineWords;
    uint32_t tag = ld_device_scope(call_line) + 1u;
    if (tag > kLastTag) tag = 1u;
    const uint32_t nlines = (nwg + kGroupSize - 1) / kGroupSize;
    uint32_t *my_verdict = lines + (size_t)(wg / kGroupSize) * kLineWords + kVerdictWord;

    // Gradients: tile k of this workgroup is tile k * nwg + wg of the block (so that the grid
    // reads each of the K rounds as one contiguous span).  A tile index past the end is clamped
    // to the last tile: the load is then redundant but in bounds and unconditional, and its
    // values are never used.
    u32x2 gv[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        uint64_t tile = (uint64_t)k * nwg + wg;
        if (tile >= ntiles) tile = ntiles - 1;
        gv[k] = *reinterpret_cast<const u32x2 *>(g + tile * kFusedTile + lane_off);
    }
    uint32_t ovf = 0;
    double acc = 0.0;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const bool valid = (uint64_t)k * nwg + wg < ntiles;
        const uint32_t x = valid ? gv[k].x : 0u, y = valid ? gv[k].y : 0u;
        ovf = overflow_bits(x, ovf);
        ovf = overflow_bits(y, ovf);
        float sq = square_pair(x, 0.0f);
        sq = square_pair(y, sq);
        acc += (double)sq;
    }
    if (wg == 0) fused_tail_reduce(g, tail_start, n, tid, ovf, acc);
    const bool wave_ovf = __builtin_amdgcn_ballot_w64(ovf != 0u) != 0;
    if ((tid & 63u) == 0u) s_ovf[tid >> 6] = wave_ovf ? 1u : 0u;
    const double part = fused_workgroup_sum(tid, acc, s_sum[0]);

    // Wavefront 0 arrives before it issues its share of the big loads (the results of its atomics
    // would otherwise queue behind them); the other wavefronts go straight on.  In the workgroup
    // that arrives last the wavefront also publishes the verdict, one lane per group line, and
    // only then looks for the mark of a workgroup that gave up: see the header comment.
    uint32_t state = 0;
    if (tid < 64u) {
        if (tid == 0) {
            uint32_t any = 0;
#pragma unroll
            for (int w = 0; w < kFusedWaves; ++w) any |= s_ovf[w];
            state = fused_arrive(wg, nwg, part, any != 0u, partial_sum, counters, lines, tag);
        }
        state = __builtin_amdgcn_readfirstlane(state);
        if ((state & kArrivedLast) != 0u) {
            const uint32_t word = (tag << 1) | (state & kOverflowed);
            uint32_t seen = 0;
            for (uint32_t l = tid; l < nlines; l += 64u)
                seen |= publish_device_scope(lines + (size_t)l * kLineWords + kVerdictWord, word);
            if (tid == 0) {
                const uint32_t mark = ld_device_scope(call_line + 1 + zero_after(seen, seen));
                *flag = (state & kOverflowed) | (mark == tag ? kFlagIncomplete : 0u);
                st_device_scope(call_line, tag);
            }
        } else if (tid == 0 && spin_limit == 0u) {
            // No waiting allowed at all (a test of the give-up path): decide here, before the
            // update is computed, while the verdict is most likely still out.
            const uint32_t old = publish_device_scope(call_line + 1, tag);
            const uint32_t word = ld_device_scope(my_verdict + zero_after(old, old));
            state = (word >> 1) == tag ? (kVerdictKnown | (word & kOverflowed)) : kGaveUp;
        }
    }
    __builtin_amdgcn_sched_barrier(0);

    // The state, every load issued before anything below consumes one.
    f32x4 pv[K], mv[K], vv[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        uint64_t tile = (uint64_t)k * nwg + wg;
        if (tile >= ntiles) tile = ntiles - 1;
        const uint64_t off = tile * kFusedTile + lane_off;
        pv[k] = *reinterpret_cast<const f32x4 *>(p + off);
        mv[k] = *reinterpret_cast<const f32x4 *>(m + off);
        vv[k] = *reinterpret_cast<const f32x4 *>(v + off);
    }
    __builtin_amdgcn_sched_barrier(0);

    // The update, in registers (wasted if the verdict turns out to be an overflow, which is
    // rare), tile by tile in the order the loads were issued.  The empty asm makes the results
    // exist HERE, ahead of the wait: left alone, the compiler sinks the whole computation into
    // the branch that stores them, behind the verdict.
    u32x2 hv[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        adam_vec4<L2, HALF_OUT>(pv[k], mv[k], vv[k], __builtin_bit_cast(f16x4, gv[k]), s, hv[k]);
        asm volatile("" : "+v"(pv[k]), "+v"(mv[k]), "+v"(vv[k]), "+v"(hv[k]));
        __builtin_amdgcn_sched_barrier(0);
    }
    asm volatile("" ::: "memory");

    // The verdict: by now it is normally there.
    if (tid == 0) {
        if ((state & (kVerdictKnown | kGaveUp)) == 0u) {
            uint32_t word = 0;
            bool there = false;
            for (uint32_t poll = 0; poll < spin_limit && !there; ++poll) {
                word = ld_device_scope(my_verdict);
                there = (word >> 1) == tag;
                if (!there) __builtin_amdgcn_s_sleep(8);
            }
            if (!there) {
                const uint32_t old = publish_device_scope(call_line + 1, tag);
                word = ld_device_scope(my_verdict + zero_after(old, old));
                there = (word >> 1) == tag;
            }
            state |= there ? (kVerdictKnown | (word & kOverflowed)) : kGaveUp;
        }
        s_verdict = state;
    }
    lds_barrier();
    const uint32_t verdict = s_verdict;

    // Skip rule: with the flag set nothing is written.
    if ((verdict & (kOverflowed | kGaveUp)) == 0u) {
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const uint64_t tile = (uint64_t)k * nwg + wg;
            if (tile < ntiles) {
                const uint64_t off = tile * kFusedTile + lane_off;
                *reinterpret_cast<f32x4 *>(p + off) = pv[k];
                *reinterpret_cast<f32x4 *>(m + off) = mv[k];
                *reinterpret_cast<f32x4 *>(v + off) = vv[k];
                *reinterpret_cast<u32x2 *>(p16 + off) = hv[k];
            }
        }
        if (wg == 0) fused_tail_update<L2, HALF_OUT>(p, m, v, g, p16, tail_start, n, tid, s);
    }

    // The workgroup that arrived last combines the partial sums in a fixed order, with its stores
    // already under way.
    if ((verdict & kArrivedLast) != 0u && sqnorm != nullptr) {
        constexpr uint32_t kRounds = kMaxPartials / kFusedThreads;
        double mine[kRounds];
#pragma unroll
        for (uint32_t j = 0; j < kRounds; ++j) {
            const uint32_t i = j * kFusedThreads + tid;
            mine[j] = i < nwg ? ld_device_scope(partial_sum + i) : 0.0;
        }
        double total = 0.0;
#pragma unroll
        for (uint32_t j = 0; j < kRounds; ++j) total += mine[j];
        total = fused_workgroup_sum(tid, total, s_sum[1]);
        if (tid == 0) *sqnorm = total * inv2;
    }
}

// ------------------------------------------------------------------------------------------------
// Host-side launchers (no validation here: the C ABI layer has done it).
// ------------------------------------------------------------------------------------------------

static uint32_t reduce_grid(uint64_t n, uint64_t tile, uint32_t max_wgs)
{
    uint64_t want = (n + tile - 1) / tile;
    if (want < 1) want = 1;
    return (uint32_t)(want < max_wgs ? want : max_wgs);
}

// The parts of a workspace (layout in lohan_kernels.h).
struct WorkspaceView {
    double *partial_sum;
    uint32_t *partial_flag;
    uint32_t *counters;
    uint64_t *magic;
    uint32_t *lines;
};

static WorkspaceView workspace_view(void *workspace)
{
    char *base = reinterpret_cast<char *>(workspace);
    return WorkspaceView{reinterpret_cast<double *>(base),
                         reinterpret_cast<uint32_t *>(base + sizeof(double) * kMaxPartials),
                         reinterpret_cast<uint32_t *>(base + kCountersOffset),
                         reinterpret_cast<uint64_t *>(base + kMagicOffset),
                         reinterpret_cast<uint32_t *>(base + kLinesOffset)};
}

hipError_t launch_workspace_init(void *workspace, hipStream_t stream)
{
    const WorkspaceView ws = workspace_view(workspace);
    constexpr uint32_t kWords = kGroupLines * kLineWords;
    static_assert(kWords >= kMultiMaxBlocks, "one thread per word covers the counters too");
    hipLaunchKernelGGL(k_workspace_init, dim3(kWords / 256), dim3(256), 0, stream, ws.counters,
                       kMultiMaxBlocks, ws.lines, kWords, ws.magic);
    return hipGetLastError();
}

template <bool WITH_NORM>
static void launch_reduce_policy(bool stream_past_caches, uint32_t grid, hipStream_t stream,
                                 const uint16_t *g, uint64_t n, const WorkspaceView &ws,
                                 double inv2, double *sqnorm, uint32_t *flag)
{
    constexpr int kUnroll = kReduceUnroll;
    if (stream_past_caches)
        hipLaunchKernelGGL((k_grad_reduce<WITH_NORM, kUnroll, true>), dim3(grid),
                           dim3(kReduceThreads), 0, stream, g, n, ws.partial_sum, ws.partial_flag,
                           ws.counters, ws.magic, inv2, sqnorm, flag);
    else
        hipLaunchKernelGGL((k_grad_reduce<WITH_NORM, kUnroll, false>), dim3(grid),
                           dim3(kReduceThreads), 0, stream, g, n, ws.partial_sum, ws.partial_flag,
                           ws.counters, ws.magic, inv2, sqnorm, flag);
}

hipError_t launch_grad_reduce(const void *grad_fp16, uint64_t n, bool with_norm, double inv2,
                              double *sqnorm, uint32_t *flag, void *workspace, uint32_t max_wgs,
                              bool stream_past_caches, hipStream_t stream)
{
    if (n == 0) {
        hipLaunchKernelGGL(k_grad_empty, dim3(1), dim3(64), 0, stream, sqnorm, flag);
        return hipGetLastError();
    }
    if (max_wgs > kMaxPartials) max_wgs = kMaxPartials;
    const uint32_t grid =
        reduce_grid(n, (uint64_t)kReduceThreads * 8 * kReduceUnroll, max_wgs);
    const WorkspaceView ws = workspace_view(workspace);
    const uint16_t *g = reinterpret_cast<const uint16_t *>(grad_fp16);
    if (with_norm)
        launch_reduce_policy<true>(stream_past_caches, grid, stream, g, n, ws, inv2, sqnorm, flag);
    else
        launch_reduce_policy<false>(stream_past_caches, grid, stream, g, n, ws, inv2, sqnorm,
                                    flag);
    return hipGetLastError();
}

template <bool WITH_NORM>
static void launch_produce_policy(bool stream_past_caches, uint32_t grid, hipStream_t stream,
                                  const float *src, uint64_t n, float mul, uint16_t *out,
                                  const WorkspaceView &ws, double inv2, double *sqnorm,
                                  uint32_t *flag)
{
    constexpr int kUnroll = kReduceUnroll;
    if (stream_past_caches)
        hipLaunchKernelGGL((k_grad_produce<WITH_NORM, kUnroll, true>), dim3(grid),
                           dim3(kReduceThreads), 0, stream, src, n, mul, out, ws.partial_sum,
                           ws.partial_flag, ws.counters, ws.magic, inv2, sqnorm, flag);
    else
        hipLaunchKernelGGL((k_grad_produce<WITH_NORM, kUnroll, false>), dim3(grid),
                           dim3(kReduceThreads), 0, stream, src, n, mul, out, ws.partial_sum,
                           ws.partial_flag, ws.counters, ws.magic, inv2, sqnorm, flag);
}

hipError_t launch_grad_produce(const float *grad_fp32, uint64_t n, float multiplier,
                               void *grad_fp16_out, double inv2, double *sqnorm, uint32_t *flag,
                               void *workspace, uint32_t max_wgs, bool stream_past_caches,
                               hipStream_t stream)
{
    if (n == 0) {
        hipLaunchKernelGGL(k_grad_empty, dim3(1), dim3(64), 0, stream, sqnorm, flag);
        return hipGetLastError();
    }
    if (max_wgs > kMaxPartials) max_wgs = kMaxPartials;
    const uint32_t grid =
        reduce_grid(n, (uint64_t)kReduceThreads * 4 * kReduceUnroll, max_wgs);
    const WorkspaceView ws = workspace_view(workspace);
    uint16_t *out = reinterpret_cast<uint16_t *>(grad_fp16_out);
    if (sqnorm != nullptr)
        launch_produce_policy<true>(stream_past_caches, grid, stream, grad_fp32, n, multiplier,
                                    out, ws, inv2, sqnorm, flag);
    else
        launch_produce_policy<false>(stream_past_caches, grid, stream, grad_fp32, n, multiplier,
                                     out, ws, inv2, sqnorm, flag);
    return hipGetLastError();
}

hipError_t launch_clip_scale(const double *sqnorm, float loss_scale, float max_norm,
                             float *inv_out, uint32_t count, hipStream_t stream)
{
    hipLaunchKernelGGL(k_clip_scale, dim3((count + 63) / 64), dim3(64), 0, stream, sqnorm,
                       loss_scale, max_norm, inv_out, count);
    return hipGetLastError();
}

template <bool WITH_NORM>
static void launch_multi_reduce_policy(bool stream_past_caches, dim3 grid, hipStream_t stream,
                                       const MultiArgs &args, const WorkspaceView &ws,
                                       double inv2, double *sqnorms, uint32_t *flags)
{
    constexpr int kUnroll = kReduceUnroll;
    if (stream_past_caches)
        hipLaunchKernelGGL((k_multi_grad_reduce<WITH_NORM, kUnroll, true>), grid,
                           dim3(kReduceThreads), 0, stream, args, ws.partial_sum, ws.partial_flag,
                           ws.counters, ws.magic, inv2, sqnorms, flags);
    else
        hipLaunchKernelGGL((k_multi_grad_reduce<WITH_NORM, kUnroll, false>), grid,
                           dim3(kReduceThreads), 0, stream, args, ws.partial_sum, ws.partial_flag,
                           ws.counters, ws.magic, inv2, sqnorms, flags);
}

hipError_t launch_multi_grad_reduce(const MultiArgs &args, uint32_t num_blocks, bool with_norm,
                                    double inv2, double *sqnorms, uint32_t *flags,
                                    void *workspace, uint32_t max_wgs, bool stream_past_caches,
                                    hipStream_t stream)
{
    if (num_blocks == 0 || num_blocks > kMultiMaxBlocks) return hipErrorInvalidValue;
    constexpr uint64_t kTile = (uint64_t)kReduceThreads * 8 * kReduceUnroll;
    uint64_t longest = 0;
    for (uint32_t b = 0; b < num_blocks; ++b)
        if (args.d[b].n > longest) longest = args.d[b].n;
    // The same total number of workgroups as a single-block call, split evenly over the blocks.
    uint32_t per_block = (max_wgs + num_blocks - 1) / num_blocks;
    if (per_block > kMaxPartials / num_blocks) per_block = kMaxPartials / num_blocks;
    per_block = reduce_grid(longest, kTile, per_block);
    const WorkspaceView ws = workspace_view(workspace);
    const dim3 grid(per_block, num_blocks);
    if (with_norm)
        launch_multi_reduce_policy<true>(stream_past_caches, grid, stream, args, ws, inv2, sqnorms,
                                         flags);
    else
        launch_multi_reduce_policy<false>(stream_past_caches, grid, stream, args, ws, inv2,
                                          sqnorms, flags);
    return hipGetLastError();
}

typedef void (*adam_kernel_t)(float *, float *, float *, const uint16_t *, uint16_t *, uint64_t,
                              StepScalars, const uint32_t *, const float *);
typedef void (*adam_oop_kernel_t)(const float *, const float *, const float *, const uint16_t *,
                                  float *, float *, float *, uint16_t *, uint64_t, StepScalars,
                                  uint32_t *, const float *);

typedef void (*adam_multi_kernel_t)(MultiArgs, StepScalars, const uint32_t *, const float *);
typedef void (*adam_ring_kernel_t)(const RingSlot *, const uint32_t *, const uint32_t *,
                                   const uint32_t *, const unsigned long long *,
                                   unsigned long long *, uint32_t, const uint16_t *, uint64_t,
                                   StepScalars, const float *);

// The kernel families share the variant space; a family names the function-pointer type and
// the instantiation for one point of it.
struct InPlaceFamily {
    typedef adam_kernel_t fn;
    template <int WG, int UNROLL, int POLICY, int MODE>
    static fn get() { return k_adam_block_step<WG, UNROLL, POLICY, MODE>; }
};
struct OutOfPlaceFamily {
    typedef adam_oop_kernel_t fn;
    template <int WG, int UNROLL, int POLICY, int MODE>
    static fn get() { return k_adam_block_step_oop<WG, UNROLL, POLICY, MODE>; }
};

struct RingFamily {
    typedef adam_ring_kernel_t fn;
    template <int WG, int UNROLL, int POLICY, int MODE>
    static fn get() { return k_adam_ring_step<WG, UNROLL, POLICY, MODE>; }
};

struct MultiBlockFamily {
    typedef adam_multi_kernel_t fn;
    template <int WG, int UNROLL, int POLICY, int MODE>
    static fn get() { return k_adam_multi_block_step<WG, UNROLL, POLICY, MODE>; }
};

template <class F, int WG, int UNROLL, int POLICY>
static typename F::fn pick_mode(int mode)
{
    switch (mode & 3) {
    case 0: return F::template get<WG, UNROLL, POLICY, 0>();
    case 1: return F::template get<WG, UNROLL, POLICY, 1>();
    case 2: return F::template get<WG, UNROLL, POLICY, 2>();
    default: return F::template get<WG, UNROLL, POLICY, 3>();
    }
}

template <class F, int WG, int UNROLL>
static typename F::fn pick_policy(int policy, int mode)
{
    switch (policy) {
    case 0: return pick_mode<F, WG, UNROLL, 0>(mode);
    case 1: return pick_mode<F, WG, UNROLL, 1>(mode);
    case 2: return pick_mode<F, WG, UNROLL, 2>(mode);
    default: return nullptr;
    }
}

template <class F, int WG>
static typename F::fn pick_unroll(int unroll_index, int policy, int mode)
{
    switch (unroll_index) {
    case 0: return pick_policy<F, WG, 1>(policy, mode);
    case 1: return pick_policy<F, WG, 2>(policy, mode);
    default: return nullptr;
    }
}

// variant bits: [1:0] workgroup size index (64, 128, 256 lanes), [3:2] unroll index (1 or 2
// vectors per lane per tile), [5:4] cache policy (0 default, 1 nontemporal, 2 nontemporal loads
// with write-through streaming stores).
bool adam_variant_valid(int variant)
{
    return variant >= 0 && variant < 64 && (variant & 3) < 3 && ((variant >> 2) & 3) < 2 &&
           ((variant >> 4) & 3) < 3;
}

template <class F>
static typename F::fn pick_kernel(int variant, int mode)
{
    const int wg_index = variant & 3, unroll_index = (variant >> 2) & 3;
    const int policy = (variant >> 4) & 3;
    switch (wg_index) {
    case 0: return pick_unroll<F, 64>(unroll_index, policy, mode);
    case 1: return pick_unroll<F, 128>(unroll_index, policy, mode);
    default: return pick_unroll<F, 256>(unroll_index, policy, mode);
    }
}

// Grid, workgroup size and the dynamic LDS request for n elements under cfg.
struct AdamGeometry {
    uint32_t grid;
    int wg;
    size_t lds;
};

static hipError_t adam_geometry(const void *kernel, uint64_t n, const AdamLaunch &cfg,
                                const DeviceInfo &dev, AdamGeometry &out)
{
    const int wg_index = cfg.variant & 3, unroll_index = (cfg.variant >> 2) & 3;
    const int wg = 64 << wg_index, unroll = 1 << unroll_index;
    const uint64_t tile = (uint64_t)wg * 4 * unroll;
    uint64_t want = n / tile;
    if (want < 1) want = 1;
    if (cfg.max_wgs_per_cu > 0) {
        const uint64_t cap = (uint64_t)dev.cus * (uint64_t)cfg.max_wgs_per_cu;
        if (want > cap) want = cap;
    }
    if (want > 0x7FFFFFFFull) want = 0x7FFFFFFFull;      // grid-stride loop covers the rest

    // Occupancy throttle: the kernels use no LDS, so a dynamic LDS request per workgroup sized
    // as a fraction of the CU's LDS bounds how many workgroups (hence wavefronts, hence bytes in
    // flight) a CU holds at once.
    size_t lds = 0;
    const int waves_per_wg = wg / 64;
    if (cfg.waves_per_cu > 0 && cfg.waves_per_cu < 32) {
        int wgs = cfg.waves_per_cu / waves_per_wg;
        if (wgs < 1) wgs = 1;
        lds = (size_t)(dev.lds_per_cu / wgs) / 256 * 256;
        if (lds > 64 * 1024) {
            hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                               (int)lds);
            if (e != hipSuccess) return e;
        }
    }
    out.grid = (uint32_t)want;
    out.wg = wg;
    out.lds = lds;
    return hipSuccess;
}

hipError_t launch_adam_block_step(float *p, float *m, float *v, const void *grad_fp16,
                                  void *p16, uint64_t n, const StepScalars &s, int mode,
                                  const uint32_t *flag, const float *inv_override,
                                  const AdamLaunch &cfg, const DeviceInfo &dev,
                                  hipStream_t stream)
{
    if (n == 0) return hipSuccess;
    if (!adam_variant_valid(cfg.variant) || dev.cus <= 0) return hipErrorInvalidValue;
    adam_kernel_t kernel = pick_kernel<InPlaceFamily>(cfg.variant, mode);
    if (kernel == nullptr) return hipErrorInvalidValue;
    AdamGeometry geo;
    hipError_t e = adam_geometry(reinterpret_cast<const void *>(kernel), n, cfg, dev, geo);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kernel, dim3(geo.grid), dim3(geo.wg), geo.lds, stream, p, m, v,
                       reinterpret_cast<const uint16_t *>(grad_fp16),
                       reinterpret_cast<uint16_t *>(p16), n, s, flag, inv_override);
    return hipGetLastError();
}

typedef void (*adam_small_kernel_t)(float *, float *, float *, const uint16_t *, uint16_t *,
                                    uint64_t, StepScalars, double *, uint32_t *, uint32_t *,
                                    const uint64_t *, double, double *, uint32_t *, uint32_t);

template <int K>
static adam_small_kernel_t small_kernel_of_depth(int mode)
{
    switch (mode & 3) {
    case 0: return k_adam_small_block_step<K, 0>;
    case 1: return k_adam_small_block_step<K, 1>;
    case 2: return k_adam_small_block_step<K, 2>;
    default: return k_adam_small_block_step<K, 3>;
    }
}

static adam_small_kernel_t small_kernel(int depth_index, int mode)
{
    static_assert(kSmallTile == kFusedTile, "the header's tile is the kernel's");
    switch (depth_index) {
    case 0: return small_kernel_of_depth<kSmallDepths[0]>(mode);
    case 1: return small_kernel_of_depth<kSmallDepths[1]>(mode);
    default: return small_kernel_of_depth<kSmallDepths[2]>(mode);
    }
}

hipError_t small_block_occupancy(int wgs_per_cu[kSmallVariants])
{
    for (int i = 0; i < kSmallVariants; ++i) {
        int lowest = 0;
        for (int mode = 0; mode < 4; ++mode) {
            int resident = 0;
            hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(
                &resident, reinterpret_cast<const void *>(small_kernel(i, mode)), kFusedThreads, 0);
            if (e != hipSuccess) return e;
            if (mode == 0 || resident < lowest) lowest = resident;
        }
        // (What the runtime reports rests on vector registers, LDS and wavefront slots; the
        // kernels' scalar registers are kept out of the way at compile time, see above.)
        wgs_per_cu[i] = lowest;
    }
    return hipSuccess;
}

// Workgroups of depth i that are resident together on the whole device.
static uint64_t small_block_grid_limit(const DeviceInfo &dev, int i)
{
    const int per_cu = dev.small_wgs_per_cu[i] > 0 ? dev.small_wgs_per_cu[i] : 0;
    const uint64_t resident = (uint64_t)dev.cus * (uint64_t)per_cu;
    return resident < kMaxPartials ? resident : kMaxPartials;
}

uint64_t small_block_max_n(const DeviceInfo &dev)
{
    uint64_t best = 0;
    for (int i = 0; i < kSmallVariants; ++i) {
        const uint64_t tiles = small_block_grid_limit(dev, i) * (uint64_t)kSmallDepths[i];
        if (tiles > best) best = tiles;
    }
    return best == 0 ? 0 : best * kSmallTile + (kSmallTile - 1);
}

hipError_t launch_adam_small_block_step(float *p, float *m, float *v, const void *grad_fp16,
                                        void *p16, uint64_t n, const StepScalars &s, int mode,
                                        double inv2, double *sqnorm, uint32_t *flag,
                                        void *workspace, uint32_t spin_limit,
                                        const DeviceInfo &dev, hipStream_t stream)
{
    if (n == 0) {
        hipLaunchKernelGGL(k_grad_empty, dim3(1), dim3(64), 0, stream, sqnorm, flag);
        return hipGetLastError();
    }
    // The shallowest depth that holds the block: most wavefronts per CU, fewest registers.  The
    // grid is as small as that depth allows, so that every workgroup's K slots are in use.
    const uint64_t ntiles = n / kSmallTile;
    for (int i = 0; i < kSmallVariants; ++i) {
        const uint64_t limit = small_block_grid_limit(dev, i);
        const uint64_t depth = (uint64_t)kSmallDepths[i];
        if (limit == 0 || limit * depth < ntiles) continue;
        uint64_t grid = (ntiles + depth - 1) / depth;
        if (grid < 1) grid = 1;
        const WorkspaceView ws = workspace_view(workspace);
        hipLaunchKernelGGL(small_kernel(i, mode), dim3((uint32_t)grid), dim3(kFusedThreads), 0,
                           stream, p, m, v, reinterpret_cast<const uint16_t *>(grad_fp16),
                           reinterpret_cast<uint16_t *>(p16), n, s, ws.partial_sum, ws.counters,
                           ws.lines, ws.magic, inv2, sqnorm, flag, spin_limit);
        return hipGetLastError();
    }
    return hipErrorInvalidValue;
}

hipError_t launch_adam_block_step_oop(const float *p_in, const float *m_in, const float *v_in,
                                      const void *grad_fp16, float *p_out, float *m_out,
                                      float *v_out, void *p16, uint64_t n, const StepScalars &s,
                                      int mode, uint32_t *flag, const float *inv_override,
                                      const AdamLaunch &cfg, const DeviceInfo &dev,
                                      hipStream_t stream)
{
    // The flag starts at 0 on the stream; the update kernel can only raise it.
    hipLaunchKernelGGL(k_grad_empty, dim3(1), dim3(64), 0, stream, (double *)nullptr, flag);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n == 0) return e;
    if (!adam_variant_valid(cfg.variant) || dev.cus <= 0) return hipErrorInvalidValue;
    adam_oop_kernel_t kernel = pick_kernel<OutOfPlaceFamily>(cfg.variant, mode);
    if (kernel == nullptr) return hipErrorInvalidValue;
    AdamGeometry geo;
    e = adam_geometry(reinterpret_cast<const void *>(kernel), n, cfg, dev, geo);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kernel, dim3(geo.grid), dim3(geo.wg), geo.lds, stream, p_in, m_in, v_in,
                       reinterpret_cast<const uint16_t *>(grad_fp16), p_out, m_out, v_out,
                       reinterpret_cast<uint16_t *>(p16), n, s, flag, inv_override);
    return hipGetLastError();
}

hipError_t launch_adam_multi_block_step(const MultiArgs &args, uint32_t num_blocks,
                                        const StepScalars &s, int mode, const uint32_t *flags,
                                        const float *inv_override, const AdamLaunch &cfg,
                                        const DeviceInfo &dev, hipStream_t stream)
{
    if (num_blocks == 0 || num_blocks > kMultiMaxBlocks) return hipErrorInvalidValue;
    if (!adam_variant_valid(cfg.variant) || dev.cus <= 0) return hipErrorInvalidValue;
    uint64_t longest = 0;
    for (uint32_t b = 0; b < num_blocks; ++b)
        if (args.d[b].n > longest) longest = args.d[b].n;
    if (longest == 0) return hipSuccess;
    adam_multi_kernel_t kernel = pick_kernel<MultiBlockFamily>(cfg.variant, mode);
    if (kernel == nullptr) return hipErrorInvalidValue;
    AdamGeometry geo;
    hipError_t e = adam_geometry(reinterpret_cast<const void *>(kernel), longest, cfg, dev, geo);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kernel, dim3(geo.grid, num_blocks), dim3(geo.wg), geo.lds, stream, args, s,
                       flags, inv_override);
    return hipGetLastError();
}

hipError_t launch_adam_ring_step(const RingView &ring, uint32_t block, const void *grad_fp16,
                                 uint64_t n, const StepScalars &s, int mode,
                                 const float *inv_override, const AdamLaunch &cfg,
                                 const DeviceInfo &dev, hipStream_t stream)
{
    if (n == 0) return hipSuccess;
    if (!adam_variant_valid(cfg.variant) || dev.cus <= 0) return hipErrorInvalidValue;
    adam_ring_kernel_t kernel = pick_kernel<RingFamily>(cfg.variant, mode);
    if (kernel == nullptr) return hipErrorInvalidValue;
    AdamGeometry geo;
    hipError_t e = adam_geometry(reinterpret_cast<const void *>(kernel), n, cfg, dev, geo);
    if (e != hipSuccess) return e;
    unsigned long long *attempts = reinterpret_cast<unsigned long long *>(ring.attempts);
    unsigned long long *overflow_attempt =
        reinterpret_cast<unsigned long long *>(ring.overflow_attempt);
    hipLaunchKernelGGL(kernel, dim3(geo.grid), dim3(geo.wg), geo.lds, stream, ring.slots,
                       ring.slot_of, ring.class_of, ring.spare_of_class, attempts,
                       overflow_attempt, block, reinterpret_cast<const uint16_t *>(grad_fp16), n,
                       s, inv_override);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_ring_commit, dim3(1), dim3(64), 0, stream, ring.slot_of, ring.class_of,
                       ring.spare_of_class, attempts, overflow_attempt, block);
    return hipGetLastError();
}

}  // namespace lohan
