// HIP kernels (gfx950 / CDNA4) for the per-block fused mixed-precision Adam step.
//
// The step is the "CPU Compute" box of LoHan's active gradient offloading (Sec. IV-C): update the
// model states of block i (P32 and the two OS32 moments of Table II) from its G16 gradients and
// emit the P16 working copy, here moved from the host into HBM.  It is an elementwise stream of
// 28 bytes per element with ~1 flop/byte, so there is no MFMA anywhere: what matters is that every
// global access of a wavefront is one contiguous run (128-bit per lane for fp32 streams, 64-bit
// per lane for the two 16-bit streams), that enough independent loads are in flight per lane, and
// that the grid is sized to the CU count.
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

constexpr int kThreads = 256;            // 4 wavefronts of 64 lanes
constexpr int kWaves = kThreads / 64;

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

// ------------------------------------------------------------------------------------------------
// Gradient reduction: overflow flag (integer test on the raw fp16 bits) and, optionally, the sum
// of squares.  Stage 1 writes one partial per workgroup; stage 2 (one workgroup) combines the
// partials in a fixed order, so the result does not depend on scheduling.
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

template <bool WITH_NORM, int UNROLL>
__global__ __launch_bounds__(kThreads) void k_grad_reduce(const uint16_t *__restrict__ g,
                                                          uint64_t n,
                                                          double *__restrict__ partial_sum,
                                                          uint32_t *__restrict__ partial_flag)
{
    constexpr uint64_t kVec = 8;                               // halves per 128-bit load
    constexpr uint64_t kTile = (uint64_t)kThreads * kVec * UNROLL;
    const uint32_t tid = threadIdx.x;
    const uint64_t ntiles = n / kTile;

    uint32_t ovf = 0;
    double acc = 0.0;

    for (uint64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(g + tile * kTile) + tid;
        u32x4 q[UNROLL];
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) q[j] = ld<true>(src + j * kThreads);
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) reduce_vec<WITH_NORM>(q[j], ovf, acc);
    }

    // Ragged end: whole 8-element vectors first, then up to 7 single elements.
    const uint64_t rem_start = ntiles * kTile;
    const uint64_t rem_vecs = (n - rem_start) / kVec;
    for (uint64_t i = (uint64_t)blockIdx.x * kThreads + tid; i < rem_vecs;
         i += (uint64_t)gridDim.x * kThreads) {
        u32x4 q = *(reinterpret_cast<const u32x4 *>(g + rem_start) + i);
        reduce_vec<WITH_NORM>(q, ovf, acc);
    }
    const uint64_t tail_start = rem_start + rem_vecs * kVec;
    if (blockIdx.x == 0 && tail_start + tid < n) {
        uint32_t h = g[tail_start + tid];
        ovf = overflow_bits(h, ovf);
        if constexpr (WITH_NORM) acc += (double)square_pair(h, 0.0f);
    }

    // Wavefront level: butterfly over the 64 lanes (fixed pairing), then LDS across the waves.
    uint32_t any = __builtin_amdgcn_ballot_w64(ovf != 0) != 0 ? 1u : 0u;
    if constexpr (WITH_NORM) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    }
    __shared__ double s_sum[kWaves];
    __shared__ uint32_t s_flag[kWaves];
    const uint32_t wave = tid >> 6, lane = tid & 63u;
    if (lane == 0) {
        s_sum[wave] = acc;
        s_flag[wave] = any;
    }
    __syncthreads();
    if (tid == 0) {
        double total = 0.0;
        uint32_t f = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            total += s_sum[w];
            f |= s_flag[w];
        }
        if constexpr (WITH_NORM) partial_sum[blockIdx.x] = total;
        partial_flag[blockIdx.x] = f;
    }
}

// Stage 2: one workgroup.  inv2 = (1/loss_scale)^2 in float64 turns the raw sum of squares into
// the squared norm of the unscaled gradients.
template <bool WITH_NORM>
__global__ __launch_bounds__(kThreads) void k_grad_finalize(const double *__restrict__ partial_sum,
                                                            const uint32_t *__restrict__ partial_flag,
                                                            uint32_t nparts, double inv2,
                                                            double *__restrict__ sqnorm,
                                                            uint32_t *__restrict__ flag)
{
    const uint32_t tid = threadIdx.x;
    double acc = 0.0;
    uint32_t f = 0;
    for (uint32_t i = tid; i < nparts; i += kThreads) {
        if constexpr (WITH_NORM) acc += partial_sum[i];
        f |= partial_flag[i];
    }
    uint32_t any = __builtin_amdgcn_ballot_w64(f != 0) != 0 ? 1u : 0u;
    if constexpr (WITH_NORM) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    }
    __shared__ double s_sum[kWaves];
    __shared__ uint32_t s_flag[kWaves];
    const uint32_t wave = tid >> 6, lane = tid & 63u;
    if (lane == 0) {
        s_sum[wave] = acc;
        s_flag[wave] = any;
    }
    __syncthreads();
    if (tid == 0) {
        double total = 0.0;
        uint32_t r = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            total += s_sum[w];
            r |= s_flag[w];
        }
        if constexpr (WITH_NORM) {
            if (sqnorm != nullptr) *sqnorm = total * inv2;
        }
        if (flag != nullptr) *flag = r;
    }
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

__device__ __forceinline__ uint32_t bf16_rne_bits(float x)
{
    uint32_t b = __builtin_bit_cast(uint32_t, x);
    uint32_t r = (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) r = (b >> 16) | 0x0040u;   // NaN stays a quiet NaN
    return r;
}

template <bool L2>
__device__ __forceinline__ void adam_elem(float &p, float &m, float &v, float g_scaled,
                                          const StepScalars &s, uint32_t &p16)
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
    p16 = bf16_rne_bits(p_new);
}

template <bool L2>
__device__ __forceinline__ void adam_vec4(f32x4 &p, f32x4 &m, f32x4 &v, f16x4 g,
                                          const StepScalars &s, u32x2 &out16)
{
    uint32_t h[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float pe = p[k], me = m[k], ve = v[k];
        adam_elem<L2>(pe, me, ve, (float)g[k], s, h[k]);
        p[k] = pe;
        m[k] = me;
        v[k] = ve;
    }
    out16.x = h[0] | (h[1] << 16);
    out16.y = h[2] | (h[3] << 16);
}

// NT is a bit set: 1 = nontemporal G16 loads, 2 = nontemporal P32/OS32 loads,
// 4 = nontemporal P32/OS32 stores, 8 = nontemporal P16 stores.
template <int UNROLL, int NT, bool L2>
__global__ __launch_bounds__(kThreads) void k_adam_block_step(float *__restrict__ p,
                                                              float *__restrict__ m,
                                                              float *__restrict__ v,
                                                              const uint16_t *__restrict__ g,
                                                              uint16_t *__restrict__ p16,
                                                              uint64_t n, StepScalars s,
                                                              const uint32_t *__restrict__ flag,
                                                              uint32_t tiles_per_wg)
{
    // Skip rule: a set overflow flag means nothing at all is written by this kernel.
    if (*flag != 0u) return;

    constexpr bool kNtG = (NT & 1) != 0, kNtLd = (NT & 2) != 0, kNtSt = (NT & 4) != 0,
                   kNtH = (NT & 8) != 0;
    constexpr uint64_t kVec = 4;                                  // elements per lane per access
    constexpr uint64_t kRow = (uint64_t)kThreads * kVec;          // elements per wg-wide access
    constexpr uint64_t kTile = kRow * UNROLL;
    const uint32_t tid = threadIdx.x;
    const uint64_t ntiles = n / kTile;

    // tiles_per_wg == 0: tiles are dealt round-robin to workgroups (neighbouring workgroups
    // stream neighbouring tiles).  Otherwise each workgroup owns a contiguous run of tiles.
    uint64_t tile, tile_end, tile_step;
    if (tiles_per_wg == 0u) {
        tile = blockIdx.x;
        tile_end = ntiles;
        tile_step = gridDim.x;
    } else {
        tile = (uint64_t)blockIdx.x * tiles_per_wg;
        tile_end = tile + tiles_per_wg < ntiles ? tile + tiles_per_wg : ntiles;
        tile_step = 1;
    }

    for (; tile < tile_end; tile += tile_step) {
        const uint64_t base = tile * kTile + (uint64_t)tid * kVec;
        f16x4 gv[UNROLL];
        f32x4 pv[UNROLL], mv[UNROLL], vv[UNROLL];
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) {
            const uint64_t off = base + j * kRow;
            gv[j] = ld<kNtG>(reinterpret_cast<const f16x4 *>(g + off));
            pv[j] = ld<kNtLd>(reinterpret_cast<const f32x4 *>(p + off));
            mv[j] = ld<kNtLd>(reinterpret_cast<const f32x4 *>(m + off));
            vv[j] = ld<kNtLd>(reinterpret_cast<const f32x4 *>(v + off));
        }
#pragma unroll
        for (int j = 0; j < UNROLL; ++j) {
            const uint64_t off = base + j * kRow;
            u32x2 h;
            adam_vec4<L2>(pv[j], mv[j], vv[j], gv[j], s, h);
            st<kNtSt>(reinterpret_cast<f32x4 *>(p + off), pv[j]);
            st<kNtSt>(reinterpret_cast<f32x4 *>(m + off), mv[j]);
            st<kNtSt>(reinterpret_cast<f32x4 *>(v + off), vv[j]);
            st<kNtH>(reinterpret_cast<u32x2 *>(p16 + off), h);
        }
    }

    // Ragged end (fewer than kTile elements): whole 4-element vectors spread over the grid, then
    // up to 3 single elements in workgroup 0.
    const uint64_t rem_start = ntiles * kTile;
    const uint64_t rem_vecs = (n - rem_start) / kVec;
    for (uint64_t i = (uint64_t)blockIdx.x * kThreads + tid; i < rem_vecs;
         i += (uint64_t)gridDim.x * kThreads) {
        const uint64_t off = rem_start + i * kVec;
        f16x4 gq = *reinterpret_cast<const f16x4 *>(g + off);
        f32x4 pq = *reinterpret_cast<const f32x4 *>(p + off);
        f32x4 mq = *reinterpret_cast<const f32x4 *>(m + off);
        f32x4 vq = *reinterpret_cast<const f32x4 *>(v + off);
        u32x2 h;
        adam_vec4<L2>(pq, mq, vq, gq, s, h);
        *reinterpret_cast<f32x4 *>(p + off) = pq;
        *reinterpret_cast<f32x4 *>(m + off) = mq;
        *reinterpret_cast<f32x4 *>(v + off) = vq;
        *reinterpret_cast<u32x2 *>(p16 + off) = h;
    }
    const uint64_t tail = rem_start + rem_vecs * kVec + tid;
    if (blockIdx.x == 0 && tail < n) {
        _Float16 gh = __builtin_bit_cast(_Float16, g[tail]);
        float pe = p[tail], me = m[tail], ve = v[tail];
        uint32_t h;
        adam_elem<L2>(pe, me, ve, (float)gh, s, h);
        p[tail] = pe;
        m[tail] = me;
        v[tail] = ve;
        p16[tail] = (uint16_t)h;
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

hipError_t launch_grad_reduce(const void *grad_fp16, uint64_t n, bool with_norm, double inv2,
                              double *sqnorm, uint32_t *flag, void *workspace, uint32_t max_wgs,
                              hipStream_t stream)
{
    if (n == 0) {
        hipLaunchKernelGGL(k_grad_empty, dim3(1), dim3(64), 0, stream, sqnorm, flag);
        return hipGetLastError();
    }
    constexpr int kUnroll = 4;
    if (max_wgs > kMaxPartials) max_wgs = kMaxPartials;
    const uint32_t grid = reduce_grid(n, (uint64_t)kThreads * 8 * kUnroll, max_wgs);
    double *psum = reinterpret_cast<double *>(workspace);
    uint32_t *pflag = reinterpret_cast<uint32_t *>(reinterpret_cast<char *>(workspace) +
                                                   sizeof(double) * kMaxPartials);
    const uint16_t *g = reinterpret_cast<const uint16_t *>(grad_fp16);
    if (with_norm) {
        hipLaunchKernelGGL((k_grad_reduce<true, kUnroll>), dim3(grid), dim3(kThreads), 0, stream,
                           g, n, psum, pflag);
        hipLaunchKernelGGL((k_grad_finalize<true>), dim3(1), dim3(kThreads), 0, stream, psum,
                           pflag, grid, inv2, sqnorm, flag);
    } else {
        hipLaunchKernelGGL((k_grad_reduce<false, kUnroll>), dim3(grid), dim3(kThreads), 0, stream,
                           g, n, psum, pflag);
        hipLaunchKernelGGL((k_grad_finalize<false>), dim3(1), dim3(kThreads), 0, stream, psum,
                           pflag, grid, inv2, sqnorm, flag);
    }
    return hipGetLastError();
}

typedef void (*adam_kernel_t)(float *, float *, float *, const uint16_t *, uint16_t *, uint64_t,
                              StepScalars, const uint32_t *, uint32_t);

template <int UNROLL, int NT>
static adam_kernel_t pick_l2(bool l2)
{
    return l2 ? k_adam_block_step<UNROLL, NT, true> : k_adam_block_step<UNROLL, NT, false>;
}

template <int UNROLL>
static adam_kernel_t pick_nt(int nt_index, bool l2)
{
    switch (nt_index) {
    case 0: return pick_l2<UNROLL, 0>(l2);
    case 1: return pick_l2<UNROLL, 9>(l2);
    case 2: return pick_l2<UNROLL, 12>(l2);
    case 3: return pick_l2<UNROLL, 13>(l2);
    case 4: return pick_l2<UNROLL, 15>(l2);
    default: return nullptr;
    }
}

bool adam_variant_valid(int variant)
{
    if (variant < 0) return false;
    const int unroll_index = variant & 3, nt_index = (variant >> 2) & 7, rest = variant >> 6;
    return unroll_index < 3 && nt_index < 5 && rest == 0;
}

hipError_t launch_adam_block_step(float *p, float *m, float *v, const void *grad_fp16,
                                  void *p16, uint64_t n, const StepScalars &s, bool l2,
                                  const uint32_t *flag, int variant, uint32_t max_wgs,
                                  hipStream_t stream)
{
    if (n == 0) return hipSuccess;
    // variant bits: [1:0] unroll index (1, 2, 4 vectors per lane per trip), [4:2] nontemporal
    // set index, [5] contiguous tile runs per workgroup instead of round-robin.
    const int unroll_index = variant & 3, nt_index = (variant >> 2) & 7;
    const bool blocked = ((variant >> 5) & 1) != 0;
    adam_kernel_t kernel = nullptr;
    int unroll = 1;
    switch (unroll_index) {
    case 0: kernel = pick_nt<1>(nt_index, l2); unroll = 1; break;
    case 1: kernel = pick_nt<2>(nt_index, l2); unroll = 2; break;
    case 2: kernel = pick_nt<4>(nt_index, l2); unroll = 4; break;
    default: break;
    }
    if (kernel == nullptr) return hipErrorInvalidValue;
    const uint64_t tile = (uint64_t)kThreads * 4 * unroll;
    uint64_t ntiles = n / tile;
    uint64_t want = ntiles > 0 ? ntiles : 1;
    uint32_t grid = (uint32_t)(want < max_wgs ? want : max_wgs);
    uint32_t tiles_per_wg = 0;
    if (blocked && ntiles > 0) {
        uint64_t per = (ntiles + grid - 1) / grid;
        if (per > 0xFFFFFFFFull) return hipErrorInvalidValue;
        tiles_per_wg = (uint32_t)per;
    }
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(kThreads), 0, stream, p, m, v,
                       reinterpret_cast<const uint16_t *>(grad_fp16),
                       reinterpret_cast<uint16_t *>(p16), n, s, flag, tiles_per_wg);
    return hipGetLastError();
}

}  // namespace lohan
