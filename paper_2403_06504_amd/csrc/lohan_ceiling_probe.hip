// Bandwidth probes (bench-only, see include/lohan_adam_tuning.h): the access patterns of the block
// step of Sec. IV-C with trivial arithmetic, to measure what the machine sustains for pure
// reads, pure writes, a copy, and the step's own five-stream 14-bytes-in / 14-bytes-out pattern
// (Table II's tensor widths: G16 2, P32 4, OS32 8 in; P32 4, OS32 8, P16 2 out).  They use the
// launch design of the update kernel -- 64-lane workgroups in address order, 128-bit accesses per
// lane, nontemporal loads, write-through streaming stores, occupancy bounded by an unused dynamic
// LDS request -- and the five-stream probe its exact tile (256 elements per workgroup), so that
// the only difference to k_adam_block_step is the arithmetic.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lohan_adam_tuning.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kLanes = 64;
constexpr uint64_t kTile = (uint64_t)kLanes * 4;

// Write-through streaming stores (sc0 sc1 nt); the trailing s_nop covers the wait states the
// hardware needs between a store of more than 64 bits and a VALU write to its data registers.
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

// The single-stream probes give every workgroup kRows rows of 64 x 128 bits (with one row per
// workgroup they would measure the rate at which workgroups can be dispatched, about 4.7 per
// nanosecond, rather than the memory); the host launches whole groups of kRows rows only.
constexpr int kRows = 8;

__global__ __launch_bounds__(kLanes) void k_probe_read(const float *a, float *sink)
{
    const float *base = a + (uint64_t)blockIdx.x * kRows * kTile + (uint64_t)threadIdx.x * 4;
    f32x4 x[kRows];
#pragma unroll
    for (int j = 0; j < kRows; ++j)
        x[j] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(base + j * kTile));
    f32x4 acc = x[0];
#pragma unroll
    for (int j = 1; j < kRows; ++j) acc += x[j];
    // Never true for finite data, but keeps the loads alive.
    if (acc.x + acc.y + acc.z + acc.w == 1.2345678e30f) *sink = acc.x;
}

__global__ __launch_bounds__(kLanes) void k_probe_write(float *__restrict__ b)
{
    float *base = b + (uint64_t)blockIdx.x * kRows * kTile + (uint64_t)threadIdx.x * 4;
    const f32x4 x = {1.0f, 2.0f, 3.0f, (float)threadIdx.x};
#pragma unroll
    for (int j = 0; j < kRows; ++j) st_through(reinterpret_cast<f32x4 *>(base + j * kTile), x);
}

__global__ __launch_bounds__(kLanes) void k_probe_copy(const float *__restrict__ a,
                                                       float *__restrict__ b)
{
    const uint64_t off = (uint64_t)blockIdx.x * kRows * kTile + (uint64_t)threadIdx.x * 4;
    f32x4 x[kRows];
#pragma unroll
    for (int j = 0; j < kRows; ++j)
        x[j] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(a + off + j * kTile));
#pragma unroll
    for (int j = 0; j < kRows; ++j)
        st_through(reinterpret_cast<f32x4 *>(b + off + j * kTile), x[j]);
}

__global__ __launch_bounds__(kLanes) void k_probe_five_stream(float *__restrict__ a,
                                                              float *__restrict__ b,
                                                              float *__restrict__ c,
                                                              const uint16_t *__restrict__ g,
                                                              uint16_t *__restrict__ h)
{
    const uint64_t off = (uint64_t)blockIdx.x * kTile + (uint64_t)threadIdx.x * 4;
    const u32x2 gv = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(g + off));
    f32x4 av = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(a + off));
    f32x4 bv = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(b + off));
    f32x4 cv = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(c + off));
    const float gs = __uint_as_float(gv.x << 16) + __uint_as_float(gv.y & 0xFFFF0000u);
    bv = bv * 0.9f + gs;
    cv = cv * 0.999f + gs * gs;
    av = av - bv * 1e-3f;
    u32x2 out;
    out.x = (__float_as_uint(av.x) >> 16) | (__float_as_uint(av.y) & 0xFFFF0000u);
    out.y = (__float_as_uint(av.z) >> 16) | (__float_as_uint(av.w) & 0xFFFF0000u);
    st_through(reinterpret_cast<f32x4 *>(a + off), av);
    st_through(reinterpret_cast<f32x4 *>(b + off), bv);
    st_through(reinterpret_cast<f32x4 *>(c + off), cv);
    st_through(reinterpret_cast<u32x2 *>(h + off), out);
}

inline bool misaligned16(const void *ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15u) != 0; }

}  // namespace

extern "C" lohan_status_t lohan_tuning_probe(int pattern, float *a, float *b, float *c,
                                             const void *g16, void *h16, uint64_t n,
                                             int waves_per_cu, hipStream_t stream)
{
    if (pattern < LOHAN_PROBE_READ || pattern > LOHAN_PROBE_MEMCPY || waves_per_cu < 0 ||
        waves_per_cu > 32)
        return LOHAN_ERR_ARG;
    const bool needs_a = pattern != LOHAN_PROBE_WRITE;
    const bool needs_b = pattern != LOHAN_PROBE_READ;
    const bool five = pattern == LOHAN_PROBE_FIVE_STREAM;
    if ((needs_a && a == nullptr) || (needs_b && b == nullptr) ||
        (five && (c == nullptr || g16 == nullptr || h16 == nullptr)))
        return LOHAN_ERR_NULL;
    if (misaligned16(a) || misaligned16(b) || misaligned16(c) || misaligned16(g16) ||
        misaligned16(h16))
        return LOHAN_ERR_ALIGN;
    const uint64_t tiles = n / kTile;
    if (tiles > 0x7FFFFFFFull) return LOHAN_ERR_ARG;
    if (tiles == 0) return LOHAN_OK;
    if (pattern == LOHAN_PROBE_MEMCPY)
        return hipMemcpyAsync(b, a, tiles * kTile * sizeof(float), hipMemcpyDeviceToDevice,
                              stream) == hipSuccess
                   ? LOHAN_OK
                   : LOHAN_ERR_HIP;

    int cus = 0;
    size_t lds_per_cu = 0;
    if (lohan_tuning_device_info(&cus, &lds_per_cu) != LOHAN_OK) return LOHAN_ERR_HIP;
    size_t lds = 0;
    if (waves_per_cu > 0 && waves_per_cu < 32) lds = lds_per_cu / (size_t)waves_per_cu / 256 * 256;
    const dim3 grid((uint32_t)tiles), wg(kLanes);
    const dim3 grid_rows((uint32_t)(tiles / kRows));        // whole groups of rows only
    if (pattern != LOHAN_PROBE_FIVE_STREAM && grid_rows.x == 0) return LOHAN_OK;
    const void *kernel = reinterpret_cast<const void *>(k_probe_five_stream);
    if (pattern == LOHAN_PROBE_READ) kernel = reinterpret_cast<const void *>(k_probe_read);
    if (pattern == LOHAN_PROBE_WRITE) kernel = reinterpret_cast<const void *>(k_probe_write);
    if (pattern == LOHAN_PROBE_COPY) kernel = reinterpret_cast<const void *>(k_probe_copy);
    if (lds > 64 * 1024 &&
        hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) !=
            hipSuccess)
        return LOHAN_ERR_HIP;
    switch (pattern) {
    case LOHAN_PROBE_READ:
        // The sink is written only if four loaded values sum to one particular number; it is a
        // itself, so the pattern needs no second array.
        hipLaunchKernelGGL(k_probe_read, grid_rows, wg, lds, stream, a, a);
        break;
    case LOHAN_PROBE_WRITE:
        hipLaunchKernelGGL(k_probe_write, grid_rows, wg, lds, stream, b);
        break;
    case LOHAN_PROBE_COPY:
        hipLaunchKernelGGL(k_probe_copy, grid_rows, wg, lds, stream, a, b);
        break;
    default:
        hipLaunchKernelGGL(k_probe_five_stream, grid, wg, lds, stream, a, b, c,
                           reinterpret_cast<const uint16_t *>(g16),
                           reinterpret_cast<uint16_t *>(h16));
        break;
    }
    return hipGetLastError() == hipSuccess ? LOHAN_OK : LOHAN_ERR_HIP;
}
