/* A plain C client that runs the block step on the GPU through the C ABI with nothing but the HIP
 * runtime underneath (no Python, no torch): device memory from hipMalloc, the step on a stream of
 * its own, the results copied back and compared bit for bit with the CPU oracle, which this test
 * program links as well (the library itself never sees the oracle).  Built ahead of time by
 * __graft_entry__.build(); run by tests/test_gpu_c_client.py.  Usage: c_abi_gpu_client [n]. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "lohan_adam.h"

/* the oracle's C entry points (oracle/lohan_oracle.c) */
int lohan_oracle_adam_block_step(float *param_fp32, float *exp_avg, float *exp_avg_sq,
                                 const uint16_t *grad_fp16, uint16_t *param_bf16_out, uint64_t n,
                                 float lr, float beta1, float beta2, float eps, float weight_decay,
                                 int64_t step, float loss_scale, int l2_mode, int half_out,
                                 int nthreads);
double lohan_oracle_grad_sqnorm(const uint16_t *grad_fp16, uint64_t n, float loss_scale);

#define HIP_OK(x)                                                        \
    do {                                                                 \
        hipError_t e_ = (x);                                             \
        if (e_ != hipSuccess) {                                          \
            printf("HIP error %d at line %d\n", (int)e_, __LINE__);      \
            return 2;                                                    \
        }                                                                \
    } while (0)
#define LOHAN_OK_OR_DIE(x)                                               \
    do {                                                                 \
        lohan_status_t s_ = (x);                                         \
        if (s_ != LOHAN_OK) {                                            \
            printf("lohan status %d (%s) at line %d\n", (int)s_,         \
                   lohan_status_string(s_), __LINE__);                   \
            return 3;                                                    \
        }                                                                \
    } while (0)

/* Seeded test data: a 64-bit mixing function turned into uniform values (data only). */
static uint64_t mix(uint64_t x)
{
    x += 0x9E3779B97F4A7C15ull;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}
static float uniform(uint64_t i, uint64_t salt) /* in (-1, 1) */
{
    return (float)((double)(mix(i * 4 + salt) >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}

int main(int argc, char **argv)
{
    const uint64_t n = argc > 1 ? strtoull(argv[1], NULL, 10) : 1000003ull;
    const float lr = 1e-4f, b1 = 0.9f, b2 = 0.999f, eps = 1e-8f, wd = 0.01f, S = 65536.0f;
    float *p = malloc(n * 4), *m = malloc(n * 4), *v = malloc(n * 4);
    float *gp = malloc(n * 4), *gm = malloc(n * 4), *gv = malloc(n * 4);
    uint16_t *g = malloc(n * 2), *h = malloc(n * 2), *gh = malloc(n * 2);
    if (!p || !m || !v || !gp || !gm || !gv || !g || !h || !gh) return 1;
    for (uint64_t i = 0; i < n; ++i) {
        p[i] = 0.05f * uniform(i, 0);
        m[i] = 3e-4f * uniform(i, 1);
        v[i] = 2e-7f * fabsf(uniform(i, 2));
        /* a finite binary16 pattern of moderate magnitude: exponent field 1..26, any mantissa */
        const uint64_t r = mix(i * 4 + 3);
        g[i] = (uint16_t)(((r & 1) << 15) | ((1 + (r >> 1) % 26) << 10) | ((r >> 8) & 0x3FF));
        h[i] = 0xC040;
    }

    float *dp, *dm, *dv;
    void *dg, *dh, *ws;
    uint32_t *dflag;
    double *dsq;
    hipStream_t stream;
    HIP_OK(hipSetDevice(0));
    HIP_OK(hipStreamCreateWithFlags(&stream, hipStreamNonBlocking));
    HIP_OK(hipMalloc((void **)&dp, n * 4 + 16));
    HIP_OK(hipMalloc((void **)&dm, n * 4 + 16));
    HIP_OK(hipMalloc((void **)&dv, n * 4 + 16));
    HIP_OK(hipMalloc(&dg, n * 2 + 16));
    HIP_OK(hipMalloc(&dh, n * 2 + 16));
    HIP_OK(hipMalloc(&ws, lohan_workspace_bytes()));
    HIP_OK(hipMalloc((void **)&dflag, 4));
    HIP_OK(hipMalloc((void **)&dsq, 8));
    HIP_OK(hipMemcpy(dp, p, n * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(dm, m, n * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(dv, v, n * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(dg, g, n * 2, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(dh, h, n * 2, hipMemcpyHostToDevice));
    LOHAN_OK_OR_DIE(lohan_workspace_init(ws, lohan_workspace_bytes(), stream));

    /* three chained steps on the device, flag/norm pass then the prechecked update */
    double sq = -1.0;
    uint32_t flag = 9;
    for (int64_t t = 100; t < 103; ++t) {
        LOHAN_OK_OR_DIE(lohan_grad_sqnorm(dg, n, S, dsq, dflag, ws, lohan_workspace_bytes(),
                                          stream));
        LOHAN_OK_OR_DIE(lohan_adam_block_step(dp, dm, dv, dg, dh, n, lr, b1, b2, eps, wd, t, S,
                                              dflag, LOHAN_FLAG_PRECHECKED, NULL, 0, stream));
    }
    HIP_OK(hipStreamSynchronize(stream));
    HIP_OK(hipMemcpy(&flag, dflag, 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(&sq, dsq, 8, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(gp, dp, n * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(gm, dm, n * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(gv, dv, n * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(gh, dh, n * 2, hipMemcpyDeviceToHost));

    for (int64_t t = 100; t < 103; ++t)
        if (lohan_oracle_adam_block_step(p, m, v, g, h, n, lr, b1, b2, eps, wd, t, S, 0, 0, 8) != 0)
            return 4;
    const double want_sq = lohan_oracle_grad_sqnorm(g, n, S);
    const int same = memcmp(gp, p, n * 4) == 0 && memcmp(gm, m, n * 4) == 0 &&
                     memcmp(gv, v, n * 4) == 0 && memcmp(gh, h, n * 2) == 0;
    printf("flag %u state_bit_identical %d sqnorm_rel_err %.3e\n", flag, same,
           fabs(sq - want_sq) / want_sq);

    /* a fourth step in ONE launch, where the block is small enough for it */
    uint64_t small_max = 0;
    LOHAN_OK_OR_DIE(lohan_adam_small_block_max_n(&small_max));
    if (n <= small_max) {
        LOHAN_OK_OR_DIE(lohan_adam_small_block_step(dp, dm, dv, dg, dh, n, lr, b1, b2, eps, wd,
                                                    103, S, dsq, dflag, 0, ws,
                                                    lohan_workspace_bytes(), stream));
        HIP_OK(hipStreamSynchronize(stream));
        HIP_OK(hipMemcpy(&flag, dflag, 4, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(&sq, dsq, 8, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(gp, dp, n * 4, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(gm, dm, n * 4, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(gv, dv, n * 4, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(gh, dh, n * 2, hipMemcpyDeviceToHost));
        if (lohan_oracle_adam_block_step(p, m, v, g, h, n, lr, b1, b2, eps, wd, 103, S, 0, 0,
                                         8) != 0)
            return 5;
        printf("small_block flag %u state_bit_identical %d sqnorm_rel_err %.3e\n", flag,
               memcmp(gp, p, n * 4) == 0 && memcmp(gm, m, n * 4) == 0 &&
                   memcmp(gv, v, n * 4) == 0 && memcmp(gh, h, n * 2) == 0,
               fabs(sq - want_sq) / want_sq);
    } else {
        printf("small_block skipped: n exceeds %llu\n", (unsigned long long)small_max);
    }

    /* an overflowing block: flag 1, state untouched (the self-checking step this time) */
    const uint16_t inf16 = 0x7C00;
    HIP_OK(hipMemcpy((char *)dg + 2 * (n / 2), &inf16, 2, hipMemcpyHostToDevice));
    LOHAN_OK_OR_DIE(lohan_adam_block_step(dp, dm, dv, dg, dh, n, lr, b1, b2, eps, wd, 104, S,
                                          dflag, 0, ws, lohan_workspace_bytes(), stream));
    HIP_OK(hipStreamSynchronize(stream));
    HIP_OK(hipMemcpy(&flag, dflag, 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(gp, dp, n * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(gh, dh, n * 2, hipMemcpyDeviceToHost));
    printf("overflow_flag %u untouched %d\n", flag,
           memcmp(gp, p, n * 4) == 0 && memcmp(gh, h, n * 2) == 0);

    HIP_OK(hipFree(dp)); HIP_OK(hipFree(dm)); HIP_OK(hipFree(dv)); HIP_OK(hipFree(dg));
    HIP_OK(hipFree(dh)); HIP_OK(hipFree(ws)); HIP_OK(hipFree(dflag)); HIP_OK(hipFree(dsq));
    HIP_OK(hipStreamDestroy(stream));
    free(p); free(m); free(v); free(gp); free(gm); free(gv); free(g); free(h); free(gh);
    return 0;
}
