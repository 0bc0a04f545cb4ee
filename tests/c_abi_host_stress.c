/* Host-side stress of the library for a sanitizer build (AddressSanitizer + UBSan on the host
 * code only; no GPU is touched): many planner instances, many placements, and the validation
 * paths of the entry points that take host arrays.  Built and run by tests/test_abi_host.py;
 * prints "ok <checksum>" on success, any sanitizer report aborts the run. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include "lohan_adam.h"
#include "lohan_swap_planner.h"

static uint64_t state = 88172645463325252ull;
static double uniform(void) /* xorshift64, in [0, 1) */
{
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return (double)(state >> 11) / 9007199254740992.0;
}

int main(void)
{
    double checksum = 0.0;
    /* planner: instances of 0..2000 layers, ties and empty activations included */
    for (int trial = 0; trial < 200; ++trial) {
        size_t n = (size_t)(uniform() * (trial % 10 == 0 ? 2000 : 60));
        lohan_layer_t *layers = malloc(sizeof(lohan_layer_t) * (n ? n : 1));
        uint32_t *list = malloc(sizeof(uint32_t) * (n ? n : 1));
        double total_flop = 0.0, total_act = 0.0;
        for (size_t i = 0; i < n; ++i) {
            layers[i].flop = 1e9 * (1.0 + 99.0 * uniform());
            layers[i].act_bytes = i % 17 == 3 ? 0.0 : 1e6 * (1.0 + 99.0 * uniform());
            if (i % 13 == 5 && i > 0) layers[i] = layers[i - 1];
            total_flop += layers[i].flop;
            total_act += layers[i].act_bytes;
        }
        lohan_swap_hw_t hw = {pow(10.0, 11 + 3 * uniform()), pow(10.0, 9 + 2 * uniform()),
                              pow(10.0, 9 + 1.5 * uniform()), pow(10.0, 9 + 1.5 * uniform()),
                              pow(10.0, 6 + 3 * uniform()), uniform() * total_act,
                              total_flop * (1.0 + 0.5 * uniform()), uniform() * total_act};
        size_t count = 0;
        double a = 0, f = 0, t = 0, slope = 0;
        if (lohan_plan_activation_swapping(layers, n, &hw, list, &count, &a, &f, &t) != LOHAN_OK)
            return 1;
        if (count > n || !(t > 0.0) || a < 0.0 || a > total_act * (1 + 1e-12)) return 2;
        for (size_t k = 0; k < count; ++k)
            if (list[k] >= n) return 3;
        if (lohan_swap_recompute_flops(layers, n, hw.flop_f, uniform() * total_act * 1.2, &f,
                                       &slope) != LOHAN_OK)
            return 4;
        if (slope > 0.0 || f > hw.flop_f * (1 + 1e-12)) return 5;
        checksum += t + a * 1e-9 + (double)count;
        free(layers);
        free(list);
    }
    /* placement: many sizes and block counts; offsets stay inside the slab and do not collide */
    for (int trial = 0; trial < 300; ++trial) {
        uint64_t n = (uint64_t)(pow(2.0, 10 + 22 * uniform()));
        uint32_t blocks = (uint32_t)(1 + uniform() * 70);
        lohan_block_offsets_t *offs = malloc(sizeof(lohan_block_offsets_t) * blocks);
        size_t slab = 0, align = 0;
        uint32_t group = 0;
        if (lohan_model_placement(n, blocks, offs, &slab, &align, &group) != LOHAN_OK) return 6;
        if (group < 1 || align == 0) return 7;
        for (uint32_t b = 0; b < blocks; ++b) {
            if (offs[b].param_fp32 + 4 * n > slab || offs[b].exp_avg + 4 * n > slab ||
                offs[b].exp_avg_sq + 4 * n > slab || offs[b].grad_fp16 + 2 * n > slab ||
                offs[b].param_bf16 + 2 * n > slab)
                return 8;
            if (b > 0 && offs[b].param_fp32 < offs[b - 1].param_fp32 + 4 * n &&
                offs[b - 1].param_fp32 < offs[b].param_fp32 + 4 * n)
                return 9;
        }
        checksum += (double)slab * 1e-12 + group;
        free(offs);
    }
    /* entry points that read host arrays, on their validation paths */
    lohan_block_t two[2] = {{(float *)0x1000, (float *)0x2000, (float *)0x3000, (void *)0x4000,
                             (void *)0x5000, 16},
                            {NULL, (float *)0x7000, (float *)0x8000, (void *)0x9000,
                             (void *)0xA000, 16}};
    if (lohan_adam_multi_block_step(two, 2, 1e-4f, 0.9f, 0.999f, 1e-8f, 0.01f, 1, 1024.0f, 0.0f,
                                    (uint32_t *)0xB000, NULL, 0, (void *)0xC000,
                                    lohan_workspace_bytes(), NULL) != LOHAN_ERR_NULL)
        return 10;
    lohan_ring_slot_t slots[3] = {
        {(float *)0x1000, (float *)0x2000, (float *)0x3000, (void *)0x4000, 16},
        {(float *)0x5000, (float *)0x6000, (float *)0x7000, (void *)0x8000, 16},
        {(float *)0x9000, (float *)0xA000, (float *)0xB004, (void *)0xC000, 16}};
    if (lohan_ring_init((void *)0x10000, lohan_ring_bytes(2, 1), slots, 2, 1) != LOHAN_ERR_ALIGN)
        return 11;
    slots[2].exp_avg_sq = (float *)0xB000;
    slots[2].n = 17;                                    /* no spare of the blocks' length */
    if (lohan_ring_init((void *)0x10000, lohan_ring_bytes(2, 1), slots, 2, 1) != LOHAN_ERR_ARG)
        return 12;
    /* per-tensor placement: many shapes, every array inside the slab and disjoint */
    for (int trial = 0; trial < 200; ++trial) {
        uint64_t lengths[24];
        lohan_block_offsets_t off[24];
        const uint32_t count = 1 + (uint32_t)(trial % 24);
        for (uint32_t i = 0; i < count; ++i)
            lengths[i] = (uint64_t)((trial * 2654435761u + i * 40503u) % 97) *
                             (trial % 3 == 0 ? 3000001ull : 20011ull) +
                         (trial % 5 == 0 && i == 0 ? (1ull << 27) : 0);
        size_t bytes = 0, align = 0;
        if (lohan_tensor_placement(lengths, count, off, &bytes, &align) != LOHAN_OK) return 13;
        for (uint32_t i = 0; i < count; ++i) {
            if (off[i].param_fp32 + lengths[i] * 4 > bytes || off[i].param_bf16 + lengths[i] * 2 > bytes)
                return 14;
            checksum += (double)off[i].exp_avg_sq * 1e-12;
        }
    }
    printf("ok %.6e\n", checksum);
    return 0;
}
