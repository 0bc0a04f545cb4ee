/* A plain C11 client of the library: proves that the headers are valid C and that the entry
 * points link and run from C.  Host-only calls, so no GPU is needed.  Built and run by
 * tests/test_abi_host.py. */
#include <math.h>
#include <stdio.h>
#include <string.h>

#include "lohan_adam.h"
#include "lohan_swap_planner.h"

int main(void)
{
    printf("workspace_bytes %zu\n", lohan_workspace_bytes());
    printf("status_3 %s\n", lohan_status_string(LOHAN_ERR_ARG));
    printf("clip %.4f\n", (double)lohan_clip_loss_scale(5.25, 1024.0f, 1.0f));

    lohan_block_offsets_t offs[3];
    size_t slab = 0, align = 0;
    uint32_t group = 0;
    lohan_status_t st = lohan_model_placement(314572800ull, 3, offs, &slab, &align, &group);
    printf("placement %d group %u lane %zu align %zu\n", (int)st, group,
           offs[0].exp_avg - offs[0].param_fp32, align);

    /* validation happens before any launch, so this returns without touching a device */
    st = lohan_adam_block_step(NULL, NULL, NULL, NULL, NULL, 16, 1e-4f, 0.9f, 0.999f, 1e-8f, 0.01f,
                               1, 1024.0f, NULL, 0, NULL, 0, NULL);
    printf("null_step %d\n", (int)st);

    lohan_layer_t layers[3] = {{100.0, 100.0}, {300.0, 10.0}, {200.0, 20.0}};
    lohan_swap_hw_t hw = {100.0, 10.0, 5.0, 5.0, 0.1, 1e9, 600.0, 0.0};
    uint32_t swap_list[3];
    size_t n_swapped = 0;
    double a_g2m = 0, flop_r = 0, t_iter = 0, slope = 0;
    st = lohan_plan_activation_swapping(layers, 3, &hw, swap_list, &n_swapped, &a_g2m, &flop_r,
                                        &t_iter);
    printf("plan %d n %zu first %u a %.1f f %.1f t %.2f\n", (int)st, n_swapped, swap_list[0],
           a_g2m, flop_r, t_iter);
    st = lohan_swap_recompute_flops(layers, 3, 600.0, 20.0, &flop_r, &slope);
    printf("flops %d %.1f %.1f\n", (int)st, flop_r, slope);
    return 0;
}
