/*
 * lohan_swap_planner.h -- C ABI of the holistic traffic-aware activation swapping planner
 * (arxiv 2403.06504, Sec. IV-D): host-only, no GPU involved.
 *
 * Given per-layer recomputation cost and activation size and the profiled hardware numbers of
 * Sec. IV-B, the planner picks which layers' activations to swap out (the rest is recomputed) so
 * that the modelled iteration time T_iter = T_f + T_b (Eq. 1) is smallest:
 *   T_f = max( FLOP_f/THP_G,  A_G2M/BW_G,  2P/BW_G,  2P/BW_S2M + spill/BW_M2S )            (Eq. 4)
 *   T_b = max( (2 FLOP_f + FLOP_r)/THP_G,  2P/BW_G,  (2P + A_G2M)/BW_G,
 *              (14P + spill)/BW_S2M + 14P/BW_M2S )                                          (Eq. 5)
 *   spill = max(0, A_G2M - MEM_avail)  (Eq. 3: what main memory cannot hold goes to the far tier)
 * Layers are taken in order of offloading benefit OB = FLOP_layer / A_layer (Eq. 6), highest
 * first (ties keep the caller's order; a layer with A = 0 comes first), and added until T_iter
 * stops decreasing, but never stopping below A_interBlock (Algorithm 1).  T_iter is convex in
 * A_G2M along that order (Sec. IV-D), so the first non-improving layer marks the optimum.
 *
 * Units: sizes in bytes, P a parameter count, bandwidths in bytes/s, FLOP counts in operations,
 * THP_G in operations/s; all float64.  On this machine the "far tier" numbers are those of the
 * pinned-host path (BW_S2M = BW_M2S = the PCIe rate) or of whatever tier the caller models.
 */
#ifndef LOHAN_SWAP_PLANNER_H
#define LOHAN_SWAP_PLANNER_H

#include <stddef.h>
#include <stdint.h>

#include "lohan_adam.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    double flop;       /* FLOP_layer: operations to recompute this layer's activations */
    double act_bytes;  /* A_layer: bytes of this layer's activations */
} lohan_layer_t;

typedef struct {
    double thp_g;         /* THP_G   */
    double bw_g;          /* BW_G: unidirectional GPU <-> main memory */
    double bw_s2m;        /* BW_S2M: far tier -> main memory */
    double bw_m2s;        /* BW_M2S: main memory -> far tier */
    double params;        /* P       */
    double mem_avail;     /* MEM_avail: main memory left for activations, bytes */
    double flop_f;        /* FLOP_f: forward operations (backward is 2 FLOP_f) */
    double a_interblock;  /* A_interBlock: smallest safe swapped amount, bytes */
} lohan_swap_hw_t;

/* T_iter of Eq. 1-5 for a swapped amount a_g2m and a recomputation cost flop_r.  NaN if hw is
 * NULL or a rate in it is not > 0. */
double lohan_swap_iter_time(const lohan_swap_hw_t *hw, double a_g2m, double flop_r);

/*
 * FLOP_r as a function of the swapped amount (Eq. 7) and its derivative (Eq. 8): with the layers
 * taken by decreasing offloading benefit, a_g2m covers the first i layers and a fraction of
 * layer i+1, whose recomputation cost is taken proportional to the fraction left behind (the
 * paper's interpolation; no layer is really split):
 *     FLOP_r = flop_f - sum_{m<=i} FLOP_m - FLOP_{i+1} * (a_g2m - sum_{m<=i} A_m) / A_{i+1}
 *     dFLOP_r / dA_G2M = -OB_{i+1}
 * At a breakpoint the derivative is the right-hand one; at or beyond the sum of all A it is 0 and
 * FLOP_r = flop_f - sum of all FLOP.  Layers with A = 0 are swapped from the start.
 * layers[0..n): host, in.  flop_r, dflop_r: host, out (dflop_r may be NULL).
 * LOHAN_ERR_NULL for NULL layers (with n > 0) or flop_r; LOHAN_ERR_ARG for a negative or
 * non-finite a_g2m, flop_f or layer entry.
 */
lohan_status_t lohan_swap_recompute_flops(const lohan_layer_t *layers, size_t n, double flop_f,
                                          double a_g2m, double *flop_r, double *dflop_r);

/*
 * Algorithm 1.  layers[0..n): host, in; swap_list: host, out, room for n indices (indices into
 * layers, in swapping order); n_swapped, a_g2m, flop_r, t_iter: host, out (a_g2m, flop_r, t_iter
 * describe the returned swap list).  LOHAN_ERR_NULL for NULL pointers (layers may be NULL only if
 * n == 0), LOHAN_ERR_ARG if a rate is not > 0 or any size / count is negative or not finite.
 */
lohan_status_t lohan_plan_activation_swapping(const lohan_layer_t *layers, size_t n,
                                              const lohan_swap_hw_t *hw, uint32_t *swap_list,
                                              size_t *n_swapped, double *a_g2m, double *flop_r,
                                              double *t_iter);

#ifdef __cplusplus
}
#endif

#endif /* LOHAN_SWAP_PLANNER_H */
