// Holistic traffic-aware activation swapping planner (Sec. IV-D): iteration-time model of
// Eq. 1-5 and the greedy search of Algorithm 1.  Host code only; see include/lohan_swap_planner.h.

#include <algorithm>
#include <cmath>
#include <limits>
#include <numeric>
#include <vector>

#include "lohan_swap_planner.h"

namespace {

bool rates_ok(const lohan_swap_hw_t *hw)
{
    return hw != nullptr && hw->thp_g > 0.0 && hw->bw_g > 0.0 && hw->bw_s2m > 0.0 &&
           hw->bw_m2s > 0.0 && std::isfinite(hw->thp_g) && std::isfinite(hw->bw_g) &&
           std::isfinite(hw->bw_s2m) && std::isfinite(hw->bw_m2s);
}

bool nonneg_finite(double x) { return std::isfinite(x) && x >= 0.0; }

// T_f (Eq. 4) + T_b (Eq. 5); each stage is as long as its slowest resource.
double iter_time(const lohan_swap_hw_t &hw, double a_g2m, double flop_r)
{
    const double spill = std::max(0.0, a_g2m - hw.mem_avail);          // Eq. 3
    const double p2 = 2.0 * hw.params, p14 = 14.0 * hw.params;
    const double t_f = std::max(std::max(hw.flop_f / hw.thp_g, a_g2m / hw.bw_g),
                                std::max(p2 / hw.bw_g, p2 / hw.bw_s2m + spill / hw.bw_m2s));
    const double t_b = std::max(std::max((2.0 * hw.flop_f + flop_r) / hw.thp_g, p2 / hw.bw_g),
                                std::max((p2 + a_g2m) / hw.bw_g,
                                         (p14 + spill) / hw.bw_s2m + p14 / hw.bw_m2s));
    return t_f + t_b;
}

// Indices of the layers by decreasing offloading benefit OB = FLOP/A (Eq. 6); ties keep the
// caller's order, a layer without activation bytes comes first.
std::vector<uint32_t> benefit_order(const lohan_layer_t *layers, size_t n)
{
    std::vector<uint32_t> order(n);
    std::iota(order.begin(), order.end(), 0u);
    auto benefit = [&](uint32_t i) {
        return layers[i].act_bytes == 0.0 ? std::numeric_limits<double>::infinity()
                                          : layers[i].flop / layers[i].act_bytes;
    };
    std::stable_sort(order.begin(), order.end(),
                     [&](uint32_t a, uint32_t b) { return benefit(a) > benefit(b); });
    return order;
}

}  // namespace

extern "C" {

double lohan_swap_iter_time(const lohan_swap_hw_t *hw, double a_g2m, double flop_r)
{
    if (!rates_ok(hw)) return std::numeric_limits<double>::quiet_NaN();
    return iter_time(*hw, a_g2m, flop_r);
}

lohan_status_t lohan_swap_recompute_flops(const lohan_layer_t *layers, size_t n, double flop_f,
                                          double a_g2m, double *flop_r, double *dflop_r)
{
    if (flop_r == nullptr || (n != 0 && layers == nullptr)) return LOHAN_ERR_NULL;
    if (!nonneg_finite(flop_f) || !nonneg_finite(a_g2m) || n > 0xFFFFFFFFull) return LOHAN_ERR_ARG;
    for (size_t i = 0; i < n; ++i)
        if (!nonneg_finite(layers[i].flop) || !nonneg_finite(layers[i].act_bytes))
            return LOHAN_ERR_ARG;
    double left = a_g2m;             // swapped bytes not yet assigned to a layer
    double f = flop_f;
    double slope = 0.0;
    for (uint32_t idx : benefit_order(layers, n)) {
        const double a = layers[idx].act_bytes;
        if (a <= left) {             // wholly swapped (this also takes every layer with A = 0)
            f -= layers[idx].flop;
            left -= a;
            continue;
        }
        f -= layers[idx].flop * (left / a);      // Eq. 7: the partly swapped layer
        slope = -(layers[idx].flop / a);         // Eq. 8
        break;
    }
    *flop_r = f;
    if (dflop_r != nullptr) *dflop_r = slope;
    return LOHAN_OK;
}

lohan_status_t lohan_plan_activation_swapping(const lohan_layer_t *layers, size_t n,
                                              const lohan_swap_hw_t *hw, uint32_t *swap_list,
                                              size_t *n_swapped, double *a_g2m, double *flop_r,
                                              double *t_iter)
{
    if (hw == nullptr || n_swapped == nullptr || a_g2m == nullptr || flop_r == nullptr ||
        t_iter == nullptr || (n != 0 && (layers == nullptr || swap_list == nullptr)))
        return LOHAN_ERR_NULL;
    if (!rates_ok(hw) || !nonneg_finite(hw->params) || !nonneg_finite(hw->mem_avail) ||
        !nonneg_finite(hw->flop_f) || !nonneg_finite(hw->a_interblock) || n > 0xFFFFFFFFull)
        return LOHAN_ERR_ARG;
    for (size_t i = 0; i < n; ++i)
        if (!nonneg_finite(layers[i].flop) || !nonneg_finite(layers[i].act_bytes))
            return LOHAN_ERR_ARG;

    // Every candidate answer is a prefix of the benefit order.  Evaluate them all: swapped bytes,
    // recomputation left (Eq. 7 at a breakpoint) and modelled iteration time (Eq. 1-5) of the
    // first k layers, k = 0..n.
    const std::vector<uint32_t> order = benefit_order(layers, n);
    std::vector<double> swapped(n + 1, 0.0), saved(n + 1, 0.0), time(n + 1, 0.0);
    for (size_t k = 1; k <= n; ++k) {
        swapped[k] = swapped[k - 1] + layers[order[k - 1]].act_bytes;
        saved[k] = saved[k - 1] + layers[order[k - 1]].flop;
    }
    for (size_t k = 0; k <= n; ++k) time[k] = iter_time(*hw, swapped[k], hw->flop_f - saved[k]);

    // Algorithm 1 (Sec. IV-D) keeps extending the prefix until one fails to beat every shorter
    // non-empty prefix while already holding at least A_interBlock bytes; the prefix before that
    // one is the plan (T_iter is convex along the order, so this is where it turns).
    size_t count = n;
    double best = std::numeric_limits<double>::infinity();
    for (size_t k = 1; k <= n; ++k) {
        if (swapped[k] >= hw->a_interblock && time[k] >= best) {
            count = k - 1;
            break;
        }
        best = std::min(best, time[k]);
    }
    for (size_t k = 0; k < count; ++k) swap_list[k] = order[k];
    *n_swapped = count;
    *a_g2m = swapped[count];
    *flop_r = hw->flop_f - saved[count];
    *t_iter = time[count];
    return LOHAN_OK;
}

}  // extern "C"
