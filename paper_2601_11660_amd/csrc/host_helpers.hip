// Host-side helpers of the deployment flow that need no GPU: folding batch norm, bias and
// the binary activation of a layer into the integer threshold of Algorithm 1 (Sec. 3.2.2),
// and the cost-aware masking priority of Sec. 3.1.2.
#include <algorithm>
#include <cmath>
#include <numeric>
#include <vector>
#include "mbu_internal.h"

using namespace mbu;

extern "C" {

// Sec. 3.2.2: the threshold covers batch norm, bias and the binary activation.  With the
// integer sum acc of a layer, s = sqrt(var + eps):
//   bit = ( gamma * (acc + bias - mean) / s + beta >= 0 ).
//   gamma > 0:  acc >= t,  t = mean - bias - beta * s / gamma   ->  thresh = ceil(t)
//   gamma < 0:  acc <= t  <=>  -acc >= -t                      ->  flip = 1, thresh = ceil(-t)
//               (the caller negates that channel's weights before packing, which negates acc)
//   gamma = 0:  the bit is the constant (beta >= 0)             ->  thresh = -+(fan_in + 1)
// acc is an integer of magnitude <= fan_in, so thresholds are clamped to +-(fan_in + 1).
int mbu_fold_batchnorm(const double *gamma, const double *beta, const double *mean,
                       const double *var, double eps, const double *bias, int C, int fan_in,
                       int32_t *thresh, int8_t *flip)
{
    const char *fn = "mbu_fold_batchnorm";
    if (!gamma || !beta || !mean || !var || !thresh || !flip)
        return fail(MBU_ERR_NULL, "%s: a required array is NULL", fn);
    if (C <= 0 || fan_in <= 0 || fan_in > (1 << 22))
        return fail(MBU_ERR_SHAPE, "%s: need C > 0 and 0 < fan_in <= 2^22 (C=%d fan_in=%d)", fn, C, fan_in);
    if (!(eps >= 0.0)) return fail(MBU_ERR_ARG, "%s: eps must be non-negative", fn);
    const double lim = (double)fan_in + 1.0;
    for (int c = 0; c < C; ++c) {
        const double v = var[c] + eps;
        if (!(v > 0.0) || !std::isfinite(gamma[c]) || !std::isfinite(beta[c]) ||
            !std::isfinite(mean[c]) || !std::isfinite(v) || (bias && !std::isfinite(bias[c])))
            return fail(MBU_ERR_ARG, "%s: channel %d has a non-finite parameter or var + eps <= 0", fn, c);
        const double b = bias ? bias[c] : 0.0;
        double t;
        flip[c] = 0;
        if (gamma[c] == 0.0) {
            t = beta[c] >= 0.0 ? -lim : lim;
        } else {
            t = mean[c] - b - beta[c] * std::sqrt(v) / gamma[c];
            if (gamma[c] < 0.0) {
                flip[c] = 1;
                t = -t;
            }
            t = std::ceil(t);
        }
        thresh[c] = (int32_t)std::min(lim, std::max(-lim, t));
    }
    return MBU_OK;
}

// Sec. 3.1.2: s_l = w_op * ops_l^ + w_param * params_l^ with both counts normalised to [0, 1]
// over the layers (min-max) and w_op + w_param = 1; layers are masked in ascending score order.
// `order` receives the layer indices from the lowest score (first to be masked) to the highest;
// ties keep the lower index first.
int mbu_cost_rank(const double *n_ops, const double *n_params, int L, double w_op, double *score,
                  int *order)
{
    const char *fn = "mbu_cost_rank";
    if (!n_ops || !n_params || !score || !order) return fail(MBU_ERR_NULL, "%s: a required array is NULL", fn);
    if (L <= 0) return fail(MBU_ERR_SHAPE, "%s: need at least one layer", fn);
    if (!(w_op >= 0.0 && w_op <= 1.0)) return fail(MBU_ERR_ARG, "%s: w_op must lie in [0, 1]", fn);
    for (int l = 0; l < L; ++l)
        if (!(n_ops[l] >= 0.0) || !(n_params[l] >= 0.0) || !std::isfinite(n_ops[l]) || !std::isfinite(n_params[l]))
            return fail(MBU_ERR_ARG, "%s: layer %d has a negative or non-finite count", fn, l);
    auto normalise = [L](const double *v, std::vector<double> &out) {
        const double lo = *std::min_element(v, v + L), hi = *std::max_element(v, v + L);
        for (int l = 0; l < L; ++l) out[l] = hi > lo ? (v[l] - lo) / (hi - lo) : 0.0;
    };
    std::vector<double> o(L), p(L);
    normalise(n_ops, o);
    normalise(n_params, p);
    for (int l = 0; l < L; ++l) score[l] = w_op * o[l] + (1.0 - w_op) * p[l];
    std::iota(order, order + L, 0);
    std::stable_sort(order, order + L, [score](int a, int b) { return score[a] < score[b]; });
    return MBU_OK;
}

}  // extern "C"
