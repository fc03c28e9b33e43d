// Offline budget allocation (sensitivity-conditioned token budgets, Eq. 1-5): host-only fp64
// arithmetic, a few dozen values per model.  Lives in the library so that the recipe a
// deployment consumes (per-layer keep ratios and integer budgets K_l) is produced by the same
// binary that later applies it.  No device work, no allocation beyond a small host scratch.
#include <algorithm>
#include <cmath>
#include <vector>
#include "../../include/quota.h"

namespace {

double percentile_linear(const std::vector<double> &sorted, double p)
{
    const double pos = p * (double)(sorted.size() - 1) / 100.0;
    const size_t lo = (size_t)std::floor(pos);
    const size_t hi = std::min(lo + 1, sorted.size() - 1);
    return sorted[lo] + (sorted[hi] - sorted[lo]) * (pos - (double)lo);
}

}  // namespace

extern "C" int quota_sensitivity(const double *diff_norm, const double *ref_norm, int n, double eta,
                                 double *S_out)
{
    if (!diff_norm || !ref_norm || !S_out) return QUOTA_ERR_NULL;
    if (n <= 0 || !(eta >= 0.0)) return QUOTA_ERR_INVALID_ARG;
    std::vector<double> ratio((size_t)n);
    for (int i = 0; i < n; ++i) {
        if (!(diff_norm[i] >= 0.0) || !(ref_norm[i] >= 0.0) || ref_norm[i] + eta == 0.0)
            return QUOTA_ERR_INVALID_ARG;
        ratio[i] = diff_norm[i] / (ref_norm[i] + eta);
    }
    std::sort(ratio.begin(), ratio.end());
    *S_out = (n & 1) ? ratio[n / 2] : 0.5 * (ratio[n / 2 - 1] + ratio[n / 2]);
    return QUOTA_OK;
}

extern "C" int quota_make_recipe(const double *S, int m, double tau, double p_min, int V0,
                                 double *s_norm_opt, double *pi_opt, double *r_out, int32_t *K_out)
{
    if (!S || !r_out || !K_out) return QUOTA_ERR_NULL;
    if (m <= 0 || !(tau > 0.0) || !(p_min >= 0.0) || !(p_min <= 1.0) || V0 < 0)
        return QUOTA_ERR_INVALID_ARG;
    for (int i = 0; i < m; ++i)
        if (!std::isfinite(S[i])) return QUOTA_ERR_INVALID_ARG;

    // Eq. 2: percentile clipping and normalisation
    std::vector<double> sorted(S, S + m), sn((size_t)m), pi((size_t)m);
    std::sort(sorted.begin(), sorted.end());
    const double p10 = percentile_linear(sorted, 10.0), p90 = percentile_linear(sorted, 90.0);
    for (int i = 0; i < m; ++i)
        sn[i] = p90 == p10 ? 0.5 : std::min(std::max((S[i] - p10) / (p90 - p10), 0.1), 0.9);

    // Eq. 3: temperature softmax of (1 - S~): less sensitive layers take a larger share of the drop
    double zmax = (1.0 - sn[0]) / tau, sum = 0.0;
    for (int i = 1; i < m; ++i) zmax = std::max(zmax, (1.0 - sn[i]) / tau);
    for (int i = 0; i < m; ++i) { pi[i] = std::exp((1.0 - sn[i]) / tau - zmax); sum += pi[i]; }
    for (int i = 0; i < m; ++i) pi[i] /= sum;

    // Eq. 4: non-increasing keep ratios with floor p_min; Eq. 5: K = ceil(r V0), where a product
    // that is an integer up to fp64 rounding is not bumped to the next one
    double acc = 0.0;
    for (int i = 0; i < m; ++i) {
        acc += (1.0 - p_min) * pi[i];
        r_out[i] = std::max(p_min, 1.0 - acc);
        K_out[i] = (int32_t)std::ceil(r_out[i] * (double)V0 - 1e-9);
        if (s_norm_opt) s_norm_opt[i] = sn[i];
        if (pi_opt) pi_opt[i] = pi[i];
    }
    return QUOTA_OK;
}

// GFLOPs ratio of a recipe (GFLOPs-estimation appendix): C_l(S) = 2 S (4 d^2 + 3 d F) + 4 S^2 d
// with S = T + V_l, 2 FLOPs per multiply-add, attention counted in full.
static double layer_cost(double S, double d, double F)
{
    return 2.0 * S * (4.0 * d * d + 3.0 * d * F) + 4.0 * S * S * d;
}

extern "C" int quota_gflops_ratio(const int32_t *V_hat, int L, int V0, int T, int d, int F, double F_vt,
                                  double F_pj, double *ratio_percent)
{
    if (!V_hat || !ratio_percent) return QUOTA_ERR_NULL;
    if (L <= 0 || V0 < 0 || T < 0 || d <= 0 || F <= 0 || !(F_vt >= 0.0) || !(F_pj >= 0.0))
        return QUOTA_ERR_INVALID_ARG;
    double pruned = F_vt + F_pj, base = F_vt + F_pj + (double)L * layer_cost((double)T + V0, d, F);
    for (int l = 0; l < L; ++l) {
        if (V_hat[l] < 0) return QUOTA_ERR_INVALID_ARG;
        pruned += layer_cost((double)T + V_hat[l], d, F);
    }
    if (base <= 0.0) return QUOTA_ERR_INVALID_ARG;
    *ratio_percent = 100.0 * pruned / base;
    return QUOTA_OK;
}
