// Four-term wave cost model (paper Eq. 6, Sec. 4.2): least-squares fit per configuration
// and the runtime argmin over configurations.  Host code only.
//
//   T_hat(c) = a + b * w + c * m + d * l,   g = (sum_e ceil(n_e / bm_c)) * ntiles_c
//   w = g/W as printed, or max(g/W, 1) (RAMP_CM_WAVE_FLOOR: a grid below one wave still costs one wave);
//   m = g as printed, or the number of distinct weight tiles (active experts * ntiles_c) when the
//   per-block traffic term is made cache aware (RAMP_CM_DISTINCT_TILES);
//   l = ln(g + 1) as printed (used only in the sub-wave case), or the number of routed pairs
//   (RAMP_CM_PAIRS: the work that does not depend on the tiling).
//   RAMP_CM_ROUNDS: the g of the wave term counts the M-tiles of each launch in whole hand-out rounds of the
//   launch's workgroup -> tile map (persistent kernels; g_r = g for the others).
//
// The columns g/W and g of the design matrix are proportional for a fixed configuration, so
// the literal four-column system is rank deficient.  The fit returns the minimum-norm
// least-squares solution (pseudo-inverse through a one-sided Jacobi SVD, singular values below
// eps*max(n,4)*sigma_max treated as zero); every solution of the system gives the same
// predictions, which is all the selection uses.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

#include "ramp.h"

namespace ramp {
void set_error(const char *fmt, ...);
}

namespace {

constexpr int kMaxTerms = 5;

// Minimum-norm least squares  min |A x - t|  for an n x m matrix (column major, m <= kMaxTerms).
void lstsq_min_norm(std::vector<double> A, int n, int m, const double *t, double *x)
{
    double V[kMaxTerms][kMaxTerms] = {};
    for (int j = 0; j < m; ++j) V[j][j] = 1.0;
    auto col = [&](int j) { return A.data() + (size_t)j * n; };
    for (int sweep = 0; sweep < 60; ++sweep) {
        double off = 0.0;
        for (int p = 0; p < m - 1; ++p)
            for (int q = p + 1; q < m; ++q) {
                double app = 0, aqq = 0, apq = 0;
                double *cp = col(p), *cq = col(q);
                for (int i = 0; i < n; ++i) {
                    app += cp[i] * cp[i];
                    aqq += cq[i] * cq[i];
                    apq += cp[i] * cq[i];
                }
                if (apq == 0.0 || app == 0.0 || aqq == 0.0) continue;
                double rel = std::fabs(apq) / std::sqrt(app * aqq);
                off = std::max(off, rel);
                if (rel < 1e-16) continue;
                double zeta = (aqq - app) / (2.0 * apq);
                double tn = (zeta >= 0 ? 1.0 : -1.0) / (std::fabs(zeta) + std::sqrt(1.0 + zeta * zeta));
                double cs = 1.0 / std::sqrt(1.0 + tn * tn), sn = cs * tn;
                for (int i = 0; i < n; ++i) {
                    double vp = cp[i], vq = cq[i];
                    cp[i] = cs * vp - sn * vq;
                    cq[i] = sn * vp + cs * vq;
                }
                for (int i = 0; i < m; ++i) {
                    double vp = V[i][p], vq = V[i][q];
                    V[i][p] = cs * vp - sn * vq;
                    V[i][q] = sn * vp + cs * vq;
                }
            }
        if (off < 1e-15) break;
    }
    double sigma[kMaxTerms], smax = 0.0;
    for (int j = 0; j < m; ++j) {
        double s = 0;
        for (int i = 0; i < n; ++i) s += col(j)[i] * col(j)[i];
        sigma[j] = std::sqrt(s);
        smax = std::max(smax, sigma[j]);
    }
    const double cut = 2.220446049250313e-16 * std::max(n, m) * smax;
    for (int j = 0; j < m; ++j) x[j] = 0.0;
    for (int j = 0; j < m; ++j) {
        if (sigma[j] <= cut || sigma[j] == 0.0) continue;
        double ut = 0;
        for (int i = 0; i < n; ++i) ut += col(j)[i] * t[i];
        double coef = ut / (sigma[j] * sigma[j]);  // (u_j . t) / sigma_j with u_j = A_j / sigma_j
        for (int i = 0; i < m; ++i) x[i] += V[i][j] * coef;
    }
}

}  // namespace

static const int kAllFlags = RAMP_CM_RELATIVE | RAMP_CM_DISTINCT_TILES | RAMP_CM_WAVE_FLOOR | RAMP_CM_PAIRS | RAMP_CM_ROUNDS;

// n_theta = 4: Eq. 6; n_theta = 5: the ablation of Sec. 5.3 with a fifth column (g/W)^2, i.e. g^2 up to the
// configuration's constant W^2 (kept of order one for the conditioning of the system).
static int fit_impl(int n_cfg, const int32_t *wave_cap, int n_pts, const int64_t *grid, const int64_t *grid_rounds,
                    const int64_t *distinct, const int64_t *pairs, const double *time_us, int flags, float *theta,
                    int n_theta)
{
    const bool use_rounds = (flags & RAMP_CM_ROUNDS) != 0;
    const bool use_distinct = (flags & RAMP_CM_DISTINCT_TILES) != 0;
    const bool relative = (flags & RAMP_CM_RELATIVE) != 0;
    const bool wave_floor = (flags & RAMP_CM_WAVE_FLOOR) != 0;
    const bool use_pairs = (flags & RAMP_CM_PAIRS) != 0;
    if (n_cfg < 0 || n_pts <= 0 || !wave_cap || !grid || !time_us || !theta || (use_distinct && !distinct) ||
        (use_pairs && !pairs) || (use_rounds && !grid_rounds) || (flags & ~kAllFlags) || (n_theta != 4 && n_theta != 5)) {
        ramp::set_error("cost_model_fit: bad argument");
        return RAMP_EINVAL;
    }
    std::vector<double> A((size_t)kMaxTerms * n_pts), sorted_g(n_pts), rhs(n_pts);
    for (int c = 0; c < n_cfg; ++c) {
        const int64_t *g = grid + (size_t)c * n_pts;
        const double *t = time_us + (size_t)c * n_pts;
        const double W = (double)wave_cap[c];
        if (W <= 0) {
            ramp::set_error("cost_model_fit: wave_cap[%d] <= 0", c);
            return RAMP_EINVAL;
        }
        for (int i = 0; i < n_pts; ++i) sorted_g[i] = (double)g[i];
        std::sort(sorted_g.begin(), sorted_g.end());
        // fourth column: the log term only when the lower median grid is in the sub-wave region; the pair count always
        const bool use_fourth = use_pairs || sorted_g[(n_pts - 1) / 2] < W;
        const int m = (use_fourth ? 4 : 3) + (n_theta == 5 ? 1 : 0);
        const int quad_col = use_fourth ? 4 : 3;  // where the quadratic column sits in the system that is solved
        for (int i = 0; i < n_pts; ++i) {
            const double gi = (double)g[i];
            const double mi = use_distinct ? (double)distinct[(size_t)c * n_pts + i] : gi;
            double scale = 1.0;
            if (relative) {
                if (!(t[i] > 0.0)) {
                    ramp::set_error("cost_model_fit: relative fit needs positive times (config %d point %d)", c, i);
                    return RAMP_EINVAL;
                }
                scale = 1.0 / t[i];
            }
            A[0 * (size_t)n_pts + i] = 1.0 * scale;
            const double wi = (use_rounds ? (double)grid_rounds[(size_t)c * n_pts + i] : gi) / W;
            A[1 * (size_t)n_pts + i] = ((wave_floor && wi < 1.0) ? 1.0 : wi) * scale;
            A[2 * (size_t)n_pts + i] = mi * scale;
            A[3 * (size_t)n_pts + i] = (use_pairs ? (double)pairs[i] : std::log(gi + 1.0)) * scale;
            if (n_theta == 5) A[(size_t)quad_col * n_pts + i] = (gi / W) * (gi / W) * scale;
            rhs[i] = t[i] * scale;
        }
        double x[kMaxTerms] = {0, 0, 0, 0, 0};
        lstsq_min_norm(std::vector<double>(A.begin(), A.begin() + (size_t)m * n_pts), n_pts, m, rhs.data(), x);
        float *th = theta + (size_t)c * n_theta;
        for (int j = 0; j < 3; ++j) th[j] = (float)x[j];
        th[3] = use_fourth ? (float)x[3] : 0.0f;
        if (n_theta == 5) th[4] = (float)x[quad_col];
    }
    return RAMP_OK;
}

extern "C" int ramp_cost_model_fit(int n_cfg, const int32_t *wave_cap, int n_pts, const int64_t *grid,
                                   const int64_t *distinct, const int64_t *pairs, const double *time_us, int flags,
                                   float *theta)
{
    return fit_impl(n_cfg, wave_cap, n_pts, grid, nullptr, distinct, pairs, time_us, flags, theta, 4);
}

extern "C" int ramp_cost_model_fit5(int n_cfg, const int32_t *wave_cap, int n_pts, const int64_t *grid,
                                    const int64_t *distinct, const int64_t *pairs, const double *time_us, int flags,
                                    float *theta5)
{
    return fit_impl(n_cfg, wave_cap, n_pts, grid, nullptr, distinct, pairs, time_us, flags, theta5, 5);
}

extern "C" int ramp_cost_model_fit_rounds(int n_cfg, const int32_t *wave_cap, int n_pts, const int64_t *grid,
                                          const int64_t *grid_rounds, const int64_t *distinct, const int64_t *pairs,
                                          const double *time_us, int flags, int n_terms, float *theta)
{
    return fit_impl(n_cfg, wave_cap, n_pts, grid, grid_rounds, distinct, pairs, time_us, flags, theta, n_terms);
}

// g_r of one configuration: the M-tiles of each of its two launches rounded up to whole hand-out rounds
static inline int64_t rounded_grid(int64_t mt, const int32_t *r)
{
    int64_t g = 0;
    for (int s = 0; s < 2; ++s) {
        const int64_t R = r[2 * s], nt = r[2 * s + 1];
        g += (mt + R - 1) / R * R * nt;
    }
    return g;
}

static int select_impl(int E, int n_cfg, const ramp_config *cfgs, const int32_t *ntiles, const int32_t *rounds,
                       const int32_t *wave_cap, const float *theta, const int32_t *expert_counts, int flags,
                       int *best_idx, double *pred_us, int n_theta)
{
    const bool use_rounds = (flags & RAMP_CM_ROUNDS) != 0;
    if (E <= 0 || n_cfg <= 0 || !cfgs || !ntiles || !wave_cap || !theta || !expert_counts || !best_idx ||
        (use_rounds && !rounds) || (flags & ~kAllFlags) || (n_theta != 4 && n_theta != 5)) {
        ramp::set_error("cost_model_select: bad argument");
        return RAMP_EINVAL;
    }
    const bool use_distinct = (flags & RAMP_CM_DISTINCT_TILES) != 0;
    const bool wave_floor = (flags & RAMP_CM_WAVE_FLOOR) != 0;
    const bool use_pairs = (flags & RAMP_CM_PAIRS) != 0;
    int64_t active = 0, pairs = 0;
    for (int e = 0; e < E; ++e) {
        active += expert_counts[e] > 0 ? 1 : 0;
        pairs += expert_counts[e] > 0 ? expert_counts[e] : 0;
    }
    int best = -1;
    double best_t = 0.0;
    // M-tiles depend only on bm; configurations usually share a handful of bm values
    int last_bm = -1;
    int64_t last_mt = 0;
    for (int c = 0; c < n_cfg; ++c) {
        const int bm = cfgs[c].bm;
        if (bm <= 0 || wave_cap[c] <= 0) {
            ramp::set_error("cost_model_select: config %d has bm=%d wave_cap=%d", c, bm, wave_cap[c]);
            return RAMP_EINVAL;
        }
        if (bm != last_bm) {
            int64_t mt = 0;
            for (int e = 0; e < E; ++e) {
                const int64_t n = expert_counts[e] > 0 ? expert_counts[e] : 0;
                mt += (n + bm - 1) / bm;
            }
            last_bm = bm;
            last_mt = mt;
        }
        const double g = (double)(last_mt * (int64_t)ntiles[c]);
        const float *th = theta + (size_t)c * n_theta;
        double t = (double)th[0];
        if (use_rounds && (rounds[4 * c] <= 0 || rounds[4 * c + 2] <= 0)) {
            ramp::set_error("cost_model_select: config %d has a round of %d / %d M-tiles", c, rounds[4 * c], rounds[4 * c + 2]);
            return RAMP_EINVAL;
        }
        const double w = (use_rounds ? (double)rounded_grid(last_mt, rounds + 4 * c) : g) / (double)wave_cap[c];
        t = t + (double)th[1] * ((wave_floor && w < 1.0) ? 1.0 : w);
        const double m = use_distinct ? (double)(active * (int64_t)ntiles[c]) : g;
        t = t + (double)th[2] * m;
        t = t + (double)th[3] * (use_pairs ? (double)pairs : std::log(g + 1.0));
        if (n_theta == 5) t = t + (double)th[4] * ((g / (double)wave_cap[c]) * (g / (double)wave_cap[c]));  // g/W, not floored
        if (pred_us) pred_us[c] = t;
        if (best < 0 || t < best_t) {
            best = c;
            best_t = t;
        }
    }
    *best_idx = best;
    return RAMP_OK;
}

extern "C" int ramp_cost_model_select(int E, int n_cfg, const ramp_config *cfgs, const int32_t *ntiles,
                                      const int32_t *wave_cap, const float *theta, const int32_t *expert_counts,
                                      int flags, int *best_idx, double *pred_us)
{
    return select_impl(E, n_cfg, cfgs, ntiles, nullptr, wave_cap, theta, expert_counts, flags, best_idx, pred_us, 4);
}

extern "C" int ramp_cost_model_select5(int E, int n_cfg, const ramp_config *cfgs, const int32_t *ntiles,
                                       const int32_t *wave_cap, const float *theta5, const int32_t *expert_counts,
                                       int flags, int *best_idx, double *pred_us)
{
    return select_impl(E, n_cfg, cfgs, ntiles, nullptr, wave_cap, theta5, expert_counts, flags, best_idx, pred_us, 5);
}

extern "C" int ramp_cost_model_select_rounds(int E, int n_cfg, const ramp_config *cfgs, const int32_t *ntiles,
                                             const int32_t *rounds, const int32_t *wave_cap, const float *theta,
                                             const int32_t *expert_counts, int flags, int n_terms, int *best_idx,
                                             double *pred_us)
{
    return select_impl(E, n_cfg, cfgs, ntiles, rounds, wave_cap, theta, expert_counts, flags, best_idx, pred_us, n_terms);
}

// Eq. 1 for every configuration on one histogram, with the other two histogram sums the model's columns use.
extern "C" int ramp_grid(int E, int n_cfg, const ramp_config *cfgs, const int32_t *ntiles, const int32_t *expert_counts,
                         int64_t *grid, int64_t *distinct, int64_t *pairs, const int32_t *rounds, int64_t *grid_rounds)
{
    if (E <= 0 || n_cfg <= 0 || !cfgs || !ntiles || !expert_counts || !grid || (grid_rounds && !rounds)) {
        ramp::set_error("grid: bad argument");
        return RAMP_EINVAL;
    }
    int64_t active = 0, total = 0;
    for (int e = 0; e < E; ++e) {
        active += expert_counts[e] > 0 ? 1 : 0;
        total += expert_counts[e] > 0 ? expert_counts[e] : 0;
    }
    for (int c = 0; c < n_cfg; ++c) {
        const int bm = cfgs[c].bm;
        if (bm <= 0 || ntiles[c] <= 0) {
            ramp::set_error("grid: config %d has bm=%d ntiles=%d", c, bm, ntiles[c]);
            return RAMP_EINVAL;
        }
        int64_t mt = 0;
        for (int e = 0; e < E; ++e) {
            const int64_t n = expert_counts[e] > 0 ? expert_counts[e] : 0;
            mt += (n + bm - 1) / bm;
        }
        grid[c] = mt * (int64_t)ntiles[c];
        if (distinct) distinct[c] = active * (int64_t)ntiles[c];
        if (grid_rounds) {
            if (rounds[4 * c] <= 0 || rounds[4 * c + 2] <= 0) {
                ramp::set_error("grid: config %d has a round of %d / %d M-tiles", c, rounds[4 * c], rounds[4 * c + 2]);
                return RAMP_EINVAL;
            }
            grid_rounds[c] = rounded_grid(mt, rounds + 4 * c);
        }
    }
    if (pairs) *pairs = total;
    return RAMP_OK;
}

// ---- performance-region variables (Sec. 4.1, Eq. 2-5, Tab. 2) ----
extern "C" int ramp_region_classify(const ramp_shape *shape, const ramp_config *cfg, long long grid,
                                    const ramp_region_thresholds *thresholds, ramp_region *out)
{
    if (!shape || !cfg || !out || grid < 0 || cfg->bn <= 0 || cfg->bk <= 0 || shape->H <= 0 || shape->I <= 0) {
        ramp::set_error("region_classify: bad argument");
        return RAMP_EINVAL;
    }
    ramp_region_thresholds th = {RAMP_REGION_RHO_C, RAMP_REGION_L2_EFF_BYTES, 2, 256, 48.0, 0.2};
    if (thresholds) th = *thresholds;
    if (th.rho_c <= 0 || th.l2_eff_bytes <= 0 || th.elem_bytes <= 0 || th.units <= 0) {
        ramp::set_error("region_classify: thresholds must be positive");
        return RAMP_EINVAL;
    }
    const double N = 2.0 * shape->I, K = shape->H;  // the paper's N (gate and up side by side) and K of phase 1
    ramp_region r;
    r.rho = N * K / ((double)cfg->bn * cfg->bk);                       // Eq. 2
    r.lambda = (double)((2ll * shape->I + cfg->bn - 1) / cfg->bn);     // Eq. 3
    r.kappa = K / cfg->bk;                                             // Eq. 3
    r.omega = (double)grid / th.units;                                 // Eq. 5
    r.group_m_threshold = th.l2_eff_bytes / ((double)cfg->bn * cfg->bk * th.elem_bytes);  // Eq. 4, right-hand side
    const int row = r.rho >= th.rho_c ? 1 : 0;
    const int col = r.omega < 1.0 ? 0 : (r.omega <= 8.0 ? 1 : 2);
    r.region = row * 3 + col;                                          // Tab. 2: A1 A2 A3 B1 B2 B3
    r.group_m = r.lambda * r.kappa > r.group_m_threshold;
    r.split_k = r.kappa >= th.split_k_kappa && r.omega < th.split_k_omega;
    r.wide_tile = r.omega > 1.0;
    *out = r;
    return RAMP_OK;
}
