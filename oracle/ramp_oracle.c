/*
 * CPU oracle for the routing-aware fused MoE layer (RaMP, arxiv 2604.26039).
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what "correct" means for the
 * GPU library; it is slow on purpose, shares no code with the HIP path and is
 * never linked into it.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg call it.
 *
 * Everything here is the plain definition written out, in fp64, from the exact
 * values of the bf16 inputs:
 *   - oracle_align   : grouping of (token, expert) pairs into bm-padded
 *                      per-expert blocks (paper Eq. 1, first factor; Fig. 1).
 *   - oracle_moe     : per-token brute force of the fused MoE layer
 *                      (paper Sec. 2.2: up-projection, SwiGLU, down-projection,
 *                      scatter back with the router weight).
 *   - oracle_grid    : Eq. 1.
 *   - oracle_predict / oracle_select : Eq. 6 evaluated for every configuration
 *                      and the argmin (Sec. 4.2 "Runtime dispatch").
 * The least-squares fit of Eq. 6 lives in oracle.py (numpy lstsq is the one
 * library primitive it uses).
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py against
 * brute force in another language, closed forms, invariants and the numbers the
 * paper prints.  No function is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---------- bf16 helpers (own implementation; nothing shared with the GPU) ---------- */

static double bf16_bits_to_f64(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Round a double to the nearest bf16 (ties to even) in ONE rounding step.
 * bf16 = 1 sign, 8 exponent, 7 fraction bits; normal exponents -126..127. */
static uint16_t f64_to_bf16_bits(double x)
{
    if (isnan(x)) return 0x7fc0;
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    double ax = fabs(x);
    if (ax == 0.0) return sign;
    if (isinf(ax)) return (uint16_t)(sign | 0x7f80);
    int ex;
    (void)frexp(ax, &ex);               /* ax = m * 2^ex, m in [0.5, 1)            */
    int e = ex - 1;                     /* ax = s * 2^e,  s in [1, 2)              */
    if (e < -126) e = -126;             /* subnormal range shares the quantum 2^-133 */
    double quantum = ldexp(1.0, e - 7);
    double q = nearbyint(ax / quantum); /* exact division; default mode = ties-even */
    double y = q * quantum;             /* exactly representable in bf16 or overflow */
    if (y >= ldexp(1.0, 128)) return (uint16_t)(sign | 0x7f80);
    float f = (float)y;                 /* exact */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return (uint16_t)(sign | (u >> 16));
}

uint16_t oracle_f64_to_bf16(double x) { return f64_to_bf16_bits(x); }
double oracle_bf16_to_f64(uint16_t b) { return bf16_bits_to_f64(b); }

/* ---------- align (Eq. 1 first factor; Fig. 1 caption) ---------- */

/* Capacity of sorted[]: every pair plus, for each expert that can be hit, at
 * most bm-1 padding slots, rounded up to a whole tile. */
int64_t oracle_align_capacity(int T, int k, int E, int bm)
{
    int64_t P = (int64_t)T * k;
    int64_t hit = P < E ? P : E;
    int64_t cap = P + hit * (bm - 1);
    return (cap + bm - 1) / bm * bm;
}

/*
 * ids[T*k]: expert of pair p = t*k + j.  Pairs with an id outside [0,E) are
 * dropped and counted.  Output (all int32):
 *   counts[E]        n_e
 *   sorted[cap]      expert e owns slots off_e .. off_e + tiles_e*bm; its first
 *                    n_e slots are the pairs routed to e in increasing p, the
 *                    rest hold the sentinel P; slots >= P_pad hold P as well
 *   tile_expert[cap/bm]  expert of tile m, -1 beyond M_tiles
 *   meta[4]          P_pad, M_tiles, dropped, 0
 * Returns 0, or -1 on bad arguments.
 */
int oracle_align(const int32_t *ids, int T, int k, int E, int bm,
                 int32_t *sorted, int32_t *tile_expert, int32_t *counts, int32_t *meta)
{
    if (T < 0 || k < 0 || E <= 0 || bm <= 0) return -1;
    int64_t P = (int64_t)T * k;
    int64_t cap = oracle_align_capacity(T, k, E, bm);
    for (int e = 0; e < E; ++e) counts[e] = 0;
    int32_t dropped = 0;
    for (int64_t p = 0; p < P; ++p) {
        int32_t e = ids[p];
        if (e < 0 || e >= E) ++dropped; else ++counts[e];
    }
    for (int64_t s = 0; s < cap; ++s) sorted[s] = (int32_t)P;
    for (int64_t m = 0; m < cap / bm; ++m) tile_expert[m] = -1;

    int64_t off = 0;
    for (int e = 0; e < E; ++e) {
        int64_t tiles = ((int64_t)counts[e] + bm - 1) / bm;
        /* r-th smallest p with ids[p] == e goes to slot off + r */
        int64_t r = 0;
        for (int64_t p = 0; p < P; ++p)
            if (ids[p] == e) sorted[off + r++] = (int32_t)p;
        for (int64_t m = 0; m < tiles; ++m) tile_expert[off / bm + m] = e;
        off += tiles * bm;
    }
    meta[0] = (int32_t)off;
    meta[1] = (int32_t)(off / bm);
    meta[2] = dropped;
    meta[3] = 0;
    return 0;
}

/* ---------- Eq. 1 ---------- */

/* grid = (sum_e ceil(n_e / bm)) * ntiles */
int64_t oracle_grid(const int32_t *counts, int E, int bm, int ntiles)
{
    int64_t m_tiles = 0;
    for (int e = 0; e < E; ++e) m_tiles += ((int64_t)counts[e] + bm - 1) / bm;
    return m_tiles * ntiles;
}

/* ---------- fused MoE layer, per-token brute force (Sec. 2.2) ---------- */

static double silu(double x) { return x / (1.0 + exp(-x)); }

/*
 * out[r,:] = sum_j w[t,j] * ( SiLU(x_t Wg[e_j]) * (x_t Wu[e_j]) ) Wd[e_j],  t = rows[r]
 *
 * X      bf16 bits [T,H]
 * ids    int32 [T,k]; w float [T,k]
 * Wg,Wu  arrays of E pointers to bf16 bits [H,I] (row h, column i contiguous)
 * Wd     array of E pointers to bf16 bits [I,H]
 *        a NULL pointer is allowed for an expert no evaluated token uses
 * rows   token indices to evaluate (NULL: all T tokens, n_rows = T)
 * round_mid  0: no intermediate rounding; 1: the activation SiLU(g)*u is
 *            rounded to bf16 before the down-projection (what a bf16 MFMA
 *            operand forces); the output is fp64 either way
 * Pairs whose id is outside [0,E) contribute nothing.
 * Returns 0, -1 on bad arguments, -2 if a needed expert pointer is NULL.
 */
int oracle_moe(const uint16_t *X, const int32_t *ids, const float *w,
               const uint16_t *const *Wg, const uint16_t *const *Wu, const uint16_t *const *Wd,
               int T, int k, int E, int H, int I,
               const int32_t *rows, int n_rows, int round_mid, double *out)
{
    if (T < 0 || k < 0 || E <= 0 || H <= 0 || I <= 0) return -1;
    if (!rows) n_rows = T;
    int status = 0;
#pragma omp parallel
    {
        double *x = (double *)malloc(sizeof(double) * (size_t)H);
        double *g = (double *)malloc(sizeof(double) * (size_t)I);
        double *u = (double *)malloc(sizeof(double) * (size_t)I);
        double *y = (double *)malloc(sizeof(double) * (size_t)H);
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < n_rows; ++r) {
            int t = rows ? rows[r] : r;
            double *o = out + (size_t)r * H;
            for (int h = 0; h < H; ++h) o[h] = 0.0;
            if (t < 0 || t >= T) { status = -1; continue; }
            for (int h = 0; h < H; ++h) x[h] = bf16_bits_to_f64(X[(size_t)t * H + h]);
            for (int j = 0; j < k; ++j) {
                int e = ids[(size_t)t * k + j];
                if (e < 0 || e >= E) continue;
                if (!Wg[e] || !Wu[e] || !Wd[e]) { status = -2; continue; }
                for (int i = 0; i < I; ++i) { g[i] = 0.0; u[i] = 0.0; }
                for (int h = 0; h < H; ++h) {
                    const uint16_t *wg = Wg[e] + (size_t)h * I;
                    const uint16_t *wu = Wu[e] + (size_t)h * I;
                    double xh = x[h];
                    for (int i = 0; i < I; ++i) {
                        g[i] += xh * bf16_bits_to_f64(wg[i]);
                        u[i] += xh * bf16_bits_to_f64(wu[i]);
                    }
                }
                for (int h = 0; h < H; ++h) y[h] = 0.0;
                for (int i = 0; i < I; ++i) {
                    double a = silu(g[i]) * u[i];
                    if (round_mid) a = bf16_bits_to_f64(f64_to_bf16_bits(a));
                    const uint16_t *wd = Wd[e] + (size_t)i * H;
                    for (int h = 0; h < H; ++h) y[h] += a * bf16_bits_to_f64(wd[h]);
                }
                double wj = (double)w[(size_t)t * k + j];
                for (int h = 0; h < H; ++h) o[h] += wj * y[h];
            }
        }
        free(x); free(g); free(u); free(y);
    }
    return status;
}

/* ---------- Eq. 6 and the argmin ---------- */

/* T_hat = a + b*g/W + c*m + d*ln(g+1), evaluated left to right in fp64.
 * m = g is Eq. 6 as printed; m = number of distinct weight tiles is the cache-aware
 * reading of the per-block traffic term (see oracle.py). */
/* General form of the four-term model: t = a + b*w + c*m + d*l.
 * As printed (Eq. 6): w = g/W, m = g, l = ln(g+1).  Options (bit mask) of the variants the
 * GPU library also offers: 1: m is supplied by the caller (distinct weight tiles);
 * 2: w = max(g/W, 1); 4: l = pairs (routed pairs) instead of the logarithm. */
double oracle_predict_opt(const float *theta4, int64_t g, int64_t m, int64_t pairs, int wave_cap, int options)
{
    double gd = (double)g;
    double w = gd / (double)wave_cap;
    if ((options & 2) && w < 1.0) w = 1.0;
    double traffic = (options & 1) ? (double)m : gd;
    double last = (options & 4) ? (double)pairs : log(gd + 1.0);
    double t = (double)theta4[0];
    t = t + (double)theta4[1] * w;
    t = t + (double)theta4[2] * traffic;
    t = t + (double)theta4[3] * last;
    return t;
}

double oracle_predict2(const float *theta4, int64_t g, int64_t m, int wave_cap)
{
    return oracle_predict_opt(theta4, g, m, 0, wave_cap, 1);
}

double oracle_predict(const float *theta4, int64_t g, int wave_cap)
{
    return oracle_predict2(theta4, g, g, wave_cap);
}

/*
 * For each configuration c: g_c = (sum_e ceil(n_e/bm_c)) * ntiles_c, then Eq. 6.
 * Returns the lowest index attaining the minimum predicted time (-1 if
 * n_cfg <= 0).  pred (optional) receives all predictions.
 */
int oracle_select(int n_cfg, const int32_t *bm, const int32_t *ntiles, const int32_t *wave_cap,
                  const float *theta /*[n_cfg,4]*/, const int32_t *counts, int E, int options,
                  double *pred)
{
    int best = -1;
    double best_t = 0.0;
    int64_t active = 0, pairs = 0;
    for (int e = 0; e < E; ++e)
        if (counts[e] > 0) { ++active; pairs += counts[e]; }
    for (int c = 0; c < n_cfg; ++c) {
        int64_t g = oracle_grid(counts, E, bm[c], ntiles[c]);
        int64_t m = active * ntiles[c];
        double t = oracle_predict_opt(theta + 4 * (size_t)c, g, m, pairs, wave_cap[c], options);
        if (pred) pred[c] = t;
        if (best < 0 || t < best_t) { best = c; best_t = t; }
    }
    return best;
}
