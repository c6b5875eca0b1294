/*
 * ramp.h - C ABI of the MI355X (gfx950) routing-aware fused-MoE library.
 *
 * The library implements the hot path of RaMP (arxiv 2604.26039): the fused MoE
 * layer of Sec. 2.2 as a family of tile configurations (Sec. 2.2 "tile
 * configuration", Sec. 4.3) plus the four-term wave cost model of Sec. 4.2 that
 * picks one configuration per call from the runtime expert histogram.
 *
 * Notation (paper -> here): S -> T tokens; c_e -> n_e pairs routed to expert e;
 * N -> 2*I (gate and up projections side by side); K -> H; SM -> 256 compute
 * units; CTA -> workgroup; wn -> wavefronts per workgroup.
 *
 * Conventions
 *  - "dev" pointers are device (HBM) addresses valid on the current HIP device,
 *    "host" pointers are ordinary host memory.  The library never allocates or
 *    frees device memory: every buffer, including workspaces, belongs to the
 *    caller and is sized with the *_bytes / *_capacity queries below.
 *  - Device work is enqueued on the caller's stream (a hipStream_t passed as
 *    void*; NULL = the default stream) and is asynchronous.  No call syncs with
 *    the host.  Calls that share a workspace must be ordered by the caller.
 *  - Every call returns RAMP_OK or a negative status; nothing throws.
 *    ramp_last_error() returns a thread-local text for the last failure.
 *  - bf16 buffers hold raw bfloat16 bit patterns (uint16 each).
 */
#ifndef RAMP_H
#define RAMP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    RAMP_OK = 0,
    RAMP_EINVAL = -1,       /* bad argument (NULL pointer, negative size, misaligned buffer) */
    RAMP_ENOSPC = -2,       /* a caller-provided buffer or workspace is too small            */
    RAMP_EUNSUPPORTED = -3, /* configuration not instantiated / shape outside kernel limits  */
    RAMP_EHIP = -4          /* the HIP runtime reported an error on launch                   */
};

/* Problem statement of Sec. 2.1/2.2: T tokens, top-k routing over E experts,
 * hidden size H, expert intermediate size I (SwiGLU experts). */
typedef struct {
    int32_t T, k, E, H, I;
} ramp_shape;

/* Tile configuration (Sec. 2.2, c = (bm, bn, wn, stg)) in this kernel's terms:
 *   bm     token-block rows per M-tile (4..288; padded to a multiple of 16 inside the MFMA; the
 *          272- and 288-row tiles of the persistent kernel are a 256-row tile plus one or two
 *          16-row tail blocks, for experts whose pairs just miss 256)
 *   bn     weight rows (columns of the paper's N) per workgroup tile: the up-projection
 *          tile holds bn/2 gate rows and the matching bn/2 up rows, the down-projection
 *          tile holds bn output features
 *   bk     K-slice staged in LDS per pipeline step
 *   waves  wavefronts (64 lanes) per workgroup
 *   stages LDS pipeline depth
 *   mode   kernel variant: bits 0-7 = (wavefront rows along the token dimension) - 1, i.e. how
 *          the `waves` wavefronts are arranged over the tile (tokens x features);
 *          bits 8.. = 0 for the LDS-staged path; 0x100 | WK selects the weight-streaming
 *          path for small token blocks (weights go from HBM straight into MFMA operand
 *          registers, the K reduction is split WK ways over the workgroup's wavefronts;
 *          bk is then the k-extent of one register load batch); 0x200 = LDS-staged path with
 *          the register-pipelined main loop; 0x400 = persistent ping-pong kernel for the
 *          large tiles (one workgroup per compute unit walks its share of the tiles, two
 *          groups of four wavefronts alternate memory and MFMA phases); bits 12-15 = v > 0: GROUP_M
 *          mode (Sec. 4.1, Eq. 4) in its XCD-aware form: the workgroups of one XCD (one L2) take
 *          blocks of 2^v M-tiles x about 32/2^v N-tiles, so the M-tiles of a block share the weight
 *          slices of a few N-tiles in L2; v = 0: a block spans all N-tiles and the token rows of its
 *          M-tiles are what stays in L2.
 *          Take configurations from ramp_get_config rather than composing mode words. */
typedef struct {
    int32_t bm, bn, bk, waves, stages, mode;
} ramp_config;

const char *ramp_last_error(void);

/* ---- configuration family (Sec. 4.3 "Configuration diversity") ------------------------- */

/* Number of configurations that are valid for this shape under gfx950 limits
 * (LDS 160 KB per CU, register budget, MFMA 16x16x32 alignment, H % 128 == 0,
 * I % 128 == 0, tile widths dividing 2*I and H).  Host only. */
int ramp_num_configs(const ramp_shape *shape);
/* idx-th valid configuration, 0 <= idx < ramp_num_configs(). */
int ramp_get_config(const ramp_shape *shape, int idx, ramp_config *out);
/* Second factor of Eq. 1 for this kernel: work tiles per M-tile summed over the
 * two projections, ceil(2I/bn) + ceil(H/bn).  Negative status on error. */
int ramp_config_ntiles(const ramp_shape *shape, const ramp_config *cfg);
/* "SM" of Eq. 6 on this chip: 256 compute units times the workgroups of this
 * configuration that fit on one unit (from its LDS and register footprint). */
int ramp_config_wave_capacity(const ramp_config *cfg);

/* What the HIP runtime says about the same quantity on the current device: workgroups of the configuration's
 * up-projection kernel (wg_per_cu[0]) and down-projection kernel (wg_per_cu[1]) that can be resident on one
 * compute unit (hipOccupancyMaxActiveBlocksPerMultiprocessor).  Needs a GPU; ramp_config_wave_capacity is the
 * static table the cost model uses and is tested against this. */
int ramp_config_runtime_occupancy(const ramp_config *cfg, int *wg_per_cu /*host out [2]*/);

/* ---- align (Eq. 1 first factor; Fig. 1) --------------------------------------------------
 * Pair p = t*k + j is routed to expert topk_ids[p].  Expert e owns
 * ceil(n_e/bm) consecutive tiles of bm slots; its pairs fill them in increasing p,
 * unused slots hold the sentinel P = T*k.  Pairs whose id is outside [0,E) are
 * dropped and counted.  The result is unique, so it can be compared byte for byte. */

/* Slots in sorted_pair_ids: roundup(P + min(E,P)*(bm-1), bm). */
size_t ramp_align_capacity(int T, int k, int E, int bm);
/* Scratch bytes ramp_moe_align / ramp_moe_histogram need for (T,k,E). */
size_t ramp_align_workspace_bytes(int T, int k, int E);

/* expert_counts[e] = n_e (Sec. 4.4 step 1).  dev in, dev out. */
int ramp_moe_histogram(const int32_t *topk_ids /*dev [T*k]*/, int T, int k, int E,
                       int32_t *expert_counts /*dev [E]*/,
                       void *ws /*dev*/, size_t ws_bytes, void *stream);

/* Full align.  meta = {P_pad, M_tiles, dropped, 0}; tile_expert[m] = expert of tile m,
 * -1 for m >= M_tiles; sorted_pair_ids slots >= P_pad hold the sentinel.
 * Limits: E <= 1024, 1 <= bm <= 1024, T*k < 2^30. */
int ramp_moe_align(const int32_t *topk_ids /*dev [T*k]*/, int T, int k, int E, int bm,
                   int32_t *sorted_pair_ids /*dev [capacity]*/,
                   int32_t *tile_expert /*dev [capacity/bm]*/,
                   int32_t *expert_counts /*dev [E]*/, int32_t *meta /*dev [4]*/,
                   void *ws /*dev*/, size_t ws_bytes, void *stream);

/* ---- expert weights ------------------------------------------------------------------------
 * Boundary layout (Sec. 2.2): W_gate, W_up bf16 [E,H,I] (x W convention, I contiguous),
 * W_down bf16 [E,I,H].  The kernels read a packed copy made once per model, outside the
 * timed path (the analogue of the paper's offline compile step): every 16x32 block of
 * W^T is stored in the register order of one MFMA 16x16x32 operand so that a wavefront
 * loads it as one contiguous 1 KB line. */
size_t ramp_pack_bytes(const ramp_shape *shape);
int ramp_pack_weights(const ramp_shape *shape, const void *W_gate, const void *W_up,
                      const void *W_down /*dev bf16*/, void *packed /*dev, 256 B aligned*/,
                      void *stream);

/* ---- fused MoE layer (Sec. 2.2 phases 1-3, Sec. 4.3) --------------------------------------
 * out[t,:] = sum_j w[t,j] * ( SiLU(x_t W_gate[e_j]) * (x_t W_up[e_j]) ) W_down[e_j]
 * bf16 inputs, fp32 accumulation, one bf16 rounding of the activation between the
 * projections, one row per pair (already multiplied by its router weight; fp32, or bf16
 * once T*k*H reaches 8 Mi elements, where these rows dominate the memory traffic) summed in
 * fp32 in fixed j order (no atomics: results are bit-identical from run to run), one final
 * rounding to bf16.  Requires H and I to be multiples of 128, E <= 1024, k <= 1024, T*k < 2^30 and
 * T*k <= 2^24 * k (the kernels divide pair indices by k with a 64-bit multiplication).
 * Runs align(bm) + both projections + combine on `stream`; the grid is an upper
 * bound with early exit (Sec. 4.3 "grid overlaunch"), so nothing is read back. */
size_t ramp_fused_moe_workspace_bytes(const ramp_shape *shape, const ramp_config *cfg);
int ramp_fused_moe(const ramp_shape *shape, const ramp_config *cfg,
                   const void *X /*dev bf16 [T,H]*/, const int32_t *topk_ids /*dev [T,k]*/,
                   const float *topk_w /*dev fp32 [T,k]*/, const void *packed_weights /*dev*/,
                   void *out /*dev bf16 [T,H]*/, void *ws /*dev, 256 B aligned*/, size_t ws_bytes,
                   void *stream);
/* ramp_fused_moe for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The workspace is a device array inside the
 * library image, RAMP_STATIC_WS_BYTES per GPU the library runs on, held until the process ends; the call
 * allocates nothing and frees nothing.  Same kernels, same result bit for bit as ramp_fused_moe.
 * Returns RAMP_ENOSPC when ramp_fused_moe_workspace_bytes(shape, cfg) exceeds RAMP_STATIC_WS_BYTES (decode- and
 * small-prefill-sized calls fit: e.g. H=7168, I=2048, E=256, top-8 up to T=64 with bm<=16).  All calls on one
 * GPU share the array: calls that overlap on one GPU (different streams, or replays of graphs that hold it)
 * race and must be ordered by the caller.  Inputs and `out` are the caller's as in ramp_fused_moe. */
#define RAMP_STATIC_WS_BYTES (64u << 20)
int ramp_fused_moe_static(const ramp_shape *shape, const ramp_config *cfg,
                          const void *X /*dev bf16 [T,H]*/, const int32_t *topk_ids /*dev [T,k]*/,
                          const float *topk_w /*dev fp32 [T,k]*/, const void *packed_weights /*dev*/,
                          void *out /*dev bf16 [T,H]*/, void *stream);
/* Where ramp_fused_moe leaves the align result inside its workspace (byte offsets),
 * for tests: sorted_pair_ids, tile_expert, expert_counts, meta. */
int ramp_fused_moe_workspace_layout(const ramp_shape *shape, const ramp_config *cfg,
                                    size_t offsets[4]);

/* ---- W8A8 FP8 variant (Sec. 4.3 "W8A8 FP8, 128x128 block scales"; Sec. 2.2 phase 2 re-quantisation) -------------
 * Same layer, same arguments, 8-bit operands: OCP E4M3 codes (largest value 448, round to nearest even, saturating)
 * with power-of-two block scales kept as E8M0 bytes b (scale 2^(b-127), the smallest power of two with
 * amax/scale <= 448; b = 127 for an all-zero block): one scale per 128 x 128 block of every weight matrix, one per
 * token and 128 consecutive k-values for the activations.  The up-projection multiplies the quantised tokens, its
 * SwiGLU output is rounded to bf16, quantised the same way and multiplied by the quantised down-projection weights;
 * accumulation is fp32 in the matrix pipe (v_mfma_scale_f32_16x16x128_f8f6f4, which applies the block scales).
 * ramp_fp8_pack_weights quantises bf16 boundary-layout weights (as ramp_pack_weights takes them) on the device and
 * lays the codes out in MFMA fragment order, followed by the scale bytes; outside the timed path.
 * The FP8 tile family is enumerated apart from the bf16 one (mode bit 0x10000, bk = 128); its configurations
 * work with ramp_config_ntiles, ramp_grid, ramp_cost_model_fit / select like any other. */
int ramp_fp8_num_configs(const ramp_shape *shape);
int ramp_fp8_get_config(const ramp_shape *shape, int idx, ramp_config *out);
int ramp_fp8_config_wave_capacity(const ramp_config *cfg);
size_t ramp_fp8_pack_bytes(const ramp_shape *shape);
int ramp_fp8_pack_weights(const ramp_shape *shape, const void *W_gate, const void *W_up, const void *W_down /*dev bf16*/,
                          void *packed_fp8 /*dev, 256 B aligned*/, void *stream);
/* Where things sit inside the packed buffer, for tests (bytes): offsets = {gate+up codes per expert, offset of the
 * up codes inside an expert, start of the down codes, down codes per expert, start of the scale bytes, scale bytes
 * per expert}; strides = {scale row stride for k over H, for k over I} (k blocks padded to a multiple of 4).
 * Codes of one matrix: [feature/16 row blocks][k/128][2 KB], a 2 KB fragment = two 1 KB halves, half h holding
 * for lane l the bytes k = 32*(l/16) + 16*h + 0..15 of the row l%16 (row -> feature by the bf16 layout's
 * interleave).  Scale bytes per expert: gate, up [I/128][stride0], then down [H/128][stride1]. */
int ramp_fp8_pack_layout(const ramp_shape *shape, size_t offsets[6], int32_t strides[2]);
/* The activation quantiser by itself (tests): src dev bf16 [rows, K] row-major, K % 128 == 0 ->
 * codes dev uint8 [rows, K], scales dev uint8 [rows][(K/128 rounded up to 4)]. */
int ramp_fp8_quantize_rows(const void *src, int rows, int K, void *codes, void *scales, void *stream);
size_t ramp_fused_moe_fp8_workspace_bytes(const ramp_shape *shape, const ramp_config *cfg);
int ramp_fused_moe_fp8(const ramp_shape *shape, const ramp_config *cfg,
                       const void *X /*dev bf16 [T,H]*/, const int32_t *topk_ids /*dev [T,k]*/,
                       const float *topk_w /*dev fp32 [T,k]*/, const void *packed_fp8 /*dev*/,
                       void *out /*dev bf16 [T,H]*/, void *ws /*dev, 256 B aligned*/, size_t ws_bytes, void *stream);

/* ---- cost model (Eq. 6, Sec. 4.2) -----------------------------------------------------------
 * T_hat(c) = a + b*w + c*m + d*l,  g = (sum_e ceil(n_e/bm_c)) * ntiles_c.
 * flags = 0 is the paper's model as printed: w = g/W, m = g, l = ln(g+1), ordinary least squares.
 * RAMP_CM_DISTINCT_TILES: the per-block memory-traffic term counts the distinct weight tiles
 *   m = u = #{e: n_e > 0} * ntiles_c instead of all blocks.  On this chip a weight tile that a
 *   second M-tile of the same expert re-reads comes out of L2 / the 256 MB last-level cache,
 *   so HBM traffic scales with u, not g.  It also makes the four columns independent.
 * RAMP_CM_RELATIVE: least squares on relative residuals (each profiling row scaled by
 *   1/t_i), because dispatch only needs the ratio between configurations and the profiled
 *   times span three decades.
 * RAMP_CM_WAVE_FLOOR: the wave term is w = max(g/W, 1): a grid that does not fill the chip still
 *   takes the time of one wave of its blocks (the sub-wave regime of Sec. 4.1), which the kernels
 *   here show as a plateau rather than a logarithm.
 * RAMP_CM_PAIRS: the fourth term is l = P = sum_e n_e, the routed pairs, in place of ln(g+1) and
 *   always fitted: gather, SwiGLU, per-pair rows and the combine cost time per pair whatever the
 *   tiling, which g (padded tiles) does not separate from the padding.
 * RAMP_CM_ROUNDS: the wave term counts whole hand-out rounds, w = g_r/W with
 *   g_r = sum over the two launches of ceil(M_tiles/R)*R*ntiles_launch (ramp_config_rounds gives R and
 *   ntiles_launch).  A persistent kernel's fixed workgroups take the M-tiles in rounds of R = 8*group_m over the
 *   8 XCDs, so its time steps at multiples of R M-tiles: the wave staircase of Sec. 4.2 ("time jumps at wave
 *   boundaries") in the units of this kernel's workgroup -> tile map, and what tells the GROUP_M block shapes of
 *   one tile apart.  R = 1 (g_r = g) for kernels whose workgroups are dispatched tile by tile.  Needs the
 *   *_rounds entry points below. */
enum { RAMP_CM_EQ6 = 0, RAMP_CM_RELATIVE = 1, RAMP_CM_DISTINCT_TILES = 2, RAMP_CM_WAVE_FLOOR = 4, RAMP_CM_PAIRS = 8,
       RAMP_CM_ROUNDS = 16 };

/* Least-squares fit per configuration from profiling (Sec. 4.2 "Fitting").
 * grid, time_us (and distinct, required with RAMP_CM_DISTINCT_TILES, else may be NULL) are
 * host arrays [n_cfg, n_pts]; wave_cap host [n_cfg]; pairs (required with RAMP_CM_PAIRS, else may
 * be NULL) host [n_pts], the routed pairs of each profiling point.
 * The log column is used only when the lower median of a configuration's profiling
 * grids is below its wave capacity.  With m = g the columns g/W and g are proportional:
 * the minimum-norm least-squares solution is returned, predictions do not depend on
 * that choice.  theta: host out [n_cfg,4] = a,b,c,d. */
int ramp_cost_model_fit(int n_cfg, const int32_t *wave_cap, int n_pts, const int64_t *grid,
                        const int64_t *distinct, const int64_t *pairs, const double *time_us, int flags,
                        float *theta);

/* Evaluate the model for every configuration on one histogram (host [E]) and return the
 * lowest index with the smallest prediction in *best_idx (Sec. 4.2 "Runtime
 * dispatch").  flags: the column choices (all but RAMP_CM_RELATIVE) must match the fit.
 * pred_us: optional host out [n_cfg] (fp64 evaluation). */
int ramp_cost_model_select(int E, int n_cfg, const ramp_config *cfgs, const int32_t *ntiles,
                           const int32_t *wave_cap, const float *theta,
                           const int32_t *expert_counts, int flags, int *best_idx, double *pred_us);

/* The five-term ablation of Sec. 5.3 ("a 5th term g^2"): the model above plus e*(g/W)^2, i.e. g^2 up to the
 * configuration's constant W^2.  theta5: host [n_cfg,5] = a,b,c,d,e; otherwise as ramp_cost_model_fit /
 * ramp_cost_model_select (same flags, same adaptive fourth column).  For the ablation report only: the
 * device-resident dispatch evaluates the four-term model. */
int ramp_cost_model_fit5(int n_cfg, const int32_t *wave_cap, int n_pts, const int64_t *grid,
                         const int64_t *distinct, const int64_t *pairs, const double *time_us, int flags,
                         float *theta5);
int ramp_cost_model_select5(int E, int n_cfg, const ramp_config *cfgs, const int32_t *ntiles,
                            const int32_t *wave_cap, const float *theta5,
                            const int32_t *expert_counts, int flags, int *best_idx, double *pred_us);

/* The model with RAMP_CM_ROUNDS (and without: grid_rounds / rounds may then be NULL).  n_terms = 4 or 5 as in
 * ramp_cost_model_fit / fit5.  grid_rounds: host [n_cfg, n_pts], the g_r of every profiling point (ramp_grid);
 * rounds: host [n_cfg, 4] = ramp_config_rounds of every configuration.  The traffic, logarithm and g^2 columns
 * keep the plain g. */
int ramp_cost_model_fit_rounds(int n_cfg, const int32_t *wave_cap, int n_pts, const int64_t *grid,
                               const int64_t *grid_rounds, const int64_t *distinct, const int64_t *pairs,
                               const double *time_us, int flags, int n_terms, float *theta /*host out [n_cfg, n_terms]*/);
int ramp_cost_model_select_rounds(int E, int n_cfg, const ramp_config *cfgs, const int32_t *ntiles,
                                  const int32_t *rounds, const int32_t *wave_cap, const float *theta,
                                  const int32_t *expert_counts, int flags, int n_terms, int *best_idx, double *pred_us);
/* out = {R_up, ntiles_up, R_down, ntiles_down}: M-tiles handed out per round over the 8 XCDs (8*group_m of the
 * launch's workgroup -> tile map for the persistent kernels, 1 otherwise) and N-tiles (2I/bn, H/bn) of the
 * up- and the down-projection launch.  Host only. */
int ramp_config_rounds(const ramp_shape *shape, const ramp_config *cfg, int32_t out[4]);

/* Eq. 1 for every configuration on one histogram (host [E]): grid[c] = (sum_e ceil(n_e/bm_c)) * ntiles[c], the
 * g of Eq. 6.  Optional outputs (may be NULL): distinct[c] = #{e: n_e > 0} * ntiles[c] (the column of
 * RAMP_CM_DISTINCT_TILES), *pairs = sum_e n_e (the column of RAMP_CM_PAIRS) and, from rounds (host [n_cfg, 4],
 * required with it), grid_rounds[c] = the g_r of RAMP_CM_ROUNDS.  Host only. */
int ramp_grid(int E, int n_cfg, const ramp_config *cfgs, const int32_t *ntiles, const int32_t *expert_counts,
              int64_t *grid /*host out [n_cfg]*/, int64_t *distinct /*host out [n_cfg]*/, int64_t *pairs /*host out*/,
              const int32_t *rounds /*host [n_cfg,4] or NULL*/, int64_t *grid_rounds /*host out [n_cfg] or NULL*/);

/* ---- performance-region variables (Sec. 4.1: Eq. 2-5, Tab. 2) ------------------------------------
 * The four quantities the paper uses to say which optimisation modes belong in a model's pool, for
 * one configuration of this kernel (ttn -> bn, tile_k -> bk, N = 2I, K = H) and one grid (Eq. 1):
 *   rho = N*K/(bn*bk)  MMA tile operations per block        lambda = ceil(N/bn)  N-tiles
 *   kappa = K/bk       K-loop depth                         omega = grid/units   waves
 * region: 0..5 = A1 A2 A3 B1 B2 B3 of Tab. 2 (row: rho >= rho_c; column: omega < 1, 1 <= omega <= 8,
 * omega > 8).  group_m: lambda*kappa > l2_eff_bytes/(bn*bk*elem_bytes) (Eq. 4); split_k: kappa >=
 * split_k_kappa and omega < split_k_omega; wide_tile: omega > 1.  Host only.
 * thresholds == NULL takes this chip's: rho_c = RAMP_REGION_RHO_C, l2_eff_bytes =
 * RAMP_REGION_L2_EFF_BYTES (three quarters of the 4 MB L2 of one XCD, the level at which workgroups
 * share weight tiles), 2-byte elements, 256 units, the paper's 48 and 0.2 for split-K.  The paper's
 * own H200 numbers are rho_c = 186, 45 MB, 1 byte, 132 units. */
#define RAMP_REGION_RHO_C 16.0
#define RAMP_REGION_L2_EFF_BYTES (3.0 * 1024 * 1024)
typedef struct {
    double rho_c, l2_eff_bytes;
    int32_t elem_bytes, units;
    double split_k_kappa, split_k_omega;
} ramp_region_thresholds;
typedef struct {
    double rho, lambda, kappa, omega, group_m_threshold;
    int32_t region, group_m, split_k, wide_tile;
} ramp_region;
int ramp_region_classify(const ramp_shape *shape, const ramp_config *cfg, long long grid,
                         const ramp_region_thresholds *thresholds /*may be NULL*/, ramp_region *out);

/* ---- device-resident dispatch (Sec. 4.4 steps 1-3 in one enqueue; Sec. 5 "dispatch overhead") ----
 * ramp_cost_model_select needs the histogram on the host: a device-to-host copy and a stream
 * synchronisation on every call.  ramp_select_device instead enqueues the histogram and one small
 * kernel that evaluates the model for every configuration on the device (fp64, the operation order of
 * ramp_cost_model_select, lowest index among equal predictions) and writes the outcome into a result
 * block.  When that block is pinned host memory the host learns the choice by polling its first word
 * (ramp_select_poll / ramp_select_wait): no copy, no stream synchronisation.  A caller that must not
 * wait at all enqueues the selection of this call, launches the fused layer with the configuration the
 * previous call's selection produced, and reads the new result later with ramp_select_poll.
 *
 * Table (device memory, built once on the host and copied by the caller):
 *   ramp_select_table_build writes ramp_select_table_bytes(n_cfg) bytes: a 128-byte header
 *   {int32 magic, n_cfg, n_bm, flags, bm[28]} (the distinct bm values) followed by n_cfg rows of 48
 *   bytes {int32 bm_slot, ntiles, wave_cap, 0; float theta[4]; int32 rounds[4]}.  At most 28 distinct bm,
 *   n_cfg <= 1024.  rounds: host [n_cfg, 4] (ramp_config_rounds), required with RAMP_CM_ROUNDS, else may be NULL.
 * Result block (ramp_select_result_bytes(E, n_cfg) bytes, 8-byte aligned, written by the kernel):
 *   uint64 word = best << 32 | ticket | int32 n_cfg | int32 0 | double pred_us[n_cfg] | int32 expert_counts[E]
 *   The word carries the caller's ticket (nonzero, different from what the block held before) and the
 *   chosen index in one 64-bit store, made last with system-scope release ordering after a single fence:
 *   once the ticket reads back, the index is there and the rest of the block is complete.
 * ws: ramp_align_workspace_bytes(T,k,E) bytes of device scratch (unused up to 8192 pairs).
 * best_idx_dev: optional device int that also receives the index (for launches that test it on the
 *   device).  Calls that share ws or a result block must be ordered by the caller. */
size_t ramp_select_table_bytes(int n_cfg);
int ramp_select_table_build(int n_cfg, const ramp_config *cfgs, const int32_t *ntiles,
                            const int32_t *wave_cap, const float *theta /*host [n_cfg,4]*/, int flags,
                            const int32_t *rounds /*host [n_cfg,4] or NULL*/, void *table /*host out*/, size_t table_bytes);
size_t ramp_select_result_bytes(int E, int n_cfg);
int ramp_select_device(const int32_t *topk_ids /*dev [T*k]*/, int T, int k, int E, int n_cfg,
                       const void *table /*dev*/, void *result /*pinned host or dev*/,
                       uint32_t ticket, int32_t *best_idx_dev /*dev, may be NULL*/,
                       void *ws /*dev*/, size_t ws_bytes, void *stream);
/* Host side of the result block.  ramp_select_poll returns RAMP_OK and *best_idx once the block
 * carries `ticket`, 1 if it does not yet (not an error), RAMP_EINVAL if the kernel found that the
 * table was not one built for n_cfg configurations (it then evaluates nothing).  ramp_select_wait spins on it for at most
 * timeout_s seconds (then RAMP_EHIP).  Neither touches the HIP runtime. */
int ramp_select_poll(const void *result_host, uint32_t ticket, int *best_idx);
int ramp_select_wait(const void *result_host, uint32_t ticket, double timeout_s, int *best_idx);

/* ---- fused layer with the configuration chosen on the device ---------------------------------------
 * For callers that cannot branch on the host between the selection and the launch (a captured HIP graph, a
 * host thread that must not wait): every one of the n_cand candidate configurations is enqueued, and on the
 * device each of its launches first reads *selected_idx (written, e.g., by ramp_select_device through
 * best_idx_dev, over a table built from the same candidates in the same order) and does nothing unless it
 * equals the candidate's position.  One candidate runs; the others cost a few empty launches.  The result is
 * the one ramp_fused_moe gives for that candidate, bit for bit.  If *selected_idx is outside [0, n_cand)
 * nothing runs, the combine included, and `out` keeps its previous contents.  1 <= n_cand <= 16.  The workspace (size from the query below) is shared
 * by the candidates; selected_idx must not change while the call's work is in flight. */
size_t ramp_fused_moe_selected_workspace_bytes(const ramp_shape *shape, int n_cand, const ramp_config *cfgs);
int ramp_fused_moe_selected(const ramp_shape *shape, int n_cand, const ramp_config *cfgs /*host [n_cand]*/,
                            const int32_t *selected_idx /*dev*/,
                            const void *X /*dev bf16 [T,H]*/, const int32_t *topk_ids /*dev [T,k]*/,
                            const float *topk_w /*dev fp32 [T,k]*/, const void *packed_weights /*dev*/,
                            void *out /*dev bf16 [T,H]*/, void *ws /*dev, 256 B aligned*/, size_t ws_bytes,
                            void *stream);

/* ---- measurement hooks --------------------------------------------------------------------------
 * ramp_probe_enable(stage): from now on every ramp_fused_moe call of this process records a
 * HIP event pair on its stream around one stage (1 = align, 2 = up-projection + SwiGLU,
 * 3 = down-projection, 4 = combine; 0 = off).  At most 4096 pairs are kept between reads.
 * ramp_probe_read: waits for the recorded events, returns the summed stage time and the
 * number of launches, and clears the list.  The list is guarded by a mutex; a call whose stream is being
 * captured into a graph records nothing.  Read only when no probed call is in progress on another thread. */
int ramp_probe_enable(int stage);
int ramp_probe_read(double *total_ms /*host*/, int *launches /*host*/);

/* ---- measurement helper ------------------------------------------------------------------------
 * Plain device copy of `bytes` bytes (multiple of 16, both 16 B aligned): the
 * known-size reference kernel that profiler byte counters are calibrated against. */
int ramp_copy_bytes(void *dst /*dev*/, const void *src /*dev*/, size_t bytes, void *stream);


/* Register-resident matrix-pipe loop, the ceiling that the MFMA-bound kernels are compared with next to the
 * nominal peak: 256 workgroups of 8 wavefronts (two per SIMD) each run `rounds` rounds of 32 independent
 * v_mfma_f32_16x16x32_bf16 on operand fragments read once from `operands` (dev, 12 fragments of 512 bf16 = 12 KB)
 * and write their sums to `sink` (dev, 256*512*4 floats).  *flops (host, optional) receives the floating-point
 * operations of the launch; the caller times it.  The chip is power limited and its clock follows the operand
 * bits, so zeros and random values give different rates. */
int ramp_mfma_rate_probe(const void *operands /*dev bf16 [12*512]*/, int rounds, void *sink /*dev fp32 [524288]*/,
                         void *stream, double *flops /*host out, may be NULL*/);

#ifdef __cplusplus
}
#endif
#endif /* RAMP_H */
