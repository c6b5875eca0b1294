// Configuration registry, the top-k combine kernel and the fused-MoE entry point
// (paper Sec. 2.2 phases 1-3 as align -> up-projection+SwiGLU -> down-projection -> combine).
#include <mutex>

#include "ramp_internal.h"

namespace ramp {

void register_group0(KernelInfo *, int *);
void register_group1(KernelInfo *, int *);
void register_group2(KernelInfo *, int *);
void register_group3(KernelInfo *, int *);
void register_group4(KernelInfo *, int *);
void register_group5(KernelInfo *, int *);
void register_group6(KernelInfo *, int *);
void register_group7(KernelInfo *, int *);
void register_stream_group0(KernelInfo *, int *);
void register_stream_group1(KernelInfo *, int *);
void register_stream_group2(KernelInfo *, int *);

namespace {
constexpr int kMaxKernels = 128;
KernelInfo g_kernels[kMaxKernels];
int g_num_kernels = 0;
std::once_flag g_once;

void init_registry()
{
    std::call_once(g_once, [] {
        register_group0(g_kernels, &g_num_kernels);
        register_group1(g_kernels, &g_num_kernels);
        register_group2(g_kernels, &g_num_kernels);
        register_group3(g_kernels, &g_num_kernels);
        register_group4(g_kernels, &g_num_kernels);
        register_group5(g_kernels, &g_num_kernels);
        register_group6(g_kernels, &g_num_kernels);
        register_group7(g_kernels, &g_num_kernels);
        register_stream_group0(g_kernels, &g_num_kernels);
        register_stream_group1(g_kernels, &g_num_kernels);
        register_stream_group2(g_kernels, &g_num_kernels);
    });
}

// out[t,:] = sum_j Y[t*k+j,:] in increasing j, fp32, one rounding to bf16.  The router weight
// was applied by the down-projection epilogue.  Pairs with an invalid expert id have no row.
// Y rows are fp32, or bf16 (Y16) for large batches.
// With sel != NULL (device-selected layer) the kernel leaves `out` untouched unless *sel names one of the
// n_cand candidates: no projection has run then and Y holds whatever an earlier call left.
template <bool Y16>
__global__ __launch_bounds__(256) void combine_kernel(const float *__restrict__ Y, const int32_t *__restrict__ ids, int T,
                                                      int k, int E, int H, uint16_t *__restrict__ out,
                                                      const int32_t *__restrict__ sel, int n_cand, unsigned skip_mask)
{
    if (sel != nullptr) {
        const int idx = *sel;
        if (idx < 0 || idx >= n_cand) return;
        if ((skip_mask >> idx) & 1u) return;  // the selected candidate's own launches wrote `out`
    }
    const int hv = H / 8;  // 8-feature columns: one 16-byte bf16 load (or two fp32 ones) per pair row
    const size_t total = (size_t)T * hv;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int t = (int)(i / hv), c = (int)(i % hv);
        float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        const int32_t *row_ids = ids + (size_t)t * k;
#pragma unroll 4
        for (int j = 0; j < k; ++j) {
            const int id = row_ids[j];
            const bool live = id >= 0 && id < E;
            const size_t elem = ((size_t)t * k + j) * H + (size_t)c * 8;
            // the row is read whether or not the pair is live (its address is always inside Y), so the loads do
            // not wait for the ids; a dropped pair's row holds stale bytes and is replaced by zeros afterwards
            if (Y16) {
                uint4 y = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(Y) + elem);
                if (!live) y = make_uint4(0, 0, 0, 0);
                const uint32_t w[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    s[2 * q] += __builtin_bit_cast(float, w[q] << 16);
                    s[2 * q + 1] += __builtin_bit_cast(float, w[q] & 0xffff0000u);
                }
            } else {
                float4 y0 = *reinterpret_cast<const float4 *>(Y + elem);
                float4 y1 = *reinterpret_cast<const float4 *>(Y + elem + 4);
                if (!live) y0 = y1 = make_float4(0.f, 0.f, 0.f, 0.f);
                s[0] += y0.x; s[1] += y0.y; s[2] += y0.z; s[3] += y0.w;
                s[4] += y1.x; s[5] += y1.y; s[6] += y1.z; s[7] += y1.w;
            }
        }
        union {
            uint16_t h[8];
            uint4 u;
        } o;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            uint32_t b = __builtin_bit_cast(uint32_t, s[q]);
            b += 0x7fffu + ((b >> 16) & 1u);
            o.h[q] = (uint16_t)(b >> 16);
        }
        *reinterpret_cast<uint4 *>(out + (size_t)t * H + (size_t)c * 8) = o.u;
    }
}

// ---- stage probe (benchmark instrumentation) ----
// One process-wide list of HIP-event pairs, guarded by a mutex.  A call whose stream is being captured into a
// graph records nothing (event records would become graph nodes).
constexpr int kMaxProbe = 4096;
std::mutex g_probe_mutex;
int g_probe_stage = 0;
int g_probe_used = 0;
int g_probe_created = 0;
hipEvent_t g_probe_ev[kMaxProbe][2];

struct ProbeScope {
    bool on;
    int slot;
    hipStream_t st;
    ProbeScope(int stage, hipStream_t stream) : on(false), slot(-1), st(stream)
    {
        if (stage != g_probe_stage) return;  // unlocked fast path for the common case (probe off)
        std::lock_guard<std::mutex> lock(g_probe_mutex);
        if (stage != g_probe_stage || g_probe_used >= kMaxProbe) return;
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(st, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) return;
        if (g_probe_used >= g_probe_created) {
            hipEvent_t e0, e1;
            if (hipEventCreate(&e0) != hipSuccess) return;
            if (hipEventCreate(&e1) != hipSuccess) {
                (void)hipEventDestroy(e0);
                return;
            }
            g_probe_ev[g_probe_created][0] = e0;
            g_probe_ev[g_probe_created][1] = e1;
            ++g_probe_created;
        }
        slot = g_probe_used++;
        on = hipEventRecord(g_probe_ev[slot][0], st) == hipSuccess;
        if (!on) --g_probe_used;  // still under the lock: the slot was the last one handed out
    }
    ~ProbeScope()
    {
        if (on) (void)hipEventRecord(g_probe_ev[slot][1], st);
    }
};

constexpr size_t kPairRowsBf16Elems = (size_t)8 << 20;

struct Workspace {
    size_t sorted, tile_expert, tile_rows, counts, meta, align_ws, a_buf, y_buf, slot_w, total;
    size_t cap, align_ws_bytes;
};

Workspace workspace_layout(const ramp_shape &s, const ramp_config &c)
{
    Workspace w;
    w.cap = ramp_align_capacity(s.T, s.k, s.E, c.bm);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes, 256);
        return o;
    };
    w.sorted = take(w.cap * 4);
    w.tile_expert = take((w.cap / (size_t)c.bm) * 4);
    w.tile_rows = take((w.cap / (size_t)c.bm) * 4);
    w.counts = take((size_t)s.E * 4);
    w.meta = take(16);
    // router weight per sorted slot, for the kernels that read it by slot (persistent ping-pong down-projection)
    w.slot_w = (c.mode & kModePingPong) ? take(w.cap * 4) : off;
    w.align_ws_bytes = ramp_align_workspace_bytes(s.T, s.k, s.E);
    w.align_ws = take(w.align_ws_bytes);
    w.a_buf = take(align_up(w.cap, 16) * (size_t)s.I * 2);  // fragment-major: whole blocks of 16 slots
    w.y_buf = take((size_t)s.T * s.k * s.H * 4);  // last: the device-selected variant shares one copy between candidates
    w.total = off;
    return w;
}

// pair / k by multiplication: ceil(2^40 / k).  Exact for pair < 2^30 when k <= 1024 (the error term pair * (magic*k -
// 2^40) stays below 2^40); the 64-bit product must not overflow, which bounds the pairs by 2^64 / magic.
unsigned long long topk_magic_of(int k) { return ((1ull << 40) + (unsigned long long)k - 1) / (unsigned long long)k; }

bool shape_ok(const ramp_shape &s)
{
    if (!(s.T >= 0 && s.k >= 1 && s.k <= 1024 && s.E >= 1 && s.E <= kAlignMaxE && s.H >= 128 && s.I >= 128 &&
          s.H % 128 == 0 && s.I % 128 == 0 && (long long)s.T * s.k < (1ll << 30)))
        return false;
    const unsigned long long P = (unsigned long long)s.T * (unsigned long long)s.k;
    return P <= ~0ull / topk_magic_of(s.k);
}

}  // namespace

bool moe_shape_ok(const ramp_shape &s) { return shape_ok(s); }
bool moe_pair_rows_bf16(const ramp_shape &s) { return (size_t)s.T * s.k * s.H >= kPairRowsBf16Elems; }
unsigned long long moe_topk_magic(int k) { return topk_magic_of(k); }

int num_kernels()
{
    init_registry();
    return g_num_kernels;
}
const KernelInfo &kernel_info(int i)
{
    init_registry();
    return g_kernels[i];
}
const KernelInfo *find_kernel(const ramp_config &c)
{
    init_registry();
    for (int i = 0; i < g_num_kernels; ++i) {
        const ramp_config &k = g_kernels[i].cfg;
        if (k.bm == c.bm && k.bn == c.bn && k.bk == c.bk && k.waves == c.waves && k.stages == c.stages &&
            k.mode == c.mode)
            return &g_kernels[i];
    }
    return nullptr;
}
bool config_valid_for_shape(const KernelInfo &ki, const ramp_shape &s)
{
    const ramp_config &c = ki.cfg;
    if (!shape_ok(s)) return false;
    if (s.H % c.bk || s.I % c.bk) return false;      // whole k-slices
    if ((2 * s.I) % c.bn || s.H % c.bn) return false;  // whole feature tiles in both projections
    // 32-bit element offsets inside the kernels
    const size_t cap = ramp_align_capacity(s.T, s.k, s.E, c.bm);
    if ((cap + 16) * (size_t)s.I >= (1ull << 32) || (size_t)s.T * s.H >= (1ull << 32)) return false;
    if (2ull * s.I * s.H >= (1ull << 32)) return false;
    // the ping-pong kernel keeps stages-1 slices in flight across tile boundaries: a tile must be at least that long
    // (and the up-projection loads its token batches up to four slices ahead)
    if ((c.mode & kModePingPong) && (s.H / c.bk < (c.stages > 4 ? c.stages : 4) || s.I / c.bk < c.stages)) return false;

    return true;
}
// Pool membership (what ramp_get_config enumerates) on top of "runs on this shape": the region analysis of Sec. 4.1
// re-derived for this chip.  GROUP_M variants enter the pool of a shape only where their premise holds: an XCD that
// works on a block of group_m M-tiles x a few N-tiles re-reads the token rows of those M-tiles for every N-block, so
// they must stay in its 4 MB L2: group_m * bm * H * 2 bytes <= 4 MiB.  Outside the pool a variant still runs when
// asked for by name (profiling).
bool config_in_pool(const KernelInfo &ki, const ramp_shape &s)
{
    if (!config_valid_for_shape(ki, s)) return false;
    const int gm = group_m_of_mode(ki.cfg.mode);
    if (gm > 0 && (size_t)gm * ki.cfg.bm * s.H * 2 > ((size_t)4 << 20)) return false;
    return true;
}

int occupancy_estimate(const KernelInfo &ki)
{
    // Workgroups of this configuration resident on one compute unit, from what the compiler reported for its
    // up-projection kernel when the library was built: wavefronts per SIMD allowed by the register allocation
    // (4 SIMDs per unit, at most 8 wavefronts each), and 160 KB of LDS.  The persistent kernels launch one
    // workgroup per unit whatever would fit.
    if (ki.cfg.mode & kModePingPong) return 1;
    const KernelResources *r = find_resources(ki.family, ki.targs, ki.n_targs);
    if (!r) return 0;  // no record for this kernel: the library was not built by its build script
    int waves_per_simd = r->waves_per_simd < 8 ? r->waves_per_simd : 8;
    if (waves_per_simd < 1) waves_per_simd = 1;
    int by_regs = waves_per_simd * 4 / ki.cfg.waves;
    const int by_lds = r->lds_bytes > 0 ? kLdsBytesPerCU / r->lds_bytes : 64;
    int occ = by_lds < by_regs ? by_lds : by_regs;
    return occ < 1 ? 1 : occ;
}

int launch_combine(const float *Y, int y_bf16, const int32_t *ids, int T, int k, int E, int H, uint16_t *out,
                   hipStream_t stream, const int32_t *sel, int n_cand, unsigned skip_mask)
{
    if (T == 0) return RAMP_OK;
    size_t total = (size_t)T * (H / 8);
    unsigned grid = (unsigned)((total + 255) / 256);
    if (grid > (unsigned)kNumCU * 16) grid = kNumCU * 16;
    if (y_bf16)
        hipLaunchKernelGGL(combine_kernel<true>, dim3(grid), dim3(256), 0, stream, Y, ids, T, k, E, H, out, sel, n_cand, skip_mask);
    else
        hipLaunchKernelGGL(combine_kernel<false>, dim3(grid), dim3(256), 0, stream, Y, ids, T, k, E, H, out, sel, n_cand, skip_mask);
    return check_launch("combine_kernel");
}

}  // namespace ramp

using namespace ramp;

extern "C" int ramp_num_configs(const ramp_shape *shape)
{
    if (!shape) {
        set_error("num_configs: NULL shape");
        return RAMP_EINVAL;
    }
    int n = 0;
    for (int i = 0; i < num_kernels(); ++i) n += config_in_pool(kernel_info(i), *shape) ? 1 : 0;
    return n;
}

extern "C" int ramp_get_config(const ramp_shape *shape, int idx, ramp_config *out)
{
    if (!shape || !out || idx < 0) {
        set_error("get_config: bad argument");
        return RAMP_EINVAL;
    }
    int n = 0;
    for (int i = 0; i < num_kernels(); ++i) {
        if (!config_in_pool(kernel_info(i), *shape)) continue;
        if (n++ == idx) {
            *out = kernel_info(i).cfg;
            return RAMP_OK;
        }
    }
    set_error("get_config: index %d out of range (%d valid)", idx, n);
    return RAMP_EINVAL;
}

extern "C" int ramp_config_ntiles(const ramp_shape *shape, const ramp_config *cfg)
{
    if (!shape || !cfg || cfg->bn <= 0) {
        set_error("config_ntiles: bad argument");
        return RAMP_EINVAL;
    }
    return (2 * shape->I + cfg->bn - 1) / cfg->bn + (shape->H + cfg->bn - 1) / cfg->bn;
}

extern "C" int ramp_config_rounds(const ramp_shape *shape, const ramp_config *cfg, int32_t out[4])
{
    if (!shape || !cfg || !out || cfg->bn <= 0 || shape->H <= 0 || shape->I <= 0) {
        set_error("config_rounds: bad argument");
        return RAMP_EINVAL;
    }
    const int nt[2] = {(2 * shape->I + cfg->bn - 1) / cfg->bn, (shape->H + cfg->bn - 1) / cfg->bn};
    for (int s = 0; s < 2; ++s) {
        int gm = 1, gn = 1;
        // only the persistent kernels walk the map with a fixed set of workgroups; the others are dispatched
        // tile by tile as compute units free up
        if ((cfg->mode & kModePingPong) && !(cfg->mode & kModeFp8)) xcd_block_shape(nt[s], group_m_of_mode(cfg->mode), &gm, &gn);
        out[2 * s] = (cfg->mode & kModePingPong) && !(cfg->mode & kModeFp8) ? 8 * gm : 1;
        out[2 * s + 1] = nt[s];
    }
    return RAMP_OK;
}

extern "C" int ramp_config_wave_capacity(const ramp_config *cfg)
{
    if (!cfg) {
        set_error("config_wave_capacity: NULL config");
        return RAMP_EINVAL;
    }
    const KernelInfo *ki = find_kernel(*cfg);
    if (!ki) {
        set_error("config_wave_capacity: configuration not instantiated");
        return RAMP_EUNSUPPORTED;
    }
    const int occ = occupancy_estimate(*ki);
    if (occ <= 0) {
        set_error("config_wave_capacity: no compiler resource record for this kernel (rebuild with paper_2604_26039_amd.build)");
        return RAMP_EUNSUPPORTED;
    }
    return kNumCU * occ;
}

extern "C" int ramp_config_runtime_occupancy(const ramp_config *cfg, int *wg_per_cu)
{
    if (!cfg || !wg_per_cu) {
        set_error("config_runtime_occupancy: NULL argument");
        return RAMP_EINVAL;
    }
    const KernelInfo *ki = find_kernel(*cfg);
    if (!ki) {
        set_error("config_runtime_occupancy: configuration not instantiated");
        return RAMP_EUNSUPPORTED;
    }
    for (int st = 0; st < 2; ++st) {
        int n = 0;
        hipError_t err = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, ki->kernel_fn[st], ki->block_threads, 0);
        if (err != hipSuccess) {
            set_error("config_runtime_occupancy: %s", hipGetErrorString(err));
            return RAMP_EHIP;
        }
        wg_per_cu[st] = n;
    }
    return RAMP_OK;
}

extern "C" size_t ramp_fused_moe_workspace_bytes(const ramp_shape *shape, const ramp_config *cfg)
{
    if (!shape || !cfg || cfg->bm <= 0 || !shape_ok(*shape)) return 0;
    return workspace_layout(*shape, *cfg).total;
}

extern "C" int ramp_fused_moe_workspace_layout(const ramp_shape *shape, const ramp_config *cfg, size_t offsets[4])
{
    if (!shape || !cfg || !offsets || cfg->bm <= 0 || !shape_ok(*shape)) {
        set_error("workspace_layout: bad argument");
        return RAMP_EINVAL;
    }
    Workspace w = workspace_layout(*shape, *cfg);
    offsets[0] = w.sorted;
    offsets[1] = w.tile_expert;
    offsets[2] = w.counts;
    offsets[3] = w.meta;
    return RAMP_OK;
}

namespace {

// Checks shared by the fused entry points.  Returns RAMP_OK and the kernel of cfg, or a status.
int check_fused_call(const char *who, const ramp_shape *shape, const ramp_config *cfg, const KernelInfo **ki)
{
    if (!shape || !cfg) {
        set_error("%s: NULL shape or config", who);
        return RAMP_EINVAL;
    }
    const ramp_shape &s = *shape;
    if (!shape_ok(s)) {
        set_error("%s: unsupported shape T=%d k=%d E=%d H=%d I=%d (need H, I multiples of 128, E<=%d)", who, s.T, s.k,
                  s.E, s.H, s.I, kAlignMaxE);
        return RAMP_EUNSUPPORTED;
    }
    *ki = find_kernel(*cfg);
    if (!*ki) {
        set_error("%s: configuration (bm=%d bn=%d bk=%d waves=%d stages=%d mode=%d) is not instantiated", who,
                  cfg->bm, cfg->bn, cfg->bk, cfg->waves, cfg->stages, cfg->mode);
        return RAMP_EUNSUPPORTED;
    }
    if (!config_valid_for_shape(**ki, s)) {
        set_error("%s: configuration bm=%d bn=%d bk=%d does not tile H=%d I=%d", who, cfg->bm, cfg->bn, cfg->bk, s.H,
                  s.I);
        return RAMP_EUNSUPPORTED;
    }
    return RAMP_OK;
}

int check_fused_buffers(const char *who, const void *X, const void *topk_ids, const void *topk_w, const void *packed,
                        const void *out, const void *ws)
{
    if (!X || !topk_ids || !topk_w || !packed || !out || !ws) {
        set_error("%s: NULL buffer", who);
        return RAMP_EINVAL;
    }
    if (reinterpret_cast<uintptr_t>(ws) % 256 || reinterpret_cast<uintptr_t>(packed) % 256 ||
        reinterpret_cast<uintptr_t>(X) % 16 || reinterpret_cast<uintptr_t>(out) % 16) {
        set_error("%s: misaligned buffer (ws/packed 256 B, X and out 16 B)", who);
        return RAMP_EINVAL;
    }
    return RAMP_OK;
}

bool pair_rows_bf16(const ramp_shape &s)
{
    // per-pair rows: fp32 while they are small, bf16 once they would exceed 32 MB
    return (size_t)s.T * s.k * s.H >= kPairRowsBf16Elems;
}

// align(bm) + both projections of one configuration; `base` holds every workspace section but the per-pair rows,
// which go to y_buf.  With pred != NULL every launch is a no-op unless *pred == pred_value on the device.
// *wrote_out is set when the configuration's launches wrote `out` themselves (two-launch decode form): no combine then.
int enqueue_projections(const ramp_shape &s, const ramp_config &cfg, const KernelInfo &ki, const Workspace &w, const void *X,
                        const int32_t *topk_ids, const float *topk_w, const void *packed_weights, char *base,
                        float *y_buf, void *out, const int32_t *pred, int pred_value, hipStream_t st, bool *wrote_out)
{
    *wrote_out = false;
    int32_t *sorted = reinterpret_cast<int32_t *>(base + w.sorted);
    int32_t *tile_expert = reinterpret_cast<int32_t *>(base + w.tile_expert);
    int32_t *tile_rows = reinterpret_cast<int32_t *>(base + w.tile_rows);
    int32_t *counts = reinterpret_cast<int32_t *>(base + w.counts);
    int32_t *meta = reinterpret_cast<int32_t *>(base + w.meta);
    uint16_t *a_buf = reinterpret_cast<uint16_t *>(base + w.a_buf);

    const PackedLayout L = packed_layout(s);
    const uint16_t *packed = static_cast<const uint16_t *>(packed_weights);
    const int P = s.T * s.k;
    if (ki.launch_decode_up && P <= kDecodeMaxPairs && 16 % s.k == 0) {
        // decode-sized call: align + up-projection + SwiGLU in one launch, down-projection + top-k sum in the other
        GemmArgs g = {};
        g.act = static_cast<const uint16_t *>(X);
        g.wpacked = packed;
        g.expert_stride = L.w1_expert_elems;
        g.up_offset = L.up_offset_elems;
        g.a_out = a_buf;
        g.a_row_major = 1;
        g.K = s.H;
        g.F = s.I;
        g.P = P;
        g.topk = s.k;
        g.n_tiles = 2 * s.I / cfg.bn;
        g.m_tiles_cap = (int)(w.cap / (size_t)cfg.bm);
        g.pred = pred;
        g.pred_value = pred_value;
        DecodeArgs da = {topk_ids, s.E, cfg.bm, (int)w.cap, sorted, tile_expert, tile_rows, counts, meta};
        {
            ProbeScope probe(2, st);
            ki.launch_decode_up(g, da, st);
        }
        if (int rc = check_launch("moe_decode_up_kernel")) return rc;
        DecodeDownArgs dd = {a_buf, packed + L.w2_base_elems, L.w2_expert_elems, topk_ids, topk_w, static_cast<uint16_t *>(out),
                             s.T, s.k, s.E, s.H, s.I, pred, pred_value};
        {
            ProbeScope probe(3, st);
            launch_decode_down_any(dd, st);
        }
        *wrote_out = true;
        return check_launch("moe_decode_down_kernel");
    }

    int rc;
    {
        ProbeScope probe(1, st);
        AlignSlotWeights sw = {nullptr, nullptr};
        if (cfg.mode & kModePingPong) sw = AlignSlotWeights{topk_w, reinterpret_cast<float *>(base + w.slot_w)};
        rc = launch_align(topk_ids, s.T, s.k, s.E, cfg.bm, sorted, tile_expert, tile_rows, counts, meta, base + w.align_ws,
                          w.align_ws_bytes, st, pred, pred_value, sw);
    }
    if (rc) return rc;

    GemmArgs g = {};
    g.sorted = sorted;
    g.slot_w = (cfg.mode & kModePingPong) ? reinterpret_cast<const float *>(base + w.slot_w) : nullptr;
    g.tile_expert = tile_expert;
    g.tile_rows = tile_rows;
    g.topk_magic = topk_magic_of(s.k);
    g.meta = meta;
    g.topk_w = topk_w;
    g.a_out = a_buf;
    g.y_out = y_buf;
    g.y_bf16 = pair_rows_bf16(s) ? 1 : 0;
    g.P = s.T * s.k;
    g.topk = s.k;
    g.m_tiles_cap = (int)(w.cap / (size_t)cfg.bm);
    g.pred = pred;
    g.pred_value = pred_value;
    g.group_m_req = group_m_of_mode(cfg.mode);

    // phase 1 + 2: up-projection with SwiGLU epilogue
    g.act = static_cast<const uint16_t *>(X);
    g.wpacked = packed;
    g.expert_stride = L.w1_expert_elems;
    g.up_offset = L.up_offset_elems;
    g.K = s.H;
    g.F = s.I;
    g.n_tiles = 2 * s.I / cfg.bn;
    {
        ProbeScope probe(2, st);
        ki.launch(1, g, st);
    }
    rc = check_launch("moe_gemm_kernel<1>");
    if (rc) return rc;

    // phase 3: down-projection, router weight applied, one row per pair
    g.act = a_buf;
    g.wpacked = packed + L.w2_base_elems;
    g.expert_stride = L.w2_expert_elems;
    g.up_offset = 0;
    g.K = s.I;
    g.F = s.H;
    g.n_tiles = s.H / cfg.bn;
    {
        ProbeScope probe(3, st);
        ki.launch(2, g, st);
    }
    return check_launch("moe_gemm_kernel<2>");
}

}  // namespace

extern "C" int ramp_fused_moe(const ramp_shape *shape, const ramp_config *cfg, const void *X, const int32_t *topk_ids,
                              const float *topk_w, const void *packed_weights, void *out, void *ws, size_t ws_bytes,
                              void *stream)
{
    const KernelInfo *ki = nullptr;
    if (int rc = check_fused_call("fused_moe", shape, cfg, &ki)) return rc;
    const ramp_shape &s = *shape;
    if (s.T == 0) return RAMP_OK;
    if (int rc = check_fused_buffers("fused_moe", X, topk_ids, topk_w, packed_weights, out, ws)) return rc;
    const Workspace w = workspace_layout(s, *cfg);
    if (ws_bytes < w.total) {
        set_error("fused_moe: workspace %zu < %zu bytes", ws_bytes, w.total);
        return RAMP_ENOSPC;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *base = static_cast<char *>(ws);
    float *y_buf = reinterpret_cast<float *>(base + w.y_buf);
    bool wrote_out = false;
    if (int rc = enqueue_projections(s, *cfg, *ki, w, X, topk_ids, topk_w, packed_weights, base, y_buf, out, nullptr, 0, st,
                                     &wrote_out))
        return rc;
    if (wrote_out) return RAMP_OK;
    ProbeScope probe(4, st);
    return launch_combine(y_buf, pair_rows_bf16(s) ? 1 : 0, topk_ids, s.T, s.k, s.E, s.H, static_cast<uint16_t *>(out), st);
}

// ---- fused layer for callers that cannot allocate -------------------------------------------------------------
// The workspace of ramp_fused_moe (align result, activation A, per-pair rows Y) lives in a device array that is
// part of the library image: every GPU the library runs on holds its own copy at its own address until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the address it returns
// for the current device is what kernels and size checks use.
static __device__ __align__(256) unsigned char scratch[RAMP_STATIC_WS_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up once per device), or NULL with the error set.
void *static_workspace()
{
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        set_error("fused_moe_static: hipGetDevice: %s (device %d)", hipGetErrorString(err), dev);
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (err != hipSuccess || !ptr) {
            set_error("fused_moe_static: hipGetSymbolAddress: %s", hipGetErrorString(err));
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

extern "C" int ramp_fused_moe_static(const ramp_shape *shape, const ramp_config *cfg, const void *X,
                                     const int32_t *topk_ids, const float *topk_w, const void *packed_weights, void *out,
                                     void *stream)
{
    const KernelInfo *ki = nullptr;
    if (int rc = check_fused_call("fused_moe_static", shape, cfg, &ki)) return rc;
    const size_t need = workspace_layout(*shape, *cfg).total;
    if (need > (size_t)RAMP_STATIC_WS_BYTES) {
        set_error("fused_moe_static: this shape and configuration need %zu bytes of workspace, the built-in one has %zu; "
                  "use ramp_fused_moe with a caller-provided workspace",
                  need, (size_t)RAMP_STATIC_WS_BYTES);
        return RAMP_ENOSPC;
    }
    if (shape->T == 0) return RAMP_OK;
    void *ws = static_workspace();
    if (!ws) return RAMP_EHIP;
    // nothing in the workspace has to start at zero: every section is written before it is read
    return ramp_fused_moe(shape, cfg, X, topk_ids, topk_w, packed_weights, out, ws, (size_t)RAMP_STATIC_WS_BYTES, stream);
}

// Workspace of the device-selected variant: the per-pair rows first (their size does not depend on the
// configuration), then room for the other sections of the largest candidate.
static size_t selected_rest_bytes(const ramp_shape &s, int n_cand, const ramp_config *cfgs)
{
    size_t rest = 0;
    for (int c = 0; c < n_cand; ++c) {
        const Workspace w = workspace_layout(s, cfgs[c]);
        rest = w.y_buf > rest ? w.y_buf : rest;  // y_buf is the last section: its offset is the size of the others
    }
    return rest;
}

extern "C" size_t ramp_fused_moe_selected_workspace_bytes(const ramp_shape *shape, int n_cand, const ramp_config *cfgs)
{
    if (!shape || !cfgs || n_cand <= 0 || !shape_ok(*shape)) return 0;
    for (int c = 0; c < n_cand; ++c)
        if (cfgs[c].bm <= 0) return 0;
    return align_up((size_t)shape->T * shape->k * shape->H * 4, 256) + selected_rest_bytes(*shape, n_cand, cfgs);
}

extern "C" int ramp_fused_moe_selected(const ramp_shape *shape, int n_cand, const ramp_config *cfgs,
                                       const int32_t *selected_idx, const void *X, const int32_t *topk_ids,
                                       const float *topk_w, const void *packed_weights, void *out, void *ws,
                                       size_t ws_bytes, void *stream)
{
    if (n_cand <= 0 || n_cand > 16 || !cfgs || !selected_idx) {
        set_error("fused_moe_selected: need 1..16 candidate configurations and a device index");
        return RAMP_EINVAL;
    }
    const KernelInfo *ki[16];
    for (int c = 0; c < n_cand; ++c)
        if (int rc = check_fused_call("fused_moe_selected", shape, &cfgs[c], &ki[c])) return rc;
    const ramp_shape &s = *shape;
    if (s.T == 0) return RAMP_OK;
    if (int rc = check_fused_buffers("fused_moe_selected", X, topk_ids, topk_w, packed_weights, out, ws)) return rc;
    const size_t need = ramp_fused_moe_selected_workspace_bytes(shape, n_cand, cfgs);
    if (ws_bytes < need) {
        set_error("fused_moe_selected: workspace %zu < %zu bytes", ws_bytes, need);
        return RAMP_ENOSPC;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    float *y_buf = static_cast<float *>(ws);
    char *base = static_cast<char *>(ws) + align_up((size_t)s.T * s.k * s.H * 4, 256);
    // every candidate is enqueued; on the device only the one whose position equals *selected_idx does anything
    unsigned self_combined = 0;  // candidates whose own launches write `out` (two-launch decode form)
    for (int c = 0; c < n_cand; ++c) {
        const Workspace w = workspace_layout(s, cfgs[c]);
        bool wrote_out = false;
        if (int rc = enqueue_projections(s, cfgs[c], *ki[c], w, X, topk_ids, topk_w, packed_weights, base, y_buf, out,
                                         selected_idx, c, st, &wrote_out))
            return rc;
        if (wrote_out) self_combined |= 1u << c;
    }
    ProbeScope probe(4, st);
    return launch_combine(y_buf, pair_rows_bf16(s) ? 1 : 0, topk_ids, s.T, s.k, s.E, s.H, static_cast<uint16_t *>(out), st,
                          selected_idx, n_cand, self_combined);
}

extern "C" int ramp_probe_enable(int stage)
{
    if (stage < 0 || stage > 4) {
        set_error("probe_enable: stage must be 0..4");
        return RAMP_EINVAL;
    }
    std::lock_guard<std::mutex> lock(g_probe_mutex);
    g_probe_stage = stage;
    return RAMP_OK;
}

extern "C" int ramp_probe_read(double *total_ms, int *launches)
{
    if (!total_ms || !launches) {
        set_error("probe_read: NULL argument");
        return RAMP_EINVAL;
    }
    std::lock_guard<std::mutex> lock(g_probe_mutex);
    double sum = 0.0;
    for (int i = 0; i < g_probe_used; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(g_probe_ev[i][1]) != hipSuccess ||
            hipEventElapsedTime(&ms, g_probe_ev[i][0], g_probe_ev[i][1]) != hipSuccess) {
            set_error("probe_read: event query failed");
            g_probe_used = 0;
            return RAMP_EHIP;
        }
        sum += ms;
    }
    *total_ms = sum;
    *launches = g_probe_used;
    g_probe_used = 0;
    return RAMP_OK;
}
