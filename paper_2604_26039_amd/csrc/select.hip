// Device-resident dispatch: histogram, cost model and argmin in one enqueue (Sec. 4.4 steps 1-3), with
// the result written straight into host-visible memory so that the host learns the chosen configuration
// by polling one word instead of copying the histogram back and synchronising the stream.
//
// The model is evaluated exactly as ramp_cost_model_select does it (fp64, same operation order, lowest
// index among equal predictions), so both pick the same configuration from the same histogram; only the
// printed model's logarithm may differ in its last bit between the device and the host math library.
#include <chrono>

#include "ramp_internal.h"

namespace ramp {
namespace {

constexpr int NT = 1024;
constexpr int NW = NT / kWave;
constexpr int kMaxBm = 28;  // distinct bm values a table can hold
constexpr int kSingleMaxP = 8192;  // up to this many pairs the select kernel makes the histogram itself

// Table in device memory (built on the host by ramp_select_table_build).
struct TableHeader {
    int32_t magic, n_cfg, n_bm, flags;
    int32_t bm[kMaxBm];
};
struct TableRow {
    int32_t bm_slot, ntiles, wave_cap, reserved;
    float theta[4];
    int32_t rounds[4];  // M-tiles per hand-out round and N-tiles of the two launches (RAMP_CM_ROUNDS)
};
static_assert(sizeof(TableHeader) == 128 && sizeof(TableRow) == 48, "table layout is part of the ABI");
constexpr int32_t kMagic = 0x52614d50;

// Result block: word = best << 32 | ticket (one 64-bit store, written last) | n_cfg | 0 | pred_us[n_cfg] (fp64) | counts[E]
struct ResultHeader {
    unsigned long long word;
    int32_t n_cfg, reserved;
};
static_assert(sizeof(ResultHeader) == 16, "result layout is part of the ABI");

__global__ __launch_bounds__(NT) void select_kernel(const int32_t *ids, int P, int B, const int32_t *block_counts, int E,
                                                    int n_cfg, const TableHeader *table, ResultHeader *res,
                                                    uint32_t ticket, int32_t *best_dev)
{
    __shared__ int hist[kAlignMaxE];
    __shared__ int mt[kMaxBm];
    __shared__ int active_pairs[2];
    const int tid = threadIdx.x, lane = tid & 63;
    // n_cfg is the caller's (the result block was sized with it); a table that is not one of
    // ramp_select_table_build's for that many configurations yields best = -1 and no predictions
    const bool table_ok = table->magic == kMagic && table->n_cfg == n_cfg && table->n_bm >= 1 && table->n_bm <= kMaxBm;
    const int n_bm = table_ok ? table->n_bm : 0, flags = table->flags;
    const int n_eval = table_ok ? n_cfg : 0;
    const TableRow *rows = reinterpret_cast<const TableRow *>(table + 1);
    double *pred = reinterpret_cast<double *>(res + 1);
    int32_t *counts_out = reinterpret_cast<int32_t *>(pred + n_cfg);

    if (tid < kMaxBm) mt[tid] = 0;
    if (tid < 2) active_pairs[tid] = 0;
    // ---- histogram: own pass over the ids (small inputs), or the per-chunk histograms of align_hist_kernel
    if (tid < E) hist[tid] = 0;
    __syncthreads();
    if (B == 0) {
        for (int p = tid; p < P; p += NT) {
            const int v = ids[p];
            if (v >= 0 && v < E) atomicAdd(&hist[v], 1);
        }
    } else {
        // all lanes share the B x E chunk counts (coalesced; integer sums do not depend on the order)
        for (int i = tid; i < B * E; i += NT) atomicAdd(&hist[i % E], block_counts[i]);
    }
    __syncthreads();
    const int n = (tid < E) ? hist[tid] : 0;
    // ---- sums over the experts: M-tiles for every distinct bm, active experts, routed pairs
    if ((tid & ~63) < E) {  // wavefronts that hold experts
        for (int j = 0; j < n_bm + 2; ++j) {
            int v;
            if (j < n_bm) {
                const int bm = table->bm[j];
                v = (n + bm - 1) / bm;
            } else {
                v = (j == n_bm) ? (n > 0 ? 1 : 0) : n;
            }
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, kWave);
            if (lane == 0) atomicAdd(j < n_bm ? &mt[j] : &active_pairs[j - n_bm], v);
        }
    }
    __syncthreads();
    if (tid >= kWave) return;
    // ---- the model for every configuration, and the lowest index with the smallest prediction
    const bool use_distinct = (flags & RAMP_CM_DISTINCT_TILES) != 0;
    const bool wave_floor = (flags & RAMP_CM_WAVE_FLOOR) != 0;
    const bool use_pairs = (flags & RAMP_CM_PAIRS) != 0;
    const bool use_rounds = (flags & RAMP_CM_ROUNDS) != 0;
    const long long active = active_pairs[0], pairs = active_pairs[1];
    int best = -1;
    double best_t = 0.0;
    for (int c = lane; c < n_eval; c += kWave) {
        const TableRow r = rows[c];
        const double g = (double)((long long)mt[r.bm_slot] * (long long)r.ntiles);
        double t = (double)r.theta[0];
        double gw = g;
        if (use_rounds) {
            const long long m = mt[r.bm_slot];
            long long gr = 0;
            for (int s = 0; s < 2; ++s) {
                const long long R = r.rounds[2 * s], nt = r.rounds[2 * s + 1];
                gr += (m + R - 1) / R * R * nt;
            }
            gw = (double)gr;
        }
        const double w = gw / (double)r.wave_cap;
        t = t + (double)r.theta[1] * ((wave_floor && w < 1.0) ? 1.0 : w);
        const double m = use_distinct ? (double)(active * (long long)r.ntiles) : g;
        t = t + (double)r.theta[2] * m;
        t = t + (double)r.theta[3] * (use_pairs ? (double)pairs : log(g + 1.0));
        pred[c] = t;
        if (best < 0 || t < best_t) {
            best = c;
            best_t = t;
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const int ob = __shfl_xor(best, d, kWave);
        const double ot = __shfl_xor(best_t, d, kWave);
        if (ob >= 0 && (best < 0 || ot < best_t || (ot == best_t && ob < best))) {
            best = ob;
            best_t = ot;
        }
    }
    // Only this wavefront writes the result block: payload, one system-scope fence (one round trip to host
    // memory), then the word that carries the ticket.
    for (int e = lane; e < E; e += kWave) counts_out[e] = hist[e];
    if (lane == 0) {
        res->n_cfg = n_cfg;
        res->reserved = 0;
        if (best_dev) *best_dev = best;
    }
    __threadfence_system();  // every lane's payload stores are complete and visible to the host ...
    if (lane == 0)           // ... before the word that announces them (the fence above is the release)
        __hip_atomic_store(&res->word, ((unsigned long long)(uint32_t)best << 32) | ticket, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_SYSTEM);
}

}  // namespace

// align.hip: per-chunk histograms of the multi-workgroup path (block_counts[B][E] at the start of ws)
int launch_chunk_histograms(const int32_t *ids, int P, int E, void *ws, size_t ws_bytes, hipStream_t stream, int *B_out);

}  // namespace ramp

extern "C" size_t ramp_select_table_bytes(int n_cfg)
{
    if (n_cfg <= 0) return 0;
    return sizeof(ramp::TableHeader) + (size_t)n_cfg * sizeof(ramp::TableRow);
}

extern "C" int ramp_select_table_build(int n_cfg, const ramp_config *cfgs, const int32_t *ntiles, const int32_t *wave_cap,
                                       const float *theta, int flags, const int32_t *rounds, void *table,
                                       size_t table_bytes)
{
    using namespace ramp;
    if (n_cfg <= 0 || n_cfg > 1024 || !cfgs || !ntiles || !wave_cap || !theta || !table ||
        ((flags & RAMP_CM_ROUNDS) && !rounds)) {
        set_error("select_table_build: bad argument (1 <= n_cfg <= 1024, no NULL)");
        return RAMP_EINVAL;
    }
    if (table_bytes < ramp_select_table_bytes(n_cfg)) {
        set_error("select_table_build: table %zu < %zu bytes", table_bytes, ramp_select_table_bytes(n_cfg));
        return RAMP_ENOSPC;
    }
    TableHeader h = {};
    h.magic = kMagic;
    h.n_cfg = n_cfg;
    h.flags = flags;
    TableRow *rows = reinterpret_cast<TableRow *>(static_cast<char *>(table) + sizeof(TableHeader));
    for (int c = 0; c < n_cfg; ++c) {
        if (cfgs[c].bm <= 0 || wave_cap[c] <= 0) {
            set_error("select_table_build: config %d has bm=%d wave_cap=%d", c, cfgs[c].bm, wave_cap[c]);
            return RAMP_EINVAL;
        }
        int slot = 0;
        while (slot < h.n_bm && h.bm[slot] != cfgs[c].bm) ++slot;
        if (slot == h.n_bm) {
            if (h.n_bm == kMaxBm) {
                set_error("select_table_build: more than %d distinct bm values", kMaxBm);
                return RAMP_EUNSUPPORTED;
            }
            h.bm[h.n_bm++] = cfgs[c].bm;
        }
        if (rounds && (rounds[4 * c] <= 0 || rounds[4 * c + 2] <= 0)) {
            set_error("select_table_build: config %d has a round of %d / %d M-tiles", c, rounds[4 * c], rounds[4 * c + 2]);
            return RAMP_EINVAL;
        }
        rows[c] = TableRow{slot, ntiles[c], wave_cap[c], 0, {theta[4 * c], theta[4 * c + 1], theta[4 * c + 2], theta[4 * c + 3]},
                           {rounds ? rounds[4 * c] : 1, rounds ? rounds[4 * c + 1] : ntiles[c], rounds ? rounds[4 * c + 2] : 1, rounds ? rounds[4 * c + 3] : 0}};
    }
    *static_cast<TableHeader *>(table) = h;
    return RAMP_OK;
}

extern "C" size_t ramp_select_result_bytes(int E, int n_cfg)
{
    if (E <= 0 || n_cfg <= 0) return 0;
    return ramp::align_up(sizeof(ramp::ResultHeader) + (size_t)n_cfg * sizeof(double) + (size_t)E * sizeof(int32_t), 64);
}

extern "C" int ramp_select_device(const int32_t *topk_ids, int T, int k, int E, int n_cfg, const void *table,
                                  void *result, uint32_t ticket, int32_t *best_idx_dev, void *ws, size_t ws_bytes,
                                  void *stream)
{
    using namespace ramp;
    if (T < 0 || k < 0 || E <= 0 || E > kAlignMaxE || n_cfg <= 0 || n_cfg > 1024 || !table || !result || ticket == 0) {
        set_error("select_device: bad argument (E <= %d, 1 <= n_cfg <= 1024, ticket != 0, no NULL table/result)", kAlignMaxE);
        return RAMP_EINVAL;
    }
    const long long P64 = (long long)T * k;
    if (P64 >= (1ll << 30) || (P64 > 0 && !topk_ids)) {
        set_error("select_device: T*k=%lld too large or NULL ids", P64);
        return RAMP_EINVAL;
    }
    const int P = (int)P64;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int B = 0;
    if (P > kSingleMaxP) {
        if (int rc = launch_chunk_histograms(topk_ids, P, E, ws, ws_bytes, s, &B)) return rc;
    }
    hipLaunchKernelGGL(select_kernel, dim3(1), dim3(NT), 0, s, topk_ids, P, B, static_cast<const int32_t *>(ws), E,
                       n_cfg, static_cast<const TableHeader *>(table), static_cast<ResultHeader *>(result), ticket,
                       best_idx_dev);
    return check_launch("select_kernel");
}

extern "C" int ramp_select_poll(const void *result_host, uint32_t ticket, int *best_idx)
{
    if (!result_host || !best_idx) {
        ramp::set_error("select_poll: NULL argument");
        return RAMP_EINVAL;
    }
    const ramp::ResultHeader *r = static_cast<const ramp::ResultHeader *>(result_host);
    const unsigned long long w = __atomic_load_n(&r->word, __ATOMIC_ACQUIRE);
    if ((uint32_t)w != ticket) return 1;
    *best_idx = (int32_t)(w >> 32);
    if (*best_idx < 0) {
        ramp::set_error("select: the kernel rejected its table (not built by ramp_select_table_build for this n_cfg)");
        return RAMP_EINVAL;
    }
    return RAMP_OK;
}

extern "C" int ramp_select_wait(const void *result_host, uint32_t ticket, double timeout_s, int *best_idx)
{
    if (!result_host || !best_idx) {
        ramp::set_error("select_wait: NULL argument");
        return RAMP_EINVAL;
    }
    const auto t0 = std::chrono::steady_clock::now();
    for (unsigned spin = 1;; ++spin) {
        const int rc = ramp_select_poll(result_host, ticket, best_idx);
        if (rc <= 0) return rc;
        if ((spin & 0x3ff) == 0 &&
            std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count() > timeout_s) {
            ramp::set_error("select_wait: ticket %u not reached within %.3f s", ticket, timeout_s);
            return RAMP_EHIP;
        }
    }
}
