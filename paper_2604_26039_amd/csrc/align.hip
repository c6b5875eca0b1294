// Route-align step: group (token, expert) pairs into bm-padded per-expert blocks
// (paper Eq. 1, first factor; Fig. 1) and the expert histogram that the cost model
// consumes (Sec. 4.4 step 1).
//
// Integer work only.  The layout is made unique by keeping pairs of one expert in
// increasing pair index, so no step may depend on the arrival order of atomics:
//   - the histogram uses LDS integer atomics (their sum is order independent);
//   - ranks inside an expert come from a wavefront ballot (lanes of lower index),
//     a per-wavefront count table in LDS (wavefronts of lower index) and a running
//     cursor (earlier chunks / earlier workgroups).
// Up to 64 pairs a single wavefront does everything; up to kAlignSingleMaxP pairs one
// 1024-lane workgroup does histogram, scan and scatter in a single launch; larger inputs take two launches (per-chunk
// histograms, then a kernel in which every workgroup scans them and scatters
// its chunk); the histogram-only entry point ends with a small scan kernel.
#include "ramp_internal.h"
#include "align_tiny.h"

namespace ramp {
namespace {

constexpr int NT = kAlignThreads;
constexpr int NW = NT / kWave;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// Exclusive prefix sum of one int per lane over the whole 1024-lane workgroup.
// wsum: LDS scratch of NW ints.  Returns the exclusive prefix; *total gets the sum.
__device__ int block_exclusive_scan(int v, int *wsum, int *total)
{
    const int lane = lane_id(), wv = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        int up = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += up;
    }
    if (lane == kWave - 1) wsum[wv] = incl;
    __syncthreads();
    int woff = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        int s = wsum[w];
        if (w < wv) woff += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return woff + incl - v;
}

// Histogram of ids[begin, end) into LDS hist[E] (must be zeroed); out-of-range ids go to *dropped.
__device__ void block_histogram(const int32_t *ids, int begin, int end, int E, int *hist, int *dropped)
{
    for (int p = begin + (int)threadIdx.x; p < end; p += NT) {
        int v = ids[p];
        if (v >= 0 && v < E) atomicAdd(&hist[v], 1);
        else atomicAdd(dropped, 1);
    }
}

// From n_e (one expert per lane, 0 beyond E): slot offsets toff[0..E] and the counts nreal[0..E) in LDS,
// counts / meta / tile_expert / tile_rows in global memory.  Called by all NT lanes; E <= NT.
__device__ void block_scan_and_emit(int n_e, int E, int bm, int cap, int dropped_total, int *toff, int *wsum,
                                    int *nreal, int32_t *counts, int32_t *meta, int32_t *tile_expert,
                                    int32_t *tile_rows, bool emit = true)
{
    const int e = threadIdx.x;
    if (e < E) nreal[e] = n_e;
    int slots = (e < E) ? (n_e + bm - 1) / bm * bm : 0;
    int p_pad;
    int off = block_exclusive_scan(slots, wsum, &p_pad);
    if (e < E) {
        toff[e] = off;
        if (emit) counts[e] = n_e;
    }
    if (e == 0) {
        toff[E] = p_pad;
        if (emit) {
            meta[0] = p_pad;
            meta[1] = p_pad / bm;
            meta[2] = dropped_total;
            meta[3] = 0;
        }
    }
    __syncthreads();
    if (!emit) return;  // the other workgroups of a launch only need the offsets
    const int m_tiles = p_pad / bm, m_cap = cap / bm;
    for (int m = threadIdx.x; m < m_cap; m += NT) {
        int owner = -1;
        if (m < m_tiles) {
            // first e with toff[e+1] > m*bm  (empty experts have toff[e+1] == toff[e] and are skipped)
            int target = m * bm, lo = 0, hi = E - 1;
            while (lo < hi) {
                int mid = (lo + hi) >> 1;
                if (toff[mid + 1] > target) hi = mid; else lo = mid + 1;
            }
            owner = lo;
        }
        tile_expert[m] = owner;
        // real rows of the tile (the rest of its bm slots is sentinel padding); optional, for the projection kernels
        if (tile_rows) {
            int rows = 0;
            if (owner >= 0) {
                rows = nreal[owner] - (m * bm - toff[owner]);
                rows = rows > bm ? bm : rows;
            }
            tile_rows[m] = rows;
        }
    }
}

// Stable scatter of pairs [base, base + NT) (clipped to P): pair p of expert e goes to
// cursor[e] + (#pairs of e before p in this chunk); cursors then advance past the chunk.
// wcnt: LDS [NW*E] words tagged with `stamp` so they never need re-zeroing.
__device__ void block_scatter_chunk(const int32_t *ids, int base, int P, int E, int *cursor, unsigned *wcnt,
                                    unsigned stamp, int32_t *sorted, AlignSlotWeights slot_weights)
{
    const int ebits = 32 - __clz((E - 1) | 1);  // bits that tell the experts apart
    const int lane = lane_id(), wv = threadIdx.x >> 6;
    const int p = base + (int)threadIdx.x;
    int e = -1;
    if (p < P) {
        int v = ids[p];
        if (v >= 0 && v < E) e = v;
    }
    // Lanes of this wavefront with the same expert, without a loop over the distinct experts: one
    // ballot per bit of the expert index, each lane keeping the side of the ballot its own bit is on.
    const unsigned long long valid = __ballot(e >= 0);
    unsigned long long same = valid;
#pragma unroll
    for (int b = 0; b < 10; ++b) {  // E <= 1024
        if (b < ebits) {
            const bool bit = (e >> b) & 1;
            const unsigned long long m = __ballot(e >= 0 && bit);
            same &= bit ? m : ~m;
        }
    }
    const int rank = __popcll(same & ((1ull << lane) - 1ull));
    if (e >= 0 && rank == 0) wcnt[wv * E + e] = (stamp << 8) | (unsigned)__popcll(same);
    __syncthreads();
    if (e >= 0) {
        int before = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            unsigned v = wcnt[w * E + e];
            if (w < wv && (v >> 8) == stamp) before += (int)(v & 0xffu);
        }
        sorted[cursor[e] + before + rank] = p;
        if (slot_weights.slot_w) slot_weights.slot_w[cursor[e] + before + rank] = slot_weights.topk_w[p];
    }
    __syncthreads();
    for (int x = threadIdx.x; x < E; x += NT) {
        int add = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            unsigned v = wcnt[w * E + x];
            if ((v >> 8) == stamp) add += (int)(v & 0xffu);
        }
        cursor[x] += add;
    }
    __syncthreads();
}

// LDS carve-up (ints): hist[E] | toff[E+1] | wsum[NW] | misc[1] | wcnt[NW*E]
__device__ __forceinline__ void carve(int *lds, int E, int *&hist, int *&toff, int *&wsum, int *&misc, unsigned *&wcnt)
{
    hist = lds;
    toff = hist + E;
    wsum = toff + E + 1;
    misc = wsum + NW;
    wcnt = reinterpret_cast<unsigned *>(misc + 1);
}
size_t lds_ints(int E) { return (size_t)E + (E + 1) + NW + 1 + (size_t)NW * E; }

// ---- single workgroup: everything in one launch ----
__global__ __launch_bounds__(NT) void align_single_kernel(const int32_t *ids, int P, int E, int bm, int cap,
                                                          int32_t *sorted, int32_t *tile_expert, int32_t *tile_rows,
                                                          int32_t *counts, int32_t *meta, int scatter,
                                                          const int32_t *pred, int pred_value,
                                                          AlignSlotWeights slot_weights)
{
    if (launch_deselected(pred, pred_value)) return;
    extern __shared__ int lds[];
    int *hist, *toff, *wsum, *misc;
    unsigned *wcnt;
    carve(lds, E, hist, toff, wsum, misc, wcnt);
    for (int x = threadIdx.x; x < E; x += NT) hist[x] = 0;
    for (int x = threadIdx.x; x < NW * E; x += NT) wcnt[x] = 0;
    if (threadIdx.x == 0) misc[0] = 0;
    __syncthreads();
    block_histogram(ids, 0, P, E, hist, misc);
    if (scatter)
        for (int s = threadIdx.x; s < cap; s += NT) sorted[s] = P;
    __syncthreads();
    if (!scatter) {  // histogram only
        for (int x = threadIdx.x; x < E; x += NT) counts[x] = hist[x];
        return;
    }
    int n_e = ((int)threadIdx.x < E) ? hist[threadIdx.x] : 0;
    int dropped = misc[0];
    block_scan_and_emit(n_e, E, bm, cap, dropped, toff, wsum, hist, counts, meta, tile_expert, tile_rows);
    __syncthreads();
    int *cursor = hist;  // histogram no longer needed
    for (int x = threadIdx.x; x < E; x += NT) cursor[x] = toff[x];
    __syncthreads();
    unsigned stamp = 1;
    for (int base = 0; base < P; base += NT, ++stamp)
        block_scatter_chunk(ids, base, P, E, cursor, wcnt, stamp, sorted, slot_weights);
}

// ---- up to 64 pairs (decode-sized calls): one wavefront, one pair per lane, no workgroup-wide steps ----
constexpr int kAlignTinyMaxP = 64;
constexpr int kAlignTinyMaxCap = 4096;
__global__ __launch_bounds__(kWave) void align_tiny_kernel(const int32_t *ids, int P, int E, int bm, int cap,
                                                           int32_t *sorted, int32_t *tile_expert, int32_t *tile_rows,
                                                           int32_t *counts, int32_t *meta, const int32_t *pred,
                                                           int pred_value, AlignSlotWeights slot_weights)
{
    if (launch_deselected(pred, pred_value)) return;
    __shared__ int n_lds[kAlignMaxE];
    __shared__ int toff[kAlignMaxE + 1];
    int e, rank;
    tiny_align_wavefront(ids, P, E, bm, (int)threadIdx.x, n_lds, toff, e, rank);
    tiny_align_emit(P, E, bm, cap, (int)threadIdx.x, n_lds, toff, e, rank, ids, sorted, tile_expert, tile_rows, counts, meta,
                    slot_weights);
}

// ---- several workgroups: histogram per chunk -> scan -> scatter ----
__global__ __launch_bounds__(NT) void align_hist_kernel(const int32_t *ids, int P, int E, int cap, int32_t *sorted,
                                                        int32_t *block_counts, int32_t *block_dropped, int fill,
                                                        const int32_t *pred, int pred_value)
{
    if (launch_deselected(pred, pred_value)) return;
    extern __shared__ int lds[];
    int *hist = lds, *dropped = lds + E;
    for (int x = threadIdx.x; x < E; x += NT) hist[x] = 0;
    if (threadIdx.x == 0) *dropped = 0;
    __syncthreads();
    const int begin = blockIdx.x * kAlignChunk;
    const int end = min(P, begin + kAlignChunk);
    block_histogram(ids, begin, end, E, hist, dropped);
    if (fill)
        for (int s = blockIdx.x * NT + threadIdx.x; s < cap; s += gridDim.x * NT) sorted[s] = P;
    __syncthreads();
    for (int x = threadIdx.x; x < E; x += NT) block_counts[(size_t)blockIdx.x * E + x] = hist[x];
    if (threadIdx.x == 0) block_dropped[blockIdx.x] = *dropped;
}

__global__ __launch_bounds__(NT) void align_scan_kernel(int B, int E, int bm, int cap, const int32_t *block_counts,
                                                        const int32_t *block_dropped, int32_t *block_base,
                                                        int32_t *tile_expert, int32_t *tile_rows, int32_t *counts,
                                                        int32_t *meta, int scatter)
{
    extern __shared__ int lds[];
    int *toff = lds, *wsum = lds + E + 1, *nreal = wsum + NW;
    const int e = threadIdx.x;
    int n_e = 0;
    if (e < E) {
#pragma unroll 8
        for (int b = 0; b < B; ++b) n_e += block_counts[(size_t)b * E + e];
    }
    if (!scatter) {
        if (e < E) counts[e] = n_e;
        return;
    }
    int dropped = 0;
#pragma unroll 8
    for (int b = 0; b < B; ++b) dropped += block_dropped[b];
    block_scan_and_emit(n_e, E, bm, cap, dropped, toff, wsum, nreal, counts, meta, tile_expert, tile_rows);
    __syncthreads();
    if (e < E) {
        int run = toff[e];
#pragma unroll 8
        for (int b = 0; b < B; ++b) {
            block_base[(size_t)b * E + e] = run;
            run += block_counts[(size_t)b * E + e];
        }
    }
}

// Scan + scatter in one launch: every workgroup sums the per-chunk histograms itself (B x E ints), scans the
// experts, and scatters its own chunk; workgroup 0 also writes counts, meta and the per-tile arrays.
__global__ __launch_bounds__(NT) void align_scan_scatter_kernel(const int32_t *ids, int P, int B, int E, int bm, int cap,
                                                                const int32_t *block_counts,
                                                                const int32_t *block_dropped, int32_t *sorted,
                                                                int32_t *tile_expert, int32_t *tile_rows,
                                                                int32_t *counts, int32_t *meta, const int32_t *pred,
                                                                int pred_value, AlignSlotWeights slot_weights)
{
    if (launch_deselected(pred, pred_value)) return;
    extern __shared__ int lds[];
    int *toff = lds, *wsum = toff + E + 1, *cursor = wsum + NW;
    unsigned *wcnt = reinterpret_cast<unsigned *>(cursor + E);
    const int e = threadIdx.x;
    int n_e = 0, before = 0;
    if (e < E) {
#pragma unroll 8
        for (int b = 0; b < B; ++b) {
            const int c = block_counts[(size_t)b * E + e];
            if (b < (int)blockIdx.x) before += c;
            n_e += c;
        }
    }
    for (int x = threadIdx.x; x < NW * E; x += NT) wcnt[x] = 0;
    int dropped = 0;
    if (blockIdx.x == 0) {
#pragma unroll 8
        for (int b = 0; b < B; ++b) dropped += block_dropped[b];
    }
    // the cursor array holds the counts while workgroup 0 emits the per-tile arrays
    block_scan_and_emit(n_e, E, bm, cap, dropped, toff, wsum, cursor, counts, meta, tile_expert, tile_rows,
                        blockIdx.x == 0);
    __syncthreads();
    if (e < E) cursor[e] = toff[e] + before;
    __syncthreads();
    const int begin = blockIdx.x * kAlignChunk;
    const int end = min(P, begin + kAlignChunk);
    unsigned stamp = 1;
    for (int base = begin; base < end; base += NT, ++stamp)
        block_scatter_chunk(ids, base, end, E, cursor, wcnt, stamp, sorted, slot_weights);
}

int num_blocks(int P) { return (P + kAlignChunk - 1) / kAlignChunk; }

// Dynamic LDS above 64 KB has to be opted into per kernel.
template <typename Kernel>
int allow_lds(Kernel kernel, size_t bytes)
{
    if (bytes <= 64 * 1024) return RAMP_OK;
    hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (err != hipSuccess) {
        set_error("align: cannot reserve %zu bytes of LDS: %s", bytes, hipGetErrorString(err));
        return RAMP_EHIP;
    }
    return RAMP_OK;
}

}  // namespace

// scatter = 0: histogram only (sorted / tile_expert / meta untouched, may be NULL)
static int launch_align_impl(const int32_t *ids, int T, int k, int E, int bm, int32_t *sorted, int32_t *tile_expert,
                             int32_t *tile_rows, int32_t *counts, int32_t *meta, void *ws, size_t ws_bytes,
                             hipStream_t stream, int scatter, const int32_t *pred = nullptr, int pred_value = 0,
                             AlignSlotWeights slot_weights = {nullptr, nullptr})
{
    if (T < 0 || k < 0 || E <= 0 || E > kAlignMaxE || bm < 1 || bm > 1024) {
        set_error("align: bad sizes T=%d k=%d E=%d bm=%d (need E<=%d, 1<=bm<=1024)", T, k, E, bm, kAlignMaxE);
        return RAMP_EINVAL;
    }
    const long long P64 = (long long)T * k;
    if (P64 >= (1ll << 30)) {
        set_error("align: T*k=%lld too large", P64);
        return RAMP_EINVAL;
    }
    const int P = (int)P64;
    if (!counts || (P > 0 && !ids) || (scatter && (!meta || (P > 0 && (!sorted || !tile_expert))))) {
        set_error("align: NULL buffer");
        return RAMP_EINVAL;
    }
    const int cap = scatter ? (int)ramp_align_capacity(T, k, E, bm) : 0;
    if (scatter && P <= kAlignTinyMaxP && cap <= kAlignTinyMaxCap) {
        hipLaunchKernelGGL(align_tiny_kernel, dim3(1), dim3(kWave), 0, stream, ids, P, E, bm, cap, sorted, tile_expert,
                           tile_rows, counts, meta, pred, pred_value, slot_weights);
        return check_launch("align_tiny_kernel");
    }
    if (P <= kAlignSingleMaxP) {
        size_t lds = lds_ints(E) * sizeof(int);
        if (int rc = allow_lds(align_single_kernel, lds)) return rc;
        hipLaunchKernelGGL(align_single_kernel, dim3(1), dim3(NT), lds, stream, ids, P, E, bm, cap, sorted,
                           tile_expert, tile_rows, counts, meta, scatter, pred, pred_value, slot_weights);
        return check_launch("align_single_kernel");
    }
    const int B = num_blocks(P);
    const size_t need = ramp_align_workspace_bytes(T, k, E);
    if (!ws || ws_bytes < need) {
        set_error("align: workspace %zu < %zu bytes", ws_bytes, need);
        return RAMP_ENOSPC;
    }
    int32_t *block_counts = static_cast<int32_t *>(ws);
    int32_t *block_base = block_counts + (size_t)B * E;
    int32_t *block_dropped = block_base + (size_t)B * E;
    hipLaunchKernelGGL(align_hist_kernel, dim3(B), dim3(NT), (E + 1) * sizeof(int), stream, ids, P, E, cap, sorted,
                       block_counts, block_dropped, scatter, pred, pred_value);
    int rc = check_launch("align_hist_kernel");
    if (rc) return rc;
    if (!scatter) {
        hipLaunchKernelGGL(align_scan_kernel, dim3(1), dim3(NT), (2 * E + 1 + NW) * sizeof(int), stream, B, E, bm, cap,
                           block_counts, block_dropped, block_base, tile_expert, tile_rows, counts, meta, scatter);
        return check_launch("align_scan_kernel");
    }
    const size_t scatter_lds = ((size_t)(E + 1) + NW + E + (size_t)NW * E) * sizeof(int);
    if (int rc2 = allow_lds(align_scan_scatter_kernel, scatter_lds)) return rc2;
    hipLaunchKernelGGL(align_scan_scatter_kernel, dim3(B), dim3(NT), scatter_lds, stream, ids, P, B, E, bm, cap,
                       block_counts, block_dropped, sorted, tile_expert, tile_rows, counts, meta, pred, pred_value,
                       slot_weights);
    return check_launch("align_scan_scatter_kernel");
}

// Per-chunk histograms only (block_counts[B][E] at the start of ws), for the device-resident dispatch kernel.
int launch_chunk_histograms(const int32_t *ids, int P, int E, void *ws, size_t ws_bytes, hipStream_t stream, int *B_out)
{
    const int B = num_blocks(P);
    const size_t need = (size_t)(2 * (size_t)B * E + B) * sizeof(int32_t);
    if (!ws || ws_bytes < need) {
        set_error("select: workspace %zu < %zu bytes (size it with ramp_align_workspace_bytes)", ws_bytes, need);
        return RAMP_ENOSPC;
    }
    int32_t *block_counts = static_cast<int32_t *>(ws);
    int32_t *block_dropped = block_counts + 2 * (size_t)B * E;
    hipLaunchKernelGGL(align_hist_kernel, dim3(B), dim3(NT), (E + 1) * sizeof(int), stream, ids, P, E, 0,
                       static_cast<int32_t *>(nullptr), block_counts, block_dropped, 0,
                       static_cast<const int32_t *>(nullptr), 0);
    *B_out = B;
    return check_launch("align_hist_kernel");
}

int launch_align(const int32_t *ids, int T, int k, int E, int bm, int32_t *sorted, int32_t *tile_expert,
                 int32_t *tile_rows, int32_t *counts, int32_t *meta, void *ws, size_t ws_bytes, hipStream_t stream,
                 const int32_t *pred, int pred_value, AlignSlotWeights slot_weights)
{
    if ((slot_weights.slot_w != nullptr) != (slot_weights.topk_w != nullptr)) {
        set_error("align: slot weights need both the router weights and the output");
        return RAMP_EINVAL;
    }
    return launch_align_impl(ids, T, k, E, bm, sorted, tile_expert, tile_rows, counts, meta, ws, ws_bytes, stream, 1,
                             pred, pred_value, slot_weights);
}

}  // namespace ramp

extern "C" size_t ramp_align_capacity(int T, int k, int E, int bm)
{
    if (T < 0 || k < 0 || E <= 0 || bm <= 0) return 0;
    long long P = (long long)T * k;
    long long hit = P < E ? P : E;
    long long cap = P + hit * (bm - 1);
    return (size_t)((cap + bm - 1) / bm * bm);
}

extern "C" size_t ramp_align_workspace_bytes(int T, int k, int E)
{
    if (T < 0 || k < 0 || E <= 0) return 0;
    long long P = (long long)T * k;
    long long B = (P + ramp::kAlignChunk - 1) / ramp::kAlignChunk;
    return ramp::align_up((size_t)(2 * B * E + B) * sizeof(int32_t) + 256, 256);
}

extern "C" int ramp_moe_histogram(const int32_t *topk_ids, int T, int k, int E, int32_t *expert_counts, void *ws,
                                  size_t ws_bytes, void *stream)
{
    return ramp::launch_align_impl(topk_ids, T, k, E, 1, nullptr, nullptr, nullptr, expert_counts, nullptr, ws, ws_bytes,
                                   static_cast<hipStream_t>(stream), 0);
}

extern "C" int ramp_moe_align(const int32_t *topk_ids, int T, int k, int E, int bm, int32_t *sorted_pair_ids,
                              int32_t *tile_expert, int32_t *expert_counts, int32_t *meta, void *ws, size_t ws_bytes,
                              void *stream)
{
    return ramp::launch_align(topk_ids, T, k, E, bm, sorted_pair_ids, tile_expert, nullptr, expert_counts, meta, ws, ws_bytes,
                              static_cast<hipStream_t>(stream));
}
