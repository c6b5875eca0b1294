// Align for decode-sized calls (at most 64 pairs): one wavefront, one pair per lane, shared by the stand-alone
// align kernel and by the projection kernels that align in their own prologue (Eq. 1 first factor; Fig. 1).
#pragma once

#include "ramp_internal.h"

namespace ramp {

// Called by the 64 lanes of one wavefront (lane = pair index).  Leaves in LDS the pairs per expert n_lds[E] and the
// first padded slot of every expert toff[E+1] (toff[E] = padded length), and returns this lane's expert (-1: no pair
// or id out of range) and its rank among the lanes of the same expert, so that its slot is toff[e] + rank.
// The LDS arrays are complete for the calling wavefront when the function returns.
__device__ __forceinline__ void tiny_align_wavefront(const int32_t *ids, int P, int E, int bm, int lane, int *n_lds, int *toff,
                                                     int &e, int &rank)
{
    for (int x = lane; x < E; x += kWave) n_lds[x] = 0;
    e = -1;
    if (lane < P) {
        const int v = ids[lane];
        if (v >= 0 && v < E) e = v;
    }
    // lanes with the same expert: one ballot per bit of the expert index
    const int ebits = 32 - __clz((E - 1) | 1);
    unsigned long long same = __ballot(e >= 0);
#pragma unroll
    for (int b = 0; b < 10; ++b) {
        if (b < ebits) {
            const bool bit = (e >> b) & 1;
            const unsigned long long m = __ballot(e >= 0 && bit);
            same &= bit ? m : ~m;
        }
    }
    rank = __popcll(same & ((1ull << lane) - 1ull));
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    if (e >= 0 && rank == 0) n_lds[e] = __popcll(same);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    // exclusive scan of the padded slot counts: lane l owns experts [l*per, (l+1)*per)
    const int per = (E + kWave - 1) / kWave;
    int local = 0;
    for (int i = 0; i < per; ++i) {
        const int x = lane * per + i;
        if (x < E) local += (n_lds[x] + bm - 1) / bm * bm;
    }
    int incl = local;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int up = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += up;
    }
    const int p_pad = __shfl(incl, kWave - 1, kWave);
    int run = incl - local;
    for (int i = 0; i < per; ++i) {
        const int x = lane * per + i;
        if (x < E) {
            toff[x] = run;
            run += (n_lds[x] + bm - 1) / bm * bm;
        }
    }
    if (lane == 0) toff[E] = p_pad;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Expert and real rows of M-tile m (m < padded length / bm), from the arrays above.
__device__ __forceinline__ void tiny_align_tile(int m, int E, int bm, const int *n_lds, const int *toff, int &owner, int &rows)
{
    int target = m * bm, lo = 0, hi = E - 1;  // first expert with toff[e+1] > m*bm (empty experts are skipped)
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (toff[mid + 1] > target) hi = mid; else lo = mid + 1;
    }
    owner = lo;
    rows = n_lds[owner] - (target - toff[owner]);
    rows = rows > bm ? bm : rows;
}

// Writes the align result to global memory (same wavefront, after tiny_align_wavefront).
__device__ __forceinline__ void tiny_align_emit(int P, int E, int bm, int cap, int lane, const int *n_lds, const int *toff, int e,
                                                int rank, const int32_t *ids, int32_t *sorted, int32_t *tile_expert,
                                                int32_t *tile_rows, int32_t *counts, int32_t *meta,
                                                AlignSlotWeights slot_weights = {nullptr, nullptr})
{
    for (int s = lane; s < cap; s += kWave) sorted[s] = P;
    const int dropped = __popcll(__ballot(lane < P && e < 0));
    const int p_pad = toff[E];
    if (lane == 0) {
        meta[0] = p_pad;
        meta[1] = p_pad / bm;
        meta[2] = dropped;
        meta[3] = 0;
    }
    for (int x = lane; x < E; x += kWave) counts[x] = n_lds[x];
    const int m_tiles = p_pad / bm, m_cap = cap / bm;
    for (int m = lane; m < m_cap; m += kWave) {
        int owner = -1, rows = 0;
        if (m < m_tiles) tiny_align_tile(m, E, bm, n_lds, toff, owner, rows);
        tile_expert[m] = owner;
        if (tile_rows) tile_rows[m] = rows;
    }
    // the sentinel fill above was done by this wavefront: order it before the scatter of the same addresses
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (e >= 0) {
        sorted[toff[e] + rank] = lane;
        if (slot_weights.slot_w) slot_weights.slot_w[toff[e] + rank] = slot_weights.topk_w[lane];
    }
    (void)ids;
}

}  // namespace ramp
