// Two-launch form of the layer for decode-sized calls (at most 64 routed pairs, i.e. T*k <= 64).
//
// With a handful of tokens the four launches of the general path (align, up-projection, down-projection, combine)
// cost as much as the weight streaming they surround (the sub-wave, start-up dominated corner of Sec. 4.1).  Here
//   launch 1 = align in the prologue + up-projection + SwiGLU: every workgroup aligns the <= 64 pairs itself with
//              one wavefront (a few hundred instructions on 256 bytes of ids) instead of waiting for an align
//              launch, then runs the weight-streaming up-projection of moe_stream_kernel on its M-tile and writes
//              the activation row of every pair, indexed by pair;
//   launch 2 = down-projection + router weights + top-k sum: a workgroup owns a slice of 16*FBW output features of
//              ONE token and all of its k pairs; wavefront (j, wk) streams expert e_j's weight rows of the slice over
//              1/WK of the reduction, the partial sums meet in LDS and are added in fixed order (wk, then j), so the
//              result is bit-identical from run to run and no per-pair rows, no combine launch and no atomics exist.
// Workgroup 0 of launch 1 also writes the align result (sorted pairs, tile tables, counts, meta) to the workspace,
// so the layout query of the general path keeps its meaning.
#pragma once

#include "align_tiny.h"
#include "moe_stream.h"

namespace ramp {

template <int BM, int FBW, int WF, int WK, int U>
__global__ __launch_bounds__(WF *WK * 64) void moe_decode_up_kernel(GemmArgs a, DecodeArgs d)
{
    using ST = StreamTraits<BM, FBW, WF, WK, U>;
    constexpr int NB = ST::NB;
    constexpr int FEAT_PER_TILE = ST::BN / 2;
    constexpr int FPW = FBW / 2;
    static_assert(BM <= kDecodeMaxPairs, "a tile holds at most the 64 pairs of a call");

    __shared__ __attribute__((aligned(16))) float red[ST::RED_FLOATS > 0 ? ST::RED_FLOATS : 4];
    __shared__ int n_lds[kAlignMaxE];
    __shared__ int toff[kAlignMaxE + 1];
    __shared__ int tile_pair[BM];
    __shared__ int tile_info[2];  // expert of this workgroup's M-tile, number of M-tiles of the call

    if (launch_deselected(a.pred, a.pred_value)) return;
    const int n_tile = blockIdx.x % a.n_tiles;
    const int m_tile = blockIdx.x / a.n_tiles;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;

    // ---- align in the prologue (wavefront 0; lane = pair)
    for (int x = threadIdx.x; x < BM; x += blockDim.x) tile_pair[x] = a.P;
    __syncthreads();
    if (wave == 0) {
        int e, rank;
        tiny_align_wavefront(d.ids, a.P, d.E, d.bm, lane, n_lds, toff, e, rank);
        if (e >= 0) {
            const int slot = toff[e] + rank;
            if (slot / BM == m_tile) tile_pair[slot - m_tile * BM] = lane;
        }
        if (lane == 0) {
            const int m_tiles = toff[d.E] / BM;
            int owner = -1, rows = 0;
            if (m_tile < m_tiles) tiny_align_tile(m_tile, d.E, BM, n_lds, toff, owner, rows);
            tile_info[0] = owner;
            tile_info[1] = m_tiles;
        }
        if (blockIdx.x == 0)
            tiny_align_emit(a.P, d.E, d.bm, d.cap, lane, n_lds, toff, e, rank, d.ids, d.sorted, d.tile_expert, d.tile_rows,
                            d.counts, d.meta);
    }
    __syncthreads();
    if (m_tile >= tile_info[1]) return;

    // ---- up-projection of this M-tile x feature tile, as moe_stream_kernel<1, ...>
    const int wf = wave % WF, wk = wave / WF;
    const int r16 = lane & 15, q = lane >> 4;
    const int e = tile_info[0];
    const int K = a.K, KST = K / 32;
    const int f0 = n_tile * FEAT_PER_TILE + wf * FPW * 16;
    const uint16_t *wexp = a.wpacked + (size_t)e * a.expert_stride;
    const int per = (KST + WK - 1) / WK;
    const int ks_begin = wk * per;
    const int ks_end = min(KST, ks_begin + per);

    uint32_t xoff[NB];
    int pair_of[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        int tr = nb * 16 + r16;
        const bool live = tr < BM;
        if (!live) tr = BM - 1;
        const int pair = tile_pair[tr];
        pair_of[nb] = live ? pair : a.P;
        xoff[nb] = ((pair < a.P) ? (uint32_t)(pair / a.topk) : 0u) * (uint32_t)K + (uint32_t)(q * 8);
    }
    uint32_t woff[FBW];
#pragma unroll
    for (int i = 0; i < FBW; ++i) {
        const int half = FBW / 2;
        const uint32_t rbg = (i < half) ? (uint32_t)((f0 / 16 + i) * KST) * kFragElems
                                        : (uint32_t)a.up_offset + (uint32_t)((f0 / 16 + i - half) * KST) * kFragElems;
        woff[i] = rbg + (uint32_t)lane * 8;
    }

    floatx4 acc[FBW][NB];
#pragma unroll
    for (int i = 0; i < FBW; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    struct Batch {
        bf16x8 x[U][NB];
        bf16x8 w[U][FBW];
    };
    auto load_batch = [&](Batch &b, int ks0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int ks = ks0 + u;
            if (ks >= ks_end) ks = ks_end - 1;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) b.x[u][nb] = *reinterpret_cast<const bf16x8 *>(a.act + xoff[nb] + (size_t)ks * 32);
#pragma unroll
            for (int i = 0; i < FBW; ++i) b.w[u][i] = *reinterpret_cast<const bf16x8 *>(wexp + woff[i] + (size_t)ks * kFragElems);
        }
    };
    auto compute_batch = [&](const Batch &b, int ks0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (ks0 + u < ks_end) {
#pragma unroll
                for (int i = 0; i < FBW; ++i)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        acc[i][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b.w[u][i], b.x[u][nb], acc[i][nb], 0, 0, 0);
            }
        }
    };
    if (ks_begin < ks_end) {
        Batch b0, b1;
        load_batch(b0, ks_begin);
        for (int ks = ks_begin; ks < ks_end; ks += 2 * U) {
            if (ks + U < ks_end) load_batch(b1, ks + U);
            compute_batch(b0, ks);
            if (ks + 2 * U < ks_end) load_batch(b0, ks + 2 * U);
            if (ks + U < ks_end) compute_batch(b1, ks + U);
        }
    }
    if (WK > 1) {
        if (wk > 0) {
#pragma unroll
            for (int i = 0; i < FBW; ++i)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    *reinterpret_cast<floatx4 *>(&red[((((wk - 1) * WF + wf) * FBW + i) * NB + nb) * 256 + lane * 4]) = acc[i][nb];
        }
        __syncthreads();
        if (wk > 0) return;
#pragma unroll
        for (int s = 0; s < WK - 1; ++s)
#pragma unroll
            for (int i = 0; i < FBW; ++i)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    acc[i][nb] += *reinterpret_cast<const floatx4 *>(&red[(((s * WF + wf) * FBW + i) * NB + nb) * 256 + lane * 4]);
    }
    // ---- epilogue: SiLU(g)*u -> bf16, one activation row per pair (row-major [P, I]; a.a_row_major is set)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int pair = pair_of[nb];
        if (pair >= a.P) continue;
        store_token_row<1, FPW>(a, &acc[0][nb], &acc[FPW][nb], NB, (size_t)pair, f0 / 16, q, 1.0f);
    }
}

// grid = (H / (16*FBW)) * T workgroups of 16 wavefronts: wavefront w handles pair j = w / WK of the token over the
// k-steps [wk*per, ...) with WK = 16 / k (k divides 16).
template <int FBW, int U>
__global__ __launch_bounds__(1024) void moe_decode_down_kernel(DecodeDownArgs d)
{
    __shared__ float red[16][FBW * 16];  // [wavefront][feature of the slice]
    if (launch_deselected(d.pred, d.pred_value)) return;
    const int n_ft = d.H / (16 * FBW);
    const int t = blockIdx.x / n_ft, ft = blockIdx.x % n_ft;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int WK = 16 / d.k;
    const int j = wave / WK, wk = wave % WK;
    const int r16 = lane & 15, q = lane >> 4;
    const int pair = t * d.k + j;
    const int e = d.ids[pair];
    const bool live = e >= 0 && e < d.E;
    const int KST = d.I / 32;
    const int per = (KST + WK - 1) / WK;
    const int ks_begin = wk * per;
    const int ks_end = min(KST, ks_begin + per);

    floatx4 acc[FBW];
#pragma unroll
    for (int i = 0; i < FBW; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    if (live && ks_begin < ks_end) {
        const uint16_t *wexp = d.wpacked + (size_t)e * d.expert_stride;
        const uint16_t *arow = d.act + (size_t)pair * d.I + q * 8;
        uint32_t woff[FBW];
#pragma unroll
        for (int i = 0; i < FBW; ++i) woff[i] = (uint32_t)((ft * FBW + i) * KST) * kFragElems + (uint32_t)lane * 8;
        struct Batch {
            bf16x8 x[U];
            bf16x8 w[U][FBW];
        };
        const bf16x8 zero = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        auto load_batch = [&](Batch &b, int ks0) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                int ks = ks0 + u;
                if (ks >= ks_end) ks = ks_end - 1;
                // the token operand has one real column (token 0 of 16): the other lanes hold zeros
                b.x[u] = (r16 == 0) ? *reinterpret_cast<const bf16x8 *>(arow + (size_t)ks * 32) : zero;
#pragma unroll
                for (int i = 0; i < FBW; ++i) b.w[u][i] = *reinterpret_cast<const bf16x8 *>(wexp + woff[i] + (size_t)ks * kFragElems);
            }
        };
        auto compute_batch = [&](const Batch &b, int ks0) {
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (ks0 + u < ks_end) {
#pragma unroll
                    for (int i = 0; i < FBW; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b.w[u][i], b.x[u], acc[i], 0, 0, 0);
                }
        };
        Batch b0, b1;
        load_batch(b0, ks_begin);
        for (int ks = ks_begin; ks < ks_end; ks += 2 * U) {
            if (ks + U < ks_end) load_batch(b1, ks + U);
            compute_batch(b0, ks);
            if (ks + 2 * U < ks_end) load_batch(b0, ks + 2 * U);
            if (ks + U < ks_end) compute_batch(b1, ks + U);
        }
    }
    // lane (q, r16 = 0) holds rows 4q .. 4q+3 of every row block for the token
    if (r16 == 0) {
#pragma unroll
        for (int i = 0; i < FBW; ++i)
#pragma unroll
            for (int c = 0; c < 4; ++c) red[wave][i * 16 + q * 4 + c] = acc[i][c];
    }
    __syncthreads();
    // one thread per output feature of the slice: sum the split-K partials in wk order, weight, sum over j in order
    if ((int)threadIdx.x < FBW * 16) {
        const int i = threadIdx.x / 16, r = threadIdx.x % 16;
        float y = 0.f;
        for (int jj = 0; jj < d.k; ++jj) {
            const int id = d.ids[t * d.k + jj];
            if (id < 0 || id >= d.E) continue;
            float s = red[jj * WK][threadIdx.x];
            for (int w = 1; w < WK; ++w) s += red[jj * WK + w][threadIdx.x];
            y += d.topk_w[t * d.k + jj] * s;
        }
        d.out[(size_t)t * d.H + packed_row_feature(ft * FBW + i, r)] = f32_to_bf16_bits(y);
    }
}

template <int BM, int FBW, int WF, int WK, int U>
void launch_decode_up(const GemmArgs &a, const DecodeArgs &d, hipStream_t stream)
{
    const dim3 grid((unsigned)a.n_tiles * (unsigned)a.m_tiles_cap), block(WF * WK * 64);
    if (grid.x == 0) return;
    hipLaunchKernelGGL((moe_decode_up_kernel<BM, FBW, WF, WK, U>), grid, block, 0, stream, a, d);
}

inline void launch_decode_down(const DecodeDownArgs &d, hipStream_t stream)
{
    if (d.T <= 0) return;
    // 16 output features per workgroup fill the chip sooner when H is small; 32 halve the launches' workgroups
    if ((size_t)d.H / 32 * d.T >= 2 * (size_t)kNumCU) {
        const dim3 grid((unsigned)(d.H / 32) * (unsigned)d.T), block(1024);
        hipLaunchKernelGGL((moe_decode_down_kernel<2, 4>), grid, block, 0, stream, d);
    } else {
        const dim3 grid((unsigned)(d.H / 16) * (unsigned)d.T), block(1024);
        hipLaunchKernelGGL((moe_decode_down_kernel<1, 4>), grid, block, 0, stream, d);
    }
}

}  // namespace ramp
