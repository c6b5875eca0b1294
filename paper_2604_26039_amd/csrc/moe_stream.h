// Weight-streaming variant of the expert projections for small token blocks (decode regime,
// HBM-bound: every weight byte is used by at most 32 tokens).
//
// Same work decomposition as the LDS-staged kernel (one workgroup = one M-tile of an expert x
// one tile of bn weight rows, Eq. 1), but nothing is shared between wavefronts, so nothing is
// staged in LDS and there is no barrier in the main loop:
//   - a wavefront owns FBW 16-row weight blocks and a 1/WK share of the reduction length K;
//     it reads its weight fragments from the packed layout straight into MFMA operand
//     registers (one contiguous 1 KB line per load) and the matching 16-token activation
//     fragment from the (L2-resident) activation rows, 16 B per lane;
//   - loads are issued U k-steps ahead in two register sets, so each wavefront keeps
//     2*U*(FBW+NB) KB in flight and many small wavefronts per compute unit cover HBM latency;
//   - the WK partial accumulators of a row block are summed through LDS once at the end
//     (split-K inside the workgroup fills the chip when few experts are active, the sub-wave
//     regime of Sec. 4.1), in a fixed order, so results stay bit-reproducible.
#pragma once

#include "moe_gemm.h"

namespace ramp {

template <int BM, int FBW, int WF, int WK, int U>
struct StreamTraits {
    static constexpr int NB = (BM + 15) / 16;  // 16-token blocks per tile (all handled by every wavefront)
    static constexpr int NWAVE = WF * WK;
    static constexpr int BN = WF * FBW * 16;   // weight rows per workgroup tile
    static constexpr int ACC_REGS = FBW * NB * 4;
    static constexpr int RED_FLOATS = (WK - 1) * WF * FBW * NB * 256;  // partial sums parked in LDS
    static constexpr int LDS_BYTES = RED_FLOATS * 4;
    static_assert(FBW % 2 == 0, "gate and up row blocks come in pairs");
    static_assert(LDS_BYTES <= 64 * 1024, "reduction buffer too large");
};

template <int STAGE, int BM, int FBW, int WF, int WK, int U>
__global__ __launch_bounds__(WF *WK * 64) void moe_stream_kernel(GemmArgs a)
{
    using ST = StreamTraits<BM, FBW, WF, WK, U>;
    constexpr int NB = ST::NB;
    constexpr int FEAT_PER_TILE = (STAGE == 1) ? ST::BN / 2 : ST::BN;
    constexpr int FPW = (STAGE == 1) ? FBW / 2 : FBW;  // feature blocks per wavefront in the output

    __shared__ __attribute__((aligned(16))) float red[ST::RED_FLOATS > 0 ? ST::RED_FLOATS : 4];

    if (launch_deselected(a.pred, a.pred_value)) return;
    const int n_tile = blockIdx.x % a.n_tiles;
    const int m_tile = blockIdx.x / a.n_tiles;
    if (m_tile >= a.meta[1]) return;

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wf = wave % WF, wk = wave / WF;
    const int r16 = lane & 15, q = lane >> 4;
    const int e = a.tile_expert[m_tile];
    const int K = a.K, KST = K / 32;
    const int f0 = n_tile * FEAT_PER_TILE + wf * FPW * 16;  // first output feature of this wavefront
    const uint16_t *wexp = a.wpacked + (size_t)e * a.expert_stride;

    // k-steps of this wavefront: [ks_begin, ks_end)
    const int per = (KST + WK - 1) / WK;
    const int ks_begin = wk * per;
    const int ks_end = min(KST, ks_begin + per);

    // activation row offsets (elements), one per token block
    uint32_t xoff[NB];
    int pair_of[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        int tr = nb * 16 + r16;
        const bool live = tr < BM;
        if (!live) tr = BM - 1;
        const int slot = m_tile * BM + tr;
        const int pair = a.sorted[slot];
        pair_of[nb] = live ? pair : a.P;
        if (STAGE == 1) xoff[nb] = ((pair < a.P) ? (uint32_t)(pair / a.topk) : 0u) * (uint32_t)K + (uint32_t)(q * 8);
        else xoff[nb] = act_elem((uint32_t)slot, (uint32_t)(q * 8), (uint32_t)KST);  // fragment-major, written by stage 1
    }
    // weight row-block offsets (elements) at k-step 0
    uint32_t woff[FBW];
#pragma unroll
    for (int i = 0; i < FBW; ++i) {
        uint32_t rbg;
        if (STAGE == 1) {
            const int half = FBW / 2;
            rbg = (i < half) ? (uint32_t)((f0 / 16 + i) * KST) * kFragElems
                             : (uint32_t)a.up_offset + (uint32_t)((f0 / 16 + i - half) * KST) * kFragElems;
        } else {
            rbg = (uint32_t)((f0 / 16 + i) * KST) * kFragElems;
        }
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
            if (ks >= ks_end) ks = ks_end - 1;  // tail: re-read the last step, its product is skipped
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                b.x[u][nb] = *reinterpret_cast<const bf16x8 *>(a.act + xoff[nb] + (size_t)ks * (STAGE == 1 ? 32 : kFragElems));
#pragma unroll
            for (int i = 0; i < FBW; ++i)
                b.w[u][i] = *reinterpret_cast<const bf16x8 *>(wexp + woff[i] + (size_t)ks * kFragElems);
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

    // ---- sum the WK partial accumulators in wk order ----
    if (WK > 1) {
        if (wk > 0) {
#pragma unroll
            for (int i = 0; i < FBW; ++i)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    *reinterpret_cast<floatx4 *>(&red[((((wk - 1) * WF + wf) * FBW + i) * NB + nb) * 256 + lane * 4]) =
                        acc[i][nb];
        }
        __syncthreads();
        if (wk > 0) return;
#pragma unroll
        for (int s = 0; s < WK - 1; ++s)
#pragma unroll
            for (int i = 0; i < FBW; ++i)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    acc[i][nb] += *reinterpret_cast<const floatx4 *>(
                        &red[(((s * WF + wf) * FBW + i) * NB + nb) * 256 + lane * 4]);
    }

    // ---- epilogue: lane holds features fblock*16 + 4*q + {0..3} of token r16 ----
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int tr = nb * 16 + r16;
        if (tr >= BM) continue;
        const int slot = m_tile * BM + tr;
        if (STAGE == 1) {
            store_token_row<1, FPW>(a, &acc[0][nb], &acc[FPW][nb], NB, (size_t)slot, f0 / 16, q, 1.0f);
        } else {
            const int pair = pair_of[nb];
            if (pair >= a.P) continue;
            store_token_row<2, FPW>(a, &acc[0][nb], &acc[0][nb], NB, (size_t)pair * a.F, f0 / 16, q, a.topk_w[pair]);
        }
    }
}

template <int BM, int FBW, int WF, int WK, int U>
void launch_stream(int stage, const GemmArgs &a, hipStream_t stream)
{
    const dim3 grid((unsigned)a.n_tiles * (unsigned)a.m_tiles_cap), block(WF * WK * 64);
    if (grid.x == 0) return;
    if (stage == 1)
        hipLaunchKernelGGL((moe_stream_kernel<1, BM, FBW, WF, WK, U>), grid, block, 0, stream, a);
    else
        hipLaunchKernelGGL((moe_stream_kernel<2, BM, FBW, WF, WK, U>), grid, block, 0, stream, a);
}


template <int BM, int FBW, int WF, int WK, int U>
KernelInfo make_stream_info()
{
    using ST = StreamTraits<BM, FBW, WF, WK, U>;
    KernelInfo ki = {};
    ki.cfg = ramp_config{BM, ST::BN, U * 32, WF * WK, 2, kModeStream | WK};
    ki.wm = 1;
    ki.wn = WF;
    ki.lds_bytes = ST::LDS_BYTES > 1024 ? ST::LDS_BYTES : 1024;
    ki.acc_regs = ST::ACC_REGS + 2 * U * (FBW + ST::NB) * 4;  // accumulators + the two load batches
    ki.launch = &launch_stream<BM, FBW, WF, WK, U>;
    ki.kernel_fn[0] = reinterpret_cast<const void *>(&moe_stream_kernel<1, BM, FBW, WF, WK, U>);
    ki.kernel_fn[1] = reinterpret_cast<const void *>(&moe_stream_kernel<2, BM, FBW, WF, WK, U>);
    ki.block_threads = WF * WK * 64;
    ki.family = "moe_stream_kernel";
    const int targs[8] = {1, BM, FBW, WF, WK, U, 0, 0};
    for (int i = 0; i < 8; ++i) ki.targs[i] = targs[i];
    ki.n_targs = 6;
    return ki;
}

}  // namespace ramp
