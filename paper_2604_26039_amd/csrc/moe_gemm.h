// Grouped expert projections of the fused MoE layer (paper Sec. 2.2 phases 1-3) for gfx950.
//
// One workgroup owns (M-tile m of expert e, feature tile n)  [Eq. 1: grid = M-tiles x N-tiles].
//   stage 1: G,U = X[rows] . W_gate[e], W_up[e]  over K = H, then A = SiLU(G)*U -> bf16 [slot, I]
//   stage 2: Y[p,:] = w[p] * A[slot] . W_down[e] over K = I  -> fp32 [pair, H]
// MFMA v_mfma_f32_16x16x32_bf16 with the weights as the A operand (16 output features) and
// the tokens as the B operand (16 tokens): every lane then owns 4 consecutive features of one
// token, which makes the SiLU*mul epilogue lane-local and the stores 8/16-byte wide.
//
// Both operands are staged in LDS as 1 KB "fragments" (16 rows x 32 k in MFMA lane order) by
// LDS-direct loads (global_load_lds_dwordx4: no register staging, no ds_write):
//   - a weight fragment is one contiguous 1 KB line of the packed layout;
//   - a token fragment is gathered row by row, 16 B per lane, and lands in lane order.
// Every wavefront-wide load therefore fills exactly one fragment, LDS writes and the
// ds_read_b128 operand reads are conflict free without padding or swizzles.
// The k-slices go through a ring of NSTAGE LDS buffers: loads for slice kt+NSTAGE-1 are in
// flight while slice kt is multiplied; one s_waitcnt vmcnt + one s_barrier per slice.
#pragma once

#include "ramp_internal.h"

namespace ramp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

template <int BM, int BN, int BK, int WM, int WN, int NSTAGE>
struct TileTraits {
    static constexpr int BMP = (BM + 15) / 16 * 16;  // token rows padded to the MFMA width
    static constexpr int NBT = BMP / 16;             // token blocks per tile
    static constexpr int RB = BN / 16;               // weight row blocks per tile
    static constexpr int KS = BK / 32;               // MFMA k-steps per staged slice
    static constexpr int NWAVE = WM * WN;
    static constexpr int NB = NBT / WM;              // token blocks per wavefront
    static constexpr int X_FRAGS = NBT * KS;
    static constexpr int W_FRAGS = RB * KS;
    static constexpr int FRAGS = X_FRAGS + W_FRAGS;
    static constexpr int SLOTS = FRAGS / NWAVE;      // fragment loads per wavefront per slice
    static constexpr int BUF_ELEMS = FRAGS * kFragElems;
    static constexpr int LDS_BYTES = NSTAGE * BUF_ELEMS * 2;
    static constexpr int FB1 = RB / 2 / WN;          // stage 1: feature blocks per wavefront (gate and up each)
    static constexpr int FB2 = RB / WN;              // stage 2
    static constexpr int ACC_REGS = 2 * FB1 * NB * 4;
    static_assert(NBT % WM == 0, "token blocks must split evenly over WM");
    static_assert(RB % (2 * WN) == 0, "bn must be a multiple of 32*WN");
    static_assert(BK % 32 == 0, "bk must be a multiple of 32");
    static_assert(FRAGS % NWAVE == 0, "every wavefront must issue the same number of loads per slice");
    static_assert(NSTAGE >= 2 && NSTAGE <= 4, "2..4 LDS stages");
    static_assert((NSTAGE - 1) * SLOTS <= 63, "vmcnt is a 6-bit counter");
    static_assert(LDS_BYTES <= kLdsBytesPerCU, "tile does not fit in LDS");
};

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    // round to nearest even; inputs here are finite
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float silu_f32(float x) { return x / (1.0f + __expf(-x)); }

// 16 bytes per lane from global memory straight into LDS at lds_base + lane*16.
__device__ __forceinline__ void load_to_lds_16B(const void *gptr, void *lds_base)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)gptr,
                                     (__attribute__((address_space(3))) void *)lds_base, 16, 0, 0);
}

// Wait until at most N vector-memory operations of this wavefront are outstanding.
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N <= 63, "vmcnt range");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

template <int STAGE, int BM, int BN, int BK, int WM, int WN, int NSTAGE>
__global__ __launch_bounds__(WM *WN * 64) void moe_gemm_kernel(GemmArgs a)
{
    using TT = TileTraits<BM, BN, BK, WM, WN, NSTAGE>;
    constexpr int KS = TT::KS, NB = TT::NB, SLOTS = TT::SLOTS, NWAVE = TT::NWAVE;
    constexpr int FB = (STAGE == 1) ? TT::FB1 : TT::FB2;
    constexpr int NACC = (STAGE == 1) ? 2 * FB : FB;  // accumulator row blocks per wavefront
    constexpr int FEAT_PER_TILE = (STAGE == 1) ? BN / 2 : BN;

    __shared__ __attribute__((aligned(1024))) uint16_t lds[NSTAGE * TT::BUF_ELEMS];

    const int n_tile = blockIdx.x % a.n_tiles;
    const int m_tile = blockIdx.x / a.n_tiles;
    if (m_tile >= a.meta[1]) return;  // overlaunched grid: surplus workgroups leave at once

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int e = a.tile_expert[m_tile];
    const int K = a.K, KST = K / 32;
    const int f0 = n_tile * FEAT_PER_TILE;
    const uint16_t *wexp = a.wpacked + (size_t)e * a.expert_stride;
    const int r16 = lane & 15, q = lane >> 4;

    // ---- per-slot global source pointers for k-slice 0; slot s of this wavefront fills fragment
    //      wave + s*NWAVE of the slice (token fragments first, then weight fragments) ----
    const uint16_t *gptr[SLOTS];
    int gstep[SLOTS];  // elements to advance per k-slice
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        const int idx = wave + s * NWAVE;
        if (idx < TT::X_FRAGS) {
            const int nb = idx / KS, ks = idx % KS;
            int tr = nb * 16 + r16;
            if (tr >= BM) tr = BM - 1;
            const int slot = m_tile * BM + tr;
            size_t row;
            if (STAGE == 1) {
                const int pair = a.sorted[slot];
                row = (pair < a.P) ? (size_t)(pair / a.topk) : 0;
            } else {
                row = (size_t)slot;
            }
            gptr[s] = a.act + row * (size_t)K + (size_t)(ks * 32 + q * 8);
            gstep[s] = BK;
        } else {
            const int widx = idx - TT::X_FRAGS;
            const int rb = widx / KS, ks = widx % KS;
            size_t base;
            if (STAGE == 1) {
                const int half = TT::RB / 2;
                base = (rb < half) ? (size_t)(f0 / 16 + rb) * KST * kFragElems
                                   : a.up_offset + (size_t)(f0 / 16 + rb - half) * KST * kFragElems;
            } else {
                base = (size_t)(f0 / 16 + rb) * KST * kFragElems;
            }
            gptr[s] = wexp + base + (size_t)ks * kFragElems + (size_t)lane * 8;
            gstep[s] = KS * kFragElems;
        }
    }

    floatx4 acc[NACC][NB];
#pragma unroll
    for (int i = 0; i < NACC; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    auto issue_slice = [&](int buf) {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            load_to_lds_16B(gptr[s], &lds[buf * TT::BUF_ELEMS + (wave + s * NWAVE) * kFragElems]);
            gptr[s] += gstep[s];
        }
    };
    auto compute_slice = [&](int buf) {
        const uint16_t *xs = &lds[buf * TT::BUF_ELEMS + lane * 8];
        const uint16_t *ws = xs + TT::X_FRAGS * kFragElems;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bf16x8 b[NB];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                b[nb] = *reinterpret_cast<const bf16x8 *>(xs + ((wm * NB + nb) * KS + ks) * kFragElems);
#pragma unroll
            for (int i = 0; i < NACC; ++i) {
                int rb;
                if (STAGE == 1) rb = (i < FB) ? (wn * FB + i) : (TT::RB / 2 + wn * FB + (i - FB));
                else rb = wn * FB + i;
                const bf16x8 w = *reinterpret_cast<const bf16x8 *>(ws + (rb * KS + ks) * kFragElems);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    acc[i][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w, b[nb], acc[i][nb], 0, 0, 0);
            }
        }
    };

    const int KT = K / BK;
    // prologue: slices 0 .. NSTAGE-2 in flight
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s)
        if (s < KT) issue_slice(s);

    int buf_cur = 0, buf_issue = NSTAGE - 1;
    for (int kt = 0; kt < KT; ++kt) {
        // slices kt+1 .. kt+NSTAGE-2 may stay in flight; slice kt must have landed
        const int later = min(NSTAGE - 2, KT - 1 - kt);
        if (NSTAGE >= 4 && later >= 2) wait_vmcnt<(NSTAGE >= 4 ? 2 : 0) * SLOTS>();
        else if (NSTAGE >= 3 && later >= 1) wait_vmcnt<(NSTAGE >= 3 ? 1 : 0) * SLOTS>();
        else wait_vmcnt<0>();
        // all wavefronts' parts of slice kt are in LDS, and everyone has finished reading the
        // buffer that the next loads overwrite (it held slice kt-1)
        __builtin_amdgcn_s_barrier();
        if (kt + NSTAGE - 1 < KT) issue_slice(buf_issue);
        compute_slice(buf_cur);
        buf_cur = (buf_cur + 1 == NSTAGE) ? 0 : buf_cur + 1;
        buf_issue = (buf_issue + 1 == NSTAGE) ? 0 : buf_issue + 1;
    }

    // ---- epilogue: lane holds features f = fblock*16 + 4*q + {0..3} of token n = r16 ----
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int tr = (wm * NB + nb) * 16 + r16;
        if (tr >= BM) continue;
        const int slot = m_tile * BM + tr;
        if (STAGE == 1) {
#pragma unroll
            for (int i = 0; i < FB; ++i) {
                const floatx4 g = acc[i][nb], u = acc[FB + i][nb];
                const int f = f0 + (wn * FB + i) * 16 + q * 4;
                union {
                    uint16_t h[4];
                    uint2 v;
                } o;
#pragma unroll
                for (int c = 0; c < 4; ++c) o.h[c] = f32_to_bf16_bits(silu_f32(g[c]) * u[c]);
                *reinterpret_cast<uint2 *>(a.a_out + (size_t)slot * a.F + f) = o.v;
            }
        } else {
            const int pair = a.sorted[slot];
            if (pair >= a.P) continue;
            const float wgt = a.topk_w[pair];
#pragma unroll
            for (int i = 0; i < FB; ++i) {
                const floatx4 y = acc[i][nb];
                const int f = f0 + (wn * FB + i) * 16 + q * 4;
                float4 o = make_float4(wgt * y[0], wgt * y[1], wgt * y[2], wgt * y[3]);
                *reinterpret_cast<float4 *>(a.y_out + (size_t)pair * a.F + f) = o;
            }
        }
    }
}

template <int BM, int BN, int BK, int WM, int WN, int NSTAGE>
void launch_gemm(int stage, const GemmArgs &a, hipStream_t stream)
{
    const dim3 grid((unsigned)a.n_tiles * (unsigned)a.m_tiles_cap), block(WM * WN * 64);
    if (grid.x == 0) return;
    if (stage == 1)
        hipLaunchKernelGGL((moe_gemm_kernel<1, BM, BN, BK, WM, WN, NSTAGE>), grid, block, 0, stream, a);
    else
        hipLaunchKernelGGL((moe_gemm_kernel<2, BM, BN, BK, WM, WN, NSTAGE>), grid, block, 0, stream, a);
}

template <int BM, int BN, int BK, int WM, int WN, int NSTAGE>
KernelInfo make_info()
{
    using TT = TileTraits<BM, BN, BK, WM, WN, NSTAGE>;
    KernelInfo ki;
    ki.cfg = ramp_config{BM, BN, BK, WM * WN, NSTAGE, WM - 1};
    ki.wm = WM;
    ki.wn = WN;
    ki.lds_bytes = TT::LDS_BYTES;
    ki.acc_regs = TT::ACC_REGS;
    ki.launch = &launch_gemm<BM, BN, BK, WM, WN, NSTAGE>;
    return ki;
}

}  // namespace ramp
