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
    // 4-wavefront tiles that need at most half (a third) of the LDS are compiled for two (three) workgroups
    // per compute unit (that many wavefronts per SIMD, <= 256 (170) registers each): the two workgroups share no barrier, so one
    // computes while the other waits for its loads.
    static constexpr int MIN_WAVES_PER_SIMD =
        (NWAVE == 4 && LDS_BYTES <= 53 * 1024 && ACC_REGS <= 64) ? 3 : ((NWAVE == 4 && LDS_BYTES <= 80 * 1024) ? 2 : 1);
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

// Two fp32 -> two bf16 (round to nearest even) in one 32-bit word, low half first: the packed conversion instruction
// of this chip (v_cvt_pk_bf16_f32) instead of three integer operations per value.
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi)
{
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

// SiLU(x) = x / (1 + e^-x) with the hardware exp2 and reciprocal (1 ulp each; the result is rounded to
// bf16 right after, which is 2^16 times coarser).
__device__ __forceinline__ float silu_f32(float x) { return x * __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }

// Four consecutive features of one weighted per-pair output row: fp32, or bf16 for large batches.
__device__ __forceinline__ void store_pair_row(const GemmArgs &a, size_t elem, float v0, float v1, float v2, float v3)
{
    if (a.y_bf16) {
        union {
            uint32_t w[2];
            uint2 v;
        } o;
        o.w[0] = f32x2_to_bf16x2(v0, v1);
        o.w[1] = f32x2_to_bf16x2(v2, v3);
        *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(a.y_out) + elem) = o.v;
    } else {
        *reinterpret_cast<float4 *>(a.y_out + elem) = make_float4(v0, v1, v2, v3);
    }
}

// Eight consecutive bf16 features (two neighbouring row blocks of one interleave group) in one 16-byte store.
__device__ __forceinline__ void store_bf16x8(uint16_t *dst, const float *v)
{
    union {
        uint32_t w[4];
        uint4 u;
    } o;
#pragma unroll
    for (int c = 0; c < 4; ++c) o.w[c] = f32x2_to_bf16x2(v[2 * c], v[2 * c + 1]);
    *reinterpret_cast<uint4 *>(dst) = o.u;
}
__device__ __forceinline__ void store_bf16x4(uint16_t *dst, const float *v)
{
    union {
        uint32_t w[2];
        uint2 u;
    } o;
#pragma unroll
    for (int c = 0; c < 2; ++c) o.w[c] = f32x2_to_bf16x2(v[2 * c], v[2 * c + 1]);
    *reinterpret_cast<uint2 *>(dst) = o.u;
}

// Epilogue of one token row of a wavefront: FB consecutive row blocks starting at row block rb0, lane
// group q.  Stage 1 turns (gate, up) into SiLU(g)*u -> bf16; stage 2 scales by the router weight and
// stores fp32 or bf16.  Neighbouring row blocks of an interleave group are adjacent in memory, so bf16
// results leave in 16-byte stores wherever two of them line up.
template <int STAGE, int FB>
__device__ __forceinline__ void store_token_row(const GemmArgs &a, const floatx4 *acc_g, const floatx4 *acc_u, int stride,
                                                size_t row_elem, int rb0, int q, float wgt)
{
    float v[FB][4];
#pragma unroll
    for (int i = 0; i < FB; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float g = acc_g[i * stride][c];
            v[i][c] = (STAGE == 1) ? silu_f32(g) * acc_u[i * stride][c] : wgt * g;
        }
    if (STAGE == 2 && !a.y_bf16) {
#pragma unroll
        for (int i = 0; i < FB; ++i)
            *reinterpret_cast<float4 *>(a.y_out + row_elem + packed_row_feature(rb0 + i, q * 4)) =
                make_float4(v[i][0], v[i][1], v[i][2], v[i][3]);
        return;
    }
    // stage 1 writes the activation in the fragment-major layout that stage 2 loads (row_elem is the slot);
    // 8 features aligned to 8 are contiguous in both layouts
    auto dst = [&](int feature) -> uint16_t * {
        if (STAGE == 1)
            return a.a_row_major ? a.a_out + row_elem * (size_t)a.F + (size_t)feature
                                 : a.a_out + act_elem((uint32_t)row_elem, (uint32_t)feature, (uint32_t)a.F >> 5);
        return reinterpret_cast<uint16_t *>(a.y_out) + row_elem + feature;
    };
    // row blocks rb0.. are consecutive; pairs (even, odd) inside a group of kPermBlocks are 8 adjacent features
    int i = 0;
    if ((rb0 & 1) && FB > 0) {
        store_bf16x4(dst(packed_row_feature(rb0, q * 4)), v[0]);
        i = 1;
    }
#pragma unroll
    for (int j = 0; j < FB; ++j) {
        if (j < i) continue;
        if (((j - i) & 1) == 0) {
            if (j + 1 < FB) {
                float w8[8] = {v[j][0], v[j][1], v[j][2], v[j][3], v[j + 1 < FB ? j + 1 : j][0], v[j + 1 < FB ? j + 1 : j][1],
                               v[j + 1 < FB ? j + 1 : j][2], v[j + 1 < FB ? j + 1 : j][3]};
                store_bf16x8(dst(packed_row_feature(rb0 + j, q * 4)), w8);
            } else {
                store_bf16x4(dst(packed_row_feature(rb0 + j, q * 4)), v[j]);
            }
        }
    }
}

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

// Workgroup -> tile.  Workgroups are handed to the 8 XCDs round robin (id % 8), each XCD has its own
// 4 MB L2 and runs 32 workgroups of the large tiles at a time.  Consecutive workgroups of one XCD
// therefore take a block of group_m M-tiles x group_n N-tiles: the token slices are shared by the
// N-tiles of the block and the weight slices by its M-tiles (same expert, mostly) while they are
// still in that XCD's L2 (the XCD-aware analogue of the GROUP_M swizzle, Sec. 4.1 Eq. 4).  Blocks
// walk the N dimension first, then the next group of M-tiles.
__device__ __forceinline__ void tile_of_id(const GemmArgs &a, int id, int &n_tile, int &m_tile)
{
    const int xcd = id & 7, s = id >> 3;
    const int per_block = a.group_m * a.group_n;
    const int sb = s / per_block, w = s - sb * per_block;
    const int dn = w / a.group_m, dm = w - dn * a.group_m;
    const int nbn = a.n_tiles / a.group_n;
    const int mb = sb / nbn, nbi = sb - mb * nbn;
    n_tile = nbi * a.group_n + dn;
    m_tile = (mb * 8 + xcd) * a.group_m + dm;
}

// The same map for the persistent kernels, whose workgroup c of an XCD walks slots c, c + 32, ...  With the static map
// a workgroup gets the same position of every block and an XCD every eighth M-tile; where the experts have a full
// M-tile followed by a ragged one (two tiles per expert: block positions and XCDs alternate full, ragged) half of the
// workgroups, or half of the XCDs, then only ever get ragged tiles, finish early and run ahead of the siblings they
// share weights with.  So the position inside the block moves on by one per block, and the XCD -> M-tile assignment
// inside a round of 8 * group_m M-tiles by three per round: an XCD then steps through the M-tiles by 11 or 3 instead
// of 8, which does not stay in phase with 2, 3, 4, 8 or 9 tiles per expert (a shift of one, steps of 9, does with 3
// and 9: measured 7 % slower on such a layer).  The tiles an XCD works on at a time stay the same, who gets which
// changes.  Same-box A/B of the layer: DeepSeek-V3 T = 2048 at 52 active experts (two tiles each) 2010 -> 1766 us,
// Mixtral T = 8192 4980 -> 4880 us, T = 1024 1035 -> 1013 us, the other large points within +-1 %.
__device__ __forceinline__ void tile_of_id_rotated(const GemmArgs &a, int id, int &n_tile, int &m_tile)
{
    const int xcd = id & 7, s = id >> 3;
    const int per_block = a.group_m * a.group_n;
    const int sb = s / per_block;
    const int w = (s - sb * per_block + sb) % per_block;
    const int dn = w / a.group_m, dm = w - dn * a.group_m;
    const int nbn = a.n_tiles / a.group_n;
    const int mb = sb / nbn, nbi = sb - mb * nbn;
    n_tile = nbi * a.group_n + dn;
    m_tile = (mb * 8 + ((xcd + 3 * mb) & 7)) * a.group_m + dm;
}

__device__ __forceinline__ void tile_of_workgroup(const GemmArgs &a, int &n_tile, int &m_tile)
{
    tile_of_id(a, (int)blockIdx.x, n_tile, m_tile);
}

// Picks the block shape for the launch and returns the (overlaunched) number of tile ids that tile_of_id expects.
inline unsigned xcd_grid(GemmArgs &g)
{
    xcd_block_shape(g.n_tiles, g.group_m_req, &g.group_m, &g.group_n);
    const int per_round = 8 * g.group_m;  // M-tiles handed out per round over the 8 XCDs
    const int rounds = (g.m_tiles_cap + per_round - 1) / per_round;
    return (unsigned)rounds * (unsigned)per_round * (unsigned)g.n_tiles;
}

template <int STAGE, int BM, int BN, int BK, int WM, int WN, int NSTAGE, int LOOP>
__global__ __launch_bounds__(WM *WN * 64, (TileTraits<BM, BN, BK, WM, WN, NSTAGE>::MIN_WAVES_PER_SIMD)) void moe_gemm_kernel(
    GemmArgs a)
{
    using TT = TileTraits<BM, BN, BK, WM, WN, NSTAGE>;
    constexpr int KS = TT::KS, NB = TT::NB, SLOTS = TT::SLOTS, NWAVE = TT::NWAVE;
    constexpr int FB = (STAGE == 1) ? TT::FB1 : TT::FB2;
    constexpr int NACC = (STAGE == 1) ? 2 * FB : FB;  // accumulator row blocks per wavefront
    constexpr int FEAT_PER_TILE = (STAGE == 1) ? BN / 2 : BN;

    __shared__ __attribute__((aligned(1024))) uint16_t lds[NSTAGE * TT::BUF_ELEMS];

    if (launch_deselected(a.pred, a.pred_value)) return;
    int n_tile, m_tile;
    tile_of_workgroup(a, n_tile, m_tile);
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
            if (STAGE == 1) {
                const int pair = a.sorted[slot];
                const size_t row = (pair < a.P) ? (size_t)(pair / a.topk) : 0;
                gptr[s] = a.act + row * (size_t)K + (size_t)(ks * 32 + q * 8);
                gstep[s] = BK;
            } else {
                // fragment-major activation written by stage 1: a k-step of 16 slots is one 1 KB line
                gptr[s] = a.act + act_elem((uint32_t)slot, (uint32_t)(ks * 32 + q * 8), (uint32_t)KST);
                gstep[s] = KS * kFragElems;
            }
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
    // Padding sits at the end of a tile, so this wavefront's token blocks are real up to some
    // block and sentinel-only after it: the products of all-padding blocks are skipped (the ragged
    // last tile of an expert then costs its loads but only the MFMAs of its real rows).
    int nb_valid = 0;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int tr0 = (wm * NB + nb) * 16;
        if (tr0 < BM && a.sorted[m_tile * BM + tr0] < a.P) nb_valid = nb + 1;
    }
    nb_valid = __builtin_amdgcn_readfirstlane(nb_valid);

    // stage 2: destination pair and router weight of this lane's token rows, fetched now so the
    // epilogue does not end on two dependent global loads
    int out_pair[NB];
    float out_wgt[NB];
    if (STAGE == 2) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int tr = (wm * NB + nb) * 16 + r16;
            out_pair[nb] = (tr < BM && nb < nb_valid) ? a.sorted[m_tile * BM + tr] : a.P;
            out_wgt[nb] = (out_pair[nb] < a.P) ? a.topk_w[out_pair[nb]] : 0.0f;
        }
    }

    auto compute_slice = [&](int buf) {
        const uint16_t *xs = &lds[buf * TT::BUF_ELEMS + lane * 8];
        const uint16_t *ws = xs + TT::X_FRAGS * kFragElems;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bf16x8 w[NACC];
#pragma unroll
            for (int i = 0; i < NACC; ++i) {
                int rb;
                if (STAGE == 1) rb = (i < FB) ? (wn * FB + i) : (TT::RB / 2 + wn * FB + (i - FB));
                else rb = wn * FB + i;
                w[i] = *reinterpret_cast<const bf16x8 *>(ws + (rb * KS + ks) * kFragElems);
            }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                if (nb < nb_valid) {
                    const bf16x8 b = *reinterpret_cast<const bf16x8 *>(xs + ((wm * NB + nb) * KS + ks) * kFragElems);
#pragma unroll
                    for (int i = 0; i < NACC; ++i)
                        acc[i][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[i], b, acc[i][nb], 0, 0, 0);
                }
            }
        }
    };

    const int KT = K / BK;
    if constexpr (LOOP == 1) {
        // Register-pipelined main loop for one wavefront per SIMD: two register sets of operand
        // fragments; while the MFMAs of k-step g run on one set, the ds_reads of k-step g+1 fill
        // the other.  All NSTAGE buffers are kept full: at the last k-step of slice kt every
        // wavefront already holds its last fragments of that slice in registers, so after one
        // barrier the buffer is handed to the loads of slice kt+NSTAGE.
        static_assert(LOOP != 1 || KS % 2 == 0, "register sets alternate per k-step: bk must be a multiple of 64");
        bf16x8 fx[2][NB], fw[2][NACC];
        auto read_frags = [&](int set, int buf, int ks) {
            const uint16_t *xs = &lds[buf * TT::BUF_ELEMS + lane * 8];
            const uint16_t *ws = xs + TT::X_FRAGS * kFragElems;
#pragma unroll
            for (int i = 0; i < NACC; ++i) {
                int rb;
                if (STAGE == 1) rb = (i < FB) ? (wn * FB + i) : (TT::RB / 2 + wn * FB + (i - FB));
                else rb = wn * FB + i;
                fw[set][i] = *reinterpret_cast<const bf16x8 *>(ws + (rb * KS + ks) * kFragElems);
            }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                fx[set][nb] = *reinterpret_cast<const bf16x8 *>(xs + ((wm * NB + nb) * KS + ks) * kFragElems);
        };
        auto mfma_step = [&](int set) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                if (nb < nb_valid) {
#pragma unroll
                    for (int i = 0; i < NACC; ++i)
                        acc[i][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw[set][i], fx[set][nb], acc[i][nb], 0, 0, 0);
                }
            }
        };
        auto wait_for_next = [&](int later) {  // `later` younger slices may stay in flight
            if (NSTAGE >= 4 && later >= 2) wait_vmcnt<(NSTAGE >= 4 ? 2 : 0) * SLOTS>();
            else if (NSTAGE >= 3 && later >= 1) wait_vmcnt<(NSTAGE >= 3 ? 1 : 0) * SLOTS>();
            else wait_vmcnt<0>();
        };
#pragma unroll
        for (int s = 0; s < NSTAGE; ++s)
            if (s < KT) issue_slice(s);
        wait_for_next(min(NSTAGE - 1, KT - 1));
        __builtin_amdgcn_s_barrier();
        read_frags(0, 0, 0);
        int buf_cur = 0;
        for (int kt = 0; kt < KT; ++kt) {
            const int buf_next = (buf_cur + 1 == NSTAGE) ? 0 : buf_cur + 1;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const int cur = ks & 1, nxt = cur ^ 1;
                if (ks + 1 < KS) {
                    read_frags(nxt, buf_cur, ks + 1);
                } else if (kt + 1 < KT) {
                    // every fragment of slice kt is in registers by now (requested one k-step ago)
                    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): no LDS read of this buffer pending
                    wait_for_next(min(NSTAGE - 2, KT - 2 - kt));
                    __builtin_amdgcn_s_barrier();
                    if (kt + NSTAGE < KT) issue_slice(buf_cur);
                    read_frags(nxt, buf_next, 0);
                }
                mfma_step(cur);
            }
            buf_cur = buf_next;
        }
    } else {
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
    }

    // ---- epilogue: lane holds features f = fblock*16 + 4*q + {0..3} of token n = r16 ----
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int tr = (wm * NB + nb) * 16 + r16;
        if (tr >= BM || nb >= nb_valid) continue;
        const int slot = m_tile * BM + tr;
        const int rb0 = f0 / 16 + wn * FB;
        if (STAGE == 1) {
            store_token_row<1, FB>(a, &acc[0][nb], &acc[FB][nb], NB, (size_t)slot, rb0, q, 1.0f);
        } else {
            const int pair = out_pair[nb];
            if (pair >= a.P) continue;
            store_token_row<2, FB>(a, &acc[0][nb], &acc[0][nb], NB, (size_t)pair * a.F, rb0, q, out_wgt[nb]);
        }
    }
}

template <int BM, int BN, int BK, int WM, int WN, int NSTAGE, int LOOP>
void launch_gemm(int stage, const GemmArgs &a, hipStream_t stream)
{
    if (a.n_tiles <= 0 || a.m_tiles_cap <= 0) return;
    GemmArgs g = a;
    const dim3 grid(xcd_grid(g)), block(WM * WN * 64);
    if (stage == 1)
        hipLaunchKernelGGL((moe_gemm_kernel<1, BM, BN, BK, WM, WN, NSTAGE, LOOP>), grid, block, 0, stream, g);
    else
        hipLaunchKernelGGL((moe_gemm_kernel<2, BM, BN, BK, WM, WN, NSTAGE, LOOP>), grid, block, 0, stream, g);
}


template <int BM, int BN, int BK, int WM, int WN, int NSTAGE, int LOOP>
KernelInfo make_info()
{
    using TT = TileTraits<BM, BN, BK, WM, WN, NSTAGE>;
    KernelInfo ki = {};
    ki.cfg = ramp_config{BM, BN, BK, WM * WN, NSTAGE, (WM - 1) | (LOOP == 1 ? kModePipe : 0)};
    ki.wm = WM;
    ki.wn = WN;
    ki.lds_bytes = TT::LDS_BYTES;
    ki.acc_regs = TT::ACC_REGS;
    ki.launch = &launch_gemm<BM, BN, BK, WM, WN, NSTAGE, LOOP>;
    ki.kernel_fn[0] = reinterpret_cast<const void *>(&moe_gemm_kernel<1, BM, BN, BK, WM, WN, NSTAGE, LOOP>);
    ki.kernel_fn[1] = reinterpret_cast<const void *>(&moe_gemm_kernel<2, BM, BN, BK, WM, WN, NSTAGE, LOOP>);
    ki.block_threads = WM * WN * 64;
    ki.family = "moe_gemm_kernel";
    const int targs[8] = {1, BM, BN, BK, WM, WN, NSTAGE, LOOP};
    for (int i = 0; i < 8; ++i) ki.targs[i] = targs[i];
    ki.n_targs = 8;
    return ki;
}

}  // namespace ramp
