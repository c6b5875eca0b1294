// W8A8 FP8 variant of the fused MoE layer (paper Sec. 4.3: "W8A8 FP8, 128x128 block scales"; Sec. 2.2 phase 2:
// the activation is re-quantised between the projections) on the scaled FP8 matrix instruction of gfx950.
//
// Numbers.  FP8 = OCP E4M3 (bias 7, largest value 448, round to nearest even, saturating).  A block scale is a
// power of two kept as an E8M0 byte b (scale 2^(b-127)): the smallest one with amax/scale <= 448.  Weights carry
// one scale per 128 x 128 block, activations one per token and 128 consecutive k-values.  Power-of-two scales are
// what v_mfma_scale_f32_16x16x128_f8f6f4 applies by itself: one instruction multiplies 16 weight rows by 16 tokens
// over exactly one scale block of 128 k-values and scales the products by 2^(a+b), so the block scales cost no
// vector ALU work at all.
//
// Path:  align(bm) -> quantise X per token and 128-group -> up-projection (FP8 MFMA, fp32 accumulate) + SwiGLU ->
// A in bf16, row-major -> quantise A -> down-projection (FP8 MFMA) x router weight -> per-pair rows -> combine.
//
// Layouts.  A "fragment" here is 16 rows x 128 k-values of E4M3 = 2 KB: the operand of one MFMA, lane l holding
// row l%16 and the 32 consecutive k-values 32*(l/16) ...  It is stored as two 1 KB halves, half h holding bytes
// [16h, 16h+16) of every lane in lane order, so each half is one conflict-free 16-byte-per-lane LDS image exactly
// like a bf16 fragment, and LDS-direct loads fill it the same way.
//   packed weights: [E][gate: I/16 row blocks][H/128][2 KB] [up: same] | [E][H/16][I/128][2 KB] | scale bytes
//   scale bytes:    [E][gate, up, down][feature block of 128][k block, row stride padded to 4 bytes]
//   quantised activations: codes row-major [rows, K], scale bytes [rows][K/128 padded to 4]
// Which feature sits in row r of row block rb is the interleave of the bf16 layout (packed_row_feature).
#include "moe_gemm.h"

namespace ramp {

typedef int intx8 __attribute__((ext_vector_type(8)));
typedef int intx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kGroup = 128;  // k-values per scale block

__host__ __device__ inline int scale_stride(int K) { return (K / kGroup + 3) / 4 * 4; }

struct Fp8Layout {
    size_t w1_expert_bytes, up_offset_bytes, w2_expert_bytes, w2_base_bytes;
    size_t scale_base, scale_g, scale_u, scale_d, scale_expert_bytes;  // offsets of the three scale arrays inside an expert's scales
    int stride1, stride2;                                               // scale row strides: k blocks of H / of I, padded
    size_t total_bytes;
};
Fp8Layout fp8_layout(const ramp_shape &s)
{
    Fp8Layout L;
    L.up_offset_bytes = (size_t)s.I * s.H;
    L.w1_expert_bytes = 2 * L.up_offset_bytes;
    L.w2_expert_bytes = (size_t)s.H * s.I;
    L.w2_base_bytes = (size_t)s.E * L.w1_expert_bytes;
    L.scale_base = align_up((size_t)s.E * (L.w1_expert_bytes + L.w2_expert_bytes), 256);
    L.stride1 = scale_stride(s.H);
    L.stride2 = scale_stride(s.I);
    L.scale_g = 0;
    L.scale_u = (size_t)(s.I / kGroup) * L.stride1;
    L.scale_d = 2 * L.scale_u;
    L.scale_expert_bytes = L.scale_d + (size_t)(s.H / kGroup) * L.stride2;
    L.total_bytes = align_up(L.scale_base + (size_t)s.E * L.scale_expert_bytes, 256);
    return L;
}

// ---- number formats -------------------------------------------------------------------------------------------

// E8M0 byte of the smallest power of two s with amax / s <= 448 (448 = 1.75 * 2^8): from the fp32 bits of amax.
__device__ __forceinline__ uint32_t e8m0_of_amax(float amax)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, amax) & 0x7fffffffu;
    if (u == 0u || u >= 0x7f800000u) return 127u;  // all-zero block (or not finite): scale 1
    const int field = (int)(u >> 23);
    const int b = field - ((u & 0x7fffffu) <= 0x600000u ? 8 : 7);
    return (uint32_t)(b < 0 ? 0 : (b > 254 ? 254 : b));
}
// 2^(127-b): the factor that brings a block into the E4M3 range.
__device__ __forceinline__ float inv_scale_of(uint32_t b) { return __builtin_bit_cast(float, (254u - b) << 23); }

// fp32 -> E4M3 code: round to nearest, ties to even, saturate at 448.
__device__ __forceinline__ uint32_t e4m3_of_f32(float v)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, v);
    const uint32_t sign = (u >> 24) & 0x80u;
    uint32_t a = u & 0x7fffffffu;
    if (a > 0x43e00000u) a = 0x43e00000u;  // 448
    if (a >= 0x3c800000u) {                // >= 2^-6: normal code; keep 3 mantissa bits
        const uint32_t r = a + 0x7ffffu + ((a >> 20) & 1u);
        uint32_t code = (r >> 20) - (120u << 3);
        if (code > 0x7eu) code = 0x7eu;
        return sign | code;
    }
    // subnormal range: multiples of 2^-9 (8 of them reach the smallest normal value, code 8)
    const float f = __builtin_bit_cast(float, a) * 512.0f;
    return sign | (uint32_t)__builtin_rintf(f);
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __builtin_bit_cast(float, h << 16); }

// ---- quantisers -----------------------------------------------------------------------------------------------

// src bf16 [rows, K] row-major -> codes [rows, K], scale bytes [rows, stride].  One wavefront per (row, 128-group),
// two values per lane.  Rows at or past *n_rows_dev (when given) are skipped.
__global__ __launch_bounds__(256) void quant_rows_kernel(const uint16_t *__restrict__ src, int rows, int K,
                                                         uint8_t *__restrict__ codes, uint8_t *__restrict__ sb, int stride,
                                                         const int32_t *__restrict__ n_rows_dev, const int32_t *pred,
                                                         int pred_value)
{
    if (launch_deselected(pred, pred_value)) return;
    const int lane = threadIdx.x & 63;
    const int groups = K / kGroup;
    const int live_rows = n_rows_dev ? min(rows, *n_rows_dev) : rows;
    const size_t total = (size_t)live_rows * groups;
    const size_t wave0 = (size_t)blockIdx.x * (blockDim.x / 64) + (threadIdx.x >> 6);
    const size_t nwaves = (size_t)gridDim.x * (blockDim.x / 64);
    for (size_t w = wave0; w < total; w += nwaves) {
        const size_t row = w / groups;
        const int g = (int)(w % groups);
        const uint32_t two = *reinterpret_cast<const uint32_t *>(src + row * (size_t)K + (size_t)g * kGroup + 2 * lane);
        const float v0 = bf16_bits_to_f32(two & 0xffffu), v1 = bf16_bits_to_f32(two >> 16);
        float amax = fmaxf(fabsf(v0), fabsf(v1));
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) amax = fmaxf(amax, __shfl_xor(amax, d));
        const uint32_t b = e8m0_of_amax(amax);
        const float inv = inv_scale_of(b);
        const uint32_t c = e4m3_of_f32(v0 * inv) | (e4m3_of_f32(v1 * inv) << 8);
        *reinterpret_cast<uint16_t *>(codes + row * (size_t)K + (size_t)g * kGroup + 2 * lane) = (uint16_t)c;
        if (lane == 0) sb[row * (size_t)stride + g] = (uint8_t)b;
    }
}

// One workgroup per 128 x 128 block of src [E][K][F] (F contiguous): scale byte into sb[e][f block][k block].
__global__ __launch_bounds__(256) void block_scale_kernel(const uint16_t *__restrict__ src, int K, int F,
                                                          uint8_t *__restrict__ sb, size_t sb_expert_stride, int stride)
{
    __shared__ float red[4];
    const int kb = blockIdx.x, fb = blockIdx.y, e = blockIdx.z;
    const int ff = threadIdx.x & 127, k0 = threadIdx.x >> 7;
    const uint16_t *p = src + (size_t)e * K * F + (size_t)(kb * kGroup) * F + (size_t)fb * kGroup + ff;
    float amax = 0.f;
    for (int kk = k0; kk < kGroup; kk += 2) amax = fmaxf(amax, fabsf(bf16_bits_to_f32(p[(size_t)kk * F])));
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) amax = fmaxf(amax, __shfl_xor(amax, d));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = amax;
    __syncthreads();
    if (threadIdx.x == 0) {
        amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        sb[(size_t)e * sb_expert_stride + (size_t)fb * stride + kb] = (uint8_t)e8m0_of_amax(amax);
    }
}

// src [E][K][F] bf16 -> packed E4M3 fragments [E][F/16][K/128][2 KB]; one lane writes one 16-byte chunk
// (16 consecutive k of one weight row).
__global__ __launch_bounds__(256) void pack_fp8_kernel(const uint16_t *__restrict__ src, uint8_t *__restrict__ dst, int E, int K,
                                                       int F, size_t dst_expert_stride, const uint8_t *__restrict__ sb,
                                                       size_t sb_expert_stride, int stride)
{
    const size_t chunks_per_expert = (size_t)K * F / 16;
    const size_t total = chunks_per_expert * E;
    const int kt = K / kGroup;
    for (size_t c = (size_t)blockIdx.x * blockDim.x + threadIdx.x; c < total; c += (size_t)gridDim.x * blockDim.x) {
        const int e = (int)(c / chunks_per_expert);
        const size_t ce = c % chunks_per_expert;
        const int lane = (int)(ce % 64);
        const int h = (int)((ce / 64) % 2);
        const size_t frag = ce / 128;
        const int ks = (int)(frag % kt);
        const int rb = (int)(frag / kt);
        const int f = packed_row_feature(rb, lane % 16);
        const int k0 = ks * kGroup + (lane / 16) * 32 + h * 16;
        const float inv = inv_scale_of(sb[(size_t)e * sb_expert_stride + (size_t)(f / kGroup) * stride + ks]);
        const uint16_t *s = src + (size_t)e * K * F + (size_t)k0 * F + f;
        union {
            uint8_t b[16];
            uint4 v;
        } u;
#pragma unroll
        for (int j = 0; j < 16; ++j) u.b[j] = (uint8_t)e4m3_of_f32(bf16_bits_to_f32(s[(size_t)j * F]) * inv);
        *reinterpret_cast<uint4 *>(dst + (size_t)e * dst_expert_stride + frag * 2048 + (size_t)h * 1024 + (size_t)lane * 16) = u.v;
    }
}

// ---- projections ----------------------------------------------------------------------------------------------

struct Fp8Args {
    const uint8_t *act_q;      // quantised token operand, row-major [rows, K]
    const uint8_t *act_scale;  // [rows][act_stride] E8M0 bytes
    int act_stride;
    const uint8_t *wq;         // packed codes of this stage
    size_t expert_stride;      // bytes between experts
    size_t up_offset;          // stage 1: byte offset of the up rows inside an expert
    const uint8_t *wscale;     // this stage's first scale array of expert 0 (gate, or down)
    size_t wscale_expert_stride;
    size_t wscale_up_offset;   // stage 1: gate -> up scale array
    int w_stride;              // scale row stride of this stage's weight scales
};

// One workgroup = (M-tile of an expert) x (tile of BN weight rows), k-slices of 128 through a ring of NSTAGE LDS
// buffers (LDS-direct loads, one vmcnt wait + one barrier per slice), as moe_gemm_kernel with LOOP = 0.  TileTraits
// is instantiated with BK = 64: a slice of 128 one-byte values occupies the bytes of 64 bf16 values, i.e. two 1 KB
// half-fragments per 16-row block.
template <int STAGE, int BM, int BN, int WM, int WN, int NSTAGE>
__global__ __launch_bounds__(WM *WN * 64) void moe_fp8_kernel(GemmArgs a, Fp8Args f)
{
    using TT = TileTraits<BM, BN, 64, WM, WN, NSTAGE>;
    constexpr int NB = TT::NB, SLOTS = TT::SLOTS, NWAVE = TT::NWAVE;
    constexpr int FB = (STAGE == 1) ? TT::FB1 : TT::FB2;
    constexpr int NACC = (STAGE == 1) ? 2 * FB : FB;
    constexpr int FEAT_PER_TILE = (STAGE == 1) ? BN / 2 : BN;
    constexpr int BUF_BYTES = TT::BUF_ELEMS * 2;
    static_assert(FB * 16 <= kGroup && kGroup % (FB * 16) == 0, "a wavefront's weight rows must share one scale block");

    __shared__ __attribute__((aligned(1024))) char lds[NSTAGE * BUF_BYTES];

    if (launch_deselected(a.pred, a.pred_value)) return;
    int n_tile, m_tile;
    tile_of_workgroup(a, n_tile, m_tile);
    if (m_tile >= a.meta[1]) return;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int e = a.tile_expert[m_tile];
    const int K = a.K, KT = K / kGroup;
    const int f0 = n_tile * FEAT_PER_TILE;
    const uint8_t *wexp = f.wq + (size_t)e * f.expert_stride;
    const int r16 = lane & 15, q = lane >> 4;

    // token row (of the quantised operand) behind slot `slot`
    auto row_of_slot = [&](int slot) -> size_t {
        if (STAGE == 2) return (size_t)slot;
        const int pair = a.sorted[slot];
        return (pair < a.P) ? (size_t)(pair / a.topk) : 0;
    };

    // ---- per-slot global sources for k-slice 0: slot s of this wavefront fills half-fragment wave + s*NWAVE
    const uint8_t *gptr[SLOTS];
    int gstep[SLOTS];
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        const int idx = wave + s * NWAVE;
        if (idx < TT::X_FRAGS) {
            const int nb = idx >> 1, h = idx & 1;
            int tr = nb * 16 + r16;
            if (tr >= BM) tr = BM - 1;
            gptr[s] = f.act_q + row_of_slot(m_tile * BM + tr) * (size_t)K + (size_t)(q * 32 + h * 16);
            gstep[s] = kGroup;
        } else {
            const int widx = idx - TT::X_FRAGS;
            const int rb = widx >> 1, h = widx & 1;
            size_t base;
            if (STAGE == 1) {
                const int half = TT::RB / 2;
                base = (rb < half) ? (size_t)(f0 / 16 + rb) * KT * 2048 : f.up_offset + (size_t)(f0 / 16 + rb - half) * KT * 2048;
            } else {
                base = (size_t)(f0 / 16 + rb) * KT * 2048;
            }
            gptr[s] = wexp + base + (size_t)h * 1024 + (size_t)lane * 16;
            gstep[s] = 2048;
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
            load_to_lds_16B(gptr[s], lds + buf * BUF_BYTES + (wave + s * NWAVE) * 1024);
            gptr[s] += gstep[s];
        }
    };

    int nb_valid = 0;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int tr0 = (wm * NB + nb) * 16;
        if (tr0 < BM && a.sorted[m_tile * BM + tr0] < a.P) nb_valid = nb + 1;
    }
    nb_valid = __builtin_amdgcn_readfirstlane(nb_valid);

    // ---- scale bytes, four k-blocks per 32-bit load (scale rows are padded to multiples of four bytes).
    // Tokens: one row of scale bytes per lane and token block; weights: one row per scale block of the wavefront's
    // features (gate and up in the up-projection), the same for every lane.
    const uint8_t *sxp[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        int tr = (wm * NB + nb) * 16 + r16;
        if (tr >= BM) tr = BM - 1;
        sxp[nb] = f.act_scale + row_of_slot(m_tile * BM + tr) * (size_t)f.act_stride;
    }
    constexpr int NWS = (STAGE == 1) ? 2 : 1;
    const uint8_t *swp[NWS];
    {
        const uint8_t *base = f.wscale + (size_t)e * f.wscale_expert_stride + (size_t)((f0 + wn * FB * 16) / kGroup) * f.w_stride;
        swp[0] = base;
        if (STAGE == 1) swp[NWS - 1] = base + f.wscale_up_offset;
    }
    uint32_t sx_cur[NB], sx_nxt[NB], sw_cur[NWS], sw_nxt[NWS];
    auto load_scales = [&](uint32_t *sx, uint32_t *sw, int group4) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) sx[nb] = *reinterpret_cast<const uint32_t *>(sxp[nb] + group4 * 4);
#pragma unroll
        for (int i = 0; i < NWS; ++i) sw[i] = *reinterpret_cast<const uint32_t *>(swp[i] + group4 * 4);
    };
    const int last_group4 = (KT - 1) / 4;
    load_scales(sx_cur, sw_cur, 0);

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

    auto compute_slice = [&](int buf, int kt) {
        const char *xs = lds + buf * BUF_BYTES + lane * 16;
        const char *ws = xs + TT::X_FRAGS * 1024;
        const int sh = (kt & 3) * 8;
        intx8 wv[NACC];
#pragma unroll
        for (int i = 0; i < NACC; ++i) {
            int rb;
            if (STAGE == 1) rb = (i < FB) ? (wn * FB + i) : (TT::RB / 2 + wn * FB + (i - FB));
            else rb = wn * FB + i;
            const intx4 lo = *reinterpret_cast<const intx4 *>(ws + (rb * 2) * 1024);
            const intx4 hi = *reinterpret_cast<const intx4 *>(ws + (rb * 2 + 1) * 1024);
            wv[i] = intx8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
        int swb[NWS];
#pragma unroll
        for (int i = 0; i < NWS; ++i) swb[i] = (int)(sw_cur[i] >> sh);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            if (nb < nb_valid) {
                const intx4 lo = *reinterpret_cast<const intx4 *>(xs + ((wm * NB + nb) * 2) * 1024);
                const intx4 hi = *reinterpret_cast<const intx4 *>(xs + ((wm * NB + nb) * 2 + 1) * 1024);
                const intx8 xv = intx8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                const int sxb = (int)(sx_cur[nb] >> sh);
#pragma unroll
                for (int i = 0; i < NACC; ++i)
                    acc[i][nb] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                        wv[i], xv, acc[i][nb], 0, 0, 0, swb[(STAGE == 1 && i >= FB) ? NWS - 1 : 0], 0, sxb);
            }
        }
    };

#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s)
        if (s < KT) issue_slice(s);

    int buf_cur = 0, buf_issue = NSTAGE - 1;
    for (int kt = 0; kt < KT; ++kt) {
        // the scale words of the next four slices are requested before this iteration's LDS-direct loads, so the
        // waits below (counted in LDS-direct loads) can only be stricter than needed, never weaker
        if ((kt & 3) == 0) load_scales(sx_nxt, sw_nxt, min(kt / 4 + 1, last_group4));
        const int later = min(NSTAGE - 2, KT - 1 - kt);
        if (NSTAGE >= 4 && later >= 2) wait_vmcnt<(NSTAGE >= 4 ? 2 : 0) * SLOTS>();
        else if (NSTAGE >= 3 && later >= 1) wait_vmcnt<(NSTAGE >= 3 ? 1 : 0) * SLOTS>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        if (kt + NSTAGE - 1 < KT) issue_slice(buf_issue);
        compute_slice(buf_cur, kt);
        if ((kt & 3) == 3) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) sx_cur[nb] = sx_nxt[nb];
#pragma unroll
            for (int i = 0; i < NWS; ++i) sw_cur[i] = sw_nxt[i];
        }
        buf_cur = (buf_cur + 1 == NSTAGE) ? 0 : buf_cur + 1;
        buf_issue = (buf_issue + 1 == NSTAGE) ? 0 : buf_issue + 1;
    }

    // ---- epilogue: lane holds features fblock*16 + 4*q + {0..3} of token r16
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

struct Fp8Kernel {
    ramp_config cfg;
    int lds_bytes, waves_per_cu_limit;
    void (*launch)(int stage, const GemmArgs &, const Fp8Args &, hipStream_t);
};

template <int BM, int BN, int WM, int WN, int NSTAGE>
void launch_fp8(int stage, const GemmArgs &a, const Fp8Args &f, hipStream_t stream)
{
    if (a.n_tiles <= 0 || a.m_tiles_cap <= 0) return;
    GemmArgs g = a;
    const dim3 grid(xcd_grid(g)), block(WM * WN * 64);
    if (stage == 1)
        hipLaunchKernelGGL((moe_fp8_kernel<1, BM, BN, WM, WN, NSTAGE>), grid, block, 0, stream, g, f);
    else
        hipLaunchKernelGGL((moe_fp8_kernel<2, BM, BN, WM, WN, NSTAGE>), grid, block, 0, stream, g, f);
}

template <int BM, int BN, int WM, int WN, int NSTAGE>
Fp8Kernel make_fp8()
{
    using TT = TileTraits<BM, BN, 64, WM, WN, NSTAGE>;
    Fp8Kernel k;
    k.cfg = ramp_config{BM, BN, kGroup, WM * WN, NSTAGE, (WM - 1) | kModeFp8};
    k.lds_bytes = TT::LDS_BYTES;
    // workgroups per compute unit: LDS, and one wavefront per SIMD for the large register tiles
    const int by_lds = kLdsBytesPerCU / TT::LDS_BYTES;
    const int by_regs = (TT::ACC_REGS > 128 ? 1 : 2) * 4 / (WM * WN);
    k.waves_per_cu_limit = by_lds < by_regs ? by_lds : by_regs;
    if (k.waves_per_cu_limit < 1) k.waves_per_cu_limit = 1;
    k.launch = &launch_fp8<BM, BN, WM, WN, NSTAGE>;
    return k;
}

// The FP8 tile family: X(bm, bn, WM, WN, NSTAGE), bk = 128.
#define RAMP_FP8_CONFIGS(X) \
    X(16, 128, 1, 2, 4)     \
    X(32, 128, 1, 4, 3)     \
    X(64, 256, 1, 4, 3)     \
    X(128, 256, 2, 2, 3)    \
    X(128, 256, 2, 4, 3)

const Fp8Kernel *fp8_kernels(int *n)
{
    static const Fp8Kernel table[] = {
#define X(BM, BN, WM, WN, NS) make_fp8<BM, BN, WM, WN, NS>(),
        RAMP_FP8_CONFIGS(X)
#undef X
    };
    *n = (int)(sizeof(table) / sizeof(table[0]));
    return table;
}

bool fp8_valid_for_shape(const Fp8Kernel &k, const ramp_shape &s)
{
    if (!moe_shape_ok(s)) return false;
    if ((2 * s.I) % k.cfg.bn || s.H % k.cfg.bn) return false;
    const size_t cap = ramp_align_capacity(s.T, s.k, s.E, k.cfg.bm);
    if ((cap + 16) * (size_t)s.I >= (1ull << 32) || (size_t)s.T * s.H >= (1ull << 32)) return false;
    return true;
}

const Fp8Kernel *find_fp8(const ramp_config &c)
{
    int n = 0;
    const Fp8Kernel *t = fp8_kernels(&n);
    for (int i = 0; i < n; ++i) {
        const ramp_config &k = t[i].cfg;
        if (k.bm == c.bm && k.bn == c.bn && k.bk == c.bk && k.waves == c.waves && k.stages == c.stages && k.mode == c.mode)
            return &t[i];
    }
    return nullptr;
}

struct Fp8Workspace {
    size_t sorted, tile_expert, tile_rows, counts, meta, align_ws, xq, xs, a_buf, aq, as, y_buf, total;
    size_t cap, align_ws_bytes;
};
Fp8Workspace fp8_workspace(const ramp_shape &s, const ramp_config &c)
{
    Fp8Workspace w;
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
    w.align_ws_bytes = ramp_align_workspace_bytes(s.T, s.k, s.E);
    w.align_ws = take(w.align_ws_bytes);
    w.xq = take((size_t)s.T * s.H);
    w.xs = take((size_t)s.T * scale_stride(s.H));
    w.a_buf = take(w.cap * (size_t)s.I * 2);
    w.aq = take(w.cap * (size_t)s.I);
    w.as = take(w.cap * (size_t)scale_stride(s.I));
    w.y_buf = take((size_t)s.T * s.k * s.H * 4);
    w.total = off;
    return w;
}

int launch_quant_rows(const uint16_t *src, int rows, int K, uint8_t *codes, uint8_t *sb, const int32_t *n_rows_dev,
                      const int32_t *pred, int pred_value, hipStream_t st)
{
    if (rows <= 0) return RAMP_OK;
    const size_t groups = (size_t)rows * (K / kGroup);
    size_t blocks = (groups + 3) / 4;
    if (blocks > (size_t)kNumCU * 32) blocks = (size_t)kNumCU * 32;
    hipLaunchKernelGGL(quant_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, st, src, rows, K, codes, sb, scale_stride(K),
                       n_rows_dev, pred, pred_value);
    return check_launch("quant_rows_kernel");
}

}  // namespace
}  // namespace ramp

using namespace ramp;

extern "C" int ramp_fp8_num_configs(const ramp_shape *shape)
{
    if (!shape) {
        set_error("fp8_num_configs: NULL shape");
        return RAMP_EINVAL;
    }
    int n = 0, cnt = 0;
    const Fp8Kernel *t = fp8_kernels(&n);
    for (int i = 0; i < n; ++i) cnt += fp8_valid_for_shape(t[i], *shape) ? 1 : 0;
    return cnt;
}

extern "C" int ramp_fp8_get_config(const ramp_shape *shape, int idx, ramp_config *out)
{
    if (!shape || !out || idx < 0) {
        set_error("fp8_get_config: bad argument");
        return RAMP_EINVAL;
    }
    int n = 0, cnt = 0;
    const Fp8Kernel *t = fp8_kernels(&n);
    for (int i = 0; i < n; ++i) {
        if (!fp8_valid_for_shape(t[i], *shape)) continue;
        if (cnt++ == idx) {
            *out = t[i].cfg;
            return RAMP_OK;
        }
    }
    set_error("fp8_get_config: index %d out of range (%d valid)", idx, cnt);
    return RAMP_EINVAL;
}

extern "C" int ramp_fp8_config_wave_capacity(const ramp_config *cfg)
{
    const Fp8Kernel *k = cfg ? find_fp8(*cfg) : nullptr;
    if (!k) {
        set_error("fp8_config_wave_capacity: configuration not in the FP8 family");
        return RAMP_EUNSUPPORTED;
    }
    return kNumCU * k->waves_per_cu_limit;
}

extern "C" size_t ramp_fp8_pack_bytes(const ramp_shape *shape)
{
    if (!shape || shape->E <= 0 || shape->H <= 0 || shape->I <= 0 || shape->H % 128 || shape->I % 128) return 0;
    return fp8_layout(*shape).total_bytes;
}

extern "C" int ramp_fp8_pack_layout(const ramp_shape *shape, size_t offsets[6], int32_t strides[2])
{
    if (!shape || !offsets || !strides || shape->E <= 0 || shape->H <= 0 || shape->I <= 0 || shape->H % 128 || shape->I % 128) {
        set_error("fp8_pack_layout: bad argument");
        return RAMP_EINVAL;
    }
    const Fp8Layout L = fp8_layout(*shape);
    offsets[0] = L.w1_expert_bytes;
    offsets[1] = L.up_offset_bytes;
    offsets[2] = L.w2_base_bytes;
    offsets[3] = L.w2_expert_bytes;
    offsets[4] = L.scale_base;
    offsets[5] = L.scale_expert_bytes;
    strides[0] = L.stride1;
    strides[1] = L.stride2;
    return RAMP_OK;
}

extern "C" int ramp_fp8_pack_weights(const ramp_shape *shape, const void *W_gate, const void *W_up, const void *W_down,
                                     void *packed, void *stream)
{
    if (!shape || !W_gate || !W_up || !W_down || !packed) {
        set_error("fp8_pack: NULL argument");
        return RAMP_EINVAL;
    }
    const ramp_shape &s = *shape;
    if (s.E <= 0 || s.H <= 0 || s.I <= 0 || s.H % 128 || s.I % 128 || s.E > 65535) {
        set_error("fp8_pack: need 0 < E <= 65535 and H, I multiples of 128 (H=%d I=%d)", s.H, s.I);
        return RAMP_EUNSUPPORTED;
    }
    if (reinterpret_cast<uintptr_t>(packed) % 256) {
        set_error("fp8_pack: packed buffer must be 256-byte aligned");
        return RAMP_EINVAL;
    }
    const Fp8Layout L = fp8_layout(s);
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t *dst = static_cast<uint8_t *>(packed);
    uint8_t *sc = dst + L.scale_base;
    struct Part {
        const void *src;
        int K, F;
        size_t dst_off, dst_stride, sc_off;
        int stride;
    } parts[3] = {{W_gate, s.H, s.I, 0, L.w1_expert_bytes, L.scale_g, L.stride1},
                  {W_up, s.H, s.I, L.up_offset_bytes, L.w1_expert_bytes, L.scale_u, L.stride1},
                  {W_down, s.I, s.H, L.w2_base_bytes, L.w2_expert_bytes, L.scale_d, L.stride2}};
    for (const Part &p : parts) {
        const uint16_t *src = static_cast<const uint16_t *>(p.src);
        hipLaunchKernelGGL(block_scale_kernel, dim3(p.K / kGroup, p.F / kGroup, s.E), dim3(256), 0, st, src, p.K, p.F,
                           sc + p.sc_off, L.scale_expert_bytes, p.stride);
        if (int rc = check_launch("block_scale_kernel")) return rc;
        const size_t chunks = (size_t)s.E * p.K * p.F / 16;
        size_t blocks = (chunks + 255) / 256;
        if (blocks > (size_t)kNumCU * 64) blocks = (size_t)kNumCU * 64;
        hipLaunchKernelGGL(pack_fp8_kernel, dim3((unsigned)blocks), dim3(256), 0, st, src, dst + p.dst_off, s.E, p.K, p.F,
                           p.dst_stride, sc + p.sc_off, L.scale_expert_bytes, p.stride);
        if (int rc = check_launch("pack_fp8_kernel")) return rc;
    }
    return RAMP_OK;
}

extern "C" int ramp_fp8_quantize_rows(const void *src, int rows, int K, void *codes, void *scales, void *stream)
{
    if (!src || !codes || !scales || rows < 0 || K <= 0 || K % 128) {
        set_error("fp8_quantize_rows: bad argument (K must be a multiple of 128)");
        return RAMP_EINVAL;
    }
    return launch_quant_rows(static_cast<const uint16_t *>(src), rows, K, static_cast<uint8_t *>(codes),
                             static_cast<uint8_t *>(scales), nullptr, nullptr, 0, static_cast<hipStream_t>(stream));
}

extern "C" size_t ramp_fused_moe_fp8_workspace_bytes(const ramp_shape *shape, const ramp_config *cfg)
{
    if (!shape || !cfg || cfg->bm <= 0 || !moe_shape_ok(*shape)) return 0;
    return fp8_workspace(*shape, *cfg).total;
}

extern "C" int ramp_fused_moe_fp8(const ramp_shape *shape, const ramp_config *cfg, const void *X, const int32_t *topk_ids,
                                  const float *topk_w, const void *packed_fp8, void *out, void *ws, size_t ws_bytes,
                                  void *stream)
{
    if (!shape || !cfg) {
        set_error("fused_moe_fp8: NULL shape or config");
        return RAMP_EINVAL;
    }
    const ramp_shape &s = *shape;
    if (!moe_shape_ok(s)) {
        set_error("fused_moe_fp8: unsupported shape T=%d k=%d E=%d H=%d I=%d", s.T, s.k, s.E, s.H, s.I);
        return RAMP_EUNSUPPORTED;
    }
    const Fp8Kernel *k = find_fp8(*cfg);
    if (!k || !fp8_valid_for_shape(*k, s)) {
        set_error("fused_moe_fp8: configuration (bm=%d bn=%d bk=%d waves=%d stages=%d mode=%d) is not in the FP8 family of "
                  "this shape", cfg->bm, cfg->bn, cfg->bk, cfg->waves, cfg->stages, cfg->mode);
        return RAMP_EUNSUPPORTED;
    }
    if (s.T == 0) return RAMP_OK;
    if (!X || !topk_ids || !topk_w || !packed_fp8 || !out || !ws) {
        set_error("fused_moe_fp8: NULL buffer");
        return RAMP_EINVAL;
    }
    if (reinterpret_cast<uintptr_t>(ws) % 256 || reinterpret_cast<uintptr_t>(packed_fp8) % 256 ||
        reinterpret_cast<uintptr_t>(X) % 16 || reinterpret_cast<uintptr_t>(out) % 16) {
        set_error("fused_moe_fp8: misaligned buffer (ws/packed 256 B, X and out 16 B)");
        return RAMP_EINVAL;
    }
    const Fp8Workspace w = fp8_workspace(s, *cfg);
    if (ws_bytes < w.total) {
        set_error("fused_moe_fp8: workspace %zu < %zu bytes", ws_bytes, w.total);
        return RAMP_ENOSPC;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *base = static_cast<char *>(ws);
    int32_t *sorted = reinterpret_cast<int32_t *>(base + w.sorted);
    int32_t *tile_expert = reinterpret_cast<int32_t *>(base + w.tile_expert);
    int32_t *tile_rows = reinterpret_cast<int32_t *>(base + w.tile_rows);
    int32_t *counts = reinterpret_cast<int32_t *>(base + w.counts);
    int32_t *meta = reinterpret_cast<int32_t *>(base + w.meta);
    uint8_t *xq = reinterpret_cast<uint8_t *>(base + w.xq), *xs = reinterpret_cast<uint8_t *>(base + w.xs);
    uint16_t *a_buf = reinterpret_cast<uint16_t *>(base + w.a_buf);
    uint8_t *aq = reinterpret_cast<uint8_t *>(base + w.aq), *as = reinterpret_cast<uint8_t *>(base + w.as);
    float *y_buf = reinterpret_cast<float *>(base + w.y_buf);

    if (int rc = launch_align(topk_ids, s.T, s.k, s.E, cfg->bm, sorted, tile_expert, tile_rows, counts, meta, base + w.align_ws,
                              w.align_ws_bytes, st))
        return rc;
    if (int rc = launch_quant_rows(static_cast<const uint16_t *>(X), s.T, s.H, xq, xs, nullptr, nullptr, 0, st)) return rc;

    const Fp8Layout L = fp8_layout(s);
    const uint8_t *packed = static_cast<const uint8_t *>(packed_fp8);
    GemmArgs g = {};
    g.sorted = sorted;
    g.tile_expert = tile_expert;
    g.tile_rows = tile_rows;
    g.topk_magic = moe_topk_magic(s.k);
    g.meta = meta;
    g.topk_w = topk_w;
    g.a_out = a_buf;
    g.a_row_major = 1;
    g.y_out = y_buf;
    g.y_bf16 = moe_pair_rows_bf16(s) ? 1 : 0;
    g.P = s.T * s.k;
    g.topk = s.k;
    g.m_tiles_cap = (int)(w.cap / (size_t)cfg->bm);
    g.group_m_req = 0;

    Fp8Args f = {};
    // up-projection + SwiGLU
    f.act_q = xq;
    f.act_scale = xs;
    f.act_stride = L.stride1;
    f.wq = packed;
    f.expert_stride = L.w1_expert_bytes;
    f.up_offset = L.up_offset_bytes;
    f.wscale = packed + L.scale_base + L.scale_g;
    f.wscale_expert_stride = L.scale_expert_bytes;
    f.wscale_up_offset = L.scale_u - L.scale_g;
    f.w_stride = L.stride1;
    g.K = s.H;
    g.F = s.I;
    g.n_tiles = 2 * s.I / cfg->bn;
    k->launch(1, g, f, st);
    if (int rc = check_launch("moe_fp8_kernel<1>")) return rc;

    // the activation, per slot and 128 features; rows past the padded length of this call are skipped
    if (int rc = launch_quant_rows(a_buf, (int)w.cap, s.I, aq, as, meta, nullptr, 0, st)) return rc;

    // down-projection
    f.act_q = aq;
    f.act_scale = as;
    f.act_stride = L.stride2;
    f.wq = packed + L.w2_base_bytes;
    f.expert_stride = L.w2_expert_bytes;
    f.up_offset = 0;
    f.wscale = packed + L.scale_base + L.scale_d;
    f.wscale_up_offset = 0;
    f.w_stride = L.stride2;
    g.K = s.I;
    g.F = s.H;
    g.n_tiles = s.H / cfg->bn;
    k->launch(2, g, f, st);
    if (int rc = check_launch("moe_fp8_kernel<2>")) return rc;

    return launch_combine(y_buf, g.y_bf16, topk_ids, s.T, s.k, s.E, s.H, static_cast<uint16_t *>(out), st);
}
