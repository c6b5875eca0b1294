// Ping-pong variant of the LDS-staged expert projections for the large tiles (128 or 256 token rows, or
// 256 rows plus one or two 16-row tail blocks; 8 wavefronts): same tile decomposition and epilogues as
// moe_gemm_kernel, different main loop and different token staging.
//
// Main loop.  The 8 wavefronts form two groups of four, one wavefront of each group per SIMD.  A
// k-slice is handled in two phases separated by workgroup barriers: M (issue the LDS-direct loads of
// later slices, read every operand fragment of the current slice into registers) and C (its MFMAs,
// registers only).  Group 1 runs one barrier behind group 0, so while one group multiplies the other
// does its memory phase on the same SIMDs and the matrix pipe does not wait for LDS.
//
// Token blocks and wavefronts.  The 16-row token blocks of a tile are dealt to the WM wavefront rows round robin
// (block b belongs to row b % WM), so a ragged tile (the real rows come first, the sentinel padding after them)
// spreads its real blocks evenly over all wavefronts instead of leaving whole wavefront rows idle; the products
// and, in ragged tiles, the operand reads of all-padding blocks are skipped.
//
// Token staging in the up-projection.  The token rows are gathered (row = pair / k of X, 2*H bytes
// apart), so every row touched by a load instruction is another page for the address translation in
// the vector memory path, and that, not bytes, is what the gather costs: 16 rows x 64 B per
// instruction (one MFMA fragment) runs at a third of the rate of a contiguous 1 KB load.  Here a load
// instruction takes 8 rows x 128 B (64 k-values per row), which halves the row visits; the 128-byte row
// pieces land in LDS row-major in 1 KB blocks of 8 rows, with the 16-byte chunk index XOR-ed with
// (row/2)%8 on the global side so that the ds_read_b128 operand reads (16 rows x one chunk) spread
// over all banks.  One such token super-slice feeds 64/bk k-slices; weights keep one slice per load
// batch.  The down-projection reads the fragment-major activation written by the up-projection, where
// a token fragment is one contiguous 1 KB line, and stages it like the weights.
#pragma once

#include <type_traits>

#include "moe_gemm.h"

#ifndef RAMP_PP_XSPLIT
#define RAMP_PP_XSPLIT 1  // 0: a two-slice token batch is issued whole in its even slice (for comparisons)
#endif
#ifndef RAMP_PINGPONG_NX2
#define RAMP_PINGPONG_NX2 0  // 1: keep two token buffers everywhere (for comparisons)
#endif

namespace ramp {

template <int STAGE, int BM, int BN, int BK, int WM, int WN, int NSTAGE>
struct PingPongTraits {
    // The token blocks of a tile come in eights, dealt to the wavefront rows; a tile of bm = (8*n + t)*16 rows has t tail
    // blocks beyond them.  All wavefronts share a tail block, each multiplying it with part of its weight fragments.
    static constexpr int TAILB = (BM / 16) % 8;
    static constexpr int BMAIN = BM - 16 * TAILB;
    using TT = TileTraits<BMAIN, BN, BK, WM, WN, 2>;  // tile geometry only; the ring depths are defined here
    static constexpr bool ROWX = (STAGE == 1);           // gathered rows, 128-byte pieces
    static constexpr int XK = ROWX ? 64 : BK;            // k-values of one token load batch ("super-slice")
    static constexpr int XS = XK / BK;                   // k-slices fed by one super-slice
    static constexpr int W_BYTES_ = TileTraits<BMAIN, BN, BK, WM, WN, 2>::W_FRAGS * kFragElems * 2;
    static constexpr int X_BYTES_ = (BM * XK * 2 / 1024 + WM * WN - 1) / (WM * WN) * (WM * WN) * 1024;
    // token ring depth in super-slices: two-slice batches get a third buffer where LDS has room for it (a batch
    // then has three slice times to arrive instead of one)
    static constexpr int NX = (XS == 2) ? ((3 * X_BYTES_ + NSTAGE * W_BYTES_ <= kLdsBytesPerCU && !RAMP_PINGPONG_NX2) ? 3 : 2) : NSTAGE;
    static constexpr int X_BLOCKS = BM * XK * 2 / 1024;                           // 1 KB token load blocks per super-slice
    static constexpr int TSLOTS = (X_BLOCKS + TT::NWAVE - 1) / TT::NWAVE;         // token load instructions per wavefront per super-slice
    static constexpr int X_BYTES = TSLOTS * TT::NWAVE * 1024;                     // (the surplus slots of a tail tile load nothing)
    static constexpr int W_BYTES = TT::W_FRAGS * kFragElems * 2;
    static constexpr int WSLOTS = TT::W_FRAGS / TT::NWAVE;     // weight load instructions per wavefront per slice
    static constexpr int RING_BYTES = NX * X_BYTES + NSTAGE * W_BYTES;
    static constexpr int STG_BYTES = (STAGE == 2) ? 4096 * TT::NWAVE : 0;  // per-wavefront staging of bf16 output rows
    // A down-projection tile with tail blocks has no registers to spare for the destination pair and router weight of its
    // token rows through the whole tile: they wait in LDS instead (pairs and weights of up to 512 slots, two tiles deep).
    static constexpr bool SLOT_LDS = (STAGE == 2) && TAILB > 0;
    static constexpr int SLOT_BYTES = SLOT_LDS ? 2 * 4096 : 0;
    static constexpr int LDS_BYTES = RING_BYTES + STG_BYTES + SLOT_BYTES;
    static_assert(!SLOT_LDS || (BM <= 512 && BM % 4 == 0), "slot table: two 1 KB loads per array");
    static_assert(TT::NWAVE == 8, "ping-pong needs two groups of four wavefronts");
    static_assert(BK == 32 || BK == 64, "bk 32 or 64");
    static_assert(BM % 16 == 0 && TAILB <= 3, "whole token blocks, at most three tail blocks");
    static_assert(TAILB == 0 || (BK == 32 && WM == 2 && (STAGE == 1 ? TT::FB1 == 2 : TT::FB2 == 4)), "tail block: 256-wide tiles of two wavefront rows");
    static_assert(TT::W_FRAGS % TT::NWAVE == 0, "weight loads must split evenly");
    static_assert(NSTAGE >= 3 || XS == 1, "a two-slice token batch needs three weight stages");
    static_assert(LDS_BYTES <= kLdsBytesPerCU, "tile does not fit in LDS");
};

// Read-only table entry at a wave-uniform address that no launch in flight writes.
__device__ __forceinline__ int32_t load_uniform_i32(const int32_t *p)
{
    return *(const __attribute__((address_space(4))) int32_t *)(p);
}

// Wait until at most n vector-memory operations of this wavefront are outstanding (n wave-uniform).
__device__ __forceinline__ void wait_vmcnt_upto(int n)
{
    switch (n) {
    case 0: wait_vmcnt<0>(); break;
    case 1: wait_vmcnt<1>(); break;
    case 2: wait_vmcnt<2>(); break;
    case 3: wait_vmcnt<3>(); break;
    case 4: wait_vmcnt<4>(); break;
    case 5: wait_vmcnt<5>(); break;
    case 6: wait_vmcnt<6>(); break;
    case 7: wait_vmcnt<7>(); break;
    case 8: wait_vmcnt<8>(); break;
    case 9: wait_vmcnt<9>(); break;
    case 10: wait_vmcnt<10>(); break;
    case 11: wait_vmcnt<11>(); break;
    case 12: wait_vmcnt<12>(); break;
    case 13: wait_vmcnt<13>(); break;
    case 14: wait_vmcnt<14>(); break;
    case 15: wait_vmcnt<15>(); break;
    default: wait_vmcnt<16>(); break;  // n >= 16: waiting for more than asked is always safe
    }
}

template <int STAGE, int BM, int BN, int BK, int WM, int WN, int NSTAGE>
__global__ __launch_bounds__(512, 1) void moe_pingpong_kernel(GemmArgs a)
{
    using PT = PingPongTraits<STAGE, BM, BN, BK, WM, WN, NSTAGE>;
    using TT = typename PT::TT;
    constexpr int TAILB = PT::TAILB, BMAIN = PT::BMAIN;
    constexpr int KS = TT::KS, NB = TT::NB, NWAVE = TT::NWAVE;
    constexpr int FB = (STAGE == 1) ? TT::FB1 : TT::FB2;
    constexpr int NACC = (STAGE == 1) ? 2 * FB : FB;
    constexpr int FEAT_PER_TILE = (STAGE == 1) ? BN / 2 : BN;
    constexpr int XS = PT::XS, NX = PT::NX, TSLOTS = PT::TSLOTS, WSLOTS = PT::WSLOTS;

    if (launch_deselected(a.pred, a.pred_value)) return;
    __shared__ __attribute__((aligned(1024))) char lds[PT::LDS_BYTES];
    char *const lds_x = lds;
    char *const lds_w = lds + NX * PT::X_BYTES;
    char *const lds_stage = lds + PT::RING_BYTES;
    char *const lds_slot = lds + PT::RING_BYTES + PT::STG_BYTES;
    constexpr bool SLOT_LDS = PT::SLOT_LDS;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int group = wave >> 2;
    const int K = a.K, KST = K / 32, KT = K / BK;
    const int r16 = lane & 15, q = lane >> 4;
    const int m_tiles = a.meta[1];

    // Tiles of this workgroup: ids blockIdx.x, + gridDim.x, ... (gridDim.x is a multiple of 8, so every tile of a
    // workgroup maps to its own XCD); ids past the real M-tiles of this call are skipped.
    auto next_tile = [&](int id, int &n_tile, int &m_tile) __attribute__((always_inline)) -> int {
        for (; id < a.total_tiles; id += (int)gridDim.x) {
            tile_of_id_rotated(a, id, n_tile, m_tile);
            // wave-uniform by construction; saying so lets the per-tile table reads below be scalar loads, which do not
            // count on vmcnt (a vector load would have to be waited for in order, behind every LDS-direct load in flight)
            n_tile = __builtin_amdgcn_readfirstlane(n_tile);
            m_tile = __builtin_amdgcn_readfirstlane(m_tile);
            if (m_tile < m_tiles) return id;
        }
        return -1;
    };

    // ---- global element offsets of this lane's loads for k-slice 0 of a tile ----
    auto tile_offsets = [&](int n_tile, int m_tile, uint32_t *xo, uint32_t *wo, const uint16_t *&wexp, int &rows) __attribute__((always_inline)) {
        // the two per-tile table entries (written by the align launch before this one) through the constant address
        // space: m_tile is wave-uniform, so these become scalar loads, which do not count on vmcnt
        rows = load_uniform_i32(a.tile_rows + m_tile);  // real rows of the tile (they come first, the sentinel padding after them)
        const int e = load_uniform_i32(a.tile_expert + m_tile);
        wexp = a.wpacked + (size_t)e * a.expert_stride;
        const int f0 = n_tile * FEAT_PER_TILE;
        if (PT::ROWX) {
            // only the index loads here; token_offsets() turns them into offsets when the first load of the tile is
            // issued, most of a tile later: nothing waits for these loads while the LDS-direct loads are in flight
#pragma unroll
            for (int t = 0; t < TSLOTS; ++t) {
                const int tr = (wave + t * NWAVE) * 8 + (lane >> 3);
                // (the surplus load slots of a tail tile never fetch rows, see token_loads: any slot of the tile will do)
                xo[t] = (uint32_t)a.sorted[m_tile * BM + (PT::X_BLOCKS % NWAVE == 0 || tr < BM ? tr : BM - 1)];
            }
        } else {
#pragma unroll
            for (int t = 0; t < TSLOTS; ++t) {
                const int blk = wave + t * NWAVE;
                const int nb = blk / KS, ks = blk % KS;
                xo[t] = act_elem((uint32_t)(m_tile * BM + nb * 16 + r16), (uint32_t)(ks * 32 + q * 8), (uint32_t)KST);
            }
        }
#pragma unroll
        for (int s = 0; s < WSLOTS; ++s) {
            const int widx = wave + s * NWAVE;
            const int rb = widx / KS, ks = widx % KS;
            uint32_t base;
            if (STAGE == 1) {
                const int half = TT::RB / 2;
                base = (rb < half) ? (uint32_t)(f0 / 16 + rb) * (uint32_t)KST * kFragElems
                                   : (uint32_t)a.up_offset + (uint32_t)(f0 / 16 + rb - half) * (uint32_t)KST * kFragElems;
            } else {
                base = (uint32_t)(f0 / 16 + rb) * (uint32_t)KST * kFragElems;
            }
            wo[s] = base + (uint32_t)ks * kFragElems + (uint32_t)lane * 8;
        }
    };
    // pair indices (as loaded by tile_offsets) -> element offsets of the token rows (token = pair / k by multiplication)
    auto token_offsets = [&](uint32_t *xo) __attribute__((always_inline)) {
        if (!PT::ROWX) return;
#pragma unroll
        for (int t = 0; t < TSLOTS; ++t) {
            const int tr = (wave + t * NWAVE) * 8 + (lane >> 3);  // 8 rows per 1 KB block, 8 lanes (128 B) per row
            const uint32_t p = (xo[t] < (uint32_t)a.P) ? xo[t] : 0u;
            const uint32_t row = (uint32_t)(((unsigned long long)p * a.topk_magic) >> 40);
            xo[t] = row * (uint32_t)K + (uint32_t)(((lane & 7) ^ ((tr >> 1) & 7)) * 8);
        }
    };
    constexpr uint32_t XSTEP = PT::ROWX ? (uint32_t)PT::XK : (uint32_t)(KS * kFragElems);
    constexpr uint32_t WSTEP = (uint32_t)(KS * kFragElems);

    // load stream state: offsets of the next slice to issue (they run ahead of the tile being multiplied)
    uint32_t xoff[TSLOTS], woff[WSLOTS];
    const uint16_t *wexp_x = nullptr, *wexp_w = nullptr;  // expert weights of the tile the weight loads belong to
    uint32_t xoff_n[TSLOTS], woff_n[WSLOTS];               // first slice of the following tile
    const uint16_t *wexp_n = nullptr;
    // Token loads of all-padding row blocks are degenerate (a ragged last tile of an expert then costs little more
    // than its weights): only the first txv of this wavefront's TSLOTS token loads per batch fetch rows.
    int txv = TSLOTS, txv_n = TSLOTS;
    auto token_loads = [&](int rows) __attribute__((always_inline)) {
        const int blocks = PT::ROWX ? (rows + 7) / 8 : (rows + 15) / 16 * KS;  // 1 KB load blocks that hold real rows
        int v = (blocks - wave + NWAVE - 1) / NWAVE;
        return v < 0 ? 0 : (v > TSLOTS ? TSLOTS : v);
    };

    // Slot table (SLOT_LDS).  The last token load of wavefronts 4..7 is a surplus slot of the load round (past the blocks
    // of the tile, it never fetches rows).  In the first slice of a tile these four loads copy the tile's part of the two
    // per-slot tables into LDS instead, 1 KB each (16-byte pieces past the tile re-read its last piece): they ride in the
    // load stream at no cost in loads or waits, and land with the slice, a whole tile before the epilogue reads them.
    // slot_tile: tile whose first slice is issued next, or -1; slot_half: the half of the table it gets (the other half
    // belongs to the tile being multiplied).
    static_assert(!SLOT_LDS || (XS == 1 && (TSLOTS - 1) * NWAVE + 4 >= PT::X_BLOCKS), "slot table: wavefronts 4..7 need a surplus load slot");
    int slot_tile = -1, slot_half = 0;
    auto issue_x = [&](int xbuf, int t0 = 0, int t1 = PT::TSLOTS) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < TSLOTS; ++t) {
            if (t < t0 || t >= t1) continue;
            // a block of nothing but padding rows re-reads one 16-byte piece instead (one cache line request, and
            // the load count that the vmcnt waits rely on stays the same)
            const uint32_t off = (t < txv) ? xoff[t] : 0u;
            if (SLOT_LDS && t == TSLOTS - 1 && wave >= 4 && slot_tile >= 0) {
                const int arr = wave & 1, part = (wave >> 1) & 1;
                const int c0 = part * 64 + lane;
                const int c = c0 < BM / 4 ? c0 : BM / 4 - 1;
                const void *src = arr ? (const void *)(a.slot_w + (size_t)slot_tile * BM + c * 4)
                                      : (const void *)(a.sorted + (size_t)slot_tile * BM + c * 4);
                load_to_lds_16B(src, lds_slot + slot_half * 4096 + arr * 2048 + part * 1024);
            } else {
                load_to_lds_16B(a.act + off, lds_x + xbuf * PT::X_BYTES + (wave + t * NWAVE) * 1024);
            }
            xoff[t] += XSTEP;
        }
        if (SLOT_LDS) slot_tile = -1;
    };
    auto issue_w = [&](int wbuf) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < WSLOTS; ++s) {
            load_to_lds_16B(wexp_w + woff[s], lds_w + wbuf * PT::W_BYTES + (wave + s * NWAVE) * 1024);
            woff[s] += WSTEP;
        }
    };

    floatx4 acc[NACC][NB];
    // tail blocks (TAILB): wavefront row wm multiplies each with two of its weight fragments: (gate, up) of feature
    // block wm in the up-projection, feature blocks 2*wm and 2*wm + 1 in the down-projection
    constexpr int NT = TAILB ? TAILB : 1;
    floatx4 acc_t[2 * NT];
    int tail_n = 0;  // tail blocks of the current tile with real rows
    auto zero_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NACC; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
        if (TAILB) {
#pragma unroll
            for (int t = 0; t < 2 * NT; ++t) acc_t[t] = floatx4{0.f, 0.f, 0.f, 0.f};
        }
    };

    // ---- LDS read offsets of this lane's operand fragments ----
    // tokens, row-major batch: row (wm*NB+nb)*16 + r16 sits in block row/8 at (row%8)*128, chunk c at (c ^ (row/2)%8)*16
    const int xrow_off = wm * 2048 + (r16 >> 3) * 1024 + (r16 & 7) * 128;  // token block nb of this wavefront is block nb*WM + wm
    const int xsw = (r16 >> 1) & 7;
    const int xtail_off = NB * WM * 2048 + (r16 >> 3) * 1024 + (r16 & 7) * 128;
    bf16x8 fx[KS][NB], fw[KS][NACC], fx_t[KS][NT];
    int nb_valid = 0;  // token blocks of this wavefront with at least one real row in the current tile
    // kk0: 32-wide k-step of the slice inside its token batch; partial_c: skip the token fragments of all-padding blocks
    auto read_all = [&](int kk0, int xbuf, int wbuf, auto partial_c) __attribute__((always_inline)) {
        constexpr bool PARTIAL = decltype(partial_c)::value;
        const char *xs = lds_x + xbuf * PT::X_BYTES;
        const char *ws = lds_w + wbuf * PT::W_BYTES + lane * 16;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
            for (int i = 0; i < NACC; ++i) {
                int rb;
                if (STAGE == 1) rb = (i < FB) ? (wn * FB + i) : (TT::RB / 2 + wn * FB + (i - FB));
                else rb = wn * FB + i;
                fw[ks][i] = *reinterpret_cast<const bf16x8 *>(ws + (rb * KS + ks) * 1024);
            }
            if (PT::ROWX) {
                const int kk = kk0 + ks;
                const int coff = ((kk * 4 + q) ^ xsw) * 16;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    if (!PARTIAL || nb < nb_valid)
                        fx[ks][nb] = *reinterpret_cast<const bf16x8 *>(xs + xrow_off + nb * (WM * 2048) + coff);
#pragma unroll
                for (int t = 0; t < TAILB; ++t) fx_t[ks][t] = *reinterpret_cast<const bf16x8 *>(xs + xtail_off + t * 2048 + coff);
            } else {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    if (!PARTIAL || nb < nb_valid)
                        fx[ks][nb] = *reinterpret_cast<const bf16x8 *>(xs + ((nb * WM + wm) * KS + ks) * 1024 + lane * 16);
#pragma unroll
                for (int t = 0; t < TAILB; ++t) fx_t[ks][t] = *reinterpret_cast<const bf16x8 *>(xs + ((NB * WM + t) * KS + ks) * 1024 + lane * 16);
            }
        }
    };
    // FULL: every token block of the wavefront is real (no branches between the MFMAs); otherwise the products of
    // all-padding blocks are skipped.  The operand reads stay unconditional: branches between them cost more than
    // the reads they save.
    auto mfma_all = [&](auto mode_c) __attribute__((always_inline)) {
        constexpr bool FULL = decltype(mode_c)::value == 1;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                if (FULL || nb < nb_valid) {
#pragma unroll
                    for (int i = 0; i < NACC; ++i)
                        acc[i][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw[ks][i], fx[ks][nb], acc[i][nb], 0, 0, 0);
                }
            }
        if (TAILB && tail_n > 0) {
            constexpr int I0 = (STAGE == 1) ? 0 : 0, I1 = (STAGE == 1) ? FB : 1, STEP = (STAGE == 1) ? 1 : 2;
#pragma unroll
            for (int t = 0; t < TAILB; ++t) {
                if (t > 0 && t >= tail_n) continue;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    if (wm == 0) {
                        acc_t[2 * t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw[ks][I0], fx_t[ks][t], acc_t[2 * t], 0, 0, 0);
                        acc_t[2 * t + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw[ks][I1], fx_t[ks][t], acc_t[2 * t + 1], 0, 0, 0);
                    } else {
                        acc_t[2 * t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw[ks][I0 + STEP], fx_t[ks][t], acc_t[2 * t], 0, 0, 0);
                        acc_t[2 * t + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw[ks][I1 + STEP], fx_t[ks][t], acc_t[2 * t + 1], 0, 0, 0);
                    }
                }
            }
        }
    };
    auto phase_barrier = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };
    auto blocks_valid = [&](int rows) __attribute__((always_inline)) {  // token blocks of this wavefront (wm, wm + WM, ...) with at least one real row
        const int v = ((rows + 15) / 16 - wm + WM - 1) / WM;
        return v < 0 ? 0 : (v > NB ? NB : v);
    };

    auto tail_blocks = [&](int rows) __attribute__((always_inline)) {  // tail blocks with at least one real row
        const int v = (rows - BMAIN + 15) / 16;
        return !TAILB || v < 0 ? 0 : (v > TAILB ? TAILB : v);
    };

    int n_tile, m_tile;
    int id = next_tile((int)blockIdx.x, n_tile, m_tile);
    if (id < 0) return;
    int rows_cur = 0, rows_next = 0;
    tile_offsets(n_tile, m_tile, xoff, woff, wexp_w, rows_cur);
    token_offsets(xoff);
    nb_valid = blocks_valid(rows_cur);
    tail_n = tail_blocks(rows_cur);
    txv = token_loads(rows_cur);
    zero_acc();

    // The k-slices of all tiles of this workgroup form one stream: the loads run NSTAGE-1 slices ahead of the
    // multiplication and simply continue with the first slices of the next tile while the current one finishes,
    // so only the very first tile waits for a cold pipeline.  Loads are issued, and counted by vmcnt, in this
    // order: prologue X(0) W(0) [X(1)] W(1) ..., then in the M phase of slice kt: the token batch whose buffer
    // became free (if any), then weight slice kt+NSTAGE-1.
    if (SLOT_LDS) slot_tile = m_tile;
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s) {
        if (XS == 1 || s == 0 || (s == 1 && NX == 3)) issue_x(s);
        issue_w(s);
    }
    // token batch 0 and weight slice 0 have landed once only the loads issued after W(0) are outstanding
    wait_vmcnt<(NSTAGE - 2) * (XS == 1 ? TSLOTS + WSLOTS : WSLOTS) + (XS == 2 && NX == 3 ? TSLOTS : 0)>();
    phase_barrier();
    if (group == 1) phase_barrier();  // stagger
    // Loads that may stay in flight at the end of the M phase of slice kt (two-slice token batches).  Weight slice
    // kt+1 has to be there; younger than it are the weight slices kt+2 .. kt+NSTAGE-1 and the token batches issued
    // with them (one per even slice, before the weight slice of that phase).  With two token buffers the batch for
    // slice kt+1 of an odd kt was issued one phase ago and has to be there too: only what followed it may remain.
    // With three token buffers a batch has slack enough to be issued in two halves, one in each slice of the pair before:
    // the wavefronts of a group issue their loads at the same time into one address path (a 1 KB load every 16 clocks, and
    // a wavefront whose load queues there issues nothing else), so the M phase of the even slices, which carried the whole
    // batch, was the longer one.  Each slice then issues half a batch and a weight slice; behind weight slice kt+1 are the
    // loads of the NSTAGE-2 slices after it.
    constexpr bool XSPLIT = RAMP_PP_XSPLIT && XS == 2 && NX == 3 && TSLOTS % 2 == 0;
    constexpr int WAIT_EVEN = XSPLIT ? (NSTAGE - 2) * (WSLOTS + TSLOTS / 2)
                                     : (NSTAGE - 2) * WSLOTS + (NX == 3 ? (NSTAGE - 3) / 2 + 1 : 1) * TSLOTS;
    constexpr int WAIT_ODD = XSPLIT ? (NSTAGE - 2) * (WSLOTS + TSLOTS / 2)
                             : (NX == 3) ? (NSTAGE - 2) * WSLOTS + (NSTAGE >= 4 ? (NSTAGE - 4) / 2 + 1 : 0) * TSLOTS
                                         : (NSTAGE - 2 < 2 ? NSTAGE - 2 : 2) * WSLOTS;

    int wbuf_cur = 0, wbuf_issue = NSTAGE - 1;  // weight ring: buffer of the slice being read / being loaded
    int xbat_cur = 0;                           // token ring: batch being read (counts over all tiles)
    int slot_par = 0;                           // slot table: half used by the current tile
    while (true) {
        // following tile of this workgroup (its first slices are loaded while this one finishes)
        int n_next = 0, m_next = 0;
        const int id_next = next_tile(id + (int)gridDim.x, n_next, m_next);
        const bool has_next = id_next >= 0;
        if (has_next) {
            tile_offsets(n_next, m_next, xoff_n, woff_n, wexp_n, rows_next);
            txv_n = token_loads(rows_next);
        }
        // stage 2: destination pair and router weight of this lane's token rows
        int out_pair[NB];
        float out_wgt[NB];
        // All index and weight loads are issued together and unconditionally (the padding slots of a tile hold the
        // sentinel P; the weights are read by slot, from the copy the align step made, not through the pair index), and
        // nothing uses them before the epilogue: no round trip on the way into the tile.  One load, one wait, one
        // dependent load per token block would be sixteen round trips, each of them also draining the LDS-direct loads
        // in flight (vmcnt counts in order).  Tail-block tiles have no registers for them: there the two tables came into LDS
        // with the first token slice of the tile (issue_x) and the epilogue reads them back.
        int tail_pair[NT];
        float tail_wgt[NT];
        if (STAGE == 2 && !SLOT_LDS) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) out_pair[nb] = a.sorted[m_tile * BM + (nb * WM + wm) * 16 + r16];
#pragma unroll
            for (int t = 0; t < TAILB; ++t) tail_pair[t] = a.sorted[m_tile * BM + BMAIN + t * 16 + r16];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) out_wgt[nb] = a.slot_w[m_tile * BM + (nb * WM + wm) * 16 + r16];
#pragma unroll
            for (int t = 0; t < TAILB; ++t) tail_wgt[t] = a.slot_w[m_tile * BM + BMAIN + t * 16 + r16];
        }

        // mode_c: 1 = every token block of the wavefront is real, 0 = some are, 2 = none (a ragged tile that ends
        // in the other wavefront row): such a wavefront issues its loads and keeps the barriers but neither reads
        // operands nor multiplies, which leaves the LDS bandwidth of the tile to the wavefronts that do
        auto slice = [&](int kt, auto steady_c, auto mode_c, auto par_c) __attribute__((always_inline)) {
            constexpr bool STEADY = decltype(steady_c)::value;
            constexpr int MODE = decltype(mode_c)::value;
            // ---- M phase: both groups have read slice kt-1 (its buffers are free).  Operand reads first, then the
            // loads: the reads are what the barrier waits for, the loads only have to be issued.
            constexpr int par = decltype(par_c)::value;  // position of the slice inside its token batch (kt & 1 for two-slice batches)
            // (the down-projection has no registers to spare for the conditional form of the reads)
            if (MODE != 2) read_all(par * KS, xbat_cur % NX, wbuf_cur, std::integral_constant<bool, MODE == 0 && STAGE == 1>{});
            // the load stream crosses into the next tile NSTAGE-1 slices (one token batch) before this one ends
            if (kt == KT - NSTAGE + 1) {
#pragma unroll
                for (int s = 0; s < WSLOTS; ++s) woff[s] = woff_n[s];
                wexp_w = wexp_n;
            }
            if (kt == KT - (NX - 1) * XS) {
#pragma unroll
                for (int t = 0; t < TSLOTS; ++t) {
                    xoff[t] = xoff_n[t];
                    // keeps the arithmetic (and with it the wait for the index loads) here instead of in front of the slice loop
                    if (PT::ROWX) asm volatile("" : "+v"(xoff[t]));
                }
                token_offsets(xoff);
                txv = txv_n;
                if (SLOT_LDS && has_next) {
                    slot_tile = m_next;
                    slot_half = slot_par ^ 1;
                }
            }
            bool x_issued = false;
            if (XSPLIT) {
                // (in the odd slice the batch of the pair is still "current": the same buffer, the other half)
                if (STEADY || kt - par + (NX - 1) * XS < KT) issue_x((xbat_cur + NX - 1) % NX, par * (TSLOTS / 2), (par + 1) * (TSLOTS / 2));
            } else if (par == 0 && (STEADY || kt + (NX - 1) * XS < KT)) {
                issue_x((xbat_cur + NX - 1) % NX);  // into the buffer freed last
                x_issued = true;
            }
            if (STEADY || kt + NSTAGE - 1 < KT) issue_w(wbuf_issue);
            // this wavefront's part of the next slice has to be in LDS before the barrier after which the other group reads it
            if (STEADY) {
                if (XS == 1) wait_vmcnt<(NSTAGE - 2) * (TSLOTS + WSLOTS)>();
                // (the very first slice of a workgroup has the whole batches of the prologue behind it, not half batches:
                // counting only the weight slices is right there and costs the first slice of later tiles next to nothing)
                else if (XSPLIT && kt == 0) wait_vmcnt<(NSTAGE - 2) * WSLOTS>();
                else if (par == 0) wait_vmcnt<WAIT_EVEN>();
                else wait_vmcnt<WAIT_ODD>();
            } else if (XSPLIT) {
                if (kt + 1 < KT) wait_vmcnt<0>();  // the last slices of the last tile: whatever is in flight is needed next
            } else if (kt + 1 < KT) {
                const int later = min(NSTAGE - 2, KT - 2 - kt);  // younger weight slices that may stay in flight
                if (XS == 1) wait_vmcnt_upto(later * (TSLOTS + WSLOTS));
                else if (par == 0) wait_vmcnt_upto(later * WSLOTS + (x_issued ? TSLOTS : 0));
                else wait_vmcnt_upto((later < 2 ? later : 2) * WSLOTS);
            }
            __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): fragments in registers, buffers no longer read
            phase_barrier();
            // ---- C phase
            if (MODE != 2) mfma_all(mode_c);
            phase_barrier();
            wbuf_cur = (wbuf_cur + 1 == NSTAGE) ? 0 : wbuf_cur + 1;
            wbuf_issue = (wbuf_issue + 1 == NSTAGE) ? 0 : wbuf_issue + 1;
            if (par == XS - 1) ++xbat_cur;
        };
        // a tile that is followed by another keeps the load stream full to its end; the last tile of the
        // workgroup drains it (conditions evaluated for its last NSTAGE-1 slices)
        using True = std::integral_constant<bool, true>;
        using False = std::integral_constant<bool, false>;
        using Some = std::integral_constant<int, 0>;
        using Full = std::integral_constant<int, 1>;
        using None = std::integral_constant<int, 2>;
        int kt = 0;
        // (two-slice token batches: slices run in pairs, so the steady part ends on an even slice; K is a multiple of 64 there)
        const int kt_steady = (has_next ? KT : KT - (NSTAGE - 1 > (NX - 1) * XS ? NSTAGE - 1 : (NX - 1) * XS)) & ~(XS - 1);
        using P0 = std::integral_constant<int, 0>;
        using P1 = std::integral_constant<int, 1>;
        auto run = [&](int kt_end, auto steady_c, auto mode_c) __attribute__((always_inline)) {
            if (XS == 2) {
                for (; kt < kt_end; kt += 2) {
                    slice(kt, steady_c, mode_c, P0{});
                    slice(kt + 1, steady_c, mode_c, P1{});
                }
            } else {
                for (; kt < kt_end; ++kt) slice(kt, steady_c, mode_c, P0{});
            }
        };
        // In the up-projection a wavefront with more than half of its token blocks real takes the branch-free form on
        // all of them (the products of its padding blocks are computed and never stored): the conditional operand reads
        // and per-block branches of the ragged form cost more than they save until half of the products go away
        // (same-box A/B: tiles of 240 of 272 rows, up-projection 286 -> 265 us).  The down-projection's ragged form reads
        // unconditionally and only skips products; there the exact rule stays.
        if (STAGE == 1 ? 2 * nb_valid > NB : nb_valid == NB) {
            run(kt_steady, True{}, Full{});
            run(KT, False{}, Some{});
        } else if (nb_valid > 0) {
            run(kt_steady, True{}, Some{});
            run(KT, False{}, Some{});
        } else {
            run(kt_steady, True{}, None{});
            run(KT, False{}, None{});
        }

        // ---- epilogue: lane holds features fblock*16 + 4*q + {0..3} of token r16.  It runs while the other group
        // is in a C phase; the stores are not waited for here.
        const int f0 = n_tile * FEAT_PER_TILE;
        if (SLOT_LDS) {
            const int *sp = reinterpret_cast<const int *>(lds_slot + slot_par * 4096);
            const float *sw = reinterpret_cast<const float *>(lds_slot + slot_par * 4096 + 2048);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                out_pair[nb] = sp[(nb * WM + wm) * 16 + r16];
                out_wgt[nb] = sw[(nb * WM + wm) * 16 + r16];
            }
#pragma unroll
            for (int t = 0; t < TAILB; ++t) {
                tail_pair[t] = sp[BMAIN + t * 16 + r16];
                tail_wgt[t] = sw[BMAIN + t * 16 + r16];
            }
            slot_par ^= 1;
        }
        if (STAGE == 2 && a.y_bf16) {
            // bf16 per-pair rows leave through LDS: a lane holds 16 consecutive features of one token, but a store
            // instruction should cover whole 128-byte lines.  Per chunk of two token blocks the wavefront writes its
            // 32 x 64 weighted results into its own 4 KB staging area (row-major, 16-byte chunk index XOR-ed with
            // (row/2)%8 so writes and reads spread over all banks) and reads them back 8 rows x 128 B at a time.
            static_assert(STAGE != 2 || (FB == 4 && NB % 2 == 0), "staged epilogue: 64 features per wavefront, token blocks in pairs");
            char *stg = lds_stage + wave * 4096;
            uint16_t *ybase = reinterpret_cast<uint16_t *>(a.y_out) + f0 + wn * (FB * 16) + (lane & 7) * 8;
#pragma unroll
            for (int c2 = 0; c2 < NB / 2; ++c2) {
                if (2 * c2 >= nb_valid) continue;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int nb = 2 * c2 + h;
                    const int row = h * 16 + r16;
#pragma unroll
                    for (int half = 0; half < 2; ++half) {  // row blocks (0,1) and (2,3): 8 features each pair
                        float w8[8];
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            w8[c] = out_wgt[nb] * acc[2 * half][nb][c];
                            w8[4 + c] = out_wgt[nb] * acc[2 * half + 1][nb][c];
                        }
                        store_bf16x8(reinterpret_cast<uint16_t *>(stg + row * 128 + (((2 * q + half) ^ ((row >> 1) & 7)) * 16)), w8);
                    }
                }
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const int row = p * 8 + (lane >> 3);
                    const int nb = 2 * c2 + (p >> 1);
                    const int pair = __shfl(out_pair[nb], row & 15);
                    const uint4 v = *reinterpret_cast<const uint4 *>(stg + row * 128 + (((lane & 7) ^ ((row >> 1) & 7)) * 16));
                    if (pair < a.P) *reinterpret_cast<uint4 *>(ybase + (size_t)pair * a.F) = v;
                }
            }
        } else {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            if (nb >= nb_valid) continue;
            const int slot = m_tile * BM + (nb * WM + wm) * 16 + r16;
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
#pragma unroll
        for (int t = 0; t < TAILB; ++t) {
            if (t >= tail_n) continue;
            if (STAGE == 1)
                store_token_row<1, 1>(a, &acc_t[2 * t], &acc_t[2 * t + 1], 1, (size_t)(m_tile * BM + BMAIN + t * 16 + r16), f0 / 16 + wn * FB + wm, q, 1.0f);
            else if (tail_pair[t] < a.P)
                store_token_row<2, 2>(a, &acc_t[2 * t], &acc_t[2 * t], 1, (size_t)tail_pair[t] * a.F, f0 / 16 + wn * FB + 2 * wm, q, tail_wgt[t]);
        }
        if (!has_next) break;
        id = id_next;
        n_tile = n_next;
        m_tile = m_next;
        rows_cur = rows_next;
        nb_valid = blocks_valid(rows_cur);
        tail_n = tail_blocks(rows_cur);
        zero_acc();
    }
    if (group == 0) phase_barrier();  // both groups execute the same number of barriers
}

// LDS stages of the down-projection, which stages tokens and weights per slice and keeps 32 KB for its output rows:
// at most 4, and 3 for a tile with tail blocks (its token buffers are padded to whole load rounds, and it keeps 8 KB for
// the per-slot tables of two tiles).
template <int BM, int WM, int NSTAGE>
constexpr int pingpong_down_stages()
{
    return ((BM / 16) % 8) ? 3 : (NSTAGE > 4 ? 4 : NSTAGE);
}

template <int BM, int BN, int BK, int WM, int WN, int NSTAGE>
void launch_pingpong(int stage, const GemmArgs &a, hipStream_t stream)
{
    if (a.n_tiles <= 0 || a.m_tiles_cap <= 0) return;
    GemmArgs g = a;
    g.total_tiles = (int)xcd_grid(g);
    // persistent: one workgroup per compute unit walks its share of the tiles (the count is a multiple of 8)
    const dim3 grid(g.total_tiles < kNumCU ? g.total_tiles : kNumCU), block(512);
    // the down-projection stages tokens and weights per slice and needs LDS for its output rows: at most 4 stages
    constexpr int NS2 = pingpong_down_stages<BM, WM, NSTAGE>();
    if (stage == 1)
        hipLaunchKernelGGL((moe_pingpong_kernel<1, BM, BN, BK, WM, WN, NSTAGE>), grid, block, 0, stream, g);
    else
        hipLaunchKernelGGL((moe_pingpong_kernel<2, BM, BN, BK, WM, WN, NS2>), grid, block, 0, stream, g);
}

template <int BM, int BN, int BK, int WM, int WN, int NSTAGE>
KernelInfo make_pingpong_info(int group_bits = 0)
{
    using TT = typename PingPongTraits<1, BM, BN, BK, WM, WN, NSTAGE>::TT;
    constexpr int l1 = PingPongTraits<1, BM, BN, BK, WM, WN, NSTAGE>::LDS_BYTES;
    constexpr int l2 = PingPongTraits<2, BM, BN, BK, WM, WN, pingpong_down_stages<BM, WM, NSTAGE>()>::LDS_BYTES;
    KernelInfo ki = {};
    ki.cfg = ramp_config{BM, BN, BK, WM * WN, NSTAGE, (WM - 1) | kModePingPong | (group_bits << kModeGroupShift)};
    ki.wm = WM;
    ki.wn = WN;
    ki.lds_bytes = l1 > l2 ? l1 : l2;
    ki.acc_regs = TT::ACC_REGS + 8 * PingPongTraits<1, BM, BN, BK, WM, WN, NSTAGE>::TAILB;
    ki.launch = &launch_pingpong<BM, BN, BK, WM, WN, NSTAGE>;
    ki.kernel_fn[0] = reinterpret_cast<const void *>(&moe_pingpong_kernel<1, BM, BN, BK, WM, WN, NSTAGE>);
    ki.kernel_fn[1] = reinterpret_cast<const void *>(&moe_pingpong_kernel<2, BM, BN, BK, WM, WN, pingpong_down_stages<BM, WM, NSTAGE>()>);
    ki.block_threads = 512;
    ki.family = "moe_pingpong_kernel";
    const int targs[8] = {1, BM, BN, BK, WM, WN, NSTAGE, 0};
    for (int i = 0; i < 8; ++i) ki.targs[i] = targs[i];
    ki.n_targs = 7;
    return ki;
}

}  // namespace ramp
