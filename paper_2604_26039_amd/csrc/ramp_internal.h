// Internal declarations shared by the library's translation units (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "ramp.h"

namespace ramp {

// Thread-local message for ramp_last_error().
void set_error(const char *fmt, ...);

inline int check_launch(const char *what)
{
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) {
        set_error("%s: %s", what, hipGetErrorString(err));
        return RAMP_EHIP;
    }
    return RAMP_OK;
}

constexpr int kNumCU = 256;           // MI355X compute units
constexpr int kLdsBytesPerCU = 160 * 1024;
constexpr int kWave = 64;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- align ----
constexpr int kAlignThreads = 1024;   // one workgroup = 16 wavefronts
constexpr int kAlignChunk = 1024;     // pairs per workgroup in the multi-workgroup path
constexpr int kAlignSingleMaxP = 2048; // up to this many pairs one workgroup does everything
constexpr int kAlignMaxE = 1024;

// Optional second output of the scatter: slot_w[s] = topk_w[sorted[s]] for the slots that hold a pair (the others are
// left as they are), so that a kernel can read the router weight of a slot without first waiting for its pair index.
struct AlignSlotWeights {
    const float *topk_w;
    float *slot_w;
};

int launch_align(const int32_t *ids, int T, int k, int E, int bm, int32_t *sorted, int32_t *tile_expert,
                 int32_t *tile_rows, int32_t *counts, int32_t *meta, void *ws, size_t ws_bytes, hipStream_t stream,
                 const int32_t *pred = nullptr, int pred_value = 0, AlignSlotWeights slot_weights = {nullptr, nullptr});

// ---- packed weights ----
// One fragment = 16 weight rows x 32 k-values = 512 bf16 = 1 KB, stored in the lane order
// of the A operand of v_mfma_f32_16x16x32_bf16: element (row r, k = 8*q + j) at (q*16 + r)*8 + j.
constexpr int kFragElems = 512;
// Which output feature sits in row r of packed row block rb.  Inside every group of 4 row blocks
// (64 features) the rows are interleaved so that, after the MFMA, lane group q of a wavefront holds
// 4 consecutive features per row block it owns, consecutive row blocks continuing the run: a lane
// that owns all 4 row blocks of a group stores 16 consecutive features (32 B of bf16) per token
// instead of 4 separate 8-byte pieces.  Pure relabelling: the packing kernel and the epilogues agree.
constexpr int kPermBlocks = 4;
__host__ __device__ inline int packed_row_feature(int rb, int r)
{
    return (rb / kPermBlocks) * (16 * kPermBlocks) + (r >> 2) * (4 * kPermBlocks) + (rb % kPermBlocks) * 4 + (r & 3);
}
// Element offset of (slot, feature) in the intermediate activation A = SiLU(G)*U.  A is private to the
// library, so the up-projection writes it in the order the down-projection consumes it: blocks of 16
// slots x 32 features stored as the 64-lane register image of one MFMA token operand (lane =
// 16*(feature/8 % 4) + slot % 16, 8 features per lane), k-steps of a slot block contiguous.  A k-step of
// 16 slots is then one contiguous 1 KB line, like a weight fragment.  kst = I / 32.
__host__ __device__ inline uint32_t act_elem(uint32_t slot, uint32_t feature, uint32_t kst)
{
    return ((slot >> 4) * kst + (feature >> 5)) * (uint32_t)kFragElems + ((((feature >> 3) & 3u) << 4) + (slot & 15u)) * 8u +
           (feature & 7u);
}
struct PackedLayout {
    size_t w1_expert_elems;  // gate then up: 2 * I * H
    size_t up_offset_elems;  // I * H
    size_t w2_expert_elems;  // H * I
    size_t w2_base_elems;    // E * 2 * I * H
    size_t total_bytes;
};
PackedLayout packed_layout(const ramp_shape &s);

// ---- projections ----
struct GemmArgs {
    const uint16_t *act;        // stage 1: X [T,H]; stage 2: A [cap,I]
    const uint16_t *wpacked;    // base of this stage's packed weights
    size_t expert_stride;       // elements between experts
    size_t up_offset;           // stage 1: offset of the up rows inside an expert
    const int32_t *sorted;      // [cap]
    const int32_t *tile_expert; // [cap/bm]
    const int32_t *tile_rows;   // [cap/bm] real rows per tile
    unsigned long long topk_magic;  // ceil(2^40 / k): pair / k == (pair * topk_magic) >> 40 for pair < 2^30
    const int32_t *meta;        // [4]
    const float *topk_w;        // stage 2: [P]
    const float *slot_w;        // stage 2, ping-pong kernels: router weight of every sorted slot that holds a pair [cap]
    uint16_t *a_out;            // stage 1: A [cap,I]
    float *y_out;               // stage 2: Y [P,H] (fp32, or bf16 in the same buffer when y_bf16 != 0)
    int y_bf16;                 // large batches keep the per-pair rows in bf16 to halve their HBM traffic
    int K;                      // reduction length (H or I)
    int F;                      // output features (I or H)
    int P;                      // pairs = T*k (the sentinel)
    int topk;                   // k
    int n_tiles;                // feature tiles of this stage
    int m_tiles_cap;            // launched M-tiles (upper bound)
    int group_m_req;            // GROUP_M of the configuration (mode bits 12-15): M-tiles per XCD block, 0 = automatic
    int group_m, group_n;       // M-tiles x N-tiles per XCD block of the workgroup->tile map (set by the launcher)
    int total_tiles;            // persistent kernels: tile ids to walk (set by the launcher)
    int a_row_major;            // stage 1: A is written row-major [slot, I] instead of fragment-major (FP8 path)
    const int32_t *pred;        // device-side predicate: the launch does nothing unless *pred == pred_value (NULL: always runs)
    int pred_value;
};
// True when a predicated launch is not the one selected on the device.
__device__ __forceinline__ bool launch_deselected(const int32_t *pred, int pred_value)
{
    return pred != nullptr && *pred != pred_value;
}

// ramp_config.mode: bits 0-7 = WM-1 (token split of the wavefront grid), then the kernel family
constexpr int kModeStream = 0x100;    // weight-streaming kernel (moe_stream.h); bits 0-7 = WK instead
constexpr int kModePipe = 0x200;      // LDS-staged kernel with the register-pipelined main loop (moe_gemm.h)
constexpr int kModePingPong = 0x400;  // persistent ping-pong kernel (moe_pingpong.h)
// GROUP_M (Sec. 4.1, Eq. 4), XCD-aware: bits 12-15 = v > 0 makes every XCD take blocks of 2^v M-tiles x (32 >> v)
// N-tiles, so that the M-tiles of a block share the weight slices of its few N-tiles in that XCD's L2; 0 = a block
// spans all N-tiles (the token rows of its M-tiles stay in L2 instead).
constexpr int kModeDecode = 0x2000;   // with kModeStream: calls of at most 64 pairs run the two-launch form (moe_decode.h)
constexpr int kModeFp8 = 0x10000;     // W8A8 FP8 family (fp8.hip), listed by ramp_fp8_get_config
constexpr int kModeGroupShift = 12;
constexpr int kModeGroupMask = 0xF << kModeGroupShift;
inline int group_m_of_mode(int mode) { const int v = (mode & kModeGroupMask) >> kModeGroupShift; return v ? (1 << v) : 0; }

// Block shape of the XCD-aware workgroup -> tile map of one launch: every XCD takes blocks of group_m M-tiles x
// group_n N-tiles, the 8 XCDs 8 * group_m M-tiles per hand-out round.  group_m_req > 0: the GROUP_M mode of the
// configuration (group_n = the largest divisor of n_tiles up to 32 / group_m).  Default: a block spans all N-tiles, so
// the token rows of its few M-tiles (group_m * bm * K * 2 bytes) stay in the 4 MB L2 across the walk over N while the
// 8 XCDs work on neighbouring M-tiles, i.e. mostly the same expert, and share its weights through the memory-side cache.
inline void xcd_block_shape(int n_tiles, int group_m_req, int *group_m, int *group_n)
{
    if (group_m_req > 0) {
        int gn = 32 / group_m_req;
        if (gn < 1) gn = 1;
        if (gn > n_tiles) gn = n_tiles;
        while (n_tiles % gn) --gn;
        *group_m = group_m_req;
        *group_n = gn;
    } else {
        int gm = 32 / n_tiles;
        if (gm < 1) gm = 1;
        if (gm > 8) gm = 8;
        *group_m = gm;
        *group_n = n_tiles;
    }
}

struct DecodeArgs;
struct DecodeDownArgs;
struct KernelInfo {
    ramp_config cfg;
    int wm, wn;                 // wavefront grid inside the workgroup (tokens x features)
    int lds_bytes;
    int acc_regs;               // fp32 accumulators per lane (stage 1, the larger one)
    void (*launch)(int stage, const GemmArgs &, hipStream_t);
    // decode-sized calls (kModeDecode): align + up-projection in one launch; NULL for every other configuration
    void (*launch_decode_up)(const GemmArgs &, const DecodeArgs &, hipStream_t);
    const void *kernel_fn[2];   // the two projection kernels (stage 1, stage 2), for occupancy queries
    int block_threads;
    const char *family;         // kernel template name and the template arguments of the stage-1 instantiation:
    int targs[8];               // the key into the compiler's per-kernel resource table (kernel_resources.inc)
    int n_targs;
};

// What the compiler reported for one kernel instantiation when the library was built (registers, LDS,
// wavefronts per SIMD that fit); generated by the build into kernel_resources.inc.
struct KernelResources {
    const char *family;
    int n_targs;
    int targs[8];
    int vgprs, agprs, lds_bytes, waves_per_simd;
};
const KernelResources *find_resources(const char *family, const int *targs, int n_targs);
int num_kernels();
const KernelInfo &kernel_info(int i);
const KernelInfo *find_kernel(const ramp_config &cfg);
bool config_valid_for_shape(const KernelInfo &ki, const ramp_shape &s);
bool config_in_pool(const KernelInfo &ki, const ramp_shape &s);
int occupancy_estimate(const KernelInfo &ki);

// sel != NULL: the launch leaves `out` untouched unless 0 <= *sel < n_cand (device-selected layer) and bit *sel of
// skip_mask is clear (a candidate whose own launches write `out`).
// Two-launch form for decode-sized calls (moe_decode.h, instantiated in stream_group2.hip)
struct DecodeArgs {
    const int32_t *ids;      // [T*k]
    int E, bm, cap;
    int32_t *sorted, *tile_expert, *tile_rows, *counts, *meta;  // align result, written by workgroup 0
};
struct DecodeDownArgs {
    const uint16_t *act;       // A [P, I] bf16, row-major, one row per pair
    const uint16_t *wpacked;   // packed down-projection weights
    size_t expert_stride;      // elements between experts
    const int32_t *ids;        // [T, k]
    const float *topk_w;       // [T, k]
    uint16_t *out;             // [T, H] bf16
    int T, k, E, H, I;
    const int32_t *pred;
    int pred_value;
};
constexpr int kDecodeMaxPairs = 64;
void launch_decode_down_any(const DecodeDownArgs &d, hipStream_t stream);

// shape limits shared by the fused entry points (fused.hip)
bool moe_shape_ok(const ramp_shape &s);
bool moe_pair_rows_bf16(const ramp_shape &s);      // per-pair rows kept in bf16 (large batches) instead of fp32
unsigned long long moe_topk_magic(int k);

int launch_combine(const float *Y, int y_bf16, const int32_t *ids, int T, int k, int E, int H, uint16_t *out,
                   hipStream_t stream, const int32_t *sel = nullptr, int n_cand = 0, unsigned skip_mask = 0);

}  // namespace ramp
