// One-time weight re-layout, thread-local error text, and the calibration copy kernel.
//
// Boundary layout: W_gate, W_up [E,H,I] and W_down [E,I,H] (x W convention, Sec. 2.2).
// Packed layout: per expert, W^T cut into fragments of 16 output rows x 32 k-values, each
// stored as the 64-lane register image of one v_mfma_f32_16x16x32_bf16 operand
// (row r = lane % 16, k = 8*(lane / 16) + j  ->  element lane*8 + j; the feature in row r of row
// block rb is packed_row_feature(rb, r), an interleave inside groups of 128 features).  Fragments of one
// 16-row block are contiguous along k, so a wavefront streaming a row block reads one
// contiguous range and every load is a full 1 KB line.
//   [E][gate: I/16 row blocks][H/32 k-steps][512]  then  [up: same]      (up-projection)
//   [E][H/16 row blocks][I/32 k-steps][512]                               (down-projection)
#include <stdarg.h>

#include "ramp_internal.h"

namespace ramp {

static thread_local char g_error[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof g_error, fmt, ap);
    va_end(ap);
}

PackedLayout packed_layout(const ramp_shape &s)
{
    PackedLayout L;
    L.up_offset_elems = (size_t)s.I * s.H;
    L.w1_expert_elems = 2 * L.up_offset_elems;
    L.w2_expert_elems = (size_t)s.H * s.I;
    L.w2_base_elems = (size_t)s.E * L.w1_expert_elems;
    L.total_bytes = align_up(((size_t)s.E * (L.w1_expert_elems + L.w2_expert_elems)) * 2, 256);
    return L;
}

namespace {

// src: [E][K][F] (F contiguous).  dst: [E][F/16][K/32][512] (+ dst_expert_stride between experts).
// One lane writes one 16-byte chunk (8 consecutive k of one output row).
__global__ __launch_bounds__(256) void pack_kernel(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst, int E,
                                                   int K, int F, size_t dst_expert_stride)
{
    const size_t chunks_per_expert = (size_t)K * F / 8;
    const size_t total = chunks_per_expert * E;
    for (size_t c = (size_t)blockIdx.x * blockDim.x + threadIdx.x; c < total; c += (size_t)gridDim.x * blockDim.x) {
        const int e = (int)(c / chunks_per_expert);
        const size_t ce = c % chunks_per_expert;
        const int lane = (int)(ce % 64);
        const size_t frag = ce / 64;
        const int kst = K / 32;
        const int ks = (int)(frag % kst);
        const int rb = (int)(frag / kst);
        const int f = packed_row_feature(rb, lane % 16);
        const int k0 = ks * 32 + (lane / 16) * 8;
        const uint16_t *s = src + (size_t)e * K * F + (size_t)k0 * F + f;
        union {
            uint16_t h[8];
            uint4 v;
        } u;
#pragma unroll
        for (int j = 0; j < 8; ++j) u.h[j] = s[(size_t)j * F];
        *reinterpret_cast<uint4 *>(dst + (size_t)e * dst_expert_stride + frag * kFragElems + (size_t)lane * 8) = u.v;
    }
}

__global__ __launch_bounds__(256) void copy_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

// Register-resident MFMA loop: the matrix-pipe rate this chip sustains on the operand values it is given, with no
// memory traffic at all.  Two wavefronts per SIMD, each with the 4 x 8 accumulator blocks of the 256x256 ping-pong
// tile (32 independent v_mfma_f32_16x16x32_bf16 per round).  The clock, and with it the rate, depends on the
// operand bits (the chip is power limited), which is why the operands come from the caller.
typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef float probe_floatx4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(512, 1) void mfma_rate_kernel(const uint16_t *__restrict__ operands, int rounds,
                                                           float *__restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    probe_bf16x8 fw[4], fx[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) fw[i] = *reinterpret_cast<const probe_bf16x8 *>(operands + (i * 64 + lane) * 8);
#pragma unroll
    for (int j = 0; j < 8; ++j) fx[j] = *reinterpret_cast<const probe_bf16x8 *>(operands + ((4 + j) * 64 + lane) * 8);
    probe_floatx4 acc[4][8];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = probe_floatx4{0.f, 0.f, 0.f, 0.f};
    for (int r = 0; r < rounds; ++r) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw[i], fx[j], acc[i][j], 0, 0, 0);
    }
    probe_floatx4 s = probe_floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) s += acc[i][j];
    reinterpret_cast<probe_floatx4 *>(sink)[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

}  // namespace
}  // namespace ramp

extern "C" const char *ramp_last_error(void) { return ramp::g_error; }

extern "C" size_t ramp_pack_bytes(const ramp_shape *shape)
{
    if (!shape || shape->E <= 0 || shape->H <= 0 || shape->I <= 0) return 0;
    return ramp::packed_layout(*shape).total_bytes;
}

extern "C" int ramp_pack_weights(const ramp_shape *shape, const void *W_gate, const void *W_up, const void *W_down,
                                 void *packed, void *stream)
{
    using namespace ramp;
    if (!shape || !W_gate || !W_up || !W_down || !packed) {
        set_error("pack: NULL argument");
        return RAMP_EINVAL;
    }
    const ramp_shape &s = *shape;
    if (s.E <= 0 || s.H <= 0 || s.I <= 0 || s.H % 128 || s.I % 128) {
        set_error("pack: need E>0 and H, I multiples of 128 (H=%d I=%d)", s.H, s.I);
        return RAMP_EUNSUPPORTED;
    }
    if (reinterpret_cast<uintptr_t>(packed) % 256) {
        set_error("pack: packed buffer must be 256-byte aligned");
        return RAMP_EINVAL;
    }
    const PackedLayout L = packed_layout(s);
    uint16_t *dst = static_cast<uint16_t *>(packed);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int grid = kNumCU * 8;
    hipLaunchKernelGGL(pack_kernel, dim3(grid), dim3(256), 0, st, static_cast<const uint16_t *>(W_gate), dst, s.E, s.H,
                       s.I, L.w1_expert_elems);
    hipLaunchKernelGGL(pack_kernel, dim3(grid), dim3(256), 0, st, static_cast<const uint16_t *>(W_up),
                       dst + L.up_offset_elems, s.E, s.H, s.I, L.w1_expert_elems);
    hipLaunchKernelGGL(pack_kernel, dim3(grid), dim3(256), 0, st, static_cast<const uint16_t *>(W_down),
                       dst + L.w2_base_elems, s.E, s.I, s.H, L.w2_expert_elems);
    return check_launch("pack_kernel");
}

extern "C" int ramp_copy_bytes(void *dst, const void *src, size_t bytes, void *stream)
{
    using namespace ramp;
    if (!dst || !src || bytes % 16 || reinterpret_cast<uintptr_t>(dst) % 16 || reinterpret_cast<uintptr_t>(src) % 16) {
        set_error("copy: need non-NULL 16-byte aligned buffers and a multiple of 16 bytes");
        return RAMP_EINVAL;
    }
    if (bytes == 0) return RAMP_OK;
    hipLaunchKernelGGL(copy_kernel, dim3(kNumCU * 8), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<uint4 *>(dst), static_cast<const uint4 *>(src), bytes / 16);
    return check_launch("copy_kernel");
}

extern "C" int ramp_mfma_rate_probe(const void *operands, int rounds, void *sink, void *stream, double *flops)
{
    using namespace ramp;
    if (!operands || !sink || rounds <= 0 || reinterpret_cast<uintptr_t>(operands) % 16 ||
        reinterpret_cast<uintptr_t>(sink) % 16) {
        set_error("mfma_rate_probe: bad argument");
        return RAMP_EINVAL;
    }
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(kNumCU), dim3(512), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint16_t *>(operands), rounds, static_cast<float *>(sink));
    if (flops) *flops = (double)kNumCU * 8.0 * (double)rounds * 32.0 * (2.0 * 16 * 16 * 32);
    return check_launch("mfma_rate_kernel");
}
