// The polymorphic tile family (paper Sec. 4.3 "Configuration diversity"), one line per
// instantiation, with WM x WN wavefronts per workgroup.
// Split in groups only so that the groups compile in parallel.
#pragma once

// LDS-staged family (moe_gemm.h): X(bm, bn, bk, WM, WN, NSTAGE, LOOP); LOOP 0 = one barrier per slice,
// 1 = register-pipelined (explicit double buffering of the operand fragments), 2 = ping-pong (two
// groups of four wavefronts alternate memory and MFMA phases).
#define RAMP_CONFIG_GROUP0(X) \
    X(32, 128, 64, 1, 4, 3, 0)   \
    X(32, 256, 64, 1, 4, 2, 0)   \
    X(64, 128, 64, 2, 2, 3, 0)   \
    X(64, 256, 64, 2, 2, 2, 0)

#define RAMP_CONFIG_GROUP1(X) \
    X(64, 256, 64, 2, 4, 3, 0)   \
    X(128, 128, 64, 2, 2, 3, 0)  \
    X(128, 128, 64, 2, 4, 3, 0)  \
    X(128, 256, 64, 2, 4, 3, 0)

#define RAMP_CONFIG_GROUP2(X) \
    X(128, 256, 64, 2, 4, 2, 0)  \
    X(128, 256, 32, 2, 4, 4, 0)  \
    X(256, 128, 64, 4, 2, 3, 0)  \
    X(256, 128, 64, 4, 2, 2, 0)

// prefill-sized token blocks: large register tiles, one workgroup per compute unit
#define RAMP_CONFIG_GROUP3(X) \
    X(256, 256, 64, 2, 4, 2, 0)  \
    X(256, 256, 32, 2, 4, 4, 0)  \
    X(256, 256, 32, 2, 4, 3, 0)  \
    X(256, 256, 64, 2, 2, 2, 0) \
    X(256, 256, 64, 2, 2, 2, 1)  \
    X(128, 256, 64, 2, 2, 3, 1)  \
    X(128, 128, 64, 2, 2, 3, 1)

#define RAMP_CONFIG_GROUP4(X) \
    X(256, 256, 64, 2, 4, 2, 1)  \
    X(128, 256, 64, 2, 4, 3, 1)  \
    X(128, 256, 64, 2, 4, 2, 1)  \
    X(256, 128, 64, 4, 2, 3, 1)

#define RAMP_CONFIG_GROUP5(X) \
    X(64, 256, 64, 2, 4, 3, 1)   \
    X(128, 128, 64, 2, 4, 3, 1)  \
    X(64, 128, 64, 2, 2, 3, 1)   \
    X(32, 128, 64, 1, 4, 3, 1)

// two independent 4-wavefront workgroups per compute unit (72 KB of LDS each)
#define RAMP_CONFIG_GROUP6(X) \
    X(128, 256, 32, 2, 2, 3, 0) \
    X(256, 128, 32, 2, 2, 3, 0) \
    X(128, 256, 32, 1, 4, 3, 0) \
    X(128, 128, 32, 2, 2, 4, 0) \
    X(128, 128, 32, 2, 2, 3, 0) \
    X(64, 256, 32, 1, 4, 3, 0)

// Ping-pong family (moe_pingpong.h): X(bm, bn, bk, WM, WN, NSTAGE), always 8 wavefronts.
#define RAMP_CONFIG_GROUP7(X) \
    X(256, 256, 32, 2, 4, 4) \
    X(256, 256, 32, 2, 4, 3) \
    X(128, 256, 32, 2, 4, 4) \
    X(128, 256, 32, 2, 4, 3) \
    X(256, 128, 32, 4, 2, 4) \
    X(272, 256, 32, 2, 4, 4) \
    X(288, 256, 32, 2, 4, 4)

// Weight-streaming family (moe_stream.h): X(bm, FBW, WF, WK, U) ->
// bn = WF*FBW*16 weight rows per tile, WF*WK wavefronts, K split WK ways inside the workgroup,
// U k-steps per load batch.
#define RAMP_STREAM_GROUP0(X) \
    X(4, 2, 1, 8, 2)          \
    X(8, 2, 1, 8, 2)          \
    X(16, 2, 1, 8, 2)         \
    X(16, 2, 1, 4, 2)         \
    X(16, 2, 2, 4, 2)         \
    X(16, 2, 4, 2, 2)         \
    X(16, 2, 4, 1, 4)         \
    X(16, 4, 2, 2, 2)         \
    X(16, 4, 4, 1, 2)

#define RAMP_STREAM_GROUP1(X) \
    X(32, 2, 1, 8, 2)         \
    X(32, 2, 2, 4, 2)         \
    X(32, 2, 4, 1, 2)         \
    X(32, 4, 2, 2, 2)         \
    X(32, 4, 4, 1, 2)         \
    X(64, 2, 2, 4, 1)         \
    X(64, 4, 4, 1, 1)

// deeper load batches (U = 4): more bytes in flight per wavefront for the smallest batches
#define RAMP_STREAM_GROUP2(X) \
    X(16, 2, 2, 4, 4)         \
    X(16, 2, 2, 2, 4)

// Stream configurations that also have the two-launch form for calls of at most 64 pairs (moe_decode.h):
// X(bm, FBW, WF, WK, U) as above; listed as separate configurations (mode bit 0x2000).
#define RAMP_DECODE_GROUP(X) \
    X(8, 2, 1, 8, 2)         \
    X(16, 2, 1, 8, 2)        \
    X(16, 2, 2, 4, 2)        \
    X(32, 2, 1, 8, 2)        \
    X(32, 2, 2, 4, 2)        \
    X(16, 2, 2, 4, 4)        \
    X(16, 2, 1, 8, 4)
