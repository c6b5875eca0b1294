// The polymorphic tile family (paper Sec. 4.3 "Configuration diversity"), one line per
// instantiation: X(bm, bn, bk, WM, WN) with WM x WN wavefronts per workgroup.
// Split in groups only so that the groups compile in parallel.
#pragma once

// decode-sized token blocks: one MFMA column block, many small workgroups per compute unit
#define RAMP_CONFIG_GROUP0(X) \
    X(4, 64, 128, 1, 2)       \
    X(8, 64, 128, 1, 2)       \
    X(16, 32, 128, 1, 1)      \
    X(16, 64, 128, 1, 2)      \
    X(16, 64, 256, 1, 2)      \
    X(16, 128, 128, 1, 4)     \
    X(16, 128, 64, 1, 4)      \
    X(16, 256, 64, 1, 4)

#define RAMP_CONFIG_GROUP1(X) \
    X(32, 64, 128, 1, 2)      \
    X(32, 128, 64, 1, 4)      \
    X(32, 128, 128, 1, 4)     \
    X(32, 256, 64, 1, 4)      \
    X(64, 128, 64, 2, 2)      \
    X(64, 128, 64, 1, 4)

#define RAMP_CONFIG_GROUP2(X) \
    X(64, 256, 64, 2, 2)      \
    X(64, 256, 64, 1, 4)      \
    X(128, 128, 64, 2, 2)     \
    X(128, 256, 64, 2, 2)

// prefill-sized token blocks: large register tiles, one workgroup per compute unit
#define RAMP_CONFIG_GROUP3(X) \
    X(128, 256, 64, 2, 4)     \
    X(256, 256, 64, 2, 2)     \
    X(256, 256, 64, 2, 4)     \
    X(256, 128, 64, 4, 1)
