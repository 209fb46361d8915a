// The compiled variant family: workgroup tile (BM, BN, BK) and wave tile (WM, WN).
// One line per variant; the same list instantiates the SGEMM and the convolution kernels, fills
// the tables polydl_get_variant() reports, and is the candidate set of the reuse-model picker.
#pragma once

#define POLYDL_TILE_FAMILY(X) \
    X(64, 64, 16, 32, 32)     \
    X(64, 128, 16, 32, 64)    \
    X(128, 64, 16, 64, 32)    \
    X(128, 128, 16, 64, 64)   \
    X(128, 128, 8, 64, 64)    \
    X(128, 256, 16, 64, 128)  \
    X(256, 128, 16, 128, 64)

// Tiles of the row-patch convolution kernel (BM output channels x BN pixels; wave tile WM x WN).
// The third entry is unused there: the stage depth is CB*R*S with CB a run-time parameter.
#define POLYDL_PATCH_FAMILY(X) \
    X(64, 64, 0, 32, 32)       \
    X(64, 128, 0, 64, 32)      \
    X(64, 128, 0, 64, 64)      \
    X(64, 256, 0, 64, 64)      \
    X(128, 64, 0, 64, 32)      \
    X(128, 128, 0, 64, 64)

// Tiles of the bfloat16 row-patch kernel (eight-channel units, v_mfma_f32_32x32x16_bf16).
#define POLYDL_PATCH_BF16_FAMILY(X) \
    X(64, 64, 0, 32, 32)            \
    X(64, 128, 0, 64, 32)           \
    X(64, 256, 0, 64, 64)           \
    X(128, 64, 0, 64, 32)           \
    X(128, 128, 0, 64, 64)          \
    X(128, 256, 0, 64, 64)
