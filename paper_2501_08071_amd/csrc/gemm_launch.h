// Internal: host-side launch interface of the GEMM + LeakyReLU kernels (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>

struct GemmLaunch {
    const void* a;
    const void* b;
    void* c;
    int batch, M, N, K;
    float slope;
    int dtype;     // 0 binary16, 1 bfloat16
    void* stream;
};

// 1: 256 x 256 tiles, 2: 128 x 128, 3: 64 x 64, 5: 32 x 32 with K split over the wavefronts of a workgroup (all on
// the matrix cores), 4: plain kernel.  The largest tile that still gives three quarters of the 256 compute units
// a workgroup; a problem that fits the chip in one round of 32 x 32 tiles and has a K worth splitting takes those.
#ifndef GEMM_SK_TILES
#define GEMM_SK_TILES 256
#endif
inline int gemm_path_of(int batch, int M, int N, int K) {
    if (K == 0 || K % 32 != 0 || N % 8 != 0 || K > (1 << 22) || N > (1 << 22)) return 4;   // 32-bit offsets inside a tile's rows
    auto tiles = [&](int t) { return (long long)batch * ((M + t - 1) / t) * ((N + t - 1) / t); };
    if (tiles(32) <= GEMM_SK_TILES && K >= 256) return 5;
    return tiles(256) >= 192 ? 1 : tiles(128) >= 192 ? 2 : 3;
}

hipError_t gemm_launch(const GemmLaunch& a);
