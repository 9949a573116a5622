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

// 1: 128 x 128 tiles, 2: 64 x 64 tiles (both on the matrix cores), 3: plain kernel
inline int gemm_path_of(int batch, int M, int N, int K) {
    if (K == 0 || K % 32 != 0 || N % 8 != 0 || K > (1 << 22) || N > (1 << 22)) return 3;   // 32-bit offsets inside a tile's rows
    const long long big = (long long)batch * ((M + 127) / 128) * ((N + 127) / 128);
    return big >= 192 ? 1 : 2;   // fewer large tiles than three quarters of the compute units: smaller tiles
}

hipError_t gemm_launch(const GemmLaunch& a);
