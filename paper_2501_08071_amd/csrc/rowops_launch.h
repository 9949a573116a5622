// Internal: host-side launch interface of the row kernels (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>

struct RowopLaunch {
    int op;            // 0 softmax, 1 rmsnorm
    const void* x;
    const void* w;     // rmsnorm only
    void* y;
    long long n_rows;
    int n;             // row length
    float eps;
    int dtype;         // 0 binary16, 1 bfloat16
    void* stream;
};

constexpr int ROWOPS_MAX_REG_ROW = 16384;   // longest row kept in registers between its read and its write

// 1 = registers path, 2 = general path
inline int rowop_path_of(int n) { return (n % 8 == 0 && n <= ROWOPS_MAX_REG_ROW) ? 1 : 2; }

hipError_t rowop_launch(const RowopLaunch& a);
