// Row softmax and RMS normalisation for gfx950: the paper's two memory-bound kernels (Table 2).
//
// Both are bound by HBM: every element is read once and written once, 4 bytes of traffic per element
// and a handful of fp32 operations.  So the whole design is about the memory side:
//   * a row stays in registers between its read and its write (rows of up to 16384 elements whose
//     length is a multiple of 8): one pass over HBM, not two or three;
//   * every lane moves 16 bytes per instruction and neighbouring lanes neighbouring addresses, so a
//     wavefront's load or store is 1 KiB of whole 128-byte lines;
//   * short rows (rmsnorm over a head dimension of 64 is 128 bytes) share a wavefront, TPR lanes per
//     row, so that the instruction stays 1 KiB wide; long rows take a whole workgroup;
//   * reductions run across the TPR lanes with cross-lane moves, across the four wavefronts of a
//     workgroup through 32 bytes of LDS.
// Rows of any other length go through a general path that reads the row two (rmsnorm) or three
// (softmax) times with 2-byte accesses.
#include <hip/hip_runtime.h>
#include <cstdint>

#include "rowops_launch.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr float LOG2E = 1.4426950408889634f;

// row groups per step (all loads first): rows within a wavefront / rows that take a workgroup with 1 or 2 chunks
#ifndef ROWOPS_U_SHORT
#define ROWOPS_U_SHORT 4
#endif
#ifndef ROWOPS_U_LONG
#define ROWOPS_U_LONG 2
#endif

template <int DT>
__device__ __forceinline__ float widen(uint16_t b) {
    if (DT == 0) return (float)__builtin_bit_cast(_Float16, b);
    return __builtin_bit_cast(float, (uint32_t)b << 16);
}
// round to nearest even into the 16-bit type (finite values; binary16 overflows to infinity)
template <int DT>
__device__ __forceinline__ uint16_t narrow(float f) {
    if (DT == 0) return __builtin_bit_cast(uint16_t, (_Float16)f);
    const uint32_t u = __builtin_bit_cast(uint32_t, f);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
template <int DT>
__device__ __forceinline__ void widen8(const u32x4& p, float (&f)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = widen<DT>((uint16_t)(p[i] & 0xFFFFu));
        f[2 * i + 1] = widen<DT>((uint16_t)(p[i] >> 16));
    }
}
template <int DT>
__device__ __forceinline__ u32x4 narrow8(const float (&f)[8]) {
    u32x4 p;
#pragma unroll
    for (int i = 0; i < 4; ++i) p[i] = (uint32_t)narrow<DT>(f[2 * i]) | ((uint32_t)narrow<DT>(f[2 * i + 1]) << 16);
    return p;
}

struct Max {
    static __device__ __forceinline__ float op(float a, float b) { return a > b ? a : b; }
};
struct Sum {
    static __device__ __forceinline__ float op(float a, float b) { return a + b; }
};

// Reduction over the TPR threads that share a row (TPR <= 64: lanes of one wavefront; TPR == 256: the
// whole workgroup, `red` holds one float per wavefront and row), of U independent rows at once.  Every
// thread gets the results.
template <class R, int TPR, int U>
__device__ __forceinline__ void reduce_rows(float (&v)[U], float (*red)[4]) {
    constexpr int W = TPR < 64 ? TPR : 64;
#pragma unroll
    for (int off = W / 2; off >= 1; off >>= 1)
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = R::op(v[u], __shfl_xor(v[u], off, 64));
    if constexpr (TPR == 256) {
        if ((threadIdx.x & 63) == 0) {
#pragma unroll
            for (int u = 0; u < U; ++u) red[u][threadIdx.x >> 6] = v[u];
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = R::op(R::op(red[u][0], red[u][1]), R::op(red[u][2], red[u][3]));
    }
}

// Registers path.  OP 0: softmax, 1: rmsnorm.  TPR threads share a row, each holds CH chunks of 8
// elements: chunk c of thread t covers elements 8 (c TPR + t) .. +7, so the TPR threads of a row read
// 16 TPR consecutive bytes per instruction.  256 / TPR rows per workgroup at a time, and U such groups
// per step, all their loads issued before the first is used: the bytes in flight are what hides the
// latency of HBM.
template <int DT, int OP, int TPR, int CH, int U>
__global__ __launch_bounds__(256) void rowop_reg_kernel(const uint16_t* x, const uint16_t* __restrict__ w,
                                                       uint16_t* y, long long n_rows, int n, float eps) {
    constexpr int RPW = 256 / TPR;
    __shared__ float red[2][U][4];
    const int t = threadIdx.x % TPR, rin = threadIdx.x / TPR;
    const int c8 = n >> 3;

    float wf[OP == 1 ? CH : 1][8];
    if constexpr (OP == 1) {
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int chunk = c * TPR + t;
            u32x4 p = {0u, 0u, 0u, 0u};
            if (chunk < c8) p = *(const u32x4*)(w + 8 * (size_t)chunk);
            widen8<DT>(p, wf[c]);
        }
    }

    int turn = 0;   // which of the two LDS slots the next workgroup-wide reduction uses
    for (long long row0 = (long long)blockIdx.x * (RPW * U); row0 < n_rows; row0 += (long long)gridDim.x * (RPW * U)) {
        float v[U][CH][8];
        bool ok[U][CH];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long long row = row0 + u * RPW + rin;
            const uint16_t* xr = x + (size_t)row * n;
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const int chunk = c * TPR + t;
                ok[u][c] = row < n_rows && chunk < c8;
                u32x4 p = {0u, 0u, 0u, 0u};
                if (ok[u][c]) p = *(const u32x4*)(xr + 8 * (size_t)chunk);
                widen8<DT>(p, v[u][c]);
            }
        }
        if constexpr (OP == 0) {
            float m[U], s[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                m[u] = -3.0e38f;   // below every finite 16-bit value
#pragma unroll
                for (int c = 0; c < CH; ++c)
#pragma unroll
                    for (int i = 0; i < 8; ++i) m[u] = ok[u][c] && v[u][c][i] > m[u] ? v[u][c][i] : m[u];
            }
            reduce_rows<Max, TPR, U>(m, red[turn]);
            turn ^= 1;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                s[u] = 0.f;
#pragma unroll
                for (int c = 0; c < CH; ++c)
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        v[u][c][i] = ok[u][c] ? __builtin_amdgcn_exp2f((v[u][c][i] - m[u]) * LOG2E) : 0.f;
                        s[u] += v[u][c][i];
                    }
            }
            reduce_rows<Sum, TPR, U>(s, red[turn]);
            turn ^= 1;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float inv = 1.0f / s[u];
#pragma unroll
                for (int c = 0; c < CH; ++c)
#pragma unroll
                    for (int i = 0; i < 8; ++i) v[u][c][i] *= inv;
            }
        } else {
            float ss[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                ss[u] = 0.f;
#pragma unroll
                for (int c = 0; c < CH; ++c)
#pragma unroll
                    for (int i = 0; i < 8; ++i) ss[u] = __builtin_fmaf(v[u][c][i], v[u][c][i], ss[u]);   // masked chunks hold zeros
            }
            reduce_rows<Sum, TPR, U>(ss, red[turn]);
            turn ^= 1;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float r = 1.0f / __builtin_sqrtf(ss[u] / (float)n + eps);
#pragma unroll
                for (int c = 0; c < CH; ++c)
#pragma unroll
                    for (int i = 0; i < 8; ++i) v[u][c][i] = v[u][c][i] * r * wf[c][i];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint16_t* yr = y + (size_t)(row0 + u * RPW + rin) * n;
#pragma unroll
            for (int c = 0; c < CH; ++c)
                if (ok[u][c]) *(u32x4*)(yr + 8 * (size_t)(c * TPR + t)) = narrow8<DT>(v[u][c]);
        }
    }
}

// General path: one workgroup per row, 2-byte accesses, the row is read again for every pass.
template <int DT, int OP>
__global__ __launch_bounds__(256) void rowop_gen_kernel(const uint16_t* x, const uint16_t* __restrict__ w,
                                                       uint16_t* y, long long n_rows, int n, float eps) {
    __shared__ float red[2][1][4];
    int turn = 0;
    auto reduce_row = [&]<class R>(R, float v) {
        float a[1] = {v};
        reduce_rows<R, 256, 1>(a, red[turn]);
        turn ^= 1;
        return a[0];
    };
    for (long long row = blockIdx.x; row < n_rows; row += gridDim.x) {
        const uint16_t* xr = x + (size_t)row * n;
        uint16_t* yr = y + (size_t)row * n;
        if constexpr (OP == 0) {
            float m = -3.0e38f;
            for (int j = threadIdx.x; j < n; j += 256) {
                const float f = widen<DT>(xr[j]);
                m = f > m ? f : m;
            }
            m = reduce_row(Max{}, m);
            float s = 0.f;
            for (int j = threadIdx.x; j < n; j += 256) s += __builtin_amdgcn_exp2f((widen<DT>(xr[j]) - m) * LOG2E);
            s = reduce_row(Sum{}, s);
            const float inv = 1.0f / s;
            // y may be x: every thread rewrites only the elements it alone reads in this pass, and all
            // reads of the earlier passes lie before the barrier of the second reduction
            for (int j = threadIdx.x; j < n; j += 256)
                yr[j] = narrow<DT>(__builtin_amdgcn_exp2f((widen<DT>(xr[j]) - m) * LOG2E) * inv);
        } else {
            float ss = 0.f;
            for (int j = threadIdx.x; j < n; j += 256) {
                const float f = widen<DT>(xr[j]);
                ss = __builtin_fmaf(f, f, ss);
            }
            ss = reduce_row(Sum{}, ss);
            const float r = 1.0f / __builtin_sqrtf(ss / (float)n + eps);
            for (int j = threadIdx.x; j < n; j += 256) yr[j] = narrow<DT>(widen<DT>(xr[j]) * r * widen<DT>(w[j]));
        }
    }
}

template <int DT, int OP, int TPR, int CH, int U>
hipError_t launch_reg(const RowopLaunch& a) {
    constexpr int RPW = (256 / TPR) * U;
    long long groups = (a.n_rows + RPW - 1) / RPW;
    const unsigned grid = (unsigned)(groups < 2048 ? groups : 2048);   // 8 workgroups per compute unit (all that fit), then a stride
    const uint16_t* x = (const uint16_t*)a.x;
    const uint16_t* w = (const uint16_t*)a.w;
    uint16_t* y = (uint16_t*)a.y;
    long long n_rows = a.n_rows;
    int n = a.n;
    float eps = a.eps;
    void* args[] = {&x, &w, &y, &n_rows, &n, &eps};
    return hipLaunchKernel(reinterpret_cast<const void*>(&rowop_reg_kernel<DT, OP, TPR, CH, U>), dim3(grid), dim3(256), args, 0,
                           (hipStream_t)a.stream);
}

template <int DT, int OP>
hipError_t launch_gen(const RowopLaunch& a) {
    const unsigned grid = (unsigned)(a.n_rows < 2048 ? a.n_rows : 2048);
    const uint16_t* x = (const uint16_t*)a.x;
    const uint16_t* w = (const uint16_t*)a.w;
    uint16_t* y = (uint16_t*)a.y;
    long long n_rows = a.n_rows;
    int n = a.n;
    float eps = a.eps;
    void* args[] = {&x, &w, &y, &n_rows, &n, &eps};
    return hipLaunchKernel(reinterpret_cast<const void*>(&rowop_gen_kernel<DT, OP>), dim3(grid), dim3(256), args, 0,
                           (hipStream_t)a.stream);
}

template <int DT, int OP>
hipError_t dispatch(const RowopLaunch& a) {
    if (rowop_path_of(a.n) != 1) return launch_gen<DT, OP>(a);
    const int c8 = a.n / 8;   // 16-byte chunks per row
    constexpr int US = ROWOPS_U_SHORT, UL = ROWOPS_U_LONG;
    if (c8 <= 8) return launch_reg<DT, OP, 8, 1, US>(a);
    if (c8 <= 16) return launch_reg<DT, OP, 16, 1, US>(a);
    if (c8 <= 32) return launch_reg<DT, OP, 32, 1, US>(a);
    if (c8 <= 64) return launch_reg<DT, OP, 64, 1, US>(a);
    if (c8 <= 256) return launch_reg<DT, OP, 256, 1, UL>(a);
    if (c8 <= 512) return launch_reg<DT, OP, 256, 2, UL>(a);
    if (c8 <= 1024) return launch_reg<DT, OP, 256, 4, 1>(a);
    return launch_reg<DT, OP, 256, 8, 1>(a);   // c8 <= 2048 = ROWOPS_MAX_REG_ROW / 8
}

}  // namespace

hipError_t rowop_launch(const RowopLaunch& a) {
    static_assert(ROWOPS_MAX_REG_ROW == 256 * 8 * 8, "the longest registers-path row is 256 threads x 8 chunks x 8 elements");
    if (a.dtype == 0) return a.op == 0 ? dispatch<0, 0>(a) : dispatch<0, 1>(a);
    return a.op == 0 ? dispatch<1, 0>(a) : dispatch<1, 1>(a);
}
