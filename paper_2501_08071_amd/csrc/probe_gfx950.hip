// Measuring aids, not part of any product path (declared in include/probe.h): small kernels whose rates are the
// denominators the throughput of the real kernels is reported against.
//   probe_mfma     nothing but independent v_mfma_f32_32x32x16 in every wavefront, on constant or random operands
//                  (the clock under matrix load depends on how many operand bits switch)
//   probe_softmax_valu  nothing but the vector work the softmax needs per score: multiply-add, exp2, and
//                  optionally the row-sum addition and the conversion to 16 bit
//   probe_l2_read  every workgroup reads a region small enough to stay in its XCD's L2, over and over
//   probe_empty    a kernel that does nothing: what a launch costs by itself
//   probe_issue_share  two wavefronts per SIMD, one issuing matrix instructions only, the other the softmax's vector
//                  work only: what a matrix instruction takes from the issue of the wavefront next to it
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "../../include/probe.h"
#include "gfx950_common.h"

namespace {

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__device__ __forceinline__ uint32_t mix(uint32_t x) {
    x = x * 2654435761u + 12345u;
    x ^= x >> 15;
    x *= 2246822519u;
    x ^= x >> 13;
    return x;
}
// two 16-bit values of magnitude in [1, 2) with random sign and mantissa (bfloat16: 0x3f80 | 7 mantissa
// bits; binary16: 0x3c00 | 10 mantissa bits), or the constant 1.0 pair
template <int DT>
__device__ __forceinline__ uint32_t operand_pair(uint32_t r, int random) {
    const uint32_t one = DT == 0 ? 0x3c003c00u : 0x3f803f80u;
    const uint32_t mask = DT == 0 ? 0x83ff83ffu : 0x807f807fu;
    return random ? ((r & mask) | one) : one;
}

template <int DT>
__global__ __launch_bounds__(256) void mfma_probe_kernel(float* out, int iters, int random) {
    u32x4 a[4], b[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            a[j][e] = operand_pair<DT>(mix(threadIdx.x * 64 + blockIdx.x * 16384 + j * 4 + e), random);
            b[j][e] = operand_pair<DT>(mix(threadIdx.x * 64 + blockIdx.x * 16384 + 16 + j * 4 + e), random);
        }
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            if constexpr (DT == 0)
                acc[j % 4] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a[j % 4]), __builtin_bit_cast(f16x8, b[(j / 4) % 4]), acc[j % 4], 0, 0, 0);
            else
                acc[j % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[j % 4]), __builtin_bit_cast(bf16x8, b[(j / 4) % 4]), acc[j % 4], 0, 0, 0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[j][r];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}


typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

// Per score the softmax needs one multiply-add and one exp2 (FULL == 0), and in the bfloat16 kernel one addition
// for the row sum and half a conversion of two weights into one register (FULL == 1).  16 independent chains per
// lane; the values settle at the fixed point of x -> 2^(x/2 - 1) and stay finite.
template <int FULL>
__global__ __launch_bounds__(256) void softmax_valu_probe_kernel(float* out, int iters, float c, float d) {
    float x[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) x[j] = 0.001f * (float)((threadIdx.x * 16 + j) & 1023);
    float sum = 0.f;
    uint32_t packed = 0u;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            x[j] = __builtin_amdgcn_exp2f(fmaf(x[j], c, d));
            if (FULL) {
                sum += x[j];
                if (j % 2 == 1) {
                    f32x2 two = {x[j - 1], x[j]};
                    uint32_t w = __builtin_bit_cast(uint32_t, __builtin_convertvector(two, bf16x2));
                    asm volatile("" : "+v"(w));   // the conversion is kept although nothing reads its result
                    packed = w;
                }
            }
        }
    }
    float s = sum + __builtin_bit_cast(float, packed & 0x3fffffffu);
#pragma unroll
    for (int j = 0; j < 16; ++j) s += x[j];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// Workgroup b reads the region b % 8 (workgroups are dealt out to the eight XCDs in turn, so a region has one L2 to
// itself), 16 bytes per lane and instruction, eight instructions in flight per lane.
__global__ __launch_bounds__(256) void l2_read_probe_kernel(const u32x4* __restrict__ buf, float* out, int region_vec, int iters) {
    const u32x4* base = buf + (size_t)(blockIdx.x & 7) * region_vec;
    const int start = (int)(((size_t)(blockIdx.x >> 3) * 2048) % (size_t)region_vec);   // workgroups of one XCD start apart
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (int it = 0; it < iters; ++it) {
        const int first = (start + it * 2048) % region_vec;   // a pass starts one step further on than the last
        for (int off = 0; off < region_vec; off += 2048) {
            u32x4 t[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                int idx = first + off + j * 256 + threadIdx.x;
                idx = idx >= region_vec ? idx - region_vec : idx;
                t[j] = base[idx];
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) acc ^= t[j];
        }
    }
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = __builtin_bit_cast(float, (acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) & 0x3fffffffu);
}

__global__ void empty_probe_kernel() {}

typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;

// Eight wavefronts, two per SIMD (wavefront w and w + 4 share one; the dynamic LDS keeps a second workgroup off the
// compute unit).  Wavefronts 0-3 issue nothing but matrix instructions, four accumulators in turn, until their partner
// has finished (or, with the partners idle, `iters` times 32); wavefronts 4-7 do the vector work of `iters` x 32 scores
// per lane: VMODE 1 the bfloat16 kernel's (multiply-add, exp2, addition, half a conversion), VMODE 2 the binary16
// kernel's (multiply-add, exp2, half a conversion, half a two-way dot product for the row sum).  Every wavefront
// writes the shader-clock cycles of its loop and the iterations it made.
template <int VMODE>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void issue_share_probe_kernel(long long* out, int iters, int matrix_on, int max_iters, float c, float d) {
    extern __shared__ __attribute__((aligned(16))) uint32_t done[];   // done[w]: wavefront w + 4 has finished
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (threadIdx.x < 4) done[threadIdx.x] = 0u;
    __syncthreads();
    long long t0 = 0, t1 = 0;
    int made = 0;
    float keep = 0.f;
    if (wave < 4) {
        if (matrix_on) {
            const u32x4 a = {0x3f803f80u, 0x3f813f80u, 0x3f803f82u, 0x3f803f80u};
            f32x16 acc[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
            volatile LDS_AS uint32_t* flag = (volatile LDS_AS uint32_t*)done + wave;
            const int limit = VMODE ? max_iters : iters;
            t0 = __builtin_amdgcn_s_memtime();
            for (; made < limit; ++made) {
                if (VMODE && __builtin_amdgcn_readfirstlane(*flag) != 0u) break;   // one LDS read per 32 matrix instructions
#pragma unroll
                for (int u = 0; u < 32; ++u)
                    acc[u % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, a), acc[u % 4], 0, 0, 0);
            }
            t1 = __builtin_amdgcn_s_memtime();
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) keep += acc[j][r];
        }
    } else {
        if (VMODE) {
            float x[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) x[j] = 0.001f * (float)((threadIdx.x * 8 + j) & 1023);
            float sum = 0.f;
            uint32_t packed = 0u;
            t0 = __builtin_amdgcn_s_memtime();
            for (; made < iters; ++made) {
#pragma unroll
                for (int u = 0; u < 32; ++u) {
                    float& y = x[u & 7];
                    y = __builtin_amdgcn_exp2f(fmaf(y, c, d));
                    if (VMODE == 1) sum += y;
                    if (u & 1) {
                        const f32x2 two = {x[(u - 1) & 7], y};
                        uint32_t w;
                        if (VMODE == 1) w = __builtin_bit_cast(uint32_t, __builtin_convertvector(two, bf16x2));
                        else {
                            w = __builtin_bit_cast(uint32_t, __builtin_convertvector(two, f16x2));
                            sum = gfx950::Elem<0>::dot2_ones(w, sum);
                        }
                        asm volatile("" : "+v"(w));   // the conversion is kept although nothing reads its result
                        packed = w;
                    }
                    asm volatile("" : "+v"(y));
                }
            }
            t1 = __builtin_amdgcn_s_memtime();
            keep = sum + __builtin_bit_cast(float, packed & 0x3fffffffu);
#pragma unroll
            for (int j = 0; j < 8; ++j) keep += x[j];
            if (lane == 0) done[wave - 4] = 1u;
        }
    }
    asm volatile("" :: "v"(keep));
    if (lane == 0) {
        out[((size_t)blockIdx.x * 8 + wave) * 2] = t1 - t0;
        out[((size_t)blockIdx.x * 8 + wave) * 2 + 1] = made;
    }
}

}  // namespace

extern "C" long long probe_mfma(float* out, int workgroups, int iters, int dtype, int random_operands, void* stream) {
    if (out == nullptr || workgroups <= 0 || workgroups > 65536 || iters <= 0 || iters > (1 << 24)) return -1;
    if (dtype != 0 && dtype != 1) return -1;
    int it = iters, rnd = random_operands != 0;
    void* args[] = {&out, &it, &rnd};
    const void* fn = dtype == 0 ? reinterpret_cast<const void*>(&mfma_probe_kernel<0>)
                                       : reinterpret_cast<const void*>(&mfma_probe_kernel<1>);
    if (hipLaunchKernel(fn, dim3((unsigned)workgroups), dim3(256), args, 0, (hipStream_t)stream) != hipSuccess) return -1;
    return (long long)workgroups * 4 * iters * 16 * 32768LL;   // 4 wavefronts, 16 matrix instructions of 2 * 32 * 32 * 16 flop
}

extern "C" long long probe_softmax_valu(float* out, int workgroups, int iters, int full, void* stream) {
    if (out == nullptr || workgroups <= 0 || workgroups > 65536 || iters <= 0 || iters > (1 << 24)) return -1;
    int it = iters;
    float c = 0.5f, d = -1.0f;
    void* args[] = {&out, &it, &c, &d};
    const void* fn = full ? reinterpret_cast<const void*>(&softmax_valu_probe_kernel<1>)
                          : reinterpret_cast<const void*>(&softmax_valu_probe_kernel<0>);
    if (hipLaunchKernel(fn, dim3((unsigned)workgroups), dim3(256), args, 0, (hipStream_t)stream) != hipSuccess) return -1;
    return (long long)workgroups * 256 * iters * 16;   // scores
}

extern "C" long long probe_l2_read(const void* buf, float* out, int region_kib, int workgroups, int iters, void* stream) {
    if (buf == nullptr || out == nullptr || workgroups <= 0 || workgroups > 65536 || iters <= 0 || iters > (1 << 20)) return -1;
    if (region_kib < 32 || region_kib > (1 << 20) || region_kib % 32 != 0) return -1;   // whole steps of 2048 x 16 bytes
    if ((reinterpret_cast<uintptr_t>(buf) & 15u) != 0) return -1;
    int region_vec = region_kib * 64, it = iters;
    void* args[] = {&buf, &out, &region_vec, &it};
    if (hipLaunchKernel(reinterpret_cast<const void*>(&l2_read_probe_kernel), dim3((unsigned)workgroups), dim3(256), args, 0,
                        (hipStream_t)stream) != hipSuccess)
        return -1;
    return (long long)workgroups * iters * region_kib * 1024LL;   // bytes
}

extern "C" int probe_empty(int workgroups, int threads, void* stream) {
    if (workgroups <= 0 || workgroups > (1 << 20) || threads <= 0 || threads > 1024) return -1;
    void* args[] = {nullptr};
    return hipLaunchKernel(reinterpret_cast<const void*>(&empty_probe_kernel), dim3((unsigned)workgroups), dim3((unsigned)threads),
                           args, 0, (hipStream_t)stream) == hipSuccess ? 0 : -1;
}

extern "C" int probe_issue_share(long long* out, int workgroups, int iters, int matrix_on, int vector_mode, void* stream) {
    if (out == nullptr || workgroups <= 0 || workgroups > 65536 || iters <= 0 || iters > (1 << 20)) return -1;
    if (vector_mode < 0 || vector_mode > 2 || (!matrix_on && vector_mode == 0)) return -1;
    if ((reinterpret_cast<uintptr_t>(out) & 7u) != 0) return -1;
    int it = iters, mon = matrix_on != 0, max_it = iters * 8;   // a partner's 32 scores take less than 8 x 32 matrix instructions
    float c = 0.5f, d = -1.0f;
    void* args[] = {&out, &it, &mon, &max_it, &c, &d};
    const void* fn = vector_mode == 0 ? reinterpret_cast<const void*>(&issue_share_probe_kernel<0>)
                   : vector_mode == 1 ? reinterpret_cast<const void*>(&issue_share_probe_kernel<1>)
                                      : reinterpret_cast<const void*>(&issue_share_probe_kernel<2>);
    constexpr unsigned lds_bytes = 96u * 1024u;   // more than half of a compute unit's: one workgroup each
    static std::atomic<uint64_t> told[3];
    if (gfx950::announce_lds(fn, lds_bytes, told[vector_mode]) != hipSuccess) return -1;
    return hipLaunchKernel(fn, dim3((unsigned)workgroups), dim3(512), args, lds_bytes, (hipStream_t)stream) == hipSuccess ? 0 : -1;
}
