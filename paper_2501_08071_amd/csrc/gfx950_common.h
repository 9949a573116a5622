// Internal: what the matrix-core kernels of this library share -- vector types, the two 16-bit element types with
// their matrix instruction and rounding, the LDS access primitives of gfx950, and the one piece of host code
// that tells the runtime about a kernel instance's LDS size.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace gfx950 {

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

#define LDS_AS __attribute__((address_space(3)))

template <int DT> struct Elem;
template <> struct Elem<0> {  // IEEE binary16
    static __device__ __forceinline__ f32x16 mfma(u32x4 a, u32x4 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {  // round to nearest even
        f32x2 x = {lo, hi};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, f16x2));
    }
    static __device__ __forceinline__ float dot2_ones(uint32_t p, float acc) {  // acc + p.lo + p.hi
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, p), f16x2{(_Float16)1.0f, (_Float16)1.0f}, acc, false);
    }
    static __device__ __forceinline__ float widen(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
};
template <> struct Elem<1> {  // bfloat16
    static __device__ __forceinline__ f32x16 mfma(u32x4 a, u32x4 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {  // round to nearest even
        f32x2 x = {lo, hi};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
    }
    static __device__ __forceinline__ float dot2_ones(uint32_t p, float acc) {  // acc + p.lo + p.hi
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, p), bf16x2{(__bf16)1.0f, (__bf16)1.0f}, acc, false);
    }
    static __device__ __forceinline__ float widen(uint16_t b) { return __builtin_bit_cast(float, (uint32_t)b << 16); }
};

// The same matrix instruction with its accumulator pinned to accumulation registers, for kernels whose wavefronts own
// the whole register file and are compiled with matrix results in vector registers by default (so that the vector pipe
// can read the products it consumes): a long-lived accumulator that no vector instruction touches in the loop goes
// here and leaves the vector registers to the rest.  Written as asm, so the compiler knows nothing of the
// instruction's latency: the CALLER passes the accumulator through mfma_settle before anything but another such
// instruction on the same accumulator reads it.
template <int DT>
__device__ __forceinline__ void mfma_aacc(f32x16& d, u32x4 a, u32x4 b) {   // d += a.b
    if constexpr (DT == 0) asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(d) : "v"(a), "v"(b));
    else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(d) : "v"(a), "v"(b));
}
// 24 wait states, after which the results of earlier mfma_aacc on the accumulators passed here are in place.  The
// accumulators go through the statement, so that no read of them (the compiler's own copies included: they follow
// the data flow, not the order of asm statements) can be placed ahead of the wait.
// (The wait comes first and by itself: a copy the compiler makes to bring an accumulator to the second statement
// then stands behind the wait.)
__device__ __forceinline__ void mfma_settle(f32x16& a0, f32x16& a1, f32x16& a2, f32x16& a3) {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" : "+a"(a0), "+a"(a1), "+a"(a2), "+a"(a3));
}

// 16 bytes per lane from global memory straight into accumulation registers (a resident matrix operand that no vector
// instruction ever touches: an ordinary value would live in vector registers and be copied over before every use).
// The compiler does not know of the load: the CALLER waits (vmcnt) before the first use.
__device__ __forceinline__ u32x4 global_load_acc16(const void* p) {
    u32x4 r;
    asm volatile("global_load_dwordx4 %0, %1, off" : "=a"(r) : "v"(p) : "memory");
    return r;
}

// 4 x 16-bit transposing LDS read: within each group of 16 lanes, lane i receives element i%4 of
// the 8 bytes addressed by lanes i/4, 4 + i/4, 8 + i/4 and 12 + i/4 of its group.
__device__ __forceinline__ u32x2 lds_read_tr16(uint32_t addr) {
    s16x4 t = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(uintptr_t)addr);
    return __builtin_bit_cast(u32x2, t);
}
__device__ __forceinline__ u32x4 lds_read_b128(uint32_t addr) { return *(const LDS_AS u32x4*)(uintptr_t)addr; }

// 16 bytes per lane from global memory straight into LDS: lane l's data lands at lds_base + 16 l
// (lds_base wave-uniform, a multiple of 16).  Written as asm so that the compiler's wait-count
// insertion does not know about the transfer: it would otherwise wait for ALL outstanding tile
// loads in front of LDS reads of another buffer.  The wait is explicit (wait_lds_dma).
__device__ __forceinline__ void lds_dma16(uint32_t lds_base, const void* gbase, uint32_t byte_off) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_base), "v"(byte_off), "s"(gbase) : "memory", "m0");
}
// wait until at most N of this wavefront's direct-to-LDS loads are still in flight (they land in order)
template <int N>
__device__ __forceinline__ void wait_lds_dma() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }

// Host: a kernel instance that wants more dynamic LDS than the default limit has to be announced to the runtime,
// once per instance and device.  `told` holds one bit per device (one object per kernel instance, owned by the
// caller); two host threads that both find the bit clear both make the call, which is harmless.  Devices beyond
// the mask are announced on every launch.
inline hipError_t announce_lds(const void* fn, unsigned lds_bytes, std::atomic<uint64_t>& told) {
    if (lds_bytes <= 65536u) return hipSuccess;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = dev >= 0 && dev < 64 ? uint64_t(1) << dev : 0;
    if (bit != 0 && (told.load(std::memory_order_acquire) & bit) != 0) return hipSuccess;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    told.fetch_or(bit, std::memory_order_release);
    return hipSuccess;
}

}  // namespace gfx950
