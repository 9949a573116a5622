// Internal: device helpers shared by the attention kernels (row maxima, the exchange between the halves of a
// wavefront, the bank-conflict swizzle of K/V rows in LDS).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace attn_device {

// plain maxima, without the quiet-NaN canonicalisation the C library semantics would add
__device__ __forceinline__ float vmax(float a, float b) {
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float vmax3(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// value held by the other half of the wavefront (lane l <-> lane l^32)
__device__ __forceinline__ float other_half(float x) {
    uint32_t u = __builtin_bit_cast(uint32_t, x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    // lanes <32 get (own, upper's); lanes >=32 get (lower's, own)
    return __builtin_bit_cast(float, (threadIdx.x & 32) ? r[0] : r[1]);
}

// XOR swizzle of the 16-byte chunk index inside a K/V row in LDS (row = tile-local key index).
// D=128 (16 chunks/row, a row spans all 64 banks): 16 consecutive rows must land on 16 different
//   chunks (b128 reads of K) and 4 consecutive rows x 4 consecutive chunks likewise (transpose
//   reads of V): swap the two low bit pairs of the row index.
// D=64 (8 chunks/row, two rows span the banks): the same two conditions with the row parity
//   already selecting the bank half: bit-reverse bits 1..3 of the row index.
// D=32 (4 chunks/row, four rows span the banks): row % 4 selects the bank quarter, so the transpose
//   reads need nothing; for the b128 reads rows r, r+4, r+8, r+12 must differ: bits 2..3 of the row.
template <int D>
__device__ __forceinline__ constexpr int swz(int row) {
    return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3))
           : D == 64 ? ((((row >> 1) & 1) << 2) | (((row >> 2) & 1) << 1) | ((row >> 3) & 1))
                     : ((row >> 2) & 3);
}

}  // namespace attn_device
