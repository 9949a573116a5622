// Fused multi-head attention forward for gfx950 (MI355X): O = softmax(Q K^T * scale [+ causal]) V
// and the per-row logsumexp, one pass over K/V with a running (online) softmax.
//
// The operation is the "flash-attention" kernel class of the paper's Table 2; the paper's
// subject is the order of memory and compute instructions inside such a fixed kernel
// (Sections 2.4, 3.5).  Here that order is set by hand for CDNA4.
//
// Work split
//   workgroup = NW wavefronts, each owning 32 consecutive query rows of one (b,h);
//   K/V stream through LDS in tiles of BC = 64 keys shared by the whole workgroup.
//
// K/V movement
//   global -> LDS directly (global_load_lds_dwordx4, no VGPR staging), two buffers per tensor, the
//   loads of tile t+1 issued right after the single barrier of tile t.  Such a load writes 1 KiB
//   of consecutive LDS per wavefront, so rows cannot be padded; bank conflicts are avoided by an
//   XOR swizzle of the 16-byte chunk index within each row, applied on the global-address side.
//
// Register layout (64-wide wavefront, lane l, half h = l/32, l32 = l%32)
//   Everything is computed transposed so that one lane only ever holds values of ONE query row:
//     S^T (keys x queries) = K_tile . Q^T      v_mfma_f32_32x32x16: A = K rows, B = Q^T
//       accumulator register r of key block jb holds  S[q = l32][key = 32 jb + 8 (r/4) + 4 h + r%4]
//     O^T (d x queries)  += V_tile^T . P^T     A = V^T (LDS transpose read), B = P^T
//       The B operand of key step (jb,t) is registers 8t..8t+7 of block jb as they are; the
//       contraction index is therefore visited in the permuted order
//         key(slot e of half h) = 32 jb + 16 t + 8 (e/4) + 4 h + e%4,
//       and the V^T operand is fetched in that same order, so P never leaves registers.
//   Row maximum and row sum are an in-lane reduction plus one exchange between the halves.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_launch.h"

namespace {

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
};

// 4 x 16-bit transposing LDS read: within each group of 16 lanes, lane i receives element i%4 of
// the 8 bytes addressed by lanes i/4, 4 + i/4, 8 + i/4 and 12 + i/4 of its group.
__device__ __forceinline__ u32x2 lds_read_tr16(const uint8_t* p) {
    s16x4 t = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)p);
    return __builtin_bit_cast(u32x2, t);
}

// 16 bytes per lane from global memory straight into LDS: lane l's data lands at lds_base + 16 l
// (lds_base wave-uniform, a multiple of 16).  Written as asm so that the compiler's wait-count
// insertion does not know about the transfer: it would otherwise wait for ALL outstanding tile
// loads in front of LDS reads of the other buffer.  The wait is explicit, before the tile barrier.
__device__ __forceinline__ void lds_dma16(uint32_t lds_base, const void* gbase, uint32_t byte_off) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_base), "v"(byte_off), "s"(gbase) : "memory", "m0");
}
__device__ __forceinline__ void wait_tile_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

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
template <int D>
__device__ __forceinline__ constexpr int swz(int row) {
    return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3))
                    : ((((row >> 1) & 1) << 2) | (((row >> 2) & 1) << 1) | ((row >> 3) & 1));
}

extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

template <int DT, int D, bool CAUSAL, int NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(ATTN_WPE, ATTN_WPE))) void attn_fwd_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                           const uint16_t* __restrict__ v, float* __restrict__ o,
                                                           float* __restrict__ lse, int S, int BH, int nqt, float c,
                                                           uint32_t qsign) {
    using E = Elem<DT>;
    constexpr int BR = NW * 32;        // query rows per workgroup
    constexpr int BC = ATTN_BC;        // keys per tile
    constexpr int KSTEPS = D / 16;     // contraction steps of Q.K^T
    constexpr int DB = D / 32;         // 32-wide blocks of the head dimension
    constexpr int ROWB = 2 * D;        // bytes per K/V row
    constexpr int TILEB = BC * ROWB;   // bytes per tile
    constexpr int CPR = D / 8;         // 16-byte chunks per row
    constexpr int RPI = 1024 / ROWB;   // rows written by one direct-to-LDS load instruction
    constexpr int IPT = BC / RPI;      // such instructions per tile and tensor
    constexpr int IPW = IPT / NW;      // ... per wavefront
    static_assert(IPT % NW == 0, "tile loads must split evenly over the wavefronts");
    // LDS: K buffer 0 | K buffer 1 | V buffer 0 | V buffer 1

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31;
    const int h = lane >> 5;

    // heaviest query tiles first (under the causal mask tile t reads t+1 key tiles)
    const int bh = blockIdx.x % BH;
    const int qt = CAUSAL ? nqt - 1 - blockIdx.x / BH : blockIdx.x / BH;
    const int q0 = qt * BR;
    const int qw0 = q0 + 32 * wave;          // first query row of this wavefront
    const int qrow = qw0 + l32;              // this lane's query row (may lie beyond S on the last tile)
    const int qrow_ld = qrow < S ? qrow : S - 1;

    const size_t head = (size_t)bh * S * D;
    const uint16_t* qh = q + head;
    const uint16_t* kh = k + head;
    const uint16_t* vh = v + head;

    const int kv_end = CAUSAL ? (q0 + BR < S ? q0 + BR : S) : S;
    const int ntiles = (kv_end + BC - 1) / BC;

    // ---- direct-to-LDS tile loads ----
    // instruction `inst` fills LDS bytes [inst*1024, +1024) of a tile buffer = rows inst*RPI.. ; lane
    // writes chunk position lane%CPR of row lane/CPR and therefore fetches source chunk pos ^ swz(row)
    uint32_t goff[IPW];
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
        const int r = (wave * IPW + i) * RPI + lane / CPR;
        goff[i] = r * D + (((lane % CPR) ^ swz<D>(r)) << 3);
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(LDS_AS uint8_t*)smem;
    auto issue_loads = [&](int j0, int buf) {
        const uint16_t* kt = kh + (size_t)j0 * D;
        const uint16_t* vt = vh + (size_t)j0 * D;
        const bool ragged = j0 + BC > S;
#pragma unroll
        for (int i = 0; i < IPW; ++i) {
            const int inst = wave * IPW + i;
            uint32_t off = goff[i];
            if (ragged) {   // rows past the end are masked later; point them at the last valid row
                const int over = j0 + inst * RPI + lane / CPR - (S - 1);
                if (over > 0) off -= over * D;
            }
            lds_dma16(lds0 + buf * TILEB + inst * 1024, kt, off * 2);
            lds_dma16(lds0 + (2 + buf) * TILEB + inst * 1024, vt, off * 2);
        }
    };
    issue_loads(0, 0);

    // Q^T operand, resident for the whole kernel: lane holds q[qrow][16 ks + 8 h .. +7]
    u32x4 qf[KSTEPS];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
        qf[ks] = *(const u32x4*)(qh + (size_t)qrow_ld * D + 16 * ks + 8 * h);
        qf[ks] ^= qsign;   // a negative scale is folded into the sign of q (exact)
    }

    f32x16 acc_o[DB];
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[i][r] = 0.f;
    float m_run = -INFINITY;   // running row maximum of the scaled logits, base-2 units
    float l_run = 0.f;         // this lane's share of the running row sum

    // ---- per-lane LDS byte offsets (loop invariant; tile/block parts are immediate offsets) ----
    // K operand of (jb, ks): row 32 jb + l32, source chunk 2 ks + h
    uint32_t kaddr[KSTEPS];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) kaddr[ks] = l32 * ROWB + (((2 * ks + h) ^ swz<D>(l32)) << 4);
    // V^T operand of (jb, t, half hi, block i): lane addresses 8 bytes of row 32 jb + 16 t + 8 hi + 4 h + x,
    // elements 32 i + 16 g1 + 4 y .. +3, where x = (lane%16)/4, y = lane%4, g1 = (lane/16)%2
    uint32_t vaddr[2][DB];
    {
        const int x = (lane & 15) >> 2, y = lane & 3, g1 = (lane >> 4) & 1;
#pragma unroll
        for (int hi = 0; hi < 2; ++hi)
#pragma unroll
            for (int i = 0; i < DB; ++i) {
                const int chunk = 4 * i + 2 * g1 + (y >> 1);
                vaddr[hi][i] = (4 * h + x) * ROWB + ((chunk ^ swz<D>(8 * hi + 4 * h + x)) << 4) + ((y & 1) << 3);
            }
    }

    auto compute_tile = [&](int j0, const uint8_t* kb, const uint8_t* vb) {
        // ---- S^T = K . Q^T ----
        f32x16 s[2];
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[jb][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
            for (int jb = 0; jb < 2; ++jb) {
                u32x4 a = *(const u32x4*)(kb + kaddr[ks] + jb * 32 * ROWB);
                s[jb] = E::mfma(a, qf[ks], s[jb]);
            }

        // ---- mask, running maximum, exponentials ----
        const bool need_mask = (j0 + BC > S) || (CAUSAL && j0 + BC - 1 > qw0);
        float m_new;
        if (need_mask) {
            // scale first, then mask, so that scale == 0 cannot meet an infinity
            const int lim = (CAUSAL ? qrow_ld : S - 1) - j0 - 4 * h;
            float mx = -INFINITY;
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int off = 32 * jb + 8 * (r / 4) + (r % 4);
                    float x = s[jb][r] * c;
                    x = off > lim ? -INFINITY : x;
                    s[jb][r] = x;
                    mx = fmaxf(mx, x);
                }
            mx = fmaxf(mx, other_half(mx));
            m_new = fmaxf(m_run, mx);
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[jb][r] = __builtin_amdgcn_exp2f(s[jb][r] - m_new);
        } else {
            float mx = s[0][0];
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[jb][r]);
            mx = fmaxf(mx, other_half(mx));
            m_new = fmaxf(m_run, mx * c);    // c >= 0
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[jb][r] = __builtin_amdgcn_exp2f(fmaf(s[jb][r], c, -m_new));
        }

        // ---- running sum ----
        // binary16 weights keep 11 bits, so the rounded weights can be summed two per dot instruction;
        // bfloat16 keeps 8, which would cost the logsumexp its 1e-3 accuracy: sum those in fp32 first
        float psum = 0.f;
        if (DT == 1) {
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int r = 0; r < 16; ++r) psum += s[jb][r];
        }

        // ---- P^T operands: registers 8t..8t+7 of block jb, rounded to the input type ----
        u32x4 pf[2][2];
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                for (int e = 0; e < 4; ++e) pf[jb][tt][e] = E::pack2(s[jb][8 * tt + 2 * e], s[jb][8 * tt + 2 * e + 1]);
        if (DT == 0) {
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                    for (int e = 0; e < 4; ++e) psum = E::dot2_ones(pf[jb][tt][e], psum);
        }

        // ---- rescale only when some row of this wavefront got a new maximum ----
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        l_run = l_run * alpha + psum;
        if (__builtin_amdgcn_ballot_w64(m_new != m_run) != 0) {
#pragma unroll
            for (int i = 0; i < DB; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc_o[i][r] *= alpha;
        }
        m_run = m_new;

        // ---- O^T += V^T . P^T ----
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                for (int i = 0; i < DB; ++i) {
                    const uint8_t* p = vb + (32 * jb + 16 * tt) * ROWB;
                    u32x2 lo = lds_read_tr16(p + vaddr[0][i]);
                    u32x2 hi = lds_read_tr16(p + vaddr[1][i] + 8 * ROWB);
                    u32x4 a = {lo[0], lo[1], hi[0], hi[1]};
                    acc_o[i] = E::mfma(a, pf[jb][tt], acc_o[i]);
                }
    };

    // one barrier per tile: after it, tile t has landed for everybody and nobody still reads the
    // buffer that tile t+1 is about to overwrite
    for (int t = 0; t < ntiles; t += 2) {
        wait_tile_loads();
        __syncthreads();
        if (t + 1 < ntiles) issue_loads((t + 1) * BC, 1);
        if (!(CAUSAL && t * BC > qw0 + 31)) compute_tile(t * BC, smem, smem + 2 * TILEB);
        if (t + 1 < ntiles) {
            wait_tile_loads();
            __syncthreads();
            if (t + 2 < ntiles) issue_loads((t + 2) * BC, 0);
            if (!(CAUSAL && (t + 1) * BC > qw0 + 31)) compute_tile((t + 1) * BC, smem + TILEB, smem + 3 * TILEB);
        }
    }

    // ---- epilogue: O = acc / l, lse = ln 2 * (m + log2 l) ----
    const float l_tot = l_run + other_half(l_run);
    const float inv = 1.0f / l_tot;
    if (qrow < S) {
        float* orow = o + head + (size_t)qrow * D;
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 x = {acc_o[i][4 * g] * inv, acc_o[i][4 * g + 1] * inv, acc_o[i][4 * g + 2] * inv,
                           acc_o[i][4 * g + 3] * inv};
                *(f32x4*)(orow + 32 * i + 8 * g + 4 * h) = x;
            }
        if (lse != nullptr && h == 0)
            lse[(size_t)bh * S + qrow] = (m_run + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
    }
}

template <int DT, int D, bool CAUSAL, int NW>
hipError_t launch(const AttnLaunch& a) {
    constexpr int BR = NW * 32;
    const int nqt = (a.S + BR - 1) / BR;
    const long long blocks = (long long)nqt * a.BH;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    const uint16_t* q = (const uint16_t*)a.q;
    const uint16_t* k = (const uint16_t*)a.k;
    const uint16_t* v = (const uint16_t*)a.v;
    float* o = a.o;
    float* lse = a.lse;
    int S = a.S, BH = a.BH, nq = nqt;
    float c = a.c;
    uint32_t qsign = a.qsign;
    void* args[] = {&q, &k, &v, &o, &lse, &S, &BH, &nq, &c, &qsign};
    // the launch status is taken from the call itself: the thread's "last error" may hold a stale
    // value left by an unrelated earlier runtime call of the host program
    constexpr unsigned lds_bytes = 4u * ATTN_BC * 2u * D;   // two K and two V tile buffers
    const void* fn = reinterpret_cast<const void*>(&attn_fwd_kernel<DT, D, CAUSAL, NW>);
    return hipLaunchKernel(fn, dim3((unsigned)blocks), dim3(NW * 64), args, lds_bytes, (hipStream_t)a.stream);
}

}  // namespace

// dispatch on (dtype, D, causal); arguments were validated by the caller
hipError_t attn_launch(const AttnLaunch& a) {
#define ATTN_CASE(DT, DD, CZ)                                       \
    if (a.dtype == DT && a.D == DD && (a.causal != 0) == CZ) return launch<DT, DD, CZ, ATTN_NW>(a);
    ATTN_CASE(0, 64, false)
    ATTN_CASE(0, 64, true)
    ATTN_CASE(0, 128, false)
    ATTN_CASE(0, 128, true)
    ATTN_CASE(1, 64, false)
    ATTN_CASE(1, 64, true)
    ATTN_CASE(1, 128, false)
    ATTN_CASE(1, 128, true)
#undef ATTN_CASE
    return hipErrorInvalidValue;
}
