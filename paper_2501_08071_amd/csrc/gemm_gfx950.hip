// Fused GEMM + LeakyReLU for gfx950 (the paper's mmLeakyReLu, Table 2): c = f(a b), a [M,K], b [K,N]
// row-major, 16-bit in and out, fp32 accumulation.
//
// Matrix-core kernel (K % 32 == 0, N % 8 == 0):
//   * a workgroup of four wavefronts (2 x 2) owns a 64 TM x 64 TN tile of c, a wavefront 32 TM x 32 TN of
//     it as TM x TN accumulator blocks of v_mfma_f32_32x32x16; TM = TN = 2 (128 x 128) when that gives
//     the chip enough tiles, else 1 (64 x 64);
//   * computed transposed, c^T = b^T a^T: the first operand is a 32 x 16 piece of b^T, fetched from the
//     row-major b tile in LDS with transposing reads (ds_read_b64_tr_b16), the second 16 contiguous bytes
//     of a row of a; a lane then holds four consecutive n of one row m of c, and the tile of c goes out
//     through LDS so that the stores write whole rows of it;
//   * K runs in steps of 32 through four LDS stages; tiles come straight from global memory into LDS
//     (global_load_lds_dwordx4, 16 bytes per lane, 1 KiB of consecutive LDS per instruction), three
//     stages ahead, with the bank-conflict swizzle applied to the global address of each lane;
//   * the 256 x 256 tile has eight wavefronts, two per SIMD, in two groups that alternate between reading a
//     block's operands from LDS and issuing its matrix instructions, one phase apart: the matrix pipe of a
//     SIMD is fed by one wavefront while the other waits for the barrier, for LDS and for its loads;
//   * rows past M repeat the last row and column chunks past N the last chunk (results masked at the
//     store), so the loop has no edge cases.
// Small problems (at most 256 tiles of 32 x 32, K >= 256): 32 x 32 tiles with K split over the four wavefronts of
// the workgroup, see gemm_lrelu_splitk_kernel.
// Plain kernel (any shape): one thread per element of c, fp32 fused multiply-adds in the order of k.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include <utility>

#include "gemm_launch.h"
#include "gfx950_common.h"

#ifndef GEMM_PINGPONG
#define GEMM_PINGPONG 1   // eight-wavefront tiles: two groups of wavefronts alternate operand reads and matrix instructions
#endif
#ifndef GEMM_NST
#define GEMM_NST 4   // LDS stages of 32 in K; GEMM_NST - 1 of them in flight ahead of the one in use
#endif

namespace {

using namespace gfx950;

template <int N>
__device__ __forceinline__ void wait_tile_loads() { wait_lds_dma<N>(); }

// XOR swizzle of the 16-byte chunk index within a row, by row length (chunks per row 4, 8, 16): rows
// that a wavefront reads together land in different banks both for the 16-byte row reads and for
// the transposing 8-byte reads.
__device__ __forceinline__ constexpr int swz_a(int row) { return (row >> 2) & 3; }
template <int CHUNKS>
__device__ __forceinline__ constexpr int swz_b(int row) {
    return CHUNKS >= 16 ? (((row & 3) << 2) | ((row >> 2) & 3))   // the low four chunk bits = 256 bytes = all banks
                        : ((((row >> 1) & 1) << 2) | (((row >> 2) & 1) << 1) | ((row >> 3) & 1));
}

__device__ __forceinline__ float leaky(float t, float slope) { return t >= 0.f ? t : slope * t; }

extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

// dynamic LDS of a kernel instance: the stages of the loop, or (if larger) the padded blocks of c on their way out
template <int WM, int WN, int TM, int TN>
struct GemmLds {
    static constexpr int STAGES = GEMM_NST * (32 * TM * WM * 64 + 32 * 2 * 32 * TN * WN);
    static constexpr int OUT = WM * WN * (32 * TM) * (64 * TN + 16);
    static constexpr int BYTES = STAGES > OUT ? STAGES : OUT;
    static_assert(BYTES <= 160 * 1024, "LDS");
};

template <int DT, int WM, int WN, int TM, int TN>
__global__ __launch_bounds__(WM * WN * 64) void gemm_lrelu_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ B,
                                                        uint16_t* __restrict__ C, int M, int N, int K, int tiles_m,
                                                        int tiles_n, float slope) {
    using E = Elem<DT>;
    constexpr int NW = WM * WN;               // wavefronts, WM x WN over the tile
    constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN, NST = GEMM_NST;
    constexpr int A_TILE = BM * 64;          // BM rows of 32 elements
    constexpr int B_ROWB = 2 * BN;           // bytes per row of the b tile
    constexpr int B_TILE = 32 * B_ROWB;      // 32 rows (k) of BN elements
    constexpr int STAGE = A_TILE + B_TILE;
    constexpr int B_LPR = B_ROWB / 16;       // lanes (16-byte chunks) per row of the b tile
    constexpr int B_RPI = 64 / B_LPR;        // rows per load instruction
    constexpr int LA = A_TILE / 1024 / NW, LB = B_TILE / 1024 / NW;   // load instructions per stage and wavefront
    constexpr int IPS = LA + LB;
    static_assert(LA * NW * 1024 == A_TILE && LB * NW * 1024 == B_TILE && LA >= 1 && LB >= 1, "the wavefronts share the loads evenly");
    static_assert(NST * STAGE <= 160 * 1024, "LDS");

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, h = lane >> 5;
    const int wm = wave % WM, wn = wave / WM;

    const int bx = blockIdx.x;
    const int tn_i = bx % tiles_n;
    const int tm_i = (bx / tiles_n) % tiles_m;
    const int bi = bx / (tiles_n * tiles_m);
    const int m0 = tm_i * BM, n0 = tn_i * BN;
    const uint16_t* Ab = A + ((size_t)bi * M + m0) * K;
    const uint16_t* Bb = B + (size_t)bi * K * N + n0;
    uint16_t* Cb = C + (size_t)bi * M * N;
    const int nk = K / 32;

    const uint32_t lds0 = (uint32_t)(uintptr_t)(LDS_AS uint8_t*)smem;

    // ---- loads: byte offset of this lane's source chunk inside the tile's rows ----
    uint32_t goff_a[LA], goff_b[LB];
#pragma unroll
    for (int j = 0; j < LA; ++j) {
        const int r = 16 * (wave * LA + j) + lane / 4, pos = lane % 4;
        const int rr = r < M - 1 - m0 ? r : M - 1 - m0;
        goff_a[j] = (uint32_t)(rr * K + ((pos ^ swz_a(r)) << 3)) * 2u;
    }
    {
        const int nvalid = (N - n0) / 8 < BN / 8 ? (N - n0) / 8 : BN / 8;   // chunks of this tile inside the matrix
#pragma unroll
        for (int j = 0; j < LB; ++j) {
            const int r = B_RPI * (wave * LB + j) + lane / B_LPR, pos = lane % B_LPR;
            int ch = pos ^ swz_b<B_LPR>(r);
            ch = ch < nvalid - 1 ? ch : nvalid - 1;
            goff_b[j] = (uint32_t)(r * N + (ch << 3)) * 2u;
        }
    }
    // k block kb into stage st; a block past the end repeats the last one (nobody reads it): every step
    // issues the same number of loads and the wait count is a constant
    auto issue = [&](int kb, int st) {
        const int kc = kb < nk - 1 ? kb : nk - 1;
        const uint16_t* sa = Ab + (size_t)kc * 32;
        const uint16_t* sb = Bb + (size_t)kc * 32 * N;
#pragma unroll
        for (int j = 0; j < LA; ++j) lds_dma16(lds0 + st * STAGE + (wave * LA + j) * 1024, sa, goff_a[j]);
#pragma unroll
        for (int j = 0; j < LB; ++j) lds_dma16(lds0 + st * STAGE + A_TILE + (wave * LB + j) * 1024, sb, goff_b[j]);
    };

    // ---- operand addresses (stage 0, k step 0 of the b tile) ----
    uint32_t a_addr[TM][2];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
            a_addr[tm][ks] = lds0 + ((wm * TM + tm) * 32 + l32) * 64 + (((2 * ks + h) ^ swz_a(l32)) << 4);
    // b^T operand: lane addresses 8 bytes of row (k) 8 h + 4 hi + x, elements (n) 16 g1 + 4 y .. +3 of the
    // 32-wide block; the transposing read hands lane l the four k of element n = l % 32
    uint32_t b_addr[2][TN];
    {
        const int x = (lane & 15) >> 2, y = lane & 3, g1 = (lane >> 4) & 1;
#pragma unroll
        for (int hi = 0; hi < 2; ++hi)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const int row = 8 * h + 4 * hi + x;
                const int chunk = 4 * (wn * TN + tn) + 2 * g1 + (y >> 1);
                b_addr[hi][tn] = lds0 + A_TILE + row * B_ROWB + ((chunk ^ swz_b<B_LPR>(row)) << 4) + ((y & 1) << 3);
            }
    }

    f32x16 acc[TN][TM];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tn][tm][r] = 0.f;

#pragma unroll
    for (int s = 0; s < NST - 1; ++s) issue(s, s);

    // The operands of one k step (16 of the 32 of a block) of stage st
    struct Ops {
        u32x4 a[TM], b[TN];
    };
    auto read_ops = [&](Ops& o, int st_bytes, int ks) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) o.a[tm] = lds_read_b128(a_addr[tm][ks] + st_bytes);
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const u32x2 lo = lds_read_tr16(b_addr[0][tn] + st_bytes + ks * 16 * B_ROWB);
            const u32x2 hi = lds_read_tr16(b_addr[1][tn] + st_bytes + ks * 16 * B_ROWB);
            o.b[tn] = u32x4{lo[0], lo[1], hi[0], hi[1]};
        }
    };
    auto multiply = [&](const Ops& o) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) acc[tn][tm] = E::mfma(o.b[tn], o.a[tm], acc[tn][tm]);
    };

    if constexpr (NW == 8 && GEMM_PINGPONG) {
        // Eight wavefronts, two per SIMD: two groups (0-3 and 4-7; w and w + 4 share a SIMD) run the same
        // sequence of phases one phase apart, a barrier between phases.  In its read phase L(k) a wavefront
        // fetches all operands of block k from LDS into registers; in its matrix phase M(k) it issues the
        // block's matrix instructions and nothing else: on every SIMD one wavefront feeds the matrix pipe while
        // the other waits for the barrier, for LDS and for its loads.  Slot 2k: first group L(k), second
        // M(k-1); slot 2k+1: first group M(k), second L(k).  Block k is read in slots 2k and 2k+1 and those
        // reads are used up in slots 2k+1 and 2k+2: its stage takes block k + NST in slot 2k+3, from the first
        // group in its M(k+1) and from the second in its L(k+1).  Every wavefront has its share of block k in
        // LDS before the barrier that opens slot 2k: all but the loads of the NST-2 later blocks.
        const bool grp1 = wave >= NW / 2;
        Ops ops[2];
        wait_tile_loads<(NST - 2) * IPS>();
        __syncthreads();
        if (grp1) asm volatile("s_barrier" ::: "memory");
        auto step = [&](int kb, auto phase) {
            constexpr int PH = decltype(phase)::value;
            wait_tile_loads<(NST - 2) * IPS>();
            asm volatile("s_barrier" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
            read_ops(ops[0], PH * STAGE, 0);
            read_ops(ops[1], PH * STAGE, 1);
            if (grp1) issue(kb + NST - 1, (PH + NST - 1) % NST);
            __builtin_amdgcn_sched_barrier(0);
            wait_tile_loads<(NST - 2) * IPS>();
            asm volatile("s_barrier" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
            multiply(ops[0]);
            __builtin_amdgcn_sched_barrier(0);
            if (!grp1) issue(kb + NST - 1, (PH + NST - 1) % NST);
            __builtin_amdgcn_sched_barrier(0);
            multiply(ops[1]);
            __builtin_amdgcn_sched_barrier(0);
        };
        static_assert(NST >= 3, "one block in use, at least two in flight");
        for (int k0 = 0; k0 < nk; k0 += NST) {
            [&]<int... PH>(std::integer_sequence<int, PH...>) {
                ((k0 + PH < nk ? step(k0 + PH, std::integral_constant<int, PH>{}) : (void)0), ...);
            }(std::make_integer_sequence<int, NST>{});
        }
        if (!grp1) asm volatile("s_barrier" ::: "memory");   // the first group's last one
    } else {
        // Block kb: its first k step runs on operands read during block kb-1 (`ahead`), its second on operands
        // read under the first, and under the second the first operands of block kb+1 are read: the matrix
        // pipe never waits for an LDS round trip behind a barrier.  For that, block kb+1 must be complete one
        // barrier early: every wavefront checks its share of it before the barrier of block kb.
        Ops ahead;
        wait_tile_loads<(NST - 2) * IPS>();
        __syncthreads();
        read_ops(ahead, 0, 0);
        auto step = [&](int kb, auto phase) {
            constexpr int PH = decltype(phase)::value;
            // blocks up to kb+1 have landed when at most the loads of the NST-3 later blocks are still out
            wait_tile_loads<(NST - 3) * IPS>();
            asm volatile("s_barrier" ::: "memory");
            // ... for everybody, and everybody is done with block kb-1: its stage takes block kb+NST-1
            issue(kb + NST - 1, (PH + NST - 1) % NST);
            Ops second;
            read_ops(second, PH * STAGE, 1);
            __builtin_amdgcn_sched_barrier(0);
            multiply(ahead);
            __builtin_amdgcn_sched_barrier(0);
            read_ops(ahead, ((PH + 1) % NST) * STAGE, 0);
            __builtin_amdgcn_sched_barrier(0);
            multiply(second);
            __builtin_amdgcn_sched_barrier(0);
        };
        static_assert(NST >= 3, "one block in use, one read ahead, at least one in flight");
        for (int k0 = 0; k0 < nk; k0 += NST) {
            [&]<int... PH>(std::integer_sequence<int, PH...>) {
                ((k0 + PH < nk ? step(k0 + PH, std::integral_constant<int, PH>{}) : (void)0), ...);
            }(std::make_integer_sequence<int, NST>{});
        }
    }
    wait_tile_loads<0>();   // the repeated loads of the last steps must not outlive the workgroup's LDS

    // ---- epilogue: activation in fp32, round; the tile leaves through LDS ----
    // A lane holds four consecutive n of one row m: stored from there, an instruction would touch 32 rows with
    // 16 bytes each.  Every wavefront writes its 32 TM x 32 TN block into a region of its own (the stages are
    // free once every wavefront is past the loop and its loads have landed), rows padded by 16 bytes against
    // bank conflicts, and reads it back with 4 TN lanes side by side on a row: a store instruction then writes
    // whole rows of the block, 64 TN bytes each.
    __syncthreads();
    {
        constexpr int RW = 32 * TM, RB = 64 * TN, RS = RB + 16;
        static_assert(NW * RW * RS <= GemmLds<WM, WN, TM, TN>::BYTES, "LDS for the way out");
        uint8_t* reg = smem + wave * (RW * RS);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int gg = 0; gg < 4; ++gg) {
                    const f32x16& t = acc[tn][tm];
                    const u32x2 v = {E::pack2(leaky(t[4 * gg], slope), leaky(t[4 * gg + 1], slope)),
                                     E::pack2(leaky(t[4 * gg + 2], slope), leaky(t[4 * gg + 3], slope))};
                    *(u32x2*)(reg + (32 * tm + l32) * RS + 64 * tn + 16 * gg + 8 * h) = v;
                }
        constexpr int LPR = RB / 16, RPP = 64 / LPR;   // lanes per row, rows per store instruction
#pragma unroll
        for (int p = 0; p < RW / RPP; ++p) {
            const int row = p * RPP + lane / LPR, ch = lane % LPR;
            const u32x4 v = *(const u32x4*)(reg + row * RS + ch * 16);
            const int m = m0 + wm * RW + row, n = n0 + wn * (32 * TN) + ch * 8;
            if (m < M && n < N) *(u32x4*)(Cb + (size_t)m * N + n) = v;
        }
    }
}


// Small problems: 32 x 32 tiles of c, K split over the four wavefronts of the workgroup.
// A problem of few 64 x 64 tiles leaves most compute units without work, and every workgroup pulls its whole
// strip of a and b through one compute unit's memory pipeline: that, not arithmetic, is what such a launch waits
// for.  Here a workgroup owns a 32 x 32 tile (four times the workgroups, half the bytes per compute unit) and
// wavefront w the k blocks w, w + 4, w + 8, ...: it streams them through LDS stages of its own (no barrier in
// the loop: what a wavefront loads only that wavefront reads), accumulates a 32 x 32 partial result in two
// independent accumulators, and at the end the four partial results meet in LDS: wavefront q adds up, activates
// and stores columns 8q .. 8q+7 of the tile.
#ifndef GEMM_SK_NST
#define GEMM_SK_NST 4   // LDS stages per wavefront (4 KiB each); more gained nothing and a larger LDS request starts later
#endif
template <int DT>
__global__ __launch_bounds__(256) void gemm_lrelu_splitk_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ B,
                                                               uint16_t* __restrict__ C, int M, int N, int K, int tiles_m,
                                                               int tiles_n, float slope) {
    using E = Elem<DT>;
    constexpr int NST = GEMM_SK_NST, STAGE = 4096, IPS = 4;
    static_assert(NST >= 3 && 4 * NST * STAGE <= 160 * 1024 && (NST - 2) * IPS <= 63, "stages");
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, h = lane >> 5;
    const int bx = blockIdx.x;
    const int tn_i = bx % tiles_n;
    const int tm_i = (bx / tiles_n) % tiles_m;
    const int bi = bx / (tiles_n * tiles_m);
    const int m0 = tm_i * 32, n0 = tn_i * 32;
    const uint16_t* Ab = A + ((size_t)bi * M + m0) * K;
    const uint16_t* Bb = B + (size_t)bi * K * N + n0;
    uint16_t* Cb = C + (size_t)bi * M * N;
    const int nk = K / 32;
    const int mine = nk > wave ? (nk - wave + 3) / 4 : 0;   // k blocks of this wavefront: wave, wave + 4, ...

    const uint32_t lds0 = (uint32_t)(uintptr_t)(LDS_AS uint8_t*)smem;
    const uint32_t ldsw = lds0 + wave * (NST * STAGE);
    // loads: instruction j covers rows 16 j .. 16 j + 15 of a tile (64 bytes each); lane = row * 4 + chunk position
    uint32_t goff_a[2], goff_b[2];
    {
        const int nvalid = (N - n0) / 8 < 4 ? (N - n0) / 8 : 4;   // 16-byte chunks of this tile inside the matrix
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int r = 16 * j + lane / 4, pos = lane % 4;
            const int rr = r < M - 1 - m0 ? r : M - 1 - m0;
            goff_a[j] = (uint32_t)(rr * K + ((pos ^ swz_a(r)) << 3)) * 2u;
            int ch = pos ^ swz_a(r);
            ch = ch < nvalid - 1 ? ch : nvalid - 1;
            goff_b[j] = (uint32_t)(r * N + (ch << 3)) * 2u;
        }
    }
    // the i-th block of this wavefront into stage st; past its last block the last one again (nobody reads it):
    // every step issues the same number of loads.  A wavefront without blocks issues nothing.
    auto issue = [&](int i, int st) {
        if (mine == 0) return;
        const int kb = wave + 4 * (i < mine - 1 ? i : mine - 1);
        const uint16_t* sa = Ab + (size_t)kb * 32;
        const uint16_t* sb = Bb + (size_t)kb * 32 * N;
#pragma unroll
        for (int j = 0; j < 2; ++j) lds_dma16(ldsw + st * STAGE + j * 1024, sa, goff_a[j]);
#pragma unroll
        for (int j = 0; j < 2; ++j) lds_dma16(ldsw + st * STAGE + 2048 + j * 1024, sb, goff_b[j]);
    };
    // operands (stage 0): a: row l32, chunk 2 ks + h; b^T: 8 bytes of row (k) 8 h + 4 hi + x, elements 16 g1 + 4 y .. +3
    uint32_t a_addr[2], b_addr[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) a_addr[ks] = ldsw + l32 * 64 + (((2 * ks + h) ^ swz_a(l32)) << 4);
    {
        const int x = (lane & 15) >> 2, y = lane & 3, g1 = (lane >> 4) & 1;
#pragma unroll
        for (int hi = 0; hi < 2; ++hi) {
            const int row = 8 * h + 4 * hi + x, chunk = 2 * g1 + (y >> 1);
            b_addr[hi] = ldsw + 2048 + row * 64 + ((chunk ^ swz_a(row)) << 4) + ((y & 1) << 3);
        }
    }
    f32x16 acc[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[ks][r] = 0.f;

#pragma unroll
    for (int s = 0; s < NST - 1; ++s) issue(s, s);
    auto step = [&](int i, auto phase) {
        constexpr int PH = decltype(phase)::value;
        // block i has landed when at most the loads of the NST-2 later blocks are still out
        wait_tile_loads<(NST - 2) * IPS>();
        u32x4 a[2], b[2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            a[ks] = lds_read_b128(a_addr[ks] + PH * STAGE);
            const u32x2 lo = lds_read_tr16(b_addr[0] + PH * STAGE + ks * 16 * 64);
            const u32x2 hi = lds_read_tr16(b_addr[1] + PH * STAGE + ks * 16 * 64);
            b[ks] = u32x4{lo[0], lo[1], hi[0], hi[1]};
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) acc[ks] = E::mfma(b[ks], a[ks], acc[ks]);
        // the operands are in registers: the stage takes this wavefront's block i + NST - 1
        issue(i + NST - 1, (PH + NST - 1) % NST);
    };
    for (int i0 = 0; i0 < mine; i0 += NST) {
        [&]<int... PH>(std::integer_sequence<int, PH...>) {
            ((i0 + PH < mine ? step(i0 + PH, std::integral_constant<int, PH>{}) : (void)0), ...);
        }(std::make_integer_sequence<int, NST>{});
    }
    wait_tile_loads<0>();   // the repeated loads of the last steps must have landed before LDS is used again
    __syncthreads();
    // the partial results meet: [wavefront][group of four registers][lane] as 16 bytes each
    {
        float* part = (float*)smem;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            f32x4 t;
#pragma unroll
            for (int e = 0; e < 4; ++e) t[e] = acc[0][4 * g + e] + acc[1][4 * g + e];
            *(f32x4*)(part + ((wave * 4 + g) * 64 + lane) * 4) = t;
        }
        __syncthreads();
        f32x4 t = *(const f32x4*)(part + ((0 * 4 + wave) * 64 + lane) * 4);
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const f32x4 u = *(const f32x4*)(part + ((w * 4 + wave) * 64 + lane) * 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) t[e] += u[e];
        }
        // registers 4 q .. 4 q + 3 of lane (l32, h) are c[m0 + l32][n0 + 8 q + 4 h .. + 3]
        const int m = m0 + l32, n = n0 + 8 * wave + 4 * h;
        if (m < M && n < N) {
            const u32x2 v = {E::pack2(leaky(t[0], slope), leaky(t[1], slope)), E::pack2(leaky(t[2], slope), leaky(t[3], slope))};
            *(u32x2*)(Cb + (size_t)m * N + n) = v;
        }
    }
}

// any shape: one thread per element of c
template <int DT>
__global__ __launch_bounds__(256) void gemm_lrelu_plain_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ B,
                                                              uint16_t* __restrict__ C, long long total, int M, int N, int K,
                                                              float slope) {
    using E = Elem<DT>;
    for (long long idx = (long long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long long)gridDim.x * 256) {
        const int n = (int)(idx % N);
        const long long bm = idx / N;          // batch * M + m
        const long long bi = bm / M;
        const uint16_t* a = A + (size_t)bm * K;
        const uint16_t* b = B + (size_t)bi * K * N + n;
        float t = 0.f;
        for (int k = 0; k < K; ++k) t = __builtin_fmaf(E::widen(a[k]), E::widen(b[(size_t)k * N]), t);
        const uint32_t p = E::pack2(leaky(t, slope), 0.f);
        C[idx] = (uint16_t)(p & 0xFFFFu);
    }
}

template <int DT, int WM, int WN, int TM, int TN>
hipError_t launch_tiles(const GemmLaunch& g) {
    constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN;
    constexpr unsigned lds_bytes = (unsigned)GemmLds<WM, WN, TM, TN>::BYTES;
    int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    const long long blocks = (long long)tiles_m * tiles_n * g.batch;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    const uint16_t* a = (const uint16_t*)g.a;
    const uint16_t* b = (const uint16_t*)g.b;
    uint16_t* c = (uint16_t*)g.c;
    int M = g.M, N = g.N, K = g.K;
    float slope = g.slope;
    void* args[] = {&a, &b, &c, &M, &N, &K, &tiles_m, &tiles_n, &slope};
    const void* fn = reinterpret_cast<const void*>(&gemm_lrelu_kernel<DT, WM, WN, TM, TN>);
    static std::atomic<uint64_t> told{0};   // per kernel instance: the devices whose runtime knows its LDS size
    if (const hipError_t e = announce_lds(fn, lds_bytes, told); e != hipSuccess) return e;
    return hipLaunchKernel(fn, dim3((unsigned)blocks), dim3(WM * WN * 64), args, lds_bytes, (hipStream_t)g.stream);
}

template <int DT>
hipError_t launch_plain(const GemmLaunch& g) {
    const uint16_t* a = (const uint16_t*)g.a;
    const uint16_t* b = (const uint16_t*)g.b;
    uint16_t* c = (uint16_t*)g.c;
    long long total = (long long)g.batch * g.M * g.N;
    int M = g.M, N = g.N, K = g.K;
    float slope = g.slope;
    const long long groups = (total + 255) / 256;
    const unsigned grid = (unsigned)(groups < 65536 ? groups : 65536);
    void* args[] = {&a, &b, &c, &total, &M, &N, &K, &slope};
    return hipLaunchKernel(reinterpret_cast<const void*>(&gemm_lrelu_plain_kernel<DT>), dim3(grid), dim3(256), args, 0,
                           (hipStream_t)g.stream);
}


template <int DT>
hipError_t launch_splitk(const GemmLaunch& g) {
    int tiles_m = (g.M + 31) / 32, tiles_n = (g.N + 31) / 32;
    const long long blocks = (long long)tiles_m * tiles_n * g.batch;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    const uint16_t* a = (const uint16_t*)g.a;
    const uint16_t* b = (const uint16_t*)g.b;
    uint16_t* c = (uint16_t*)g.c;
    int M = g.M, N = g.N, K = g.K;
    float slope = g.slope;
    void* args[] = {&a, &b, &c, &M, &N, &K, &tiles_m, &tiles_n, &slope};
    constexpr unsigned lds_bytes = 4u * GEMM_SK_NST * 4096u;
    const void* fn = reinterpret_cast<const void*>(&gemm_lrelu_splitk_kernel<DT>);
    static std::atomic<uint64_t> told{0};   // per kernel instance: the devices whose runtime knows its LDS size
    if (const hipError_t e = announce_lds(fn, lds_bytes, told); e != hipSuccess) return e;
    return hipLaunchKernel(fn, dim3((unsigned)blocks), dim3(256), args, lds_bytes, (hipStream_t)g.stream);
}
template <int DT>
hipError_t dispatch(const GemmLaunch& g) {
    switch (gemm_path_of(g.batch, g.M, g.N, g.K)) {
        case 1: return launch_tiles<DT, 4, 2, 2, 4>(g);   // 256 x 256, eight wavefronts of 64 x 128
        case 2: return launch_tiles<DT, 2, 2, 2, 2>(g);   // 128 x 128, four wavefronts of 64 x 64
        case 3: return launch_tiles<DT, 2, 2, 1, 1>(g);   // 64 x 64, four wavefronts of 32 x 32
        case 5: return launch_splitk<DT>(g);   // 32 x 32, K split over the four wavefronts
        default: return launch_plain<DT>(g);
    }
}

}  // namespace

hipError_t gemm_launch(const GemmLaunch& g) { return g.dtype == 0 ? dispatch<0>(g) : dispatch<1>(g); }
