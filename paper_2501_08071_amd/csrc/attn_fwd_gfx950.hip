// Fused multi-head attention forward for gfx950 (MI355X): O = softmax(Q K^T * scale [+ causal]) V
// and the per-row logsumexp, one pass over K/V with a running (online) softmax.
//
// The operation is the "flash-attention" kernel class of the paper's Table 2; the paper's
// subject is the order of memory and compute instructions inside such a fixed kernel
// (Sections 2.4, 3.5).  Here that order is set by hand for CDNA4.
//
// Work split
//   workgroup = NW wavefronts, each owning 32 consecutive query rows of one (b,h);
//   K/V stream through LDS in blocks of BC keys shared by the whole workgroup (64 in the
//   alternating-phase loop, 32 in the interleaved one).
//
// K/V movement
//   global -> LDS directly (global_load_lds_dwordx4, no VGPR staging), ATTN_NBUF buffers of 32 keys per
//   tensor (half as many of 64), loads issued about that many blocks ahead of their use.  Such a load writes 1 KiB of consecutive
//   LDS per wavefront, so rows cannot be padded; bank conflicts are avoided by an XOR swizzle of the
//   16-byte chunk index within each row, applied on the global-address side.
//
// Schedule
//   The two wavefronts of a SIMD share one issue port for vector and matrix instructions, and the
//   vector work of 32 keys (16 fma, 16 exp, 16 add, 8 convert per lane) is of the order of their
//   matrix work (16 matrix instructions at D = 128, 8 at D = 64).  Two loop structures:
//   D >= 64  two groups of wavefronts run matrix phases M(k): S(k) = K(k).Q^T, O += V(k-1)^T.P(k-1)^T
//            and vector phases V(k): P(k) = exp2(c S(k) - m) half a block apart, a barrier between
//            phases: on every SIMD one wavefront feeds the matrix pipe while the other has the vector port;
//            64 keys per block, so that a phase is 32 (D = 128) or 16 (D = 64) matrix instructions long;
//   D = 32   every wavefront interleaves the matrix instructions of S(k+1) and O += V(k-1)^T.P(k-1)^T
//            with the vector work of P(k); one barrier per two blocks.
//   The softmax reference m of a row is the maximum of its first block; it is only taken again when a
//   block's weight sum overflows a threshold (no row maxima on the hot path).  After a reference had to
//   move, the alternating loop takes the row maxima first for the next ATTN_WARY blocks (a peaked
//   softmax moves its references block after block at first, and would compute every block's weights twice).
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
#include <type_traits>

#include "attn_launch.h"
#include "gfx950_common.h"
#include "attn_device.h"

namespace {

using namespace gfx950;
using namespace attn_device;

template <int N>
__device__ __forceinline__ void wait_block_loads() { wait_lds_dma<N>(); }

extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

template <int DT, int D, bool CAUSAL, int NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(ATTN_WPE, ATTN_WPE)))
void attn_fwd_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                     void* __restrict__ o, float* __restrict__ lse, int S, int BH, int nqt, float c_arg,
                     uint32_t qsign, int o16) {
    using E = Elem<DT>;
    // Row sum of the weights.  By one fp32 addition per weight, or -- binary16 at D = 64 -- from the rounded weights, two
    // per dot instruction.  A dot instruction issued while the other wavefront of the SIMD streams matrix instructions
    // waits for a gap in that stream (measured: include/probe.h, probe_issue_share), so it only pays where the vector
    // phase outlasts the other wavefront's matrix phase and the dot instructions can stand at its end: D = 64.
    constexpr bool SUM_DOT = ATTN_F16_SUM_DOT != 0 && DT == 0 && D == 64;
    constexpr int BR = NW * 32;        // query rows per workgroup, 32 per wavefront
    // keys per block: 32, or 64 (D = 128) and 128 (D = 64) in the alternating-phase loop (a phase then has more work
    // between its two barriers; half as many buffers, each larger)
    constexpr int BC = attn_block_keys(D);
    constexpr int NSUB = BC / 32;      // 32-key sub-blocks (one accumulator tile of S each)
    constexpr int NBUF = attn_buffers(D);   // LDS buffers per tensor (a power of two); block k lives in buffer k % NBUF
    // Two loop structures (see below): D = 128 and 64 alternate matrix and vector phases between two
    // groups of wavefronts; D = 32, where the vector work far outweighs the matrix work, interleaves both
    // in every wavefront.
    constexpr bool PP = attn_alternating(D);
    constexpr int BEV = ATTN_BARRIER_EVERY;    // interleaved loop: slots per workgroup barrier (1 or 2)
    static_assert((BEV == 1 || BEV == 2) && NBUF % BEV == 0, "barrier period");
    // block k's step issues the load of K(k + KAHEAD) and of V(k + VAHEAD), into buffers nobody reads
    // any more (last read before the previous barrier, by either group)
    constexpr int KAHEAD = PP ? NBUF - 1 : NBUF - (BEV - 1);
    constexpr int VAHEAD = PP ? NBUF - 2 : KAHEAD - 2;
    static_assert(PP ? KAHEAD + VAHEAD >= 5 : KAHEAD - 1 >= BEV + 1, "too few buffers for the loads that have to be in flight");
    constexpr int KSTEPS = D / 16;     // contraction steps of Q.K^T
    constexpr int DB = D / 32;         // 32-wide blocks of the head dimension
    constexpr int ROWB = 2 * D;        // bytes per K/V row
    constexpr int BLKB = BC * ROWB;    // bytes per key block
    constexpr int CPR = D / 8;         // 16-byte chunks per row
    constexpr int RPI = 1024 / ROWB;   // rows written by one direct-to-LDS load instruction
    constexpr int IPT = BC / RPI;      // such instructions per block and tensor
    constexpr int IPW = IPT >= NW ? IPT / NW : 1;   // ... per loading wavefront
    constexpr int LOADERS = IPT / IPW;              // wavefronts that issue loads
    static_assert((BC == 32 || (PP && (BC == 64 || (BC == 128 && D == 64)))) && IPT % IPW == 0 && LOADERS <= NW, "load split");
    // LDS: K buffers 0..NBUF-1 | V buffers 0..NBUF-1

    const float c = c_arg;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31;
    const int h = lane >> 5;

    // Workgroup -> tile.  Workgroups are handed to the eight XCDs in turn (workgroup b runs on XCD b % 8,
    // each with an L2 of its own), in the order of their number.  The (b,h) pairs are therefore dealt out
    // by XCD (bh % 8 = b % 8) and, on an XCD, taken ATTN_HEAD_GROUP at a time: all query tiles of those
    // few heads -- heaviest first: under the causal mask query tile t reads t+1 key tiles -- before the
    // next heads.  Tiles that stream the same K and V then run at the same time on the same L2.  With a
    // number of heads that does not divide that way: heaviest tiles first over all heads.
    int bh, qt;
    {
        constexpr int GS = ATTN_HEAD_GROUP;
        const int b = blockIdx.x;
        if (GS > 0 && BH % (8 * GS) == 0 && (gridDim.x & 7) == 0) {
            const int x = b & 7, j = b >> 3;          // XCD, and position in its queue
            const int per = GS * nqt;                 // tiles per group of heads
            const int p = j / per, r = j - p * per;
            qt = r / GS;
            bh = x + 8 * (p * GS + (r - qt * GS));
        } else {
            bh = b % BH;
            qt = b / BH;
        }
        if (CAUSAL) qt = nqt - 1 - qt;
    }
    const int q0 = qt * BR;
    const int qw0 = q0 + 32 * wave;          // first query row of this wavefront
    const int qrow = qw0 + l32;              // this lane's query row (may lie beyond S on the last tile)
    const int qrow_ld = qrow < S ? qrow : S - 1;

    const size_t head = (size_t)bh * S * D;
    const uint16_t* qh = q + head;
    const uint16_t* kh = k + head;
    const uint16_t* vh = v + head;

    const int kv_end = CAUSAL ? (q0 + BR < S ? q0 + BR : S) : S;
    const int nblk = (kv_end + BC - 1) / BC;       // key blocks the workgroup streams
    // kd: the first block this wavefront needs a mask for -- the one on its causal diagonal, or the
    // ragged last block of the sequence (which may not exist: then kd == nblk).  Later blocks of the
    // workgroup are masked entirely for it.
    const int nfull = S / BC;
    auto first_masked = [&](int w) {
        const int d = CAUSAL ? (q0 + 32 * w) / BC : nfull;
        return d < nfull ? d : nfull;
    };
    const int kd = first_masked(wave);
    const int last_max = nblk - 1;   // the last block any wavefront of the workgroup works on

    // ---- direct-to-LDS block loads ----
    // instruction `inst` fills LDS bytes [inst*1024, +1024) of a block buffer = rows inst*RPI.. ; lane
    // writes chunk position lane%CPR of row lane/CPR and therefore fetches source chunk pos ^ swz(row)
    const uint32_t lds0 = (uint32_t)(uintptr_t)(LDS_AS uint8_t*)smem;
    uint32_t goff[IPW];   // byte offset of this lane's source chunk inside a block
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
        const int r = (wave * IPW + i) * RPI + lane / CPR;
        goff[i] = (r * D + (((lane % CPR) ^ swz<D>(r)) << 3)) * 2;
    }
    // the same for the ragged last block of the sequence: rows past the end (masked later) point at the
    // last valid row
    uint32_t goff_r[IPW];
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
        const int over = nfull * BC + (wave * IPW + i) * RPI + lane / CPR - (S - 1);
        goff_r[i] = over > 0 ? goff[i] - over * ROWB : goff[i];
    }
    const uint32_t lds_wave = lds0 + wave * IPW * 1024;
    // One load instruction: piece i (0..IPW-1) of K block `blk` (which = 0) or V block `blk` (which = 1)
    // into LDS at lds_wave + dst.  A block index past the end of the stream is replaced by the last
    // block (a copy nobody reads, into a buffer nobody needs any more), so that every slot issues the
    // same number of loads and the code has no branch; the address arithmetic is scalar.
    auto issue_piece = [&](int which, int blk, int i, uint32_t dst) {
        if (LOADERS < NW && wave >= LOADERS) return;
        if constexpr (ATTN_DEBUG_POISON != 0) {
            // Debug build: what this load is about to overwrite is first filled with NaN patterns.  A wavefront that
            // still reads the buffer -- a load issued a barrier too early -- then shows in the output instead of quietly
            // reading the old block or the new one.
            *(LDS_AS u32x4*)(uintptr_t)(lds_wave + dst + lane * 16) = u32x4{0x7fff7fffu, 0x7fff7fffu, 0x7fff7fffu, 0x7fff7fffu};
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
        const int b = blk < nblk - 1 ? blk : nblk - 1;
        const uint16_t* src = (which ? vh : kh) + (size_t)b * (BC * D);
        lds_dma16(lds_wave + dst, src, b >= nfull ? goff_r[i] : goff[i]);
    };
    auto issue_load = [&](int which, int blk) {
#pragma unroll
        for (int i = 0; i < IPW; ++i) issue_piece(which, blk, i, (NBUF * which + (blk & (NBUF - 1))) * BLKB + i * 1024);
    };
    // blocks K(0 .. KAHEAD-1) and V(0 .. VAHEAD-1) start the pipeline, in the order of their use;
    // slot k adds K(k + KAHEAD) and V(k + VAHEAD)
    issue_load(0, 0);
#pragma unroll
    for (int j = 1; j < KAHEAD; ++j) {
        issue_load(0, j);
        if (j - 1 < VAHEAD) issue_load(1, j - 1);
    }

    // the last V buffer is read by slot 0 (with all-zero weights) before anything was loaded into it:
    // make its contents finite
    {
        constexpr int PER = BLKB / (NW * 64);   // bytes per thread
        static_assert(PER % 16 == 0 || PER == 8 || PER == 4, "zero fill");
        uint8_t* vb3 = smem + (2 * NBUF - 1) * BLKB + tid * PER;
        if constexpr (PER == 4) *(uint32_t*)vb3 = 0u;
        if constexpr (PER == 8) *(u32x2*)vb3 = u32x2{0u, 0u};
#pragma unroll
        for (int i = 0; i < PER / 16; ++i) *(u32x4*)(vb3 + 16 * i) = u32x4{0u, 0u, 0u, 0u};
    }

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
    float m_run = -INFINITY;   // reference maximum (base-2 units) everything accumulated so far was taken against
    float l_run = 0.f;         // this lane's share of the running row sum
    float m_ref;               // main loop: reference maximum of the block in hand

    // ---- per-lane LDS addresses (loop invariant; buffer parts become immediate offsets) ----
    // K operand of step ks: row l32 of the block, source chunk 2 ks + h
    uint32_t kaddr[KSTEPS];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) kaddr[ks] = lds0 + l32 * ROWB + (((2 * ks + h) ^ swz<D>(l32)) << 4);
    // V^T operand of (t, half hi, block i): lane addresses 8 bytes of row 16 t + 8 hi + 4 h + x,
    // elements 32 i + 16 g1 + 4 y .. +3, where x = (lane%16)/4, y = lane%4, g1 = (lane/16)%2
    uint32_t vaddr[2][DB];
    {
        const int x = (lane & 15) >> 2, y = lane & 3, g1 = (lane >> 4) & 1;
#pragma unroll
        for (int hi = 0; hi < 2; ++hi)
#pragma unroll
            for (int i = 0; i < DB; ++i) {
                const int chunk = 4 * i + 2 * g1 + (y >> 1);
                vaddr[hi][i] = lds0 + NBUF * BLKB + (8 * hi + 4 * h + x) * ROWB +
                               ((chunk ^ swz<D>(8 * hi + 4 * h + x)) << 4) + ((y & 1) << 3);
            }
    }

    constexpr int NT = BC / 16;                      // 16-key steps of the second product
    constexpr int NU = NSUB * KSTEPS + NT * DB;      // matrix instructions (units, operand fetches) per block
    auto fetch_v = [&](int VB, int tt, int i) {
        u32x2 lo = lds_read_tr16(vaddr[0][i] + VB * BLKB + 16 * tt * ROWB);
        u32x2 hi = lds_read_tr16(vaddr[1][i] + VB * BLKB + 16 * tt * ROWB);
        return u32x4{lo[0], lo[1], hi[0], hi[1]};
    };

    // scale the accumulators when the reference maximum of some row moved (rare after the first blocks)
    auto rescale_o = [&](float alpha) {
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_o[i][r] *= alpha;
    };

    // O^T += V(j)^T . P(j)^T, plain order (used once or twice per wavefront)
    auto pv_plain = [&](const u32x4 (&pf)[2], int VB) {
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int i = 0; i < DB; ++i) {
                acc_o[i] = E::mfma(fetch_v(VB, tt, i), pf[tt], acc_o[i]);
                __builtin_amdgcn_sched_barrier(0);   // no hoisting of all the reads: registers are scarce
            }
    };

    if constexpr (PP) {
        // first operands of the next matrix phase, read in the vector phase before it (the matrix phase is the one
        // short of issue slots: every operand read moved out of it shortens it)
        constexpr int FETCH = ATTN_PP_FETCH < NSUB * KSTEPS ? ATTN_PP_FETCH : NSUB * KSTEPS;   // all of them K operands
        u32x4 pre[FETCH];
        int wary = 0;    // blocks still to go whose row maxima are taken before the weights (wavefront-uniform)
        f32x16 s[NSUB];  // S(k): written by M(k), read by V(k)
        u32x4 pf[NT];    // weights of block k-1 (matrix operand layout) for M(k)

        // Two groups of wavefronts (0 .. NW/2-1 and NW/2 .. NW-1; wavefront w and w + NW/2 share a SIMD) run
        // the same sequence of phases half a block apart: while one group is in its matrix phase M(k) --
        // S(k) = K(k).Q^T and O^T += V(k-1)^T.P(k-1)^T, nothing but matrix instructions, their LDS operand reads
        // and the block loads -- the other is in its vector phase V(k') -- row maximum, weights, row sum --
        // so the two wavefronts of a SIMD never compete for the same pipe.  A workgroup barrier separates the
        // phases.
        auto m_phase = [&](int kb, auto phase) {
            constexpr int PH = decltype(phase)::value;
            constexpr int KB = PH;                             // buffer of K(k)
            constexpr int VB = (PH + NBUF - 1) & (NBUF - 1);   // buffer of V(k-1)
            u32x4 opnd[NU];
            auto fetch = [&](auto unit) {
                constexpr int U = decltype(unit)::value;
                constexpr int NQK = NSUB * KSTEPS;
                if constexpr (U < NQK) opnd[U] = lds_read_b128(kaddr[U % KSTEPS] + KB * BLKB + (U / KSTEPS) * 32 * ROWB);
                else opnd[U] = fetch_v(VB, (U - NQK) / DB, (U - NQK) % DB);
            };
            auto unit_step = [&](auto unit) {
                constexpr int U = decltype(unit)::value;
                constexpr int NQK = NSUB * KSTEPS;
                if constexpr (U + FETCH < NU) fetch(std::integral_constant<int, U + FETCH>{});
                if constexpr (U < NQK) {
                    constexpr int sub = U / KSTEPS, ks = U % KSTEPS;
                    if constexpr (ks == 0) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) s[sub][r] = 0.f;
                    }
                    s[sub] = E::mfma(opnd[U], qf[ks], s[sub]);
                } else {
                    constexpr int tt = (U - NQK) / DB, i = (U - NQK) % DB;
                    acc_o[i] = E::mfma(opnd[U], pf[tt], acc_o[i]);
                }
                // the 2 IPW load instructions of this block, evenly spread
                constexpr int NP = 2 * IPW, GAP = NU / NP;
                if constexpr (U % GAP == GAP / 2 && U / GAP < NP) {
                    constexpr int P = U / GAP;
                    constexpr int W = P / IPW, AHEAD = W ? VAHEAD : KAHEAD;
                    issue_piece(W, kb + AHEAD, P % IPW, (NBUF * W + ((PH + AHEAD) & (NBUF - 1))) * BLKB + (P % IPW) * 1024);
                }
                __builtin_amdgcn_sched_barrier(0);
            };
#pragma unroll
            for (int u = 0; u < FETCH; ++u) opnd[u] = pre[u];
            [&]<int... U>(std::integer_sequence<int, U...>) {
                (unit_step(std::integral_constant<int, U>{}), ...);
            }(std::make_integer_sequence<int, NU>{});
        };
        auto v_phase = [&](int kb, auto phase) {
            constexpr int PH = decltype(phase)::value;
            constexpr int KB1 = (PH + 1) & (NBUF - 1);   // buffer of K(k+1)
            if (kb >= kd) {
                // A block cut by the causal diagonal or by the end of the sequence: masked logits become
                // -3e38 (times c >= 1e-30 that is far below any real logit and the weight comes out as an
                // exact 0); past the diagonal that is all of them and the phase changes nothing.
                const int lim = (CAUSAL ? qrow_ld : S - 1) - kb * BC - 4 * h;
#pragma unroll
                for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int off = 32 * sub + 8 * (r / 4) + (r % 4);
                        s[sub][r] = off > lim ? -3.0e38f : s[sub][r];
                    }
            }
            float psum = 0.f;
            auto weights = [&](float nm) {
                psum = 0.f;
#pragma unroll
                for (int sub = 0; sub < NSUB; ++sub) {
                    f32x16 p;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        p[r] = __builtin_amdgcn_exp2f(fmaf(s[sub][r], c, nm));
                        if (r % 2 == 1) pf[2 * sub + r / 8][(r % 8) / 2] = E::pack2(p[r - 1], p[r]);
                        // bfloat16 keeps only 8 bits, which would cost the logsumexp its 1e-3 accuracy: sum the fp32 values
                        if (!SUM_DOT) psum += p[r];
                    }
                }
                if constexpr (SUM_DOT) {
                    __builtin_amdgcn_sched_barrier(0);   // the dot instructions last, when the other wavefront's matrix phase is over
#pragma unroll
                    for (int tt = 0; tt < NT; ++tt)
#pragma unroll
                        for (int e = 0; e < 4; ++e) psum = E::dot2_ones(pf[tt][e], psum);
                }
            };
            constexpr int WARY = ATTN_WARY;
            const bool look_first = kb == 0 || (WARY > 0 && wary > 0);
            if (!look_first) weights(-m_ref);
            const bool outgrown = !look_first && __builtin_amdgcn_ballot_w64(!(psum <= __builtin_exp2f(ATTN_MAX_SLACK))) != 0;
            if (look_first || outgrown) {
                float mx = vmax3(s[0][0], s[0][1], s[0][2]);
#pragma unroll
                for (int j = 1; j < 7; ++j) mx = vmax3(mx, s[0][2 * j + 1], s[0][2 * j + 2]);
                mx = vmax(mx, s[0][15]);
#pragma unroll
                for (int sub = 1; sub < NSUB; ++sub) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) mx = vmax3(mx, s[sub][2 * j], s[sub][2 * j + 1]);
                }
                const float m = vmax(mx, other_half(mx)) * c;    // c >= 0
                // after an overflow (and in the first block) the reference goes to the true maximum; while only
                // looking first, it moves where a logit outgrows it by more than the slack
                const float m_new = (kb == 0 || outgrown) ? (m > m_ref ? m : m_ref) : (m > m_ref + ATTN_MAX_SLACK ? m : m_ref);
                const bool moved = __builtin_amdgcn_ballot_w64(m_new != m_ref) != 0;
                if (moved) {
                    const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);
                    l_run *= alpha;
                    rescale_o(alpha);
                    m_ref = m_new;
                }
                weights(-m_ref);
                if (WARY > 0) wary = (outgrown || (moved && kb != 0)) ? WARY : wary - (wary > 0);
            }
            l_run += psum;
#pragma unroll
            for (int u = 0; u < FETCH; ++u) pre[u] = lds_read_b128(kaddr[u % KSTEPS] + KB1 * BLKB + (u / KSTEPS) * 32 * ROWB);
        };

#pragma unroll
        for (int tt = 0; tt < NT; ++tt) pf[tt] = u32x4{0u, 0u, 0u, 0u};
        m_ref = -INFINITY;
        const bool grp1 = wave >= NW / 2;
        // prologue: K(0), the first load, has to be there for the first operand reads
        wait_block_loads<(KAHEAD + VAHEAD - 1) * IPW>();
        __syncthreads();
#pragma unroll
        for (int u = 0; u < FETCH; ++u) pre[u] = lds_read_b128(kaddr[u % KSTEPS] + (u / KSTEPS) * 32 * ROWB);
        if (grp1) asm volatile("s_barrier" ::: "memory");   // the second group starts half a block late

        // In the order of issue K(j) is load number 2 j (K(0) number 1) and V(j) number 2 j + 3 (times IPW
        // pieces); before M(k), KAHEAD + VAHEAD + 2 k are out.  The barriers alternate: first group into M(k),
        // second group into M(k) (= first group into V(k)), ...  M(k) reads K(k) and V(k-1), V(k) reads the
        // first operands of K(k+1).  A wavefront's check stands in front of its own M(k); what the other group
        // starts one barrier later must be covered by it as well: the first group's V(k) needs K(k+1), the
        // first group's M(k+1) needs K(k+1) and V(k) from the second group's check.  So every wavefront makes
        // sure of its share of K(k+1) and V(k), load number 2 k + 3: all but the last KAHEAD + VAHEAD - 3.
        constexpr int IN_FLIGHT = (KAHEAD + VAHEAD - 3) * IPW;
        auto block = [&](int kb, auto phase) {
            wait_block_loads<IN_FLIGHT>();
            asm volatile("s_barrier" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
            // Where both wavefronts of a SIMD want the issue port the arbiter prefers the older one: without a priority
            // the second group's matrix phases (younger wavefronts next to older ones in their vector phase) take 12 %
            // longer than the first group's.  The wavefront that feeds the matrix pipe goes first.
            if constexpr (ATTN_PP_PRIO_M != ATTN_PP_PRIO_V) __builtin_amdgcn_s_setprio(ATTN_PP_PRIO_M);
            m_phase(kb, phase);
            asm volatile("s_barrier" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (ATTN_PP_PRIO_M != ATTN_PP_PRIO_V) __builtin_amdgcn_s_setprio(ATTN_PP_PRIO_V);
            v_phase(kb, phase);
            __builtin_amdgcn_sched_barrier(0);
        };
        // The second product of a wavefront's last block, all operand reads first.
        auto closing_product = [&](int VB) {
            u32x4 a[NT][DB];
#pragma unroll
            for (int tt = 0; tt < NT; ++tt)
#pragma unroll
                for (int i = 0; i < DB; ++i) a[tt][i] = fetch_v(VB, tt, i);
#pragma unroll
            for (int tt = 0; tt < NT; ++tt)
#pragma unroll
                for (int i = 0; i < DB; ++i) acc_o[i] = E::mfma(a[tt][i], pf[tt], acc_o[i]);
        };
        // Under the causal mask a wavefront is done with its diagonal block kd: every later block of the
        // workgroup is masked entirely for it.  In the time of block kd+1 it adds the second product of
        // block kd; from then on it only issues its share of the block loads and keeps the barriers.
        const int last_w = CAUSAL && kd < last_max ? kd : last_max;
        for (int k0 = 0; k0 <= last_w; k0 += NBUF) {
            [&]<int... PH>(std::integer_sequence<int, PH...>) {
                ((k0 + PH <= last_w ? block(k0 + PH, std::integral_constant<int, PH>{}) : (void)0), ...);
            }(std::make_integer_sequence<int, NBUF>{});
        }
        for (int kb = last_w + 1; kb <= last_max; ++kb) {
            wait_block_loads<IN_FLIGHT>();
            asm volatile("s_barrier" ::: "memory");
            if (kb == last_w + 1) closing_product(last_w & (NBUF - 1));
#pragma unroll
            for (int P = 0; P < 2 * IPW; ++P) {
                const int W = P / IPW, AHEAD = W ? VAHEAD : KAHEAD;
                issue_piece(W, kb + AHEAD, P % IPW, (NBUF * W + ((kb + AHEAD) & (NBUF - 1))) * BLKB + (P % IPW) * 1024);
            }
            asm volatile("s_barrier" ::: "memory");
        }
        if (!grp1) asm volatile("s_barrier" ::: "memory");   // the first group's last one
        // A wavefront that went through to the workgroup's last block still has that block's second
        // product open.  Every wavefront made sure of its share of V(last) two blocks ago at the latest,
        // and has passed a barrier since.
        if (last_w == last_max) closing_product(last_max & (NBUF - 1));
        m_run = m_ref;
    } else {
        // first ATTN_FETCH operands of the next slot, read before its barrier (so that the matrix pipe does not
        // sit idle for an LDS round trip after every barrier)
        constexpr int FETCH = ATTN_FETCH < KSTEPS ? ATTN_FETCH : KSTEPS;   // all of them K operands
        u32x4 pre[FETCH];

        // Slot k of the pipeline (PH = k % NBUF fixes every LDS offset).  Every wavefront: wait for its own
        // loads of K(k+2) and V(k-1) (issued NBUF-2 slots ago, so newer ones may stay in flight), barrier.
        // Then one straight line for every wavefront and every block: s_cur holds S(k) on entry, s_nxt
        // receives S(k+1); pf_prv holds the weights of block k-1, pf_cur receives those of block k.  From
        // block kd on the masked logits are first replaced by a huge negative number; past the causal
        // diagonal that is all of them, the weights come out as zeros and the slot changes nothing (the
        // wavefront would otherwise only wait for the others at the next barrier).
        auto slot = [&](int kb, auto phase, f32x16& s_cur, f32x16& s_nxt, u32x4 (&pf_prv)[2], u32x4 (&pf_cur)[2]) {
            constexpr int PH = decltype(phase)::value;
            constexpr int KB = (PH + 1) & (NBUF - 1);          // buffer of K(k+1)
            constexpr int KB2 = (PH + 2) & (NBUF - 1);         // buffer of K(k+2)
            constexpr int VB = (PH + NBUF - 1) & (NBUF - 1);   // buffer of V(k-1)
            // A barrier every BEV slots.  Before slot k issues its own loads, 2 (k + KAHEAD - 1) are out; the
            // slots up to the next barrier read K(k+2) .. K(k+BEV+1) (the last of them is load number
            // 2 (k+BEV+1) at most) and V(k-1) .. V(k+BEV-2), which come earlier in the order of issue.
            if constexpr (PH % BEV == 0) {
                wait_block_loads<(2 * (KAHEAD - 1) - 2 * (BEV + 1)) * IPW>();
                // ... landed for everybody; nobody still reads the buffers the next BEV slots load into.  The
                // bare instruction, not the fenced barrier: the operand reads issued just above stay in flight
                // across it (they read K(k+2), which nobody overwrites before this wavefront has used them).
                asm volatile("s_barrier" ::: "memory");
            }

            if (kb >= kd) {
                // A block cut by the causal diagonal or by the end of the sequence: masked logits become
                // -3e38 (times c >= 1e-30 that is far below any real logit and the weight comes out as an
                // exact 0), and the reference maximum is taken again, over what is left.
                const int lim = (CAUSAL ? qrow_ld : S - 1) - kb * BC - 4 * h;
                float m = -3.0e38f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int off = 8 * (r / 4) + (r % 4);
                    s_cur[r] = off > lim ? -3.0e38f : s_cur[r];
                    m = fmaxf(m, s_cur[r]);
                }
                m = fmaxf(m, other_half(m)) * c;
                m_ref = m > m_run + ATTN_MAX_SLACK ? m : m_run;
            }
            // Units 0 .. KSTEPS - 1: S(k+1) = K(k+1).Q^T ; units KSTEPS .. NU - 1: O^T += V(k-1)^T.P(k-1)^T.
            // A unit is: the LDS read of the operand ATTN_FETCH units ahead, one matrix instruction on the
            // unit's operand, and a share of the vector work: its part of the 16 weights of block k.  Their
            // reference maximum m_ref is the one everything so far was taken against (so the exponentials
            // start at once); no row maximum is taken here.  The order written here is the order issued:
            // nothing moves across a unit.
            f32x16 p;
            float psum = 0.f;
            const float neg_m = -m_ref;
            u32x4 opnd[NU];
            auto fetch = [&](auto unit) {
                constexpr int U = decltype(unit)::value;
                if constexpr (U < KSTEPS) opnd[U] = lds_read_b128(kaddr[U] + KB * BLKB);
                else opnd[U] = fetch_v(VB, (U - KSTEPS) / DB, (U - KSTEPS) % DB);
            };
            auto weight = [&](int r) {
                p[r] = __builtin_amdgcn_exp2f(fmaf(s_cur[r], c, neg_m));
                if (r % 2 == 1) {
                    uint32_t w = E::pack2(p[r - 1], p[r]);
                    asm volatile("" : "+v"(w));   // round here, under the matrix instruction, not later
                    pf_cur[r / 8][(r % 8) / 2] = w;
                    if (SUM_DOT) psum = E::dot2_ones(w, psum);
                }
                if (!SUM_DOT) {
                    psum += p[r];
                    asm volatile("" : "+v"(psum));   // add here, under the matrix instruction, not later
                }
            };
            auto unit_step = [&](auto unit) {
                constexpr int U = decltype(unit)::value;
                if constexpr (U + FETCH < NU) fetch(std::integral_constant<int, U + FETCH>{});
                else pre[U + FETCH - NU] = lds_read_b128(kaddr[U + FETCH - NU] + KB2 * BLKB);
                if constexpr (U < KSTEPS) {
                    if constexpr (U == 0) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) s_nxt[r] = 0.f;
                    }
                    s_nxt = E::mfma(opnd[U], qf[U], s_nxt);
                } else {
                    constexpr int tt = (U - KSTEPS) / DB, i = (U - KSTEPS) % DB;
                    acc_o[i] = E::mfma(opnd[U], pf_prv[tt], acc_o[i]);
                }
                {
                    constexpr int lo = (16 * U) / NU, hi = (16 * (U + 1)) / NU;
#pragma unroll
                    for (int r = lo; r < hi; ++r) weight(r);
                }
                // the 2 IPW load instructions of this slot, one per unit, evenly spread
                constexpr int NP = 2 * IPW, GAP = NU / NP;
                if constexpr (U % GAP == GAP / 2 && U / GAP < NP) {
                    constexpr int P = U / GAP;
                    constexpr int W = P / IPW, AHEAD = W ? VAHEAD : KAHEAD;
                    issue_piece(W, kb + AHEAD, P % IPW, (NBUF * W + ((PH + AHEAD) & (NBUF - 1))) * BLKB + (P % IPW) * 1024);
                }
                __builtin_amdgcn_sched_barrier(0);
            };
#pragma unroll
            for (int u = 0; u < FETCH; ++u) opnd[u] = pre[u];
            [&]<int... U>(std::integer_sequence<int, U...>) {
                (unit_step(std::integral_constant<int, U>{}), ...);
            }(std::make_integer_sequence<int, NU>{});
            // A weight sum above 2^ATTN_MAX_SLACK (or not a number: a weight overflowed) means that some row's
            // logits have outgrown the reference by about that much: only then the row maxima of the block are
            // taken, the references of the rows concerned moved up to them and the block's weights computed
            // again.  Weights stay below 2^ATTN_MAX_SLACK (finite in binary16 too), and the matrix pipe is not
            // held up by maxima that, after the first blocks, hardly ever change anything.
            if (__builtin_amdgcn_ballot_w64(!(psum <= __builtin_exp2f(ATTN_MAX_SLACK))) != 0) {
                float mx = vmax3(s_cur[0], s_cur[1], s_cur[2]);
#pragma unroll
                for (int j = 1; j < 7; ++j) mx = vmax3(mx, s_cur[2 * j + 1], s_cur[2 * j + 2]);
                mx = vmax(mx, s_cur[15]);
                const float m = vmax(mx, other_half(mx)) * c;    // c >= 0
                m_ref = m > m_ref ? m : m_ref;
                const float nm = -m_ref;
                psum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    p[r] = __builtin_amdgcn_exp2f(fmaf(s_cur[r], c, nm));
                    if (r % 2 == 1) {
                        const uint32_t w = E::pack2(p[r - 1], p[r]);
                        pf_cur[r / 8][(r % 8) / 2] = w;
                        if (SUM_DOT) psum = E::dot2_ones(w, psum);
                    }
                    if (!SUM_DOT) psum += p[r];
                }
            }
            // block k is done: its weights were taken against m_ref; everything older against m_run
            if (__builtin_amdgcn_ballot_w64(m_ref != m_run) != 0) {   // rare after the first blocks
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_ref);
                l_run *= alpha;
                rescale_o(alpha);
                m_run = m_ref;
            }
            l_run += psum;
        };

        f32x16 s_a, s_b;
        u32x4 pf_a[2], pf_b[2];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) pf_b[tt] = u32x4{0u, 0u, 0u, 0u};
        // prologue: S(0) and its row maximum; only K(0) and K(1), the first two loads, have to be there
        wait_block_loads<(KAHEAD + VAHEAD - 2) * IPW>();
        __syncthreads();
        {
#pragma unroll
            for (int r = 0; r < 16; ++r) s_a[r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                s_a = E::mfma(lds_read_b128(kaddr[ks]), qf[ks], s_a);
                __builtin_amdgcn_sched_barrier(0);
            }
            float mx = s_a[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s_a[r]);
            m_ref = fmaxf(mx, other_half(mx)) * c;   // the first reference: the true maxima of block 0
#pragma unroll
            for (int u = 0; u < FETCH; ++u) pre[u] = lds_read_b128(kaddr[u] + (1 & (NBUF - 1)) * BLKB);
        }

        // main loop: one slot per block, up to the last block of the workgroup's last wavefront
        for (int k0 = 0; k0 <= last_max; k0 += NBUF) {
            [&]<int... PH>(std::integer_sequence<int, PH...>) {
                ((k0 + PH <= last_max
                      ? (PH % 2 == 0 ? slot(k0 + PH, std::integral_constant<int, PH>{}, s_a, s_b, pf_b, pf_a)
                                     : slot(k0 + PH, std::integral_constant<int, PH>{}, s_b, s_a, pf_a, pf_b))
                      : (void)0),
                 ...);
            }(std::make_integer_sequence<int, NBUF>{});
        }
        // The second product of the last block is still open; its weights sit in pf_a / pf_b by parity.
        wait_block_loads<0>();
        __syncthreads();
        if (last_max & 1) pv_plain(pf_b, last_max & (NBUF - 1));
        else pv_plain(pf_a, last_max & (NBUF - 1));
    }

    // ---- epilogue: O = acc / l, lse = ln 2 * (m + log2 l) ----
    const float l_tot = l_run + other_half(l_run);
    const float inv = 1.0f / l_tot;
    if (o16 == 0) {
        // Single precision O.  A lane holds 4 consecutive elements of its own row: stored from there, one
        // instruction would touch 32 rows with 32 bytes each.  The tile goes through LDS instead, 32 columns
        // (4 KB, a region of the wavefront's own behind the block buffers) at a time, and comes back with
        // 8 lanes side by side on a row: every store instruction then writes 8 whole 128-byte lines.
        // 16-byte chunk c of row r sits at chunk position c ^ ((r / 2) % 8): the writes (16 rows, one
        // chunk column) and the reads (2 rows, all chunks) both spread over all banks.
        uint8_t* xp = smem + 2 * NBUF * BLKB + wave * 4096;
        float* obase = (float*)o + head + (size_t)qw0 * D;
#pragma unroll
        for (int i = 0; i < DB; ++i) {
#pragma unroll
            for (int gg = 0; gg < 4; ++gg) {
                f32x4 x = {acc_o[i][4 * gg] * inv, acc_o[i][4 * gg + 1] * inv, acc_o[i][4 * gg + 2] * inv,
                           acc_o[i][4 * gg + 3] * inv};
                *(f32x4*)(xp + l32 * 128 + (((2 * gg + h) ^ ((l32 >> 1) & 7)) << 4)) = x;
            }
#pragma unroll
            for (int pass = 0; pass < 4; ++pass) {
                const int row = 8 * pass + (lane >> 3), ch = lane & 7;
                const f32x4 y = *(const f32x4*)(xp + row * 128 + ((ch ^ ((row >> 1) & 7)) << 4));
                if (qw0 + row < S) *(f32x4*)(obase + (size_t)row * D + 32 * i + 4 * ch) = y;
            }
        }
    } else if (qrow < S) {   // O in the input type, rounded to nearest even: 4 elements = 8 bytes per store
        uint16_t* orow = (uint16_t*)o + head + (size_t)qrow * D;
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
            for (int gg = 0; gg < 4; ++gg) {
                u32x2 x = {E::pack2(acc_o[i][4 * gg] * inv, acc_o[i][4 * gg + 1] * inv),
                           E::pack2(acc_o[i][4 * gg + 2] * inv, acc_o[i][4 * gg + 3] * inv)};
                *(u32x2*)(orow + 32 * i + 8 * gg + 4 * h) = x;
            }
    }
    if (qrow < S) {
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
    void* o = a.o;
    float* lse = a.lse;
    int S = a.S, BH = a.BH, nq = nqt, o16 = a.o16;
    float c = a.c;
    uint32_t qsign = a.qsign;
    void* args[] = {&q, &k, &v, &o, &lse, &S, &BH, &nq, &c, &qsign, &o16};
    // the launch status is taken from the call itself: the thread's "last error" may hold a stale
    // value left by an unrelated earlier runtime call of the host program
    // NBUF K and NBUF V block buffers, and 4 KB per wavefront for the way out of the output tile
    constexpr unsigned lds_bytes = 2u * attn_buffers(D) * attn_block_keys(D) * 2u * D + NW * 4096u;
    const void* fn = reinterpret_cast<const void*>(&attn_fwd_kernel<DT, D, CAUSAL, NW>);
    static std::atomic<uint64_t> told{0};   // per kernel instance: the devices whose runtime knows its LDS size
    if (const hipError_t e = announce_lds(fn, lds_bytes, told); e != hipSuccess) return e;
    return hipLaunchKernel(fn, dim3((unsigned)blocks), dim3(NW * 64), args, lds_bytes, (hipStream_t)a.stream);
}

}  // namespace

// dispatch on (dtype, D, causal); arguments were validated by the caller
hipError_t attn_launch(const AttnLaunch& a) {
    // (a negative scale, folded into the sign of q, stays with the 32-row kernel: this one keeps q where no vector
    // instruction reaches it)
    if (attn_takes_rows64(a.BH, a.S, a.D) && a.qsign == 0) return attn_launch_rows64(a);
#define ATTN_CASE(DT, DD, CZ)                                       \
    if (a.dtype == DT && a.D == DD && (a.causal != 0) == CZ)     \
        return attn_pick_nw(a.BH, a.S) == ATTN_NW ? launch<DT, DD, CZ, ATTN_NW>(a) : launch<DT, DD, CZ, ATTN_NW / 2>(a);
    ATTN_CASE(0, 32, false)
    ATTN_CASE(0, 32, true)
    ATTN_CASE(1, 32, false)
    ATTN_CASE(1, 32, true)
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
