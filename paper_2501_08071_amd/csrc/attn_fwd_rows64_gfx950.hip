// Fused multi-head attention forward for gfx950, the schedule with 64 query rows per wavefront.
//
// Same operation, same data movement and the same register layout as attn_fwd_gfx950.hip (transposed products,
// one lane = one query row, weights straight from the accumulator registers, K/V blocks from global memory
// directly into swizzled LDS); what differs is who shares what:
//
//   workgroup = 4 wavefronts, ONE per SIMD with the whole register file, each owning TWO sub-tiles of 32 query
//   rows; every K and V operand read from LDS feeds two matrix instructions, one per sub-tile, so the loop reads
//   half the LDS bytes per matrix instruction.  With one wavefront per SIMD there is no second wavefront to take the
//   vector work: matrix and vector instructions interleave inside the wavefront -- in the step of key block k
//   (32 keys) the matrix pipe runs S(k+1) = K(k+1).Q^T and O^T += V(k-1)^T.P(k-1)^T of both sub-tiles while the
//   vector pipe turns S(k) into P(k), one weight per matrix instruction.  The order written is the order issued.
//
//   Sub-tiles: wavefront w owns rows 32 w .. 32 w + 31 (sub-tile A) and 32 (w + 4) .. 32 (w + 4) + 31 (sub-tile B)
//   of the workgroup's 256.  Under the causal mask sub-tile s is done after its diagonal block; pairing an early
//   with a late sub-tile gives every wavefront work until late in the tile's last blocks (a wavefront steps through
//   "both", "B only" and "idle" blocks; idle ones keep the barriers and issue their share of the block loads).
//
// The paper's subject is the order of memory and compute instructions inside a fixed kernel (Sections 2.4, 3.5);
// this file is one more state of that order for the attention kernel of Table 2.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include <utility>

#include "attn_launch.h"
#include "gfx950_common.h"
#include "attn_device.h"

namespace {

using namespace gfx950;
using namespace attn_device;

extern __shared__ __attribute__((aligned(1024))) uint8_t smem64[];

template <int DT, int D, bool CAUSAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void attn_fwd_rows64_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                            void* __restrict__ o, float* __restrict__ lse, int S, int BH, int nqt, float c_arg,
                            uint32_t qsign, int o16) {
    using E = Elem<DT>;
    constexpr int NW = 4;              // wavefronts per workgroup, one per SIMD
    constexpr int RS = 2;              // sub-tiles of 32 query rows per wavefront
    constexpr int BR = NW * RS * 32;   // query rows per workgroup
    constexpr int BC = 32;             // keys per block
    constexpr int NBUF = ATTN64_NBUF;  // LDS buffers per tensor (a power of two); block k lives in buffer k % NBUF
    constexpr int BEV = 2;             // blocks per workgroup barrier
    static_assert(NBUF % BEV == 0 && (NBUF & (NBUF - 1)) == 0, "buffers");
    // block k's step issues the load of K(k + KAHEAD) and of V(k + VAHEAD), into buffers nobody reads any more
    constexpr int KAHEAD = NBUF - (BEV - 1);
    constexpr int VAHEAD = KAHEAD - 2;
    static_assert(KAHEAD - 1 >= BEV + 1, "too few buffers for the loads that have to be in flight");
    constexpr int KSTEPS = D / 16;     // contraction steps of Q.K^T
    constexpr int DB = D / 32;         // 32-wide blocks of the head dimension
    constexpr int ROWB = 2 * D;        // bytes per K/V row
    constexpr int BLKB = BC * ROWB;    // bytes per key block
    constexpr int CPR = D / 8;         // 16-byte chunks per row
    constexpr int RPI = 1024 / ROWB;   // rows written by one direct-to-LDS load instruction
    constexpr int IPT = BC / RPI;      // such instructions per block and tensor
    constexpr int IPW = IPT >= NW ? IPT / NW : 1;   // ... per loading wavefront
    constexpr int LOADERS = IPT / IPW;              // wavefronts that issue loads
    static_assert(IPT % IPW == 0 && LOADERS <= NW, "load split");

    const float c = c_arg;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31;
    const int h = lane >> 5;

    // Workgroup -> tile: as in the 32-row kernel.  Workgroup b runs on XCD b % 8; the (b,h) pairs are dealt out by
    // XCD and, on an XCD, taken ATTN_HEAD_GROUP at a time, heaviest query tiles first.
    int bh, qt;
    {
        constexpr int GS = ATTN_HEAD_GROUP;
        const int b = blockIdx.x;
        if (GS > 0 && BH % (8 * GS) == 0 && (gridDim.x & 7) == 0) {
            const int x = b & 7, j = b >> 3;
            const int per = GS * nqt;
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
    int qs0[RS], qrow[RS], qrow_ld[RS];   // first row of a sub-tile, this lane's row in it, and that row clamped to the sequence
#pragma unroll
    for (int r = 0; r < RS; ++r) {
        qs0[r] = q0 + 32 * (wave + NW * r);
        qrow[r] = qs0[r] + l32;
        qrow_ld[r] = qrow[r] < S ? qrow[r] : S - 1;
    }

    const size_t head = (size_t)bh * S * D;
    const uint16_t* qh = q + head;
    const uint16_t* kh = k + head;
    const uint16_t* vh = v + head;

    const int kv_end = CAUSAL ? (q0 + BR < S ? q0 + BR : S) : S;
    const int nblk = (kv_end + BC - 1) / BC;       // key blocks the workgroup streams
    const int nfull = S / BC;
    const int last_max = nblk - 1;                 // the last block any wavefront of the workgroup works on
    // kd: the first block a sub-tile needs a mask for -- the one on its causal diagonal, or the ragged last block
    // of the sequence (which may not exist: then kd == nblk).  last: the last block it works on.
    int kd[RS], last[RS];
#pragma unroll
    for (int r = 0; r < RS; ++r) {
        const int d = CAUSAL ? qs0[r] / BC : nfull;
        kd[r] = d < nfull ? d : nfull;
        last[r] = CAUSAL && kd[r] < last_max ? kd[r] : last_max;
    }

    // Q^T operands, resident for the whole kernel in accumulation registers: lane holds q[qrow][16 ks + 8 h .. +7] of
    // both sub-tiles.  Requested first: the wait for the first K blocks below covers them.
    u32x4 qf[RS][KSTEPS];
#pragma unroll
    for (int r = 0; r < RS; ++r)
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) qf[r][ks] = global_load_acc16(qh + (size_t)qrow_ld[r] * D + 16 * ks + 8 * h);

    // ---- direct-to-LDS block loads (see attn_fwd_gfx950.hip) ----
    const uint32_t lds0 = (uint32_t)(uintptr_t)(LDS_AS uint8_t*)smem64;
    uint32_t goff[IPW], goff_r[IPW];
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
        const int r = (wave * IPW + i) * RPI + lane / CPR;
        goff[i] = (r * D + (((lane % CPR) ^ swz<D>(r)) << 3)) * 2;
        // the ragged last block of the sequence: rows past the end (masked later) point at the last valid row
        const int over = nfull * BC + r - (S - 1);
        goff_r[i] = over > 0 ? goff[i] - over * ROWB : goff[i];
    }
    const uint32_t lds_wave = lds0 + wave * IPW * 1024;
    // One load instruction: piece i of K block `blk` (which = 0) or V block `blk` (which = 1).  A block index past
    // the end of the stream is replaced by the last block (a copy nobody reads, into a buffer nobody needs any
    // more), so that every step issues the same number of loads.
    auto issue_piece = [&](int which, int blk, int i, uint32_t dst) __attribute__((always_inline)) {
        if (LOADERS < NW && wave >= LOADERS) return;
        const int b = blk < nblk - 1 ? blk : nblk - 1;
        const uint16_t* src = (which ? vh : kh) + (size_t)b * (BC * D);
        lds_dma16(lds_wave + dst, src, b >= nfull ? goff_r[i] : goff[i]);
    };
    auto issue_load = [&](int which, int blk) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < IPW; ++i) issue_piece(which, blk, i, (NBUF * which + (blk & (NBUF - 1))) * BLKB + i * 1024);
    };
    issue_load(0, 0);
#pragma unroll
    for (int j = 1; j < KAHEAD; ++j) {
        issue_load(0, j);
        if (j - 1 < VAHEAD) issue_load(1, j - 1);
    }
    // the last V buffer is read by step 0 (with all-zero weights) before anything was loaded into it: make it finite
    {
        constexpr int PER = BLKB / (NW * 64);   // bytes per thread
        static_assert(PER % 16 == 0, "zero fill");
        uint8_t* vb = smem64 + (2 * NBUF - 1) * BLKB + tid * PER;
#pragma unroll
        for (int i = 0; i < PER / 16; ++i) *(u32x4*)(vb + 16 * i) = u32x4{0u, 0u, 0u, 0u};
    }

    f32x16 acc_o[RS][DB];
#pragma unroll
    for (int r = 0; r < RS; ++r)
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc_o[r][i][e] = 0.f;
    static_assert(DB == 4, "mfma_settle takes the four accumulator blocks of a sub-tile");
    auto settle = [&](int r) __attribute__((always_inline)) { mfma_settle(acc_o[r][0], acc_o[r][1], acc_o[r][2], acc_o[r][3]); };
    float m_run[RS], l_run[RS], m_ref[RS];   // reference maximum (base-2 units) of what is accumulated, this lane's share of the row sum, reference of the block in hand
#pragma unroll
    for (int r = 0; r < RS; ++r) { m_run[r] = -INFINITY; l_run[r] = 0.f; m_ref[r] = -INFINITY; }

    // ---- per-lane LDS addresses (loop invariant; buffer parts become immediate offsets) ----
    uint32_t kaddr[KSTEPS];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) kaddr[ks] = lds0 + l32 * ROWB + (((2 * ks + h) ^ swz<D>(l32)) << 4);
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
    constexpr int NT = BC / 16;                // 16-key steps of the second product
    constexpr int NU = KSTEPS + NT * DB;       // operand fetches (units) per block; a unit feeds one matrix instruction per active sub-tile
    static_assert(16 % NU == 0 || NU % 16 == 0, "weights per unit");
    auto fetch_v = [&](int VB, int tt, int i) __attribute__((always_inline)) {
        u32x2 lo = lds_read_tr16(vaddr[0][i] + VB * BLKB + 16 * tt * ROWB);
        u32x2 hi = lds_read_tr16(vaddr[1][i] + VB * BLKB + 16 * tt * ROWB);
        return u32x4{lo[0], lo[1], hi[0], hi[1]};
    };
    auto rescale_o = [&](int r, float alpha) __attribute__((always_inline)) {
        // the accumulators live in accumulation registers (mfma_aacc): the last matrix instruction on them has to have
        // finished; then one block of 16 at a time comes over, is scaled and goes back, so that this rare path does
        // not claim vector registers the loop needs
        settle(r);
#pragma unroll
        for (int i = 0; i < DB; ++i) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int e = 0; e < 16; ++e) acc_o[r][i][e] *= alpha;
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // O^T += V(j)^T . P(j)^T of one sub-tile, plain order (a sub-tile's last block).  Called under a condition, so the
    // compiler may move the accumulators afterwards: their matrix instructions are waited out first.
    auto pv_plain = [&](int r, const u32x4 (&pf)[2], int VB) __attribute__((always_inline)) {
#pragma unroll
        for (int tt = 0; tt < NT; ++tt)
#pragma unroll
            for (int i = 0; i < DB; ++i) {
                mfma_aacc<DT>(acc_o[r][i], fetch_v(VB, tt, i), pf[tt]);
                __builtin_amdgcn_sched_barrier(0);
            }
        settle(r);
        __builtin_amdgcn_sched_barrier(0);
    };

    constexpr int FETCH = ATTN_FETCH < KSTEPS ? ATTN_FETCH : KSTEPS;   // units between an operand's LDS read and its use
    u32x4 pre[FETCH];   // first operands of the next step, read before its barrier

    // The barrier in front of every BEV-th step.  Before step k issues its own loads, 2 (k + KAHEAD - 1) are out (in
    // units of IPW pieces); the steps up to the next barrier read K(k+2) .. K(k+BEV+1) (the last of them is load
    // number 2 (k+BEV+1) at most) and V(k-1) .. V(k+BEV-2), which come earlier in the order of issue.
    auto step_barrier = [&](int ph) __attribute__((always_inline)) {
        if (ph % BEV == 0) {
            wait_lds_dma<(2 * (KAHEAD - 1) - 2 * (BEV + 1)) * IPW>();
            asm volatile("s_barrier" ::: "memory");
        }
    };
    // the weights of a whole block of one sub-tile again, against a reference moved up to the block's row maxima
    auto redo_weights = [&](int r, f32x16& s_cur, u32x4 (&pf_cur)[2], float& psum) __attribute__((always_inline)) {
        float mx = vmax3(s_cur[0], s_cur[1], s_cur[2]);
#pragma unroll
        for (int j = 1; j < 7; ++j) mx = vmax3(mx, s_cur[2 * j + 1], s_cur[2 * j + 2]);
        mx = vmax(mx, s_cur[15]);
        const float m = vmax(mx, other_half(mx)) * c;    // c >= 0
        m_ref[r] = m > m_ref[r] ? m : m_ref[r];
        const float nm = -m_ref[r];
        psum = 0.f;
        float p[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            p[e] = __builtin_amdgcn_exp2f(fmaf(s_cur[e], c, nm));
            if (e % 2 == 1) {
                const uint32_t w = E::pack2(p[e - 1], p[e]);
                pf_cur[e / 8][(e % 8) / 2] = w;
            }
            psum += p[e];   // the fp32 weights, both types (a dot instruction would wait on the matrix pipe)
        }
    };

    // Step k of the pipeline, for the sub-tiles R0 .. RS-1 (R0 = 0: both; R0 = 1: sub-tile A is done).  PH = k % NBUF
    // fixes every LDS offset: a constant in the main loop, where the steps are unrolled by phase, a run-time value
    // in the few steps after sub-tile A is done.  s_cur holds S(k) on entry, s_nxt receives S(k+1); pf_prv holds the
    // weights of block k-1, pf_cur receives those of block k.
    auto step = [&](int kb, const int PH, auto first, f32x16 (&s_cur)[RS], f32x16 (&s_nxt)[RS], u32x4 (&pf_prv)[RS][2],
                    u32x4 (&pf_cur)[RS][2]) __attribute__((always_inline)) {
        constexpr int R0 = decltype(first)::value;
        const int KB = (PH + 1) & (NBUF - 1);          // buffer of K(k+1)
        const int KB2 = (PH + 2) & (NBUF - 1);         // buffer of K(k+2)
        const int VB = (PH + NBUF - 1) & (NBUF - 1);   // buffer of V(k-1)
        step_barrier(PH);
        if constexpr (R0 == 1) {
            // sub-tile A finished with block k-1: its second product of that block is still open
            if (kb == last[0] + 1) pv_plain(0, pf_prv[0], VB);
        }
        float neg_m[RS], psum[RS];
#pragma unroll
        for (int r = R0; r < RS; ++r) {
            if (kb >= kd[r]) {
                // A block cut by the causal diagonal or by the end of the sequence: masked logits become -3e38 (times
                // c >= 1e-30 that is far below any real logit and the weight comes out as an exact 0), and the
                // reference maximum is taken again, over what is left.
                const int lim = (CAUSAL ? qrow_ld[r] : S - 1) - kb * BC - 4 * h;
                float m = -3.0e38f;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int off = 8 * (e / 4) + (e % 4);
                    s_cur[r][e] = off > lim ? -3.0e38f : s_cur[r][e];
                    m = fmaxf(m, s_cur[r][e]);
                }
                m = fmaxf(m, other_half(m)) * c;
                m_ref[r] = m > m_run[r] + ATTN_MAX_SLACK ? m : m_run[r];
            }
            neg_m[r] = -m_ref[r];
            psum[r] = 0.f;
        }
        // Units 0 .. KSTEPS-1: S(k+1) = K(k+1).Q^T; units KSTEPS .. NU-1: O^T += V(k-1)^T.P(k-1)^T.  A unit is: the LDS
        // read of the operand FETCH units ahead, then per sub-tile one matrix instruction on the unit's operand and
        // the sub-tile's share of the 16 weights of block k.  Nothing moves across a unit.
        float p[RS][16];
        u32x4 opnd[NU];
        auto fetch = [&](auto unit) __attribute__((always_inline)) {
            constexpr int U = decltype(unit)::value;
            if constexpr (U < KSTEPS) opnd[U] = lds_read_b128(kaddr[U] + KB * BLKB);
            else opnd[U] = fetch_v(VB, (U - KSTEPS) / DB, (U - KSTEPS) % DB);
        };
        // The vector work of weight e of sub-tile r in two halves, so that a matrix instruction can stand between an
        // exponential and the first use of its result: the argument and the exponential; then the row sum and, with
        // every second weight, the rounding of two weights into one register.
        auto weight_exp = [&](int r, int e) __attribute__((always_inline)) {
            p[r][e] = __builtin_amdgcn_exp2f(fmaf(s_cur[r][e], c, neg_m[r]));
            asm volatile("" : "+v"(p[r][e]));   // here, in this group, not where the compiler would sink it to
        };
        auto weight_sum = [&](int r, int e) __attribute__((always_inline)) {
            if (e % 2 == 1) {
                uint32_t w = E::pack2(p[r][e - 1], p[r][e]);
                asm volatile("" : "+v"(w));
                pf_cur[r][e / 8][(e % 8) / 2] = w;
            }
            psum[r] += p[r][e];   // row sum from the fp32 weights, both types
            asm volatile("" : "+v"(psum[r]));
        };
        // With one wavefront per SIMD nothing else fills the issue slots while a matrix instruction waits for the
        // pipe: two matrix instructions in a row cost the wavefront a whole matrix instruction's time.  So the unit
        // is written as four groups that nothing crosses: matrix instruction of the first sub-tile | arguments and
        // exponentials of both sub-tiles | matrix instruction of the second sub-tile | sums and roundings, the
        // operand read of a later unit, a block load.  Each vector group fits the matrix instruction before it.
        auto matrix = [&](auto unit, int r) __attribute__((always_inline)) {
            constexpr int U = decltype(unit)::value;
            if constexpr (U < KSTEPS) {
                if constexpr (U == 0) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) s_nxt[r][e] = 0.f;
                }
                s_nxt[r] = E::mfma(opnd[U], qf[r][U], s_nxt[r]);
            } else {
                constexpr int tt = (U - KSTEPS) / DB, i = (U - KSTEPS) % DB;
                mfma_aacc<DT>(acc_o[r][i], opnd[U], pf_prv[r][tt]);
            }
        };
        auto unit_step = [&](auto unit) __attribute__((always_inline)) {
            constexpr int U = decltype(unit)::value;
            constexpr int lo = (16 * U) / NU, hi = (16 * (U + 1)) / NU;
            if constexpr (R0 == 0) {
                matrix(unit, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int e = lo; e < hi; ++e)
#pragma unroll
                for (int r = R0; r < RS; ++r) weight_exp(r, e);
            __builtin_amdgcn_sched_barrier(0);
            matrix(unit, 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int e = lo; e < hi; ++e)
#pragma unroll
                for (int r = R0; r < RS; ++r) weight_sum(r, e);
            if constexpr (U + FETCH < NU) fetch(std::integral_constant<int, U + FETCH>{});
            else pre[U + FETCH - NU] = lds_read_b128(kaddr[U + FETCH - NU] + KB2 * BLKB);
            // the 2 IPW load instructions of this step, evenly spread
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
#pragma unroll
        for (int r = R0; r < RS; ++r) {
            // A weight sum above 2^ATTN_MAX_SLACK (or not a number: a weight overflowed) means that some row's logits
            // have outgrown the reference: only then the row maxima of the block are taken, the references of the rows
            // concerned moved up to them and the block's weights computed again.
            if (__builtin_amdgcn_ballot_w64(!(psum[r] <= __builtin_exp2f(ATTN_MAX_SLACK))) != 0)
                redo_weights(r, s_cur[r], pf_cur[r], psum[r]);
            // block k is done: its weights were taken against m_ref; everything older against m_run
            if (__builtin_amdgcn_ballot_w64(m_ref[r] != m_run[r]) != 0) {   // rare after the first blocks
                const float alpha = __builtin_amdgcn_exp2f(m_run[r] - m_ref[r]);
                l_run[r] *= alpha;
                rescale_o(r, alpha);
                m_run[r] = m_ref[r];
            }
            l_run[r] += psum[r];
        }
        // The steps of sub-tile B alone are reached by run-time conditions, behind which the compiler may move the
        // accumulators: their matrix instructions are waited out before the step is left.
        if constexpr (R0 == 1) settle(1);
    };
    // A step in which this wavefront has nothing left to compute: it keeps the barrier, closes a sub-tile that
    // finished with the previous block, and issues its share of the block loads.
    auto idle_step = [&](int kb, const int PH, u32x4 (&pf_prv)[RS][2]) __attribute__((always_inline)) {
        const int VB = (PH + NBUF - 1) & (NBUF - 1);
        step_barrier(PH);
#pragma unroll
        for (int r = 0; r < RS; ++r)
            if (kb == last[r] + 1) pv_plain(r, pf_prv[r], VB);
#pragma unroll
        for (int P = 0; P < 2 * IPW; ++P) {
            const int W = P / IPW, AHEAD = W ? VAHEAD : KAHEAD;
            issue_piece(W, kb + AHEAD, P % IPW, (NBUF * W + ((PH + AHEAD) & (NBUF - 1))) * BLKB + (P % IPW) * 1024);
        }
    };

    f32x16 s_a[RS], s_b[RS];
    u32x4 pf_a[RS][2], pf_b[RS][2];
#pragma unroll
    for (int r = 0; r < RS; ++r)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) pf_b[r][tt] = u32x4{0u, 0u, 0u, 0u};
    // prologue: S(0) and its row maxima; only K(0) and K(1), the first two loads, have to be there
    wait_lds_dma<(KAHEAD + VAHEAD - 2) * IPW>();
    __syncthreads();
    {
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const u32x4 kop = lds_read_b128(kaddr[ks]);
#pragma unroll
            for (int r = 0; r < RS; ++r) {
                if (ks == 0) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) s_a[r][e] = 0.f;
                }
                s_a[r] = E::mfma(kop, qf[r][ks], s_a[r]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int r = 0; r < RS; ++r) {
            float mx = s_a[r][0];
#pragma unroll
            for (int e = 1; e < 16; ++e) mx = fmaxf(mx, s_a[r][e]);
            m_ref[r] = fmaxf(mx, other_half(mx)) * c;   // the first reference: the true maxima of block 0
        }
#pragma unroll
        for (int u = 0; u < FETCH; ++u) pre[u] = lds_read_b128(kaddr[u] + (1 & (NBUF - 1)) * BLKB);
    }

    // main loop: one step per block while both sub-tiles work, unrolled by phase
    const int last_both = CAUSAL ? last[0] : last_max;
    for (int k0 = 0; k0 <= last_both; k0 += NBUF) {
        [&]<int... PH>(std::integer_sequence<int, PH...>) {
            auto one = [&](auto phase) __attribute__((always_inline)) {
                constexpr int P = decltype(phase)::value;
                if (k0 + P > last_both) return;
                if constexpr (P % 2 == 0) step(k0 + P, P, std::integral_constant<int, 0>{}, s_a, s_b, pf_b, pf_a);
                else step(k0 + P, P, std::integral_constant<int, 0>{}, s_b, s_a, pf_a, pf_b);
            };
            (one(std::integral_constant<int, PH>{}), ...);
        }(std::make_integer_sequence<int, NBUF>{});
    }
    // Under the causal mask sub-tile A is done first: the remaining blocks of the workgroup are steps of sub-tile B
    // alone, then idle ones; these few steps are not unrolled (the phase is a run-time value).  Where the compiler
    // moves accumulators between the two loops or between these steps, their matrix instructions have finished.
    if constexpr (CAUSAL) {
        settle(0);
        settle(1);
        __builtin_amdgcn_sched_barrier(0);
        for (int kb = last_both + 1; kb <= last_max; ++kb) {
            const int ph = kb & (NBUF - 1);
            if (kb <= last[1]) {
                if ((kb & 1) == 0) step(kb, ph, std::integral_constant<int, 1>{}, s_a, s_b, pf_b, pf_a);
                else step(kb, ph, std::integral_constant<int, 1>{}, s_b, s_a, pf_a, pf_b);
            } else {
                if ((kb & 1) == 0) idle_step(kb, ph, pf_b);
                else idle_step(kb, ph, pf_a);
            }
        }
    }
    // A sub-tile that went through to the workgroup's last block still has that block's second product open; its
    // weights sit in pf_a / pf_b by parity.
    wait_lds_dma<0>();
    __syncthreads();
#pragma unroll
    for (int r = 0; r < RS; ++r)
        if (last[r] == last_max) {
            if (last_max & 1) pv_plain(r, pf_b[r], last_max & (NBUF - 1));
            else pv_plain(r, pf_a[r], last_max & (NBUF - 1));
        }

    settle(0);   // the accumulators' last matrix instructions, of which the compiler knows nothing
    settle(1);
    __builtin_amdgcn_sched_barrier(0);
    // ---- epilogue: O = acc / l, lse = ln 2 * (m + log2 l), one sub-tile after the other ----
    uint8_t* xp = smem64 + 2 * NBUF * BLKB + wave * 4096;
#pragma unroll
    for (int r = 0; r < RS; ++r) {
        const float l_tot = l_run[r] + other_half(l_run[r]);
        const float inv = 1.0f / l_tot;
        if (o16 == 0) {
            // Single precision O leaves through LDS, 32 columns (4 KB, a region of the wavefront's own behind the
            // block buffers) at a time, and comes back with 8 lanes side by side on a row: every store instruction
            // writes 8 whole 128-byte lines.  16-byte chunk c of row x sits at chunk position c ^ ((x / 2) % 8).
            float* obase = (float*)o + head + (size_t)qs0[r] * D;
#pragma unroll
            for (int i = 0; i < DB; ++i) {
#pragma unroll
                for (int gg = 0; gg < 4; ++gg) {
                    f32x4 x = {acc_o[r][i][4 * gg] * inv, acc_o[r][i][4 * gg + 1] * inv, acc_o[r][i][4 * gg + 2] * inv,
                               acc_o[r][i][4 * gg + 3] * inv};
                    *(f32x4*)(xp + l32 * 128 + (((2 * gg + h) ^ ((l32 >> 1) & 7)) << 4)) = x;
                }
#pragma unroll
                for (int pass = 0; pass < 4; ++pass) {
                    const int row = 8 * pass + (lane >> 3), ch = lane & 7;
                    const f32x4 y = *(const f32x4*)(xp + row * 128 + ((ch ^ ((row >> 1) & 7)) << 4));
                    if (qs0[r] + row < S) *(f32x4*)(obase + (size_t)row * D + 32 * i + 4 * ch) = y;
                }
            }
        } else if (qrow[r] < S) {   // O in the input type, rounded to nearest even: 4 elements = 8 bytes per store
            uint16_t* orow = (uint16_t*)o + head + (size_t)qrow[r] * D;
#pragma unroll
            for (int i = 0; i < DB; ++i)
#pragma unroll
                for (int gg = 0; gg < 4; ++gg) {
                    u32x2 x = {E::pack2(acc_o[r][i][4 * gg] * inv, acc_o[r][i][4 * gg + 1] * inv),
                               E::pack2(acc_o[r][i][4 * gg + 2] * inv, acc_o[r][i][4 * gg + 3] * inv)};
                    *(u32x2*)(orow + 32 * i + 8 * gg + 4 * h) = x;
                }
        }
        if (qrow[r] < S && lse != nullptr && h == 0)
            lse[(size_t)bh * S + qrow[r]] = (m_run[r] + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
    }
}

template <int DT, int D, bool CAUSAL>
hipError_t launch64(const AttnLaunch& a) {
    constexpr int BR = 256;
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
    // ATTN64_NBUF K and as many V block buffers of 32 keys, and 4 KB per wavefront for the way out of the output tile
    constexpr unsigned lds_bytes = 2u * ATTN64_NBUF * 32u * 2u * D + 4u * 4096u;
    const void* fn = reinterpret_cast<const void*>(&attn_fwd_rows64_kernel<DT, D, CAUSAL>);
    static std::atomic<uint64_t> told{0};   // per kernel instance: the devices whose runtime knows its LDS size
    if (const hipError_t e = announce_lds(fn, lds_bytes, told); e != hipSuccess) return e;
    return hipLaunchKernel(fn, dim3((unsigned)blocks), dim3(256), args, lds_bytes, (hipStream_t)a.stream);
}

}  // namespace

// dispatch on (dtype, causal); D = 128 only; arguments were validated by the caller
hipError_t attn_launch_rows64(const AttnLaunch& a) {
    if (a.D != 128) return hipErrorInvalidValue;
    if (a.dtype == 0) return a.causal ? launch64<0, 128, true>(a) : launch64<0, 128, false>(a);
    return a.causal ? launch64<1, 128, true>(a) : launch64<1, 128, false>(a);
}
