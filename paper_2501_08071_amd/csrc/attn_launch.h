// Internal: validated launch request handed from the C-ABI layer to the kernel dispatcher.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#ifndef ATTN_NW
#define ATTN_NW 8   // wavefronts per workgroup, each owning 32 query rows
#endif
#ifndef ATTN_PP_KEYS
#define ATTN_PP_KEYS 64   // keys per inner-loop block in the alternating-phase loop at D = 128 (32 or 64)
#endif
#ifndef ATTN_PP_KEYS_D64
#define ATTN_PP_KEYS_D64 (2 * ATTN_PP_KEYS)   // the same at D = 64 (32, 64 or 128), where a key costs half the matrix work and half the LDS: twice the keys per phase
#endif
#define ATTN_BC 32  // keys per inner-loop block in the interleaved loop
#ifndef ATTN_MAX_SLACK
#define ATTN_MAX_SLACK 15.0f  // log2 of the largest sum of a lane's softmax weights of one block tolerated before the reference maximum is moved
#endif
#ifndef ATTN_WARY
#define ATTN_WARY 16  // alternating-phase loop: after a reference maximum moved, blocks whose row maxima are taken before the weights
#endif
#ifndef ATTN_NBUF
#define ATTN_NBUF 8   // LDS buffers per tensor for blocks of up to 8 KiB (a power of two); larger blocks get half as many: 4 x 2 x 16 KiB = 128 KiB with the shipped blocks at D = 128 and 64, one workgroup per CU
#endif
#ifndef ATTN_BARRIER_EVERY
#define ATTN_BARRIER_EVERY 2  // key blocks per workgroup barrier (1 or 2)
#endif
#ifndef ATTN_PINGPONG
#define ATTN_PINGPONG 1  // D = 128 and 64: alternate matrix and vector phases between two groups of wavefronts
#endif
#ifndef ATTN_HEAD_GROUP
#define ATTN_HEAD_GROUP 4  // (b,h) pairs whose query tiles an XCD works on at the same time (0: no grouping)
#endif
#ifndef ATTN_FETCH
#define ATTN_FETCH 4  // units between the LDS read of an operand and the matrix instruction that uses it
#endif
#ifndef ATTN_PP_FETCH
#define ATTN_PP_FETCH 4  // alternating-phase loop: K operands of the next matrix phase read ahead, in the vector phase
#endif
#ifndef ATTN_F16_SUM_DOT
#define ATTN_F16_SUM_DOT 1  // binary16 at D = 64: row sums from the rounded weights, two per v_dot2c_f32_f16, at the end of the vector phase (0: from the fp32 weights, one addition each, as everywhere else)
#endif
#ifndef ATTN_PP_PRIO_M
#define ATTN_PP_PRIO_M 1  // alternating-phase loop: issue priority of a wavefront in its matrix phase ...
#endif
#ifndef ATTN_PP_PRIO_V
#define ATTN_PP_PRIO_V 0  // ... and in its vector phase (0 .. 3; equal: the priority is never touched)
#endif
#ifndef ATTN_DEBUG_POISON
#define ATTN_DEBUG_POISON 0  // debug build: an LDS buffer is filled with NaN patterns right before the load that overwrites it
#endif
#ifndef ATTN_WPE
#define ATTN_WPE 2  // wavefronts per SIMD the register budget is sized for
#endif

#ifndef ATTN_ROWS64
#define ATTN_ROWS64 0  // D = 128, problems that fill the chip: the kernel with 64 query rows per wavefront, one wavefront per SIMD
#endif
#ifndef ATTN64_NBUF
#define ATTN64_NBUF 8  // that kernel's LDS buffers of 32 keys per tensor
#endif

// Which loop a head dimension runs, the keys per inner-loop block and the LDS buffers per tensor that go with it.
constexpr bool attn_alternating(int D) { return ATTN_PINGPONG != 0 && (D == 128 || D == 64); }
constexpr int attn_block_keys(int D) { return attn_alternating(D) ? (D == 64 ? ATTN_PP_KEYS_D64 : ATTN_PP_KEYS) : ATTN_BC; }
constexpr int attn_buffers(int D) { return attn_block_keys(D) * D > 32 * 128 ? ATTN_NBUF / 2 : ATTN_NBUF; }   // blocks of more than 8 KiB: half as many (128 KiB in all with the shipped blocks, D = 128 and 64)

static_assert(ATTN_PP_KEYS == 32 || ATTN_PP_KEYS == 64, "block size of the alternating-phase loop");
static_assert(ATTN_PP_KEYS_D64 == 32 || ATTN_PP_KEYS_D64 == 64 || ATTN_PP_KEYS_D64 == 128, "block size of the alternating-phase loop at D = 64");

// Wavefronts per workgroup for a problem of BH (b,h) pairs and S rows: ATTN_NW (256 query rows per workgroup),
// or half of that when the larger tiles would leave at least half of the 256 compute units without a
// workgroup (the smaller workgroups also fit two to a compute unit at D = 32).
#ifndef ATTN_SMALL_TILES
#define ATTN_SMALL_TILES 128
#endif
inline int attn_pick_nw(long long BH, int S) {
    const long long tiles = BH * ((S + 32 * ATTN_NW - 1) / (32 * ATTN_NW));
    return tiles <= ATTN_SMALL_TILES ? ATTN_NW / 2 : ATTN_NW;
}

struct AttnLaunch {
    const void* q;
    const void* k;
    const void* v;
    void* o;          // fp32, or the input type when o16 is set
    float* lse;       // may be null
    int BH, S, D;
    int causal;
    int dtype;        // 0 binary16, 1 bfloat16
    float c;          // |scale| * log2(e)
    uint32_t qsign;   // 0x80008000 when scale < 0 (sign folded into q), else 0
    int o16;          // write O rounded to the input type instead of fp32
    void* stream;
};

hipError_t attn_launch(const AttnLaunch& a);
hipError_t attn_launch_rows64(const AttnLaunch& a);   // D = 128 only: 64 query rows per wavefront

// Does this problem take the kernel with 64 query rows per wavefront?  (Workgroups of 256 rows either way.)
inline bool attn_takes_rows64(long long BH, int S, int D) {
    return ATTN_ROWS64 != 0 && D == 128 && attn_pick_nw(BH, S) == ATTN_NW;
}
