/*
 * probe.h -- measuring aids exported by the same library as the kernels.
 *
 * None of these is an operation of the paper and none cites a passage: they are small kernels whose measured
 * rates serve as denominators next to the published peaks (what the matrix cores sustain under load, what the
 * vector pipes need for the softmax of one score, what the L2 delivers, what a launch costs by itself).  No
 * product path calls them; the bench harness and its tests do.
 *
 * All pointers are DEVICE pointers owned by the caller; nothing is allocated, nothing synchronises; every call
 * enqueues one kernel on `stream` (a hipStream_t, NULL = the default stream) and is timed by the caller.
 * Bad arguments and refused launches return -1.
 */
#ifndef PAPER_2501_08071_PROBE_H
#define PAPER_2501_08071_PROBE_H

#ifdef __cplusplus
extern "C" {
#endif

/*
 * `workgroups` workgroups of four wavefronts that issue nothing but independent 32x32x16 matrix instructions
 * of `dtype` (0 binary16, 1 bfloat16), `iters` x 16 each, on constant (random_operands == 0) or random
 * operands.  Returns the floating-point operations of the launch.  out: workgroups * 256 floats, written.
 */
long long probe_mfma(float *out, int workgroups, int iters, int dtype, int random_operands, void *stream);

/*
 * The vector work of the softmax of one score, `iters` x 16 scores per lane in `workgroups` workgroups of 256
 * lanes: a multiply-add and an exp2 (full == 0), plus the row-sum addition and half a two-into-one conversion
 * to bfloat16 (full != 0).  Returns the number of scores.  out: workgroups * 256 floats, written.
 */
long long probe_softmax_valu(float *out, int workgroups, int iters, int full, void *stream);

/*
 * Workgroup b (256 lanes) reads region b % 8 of `buf` -- eight regions of region_kib KiB each, region_kib a
 * multiple of 32 -- `iters` times, 16 bytes per lane and instruction.  With a region that fits an XCD's L2 all
 * passes but the first are L2 hits.  Returns the bytes read.  buf: 8 * region_kib KiB, 16-byte aligned, read;
 * out: workgroups * 256 floats, written.
 */
long long probe_l2_read(const void *buf, float *out, int region_kib, int workgroups, int iters, void *stream);

/*
 * What a matrix instruction takes from the instruction issue of the other wavefront on its SIMD.  `workgroups`
 * workgroups of eight wavefronts, two per SIMD, one workgroup per compute unit (96 KiB of LDS each).  On every
 * SIMD one wavefront does the softmax's vector work of `iters` x 32 scores per lane -- vector_mode 1: multiply-add,
 * exp2, row-sum addition, half a conversion to bfloat16; 2: multiply-add, exp2, half a conversion to binary16, half
 * a two-way dot product; 0: it exits at once -- and, if matrix_on != 0, the other issues 32x32x16 bfloat16 matrix
 * instructions until its partner is done (vector_mode 0: `iters` x 32 of them).  matrix_on == 0 needs
 * vector_mode != 0.
 * out: workgroups * 8 pairs of 64-bit integers, written: for wavefront w of workgroup b, out[2 (8 b + w)] = shader
 * clock cycles its loop took, out[2 (8 b + w) + 1] = iterations of 32 (matrix instructions for w < 4, scores per lane
 * for w >= 4) it made.  Returns 0.
 */
int probe_issue_share(long long *out, int workgroups, int iters, int matrix_on, int vector_mode, void *stream);

/* A kernel that does nothing, `workgroups` x `threads`: the cost of a launch by itself.  Returns 0. */
int probe_empty(int workgroups, int threads, void *stream);

#ifdef __cplusplus
}
#endif
#endif
