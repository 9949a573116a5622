/*
 * gemm.h -- C ABI of the fused GEMM + LeakyReLU for gfx950.
 *
 * The paper's second compute-bound kernel (Table 2: mmLeakyReLu, B, M, N, K =
 * 1, 512, 512, 2048, float16; Section 5.1 describes it as a matrix product with
 * the activation fused into its epilogue; Section 5.4 analyses its schedule).  No formula is given;
 * the definition is the plain one:
 *
 *     c[i, m, n] = f( sum_k a[i, m, k] * b[i, k, n] ),   f(t) = t if t >= 0 else slope * t
 *
 * Products are accumulated in fp32; the activation is applied in fp32 and the
 * result rounded to nearest even into the input type.
 */
#ifndef PAPER_2501_08071_GEMM_H
#define PAPER_2501_08071_GEMM_H

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { GEMM_F16 = 0, GEMM_BF16 = 1 } gemm_dtype_t;

typedef enum {
    GEMM_OK = 0,
    GEMM_ERR_NULL = -1,    /* a, b or c is NULL while there is something to compute   */
    GEMM_ERR_SHAPE = -2,   /* batch, M, N < 0, K < 0, or a matrix above 2^31 elements */
    GEMM_ERR_DTYPE = -3,   /* dtype is not a gemm_dtype_t                             */
    GEMM_ERR_SLOPE = -4,   /* slope is NaN or infinite                                */
    GEMM_ERR_ALIGN = -6,   /* a pointer is not 16-byte aligned                        */
    GEMM_ERR_LAUNCH = -7   /* the HIP runtime refused the launch                      */
} gemm_status_t;

/*
 * Fused matrix product and LeakyReLU (Table 2's mmLeakyReLu row; definition above).
 *
 *   a        DEVICE pointer, [batch, M, K] contiguous (K fastest), elements of `dtype`.  Read only.
 *   b        DEVICE pointer, [batch, K, N] contiguous (N fastest), elements of `dtype`.  Read only.
 *   c        DEVICE pointer, [batch, M, N] contiguous, elements of `dtype`.  Written; must not alias a or b.
 *   batch, M, N, K   any sizes >= 0.  batch, M or N == 0: nothing to compute, nothing is launched.
 *            K == 0: every sum is empty and c is all zeros.  With K % 32 == 0 and N % 8 == 0 the matrix
 *            cores are used (any M, any such N); other shapes take a plain kernel, one thread per
 *            element of c.
 *   slope    factor of the negative side; any finite value (0.01 in the kernel the paper evaluates).
 *   dtype    gemm_dtype_t of a, b and c.
 *   stream   hipStream_t to enqueue on (NULL = the default stream).
 *
 * Ownership, asynchrony and alignment as for attn_fwd: the caller owns every buffer, the library
 * allocates nothing, keeps no state and never synchronises; pointers are 16-byte aligned.  Returns a
 * gemm_status_t; every check is made before the first HIP call.
 */
int gemm_leakyrelu_fwd(const void* a, const void* b, void* c, int batch, int M, int N, int K, float slope,
                       int dtype, void* stream);

/* Which code path serves this shape: 1, 2, 3 = matrix cores with tiles of 256 x 256, 128 x 128, 64 x 64 (the
 * largest that still gives most of the chip a workgroup); 5 = matrix cores with tiles of 32 x 32 and K split over
 * the wavefronts of a workgroup (small problems with K >= 256, the paper's 512 x 512 x 2048 among them); 4 = the
 * plain kernel; 0 = the shape or dtype is not accepted. */
int gemm_path(int batch, int M, int N, int K, int dtype);

/* Static, NUL-terminated description of a status code; never NULL. */
const char* gemm_status_str(int status);

#ifdef __cplusplus
}
#endif
#endif
