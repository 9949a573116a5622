/*
 * rowops.h -- C ABI of the two memory-bound row kernels for gfx950.
 *
 * The paper evaluates two memory-bound kernels next to the compute-bound ones
 * (Table 2: softmax, n_rows x n_cols = 512 x 4096; rmsnorm, B x n_head x
 * seq_len x d_head = 1 x 32 x 4096 x 64; float16) and names them without a
 * formula (Section 5.1).  The definitions are the standard ones:
 *
 *     softmax   y[i,j] = exp(x[i,j] - m_i) / sum_j' exp(x[i,j'] - m_i),  m_i = max_j x[i,j]
 *     rmsnorm   y[i,j] = x[i,j] / sqrt(mean_j' x[i,j']^2 + eps) * w[j]
 *
 * Both read every input byte once and write every output byte once; the
 * arithmetic is fp32, the result is rounded to nearest even into the input
 * type.
 */
#ifndef PAPER_2501_08071_ROWOPS_H
#define PAPER_2501_08071_ROWOPS_H

#ifdef __cplusplus
extern "C" {
#endif

/* Element type of x, w and y (the same numbering as attn_dtype_t). */
typedef enum { ROWOPS_F16 = 0, ROWOPS_BF16 = 1 } rowops_dtype_t;

typedef enum {
    ROWOPS_OK = 0,
    ROWOPS_ERR_NULL = -1,    /* x, y (or w) is NULL while n_rows > 0             */
    ROWOPS_ERR_SHAPE = -2,   /* n_rows < 0, row length <= 0 or above 2^24,
                                or more than 2^40 elements                       */
    ROWOPS_ERR_DTYPE = -3,   /* dtype is not a rowops_dtype_t                    */
    ROWOPS_ERR_EPS = -4,     /* eps is negative, NaN or infinite                 */
    ROWOPS_ERR_ALIGN = -6,   /* a pointer is not 16-byte aligned                 */
    ROWOPS_ERR_LAUNCH = -7   /* the HIP runtime refused the launch               */
} rowops_status_t;

/*
 * Row softmax (Table 2's softmax row; definition above).
 *
 *   x        DEVICE pointer, [n_rows, n_cols] contiguous, elements of `dtype`.  Read only.
 *   y        DEVICE pointer, [n_rows, n_cols] contiguous, elements of `dtype`.  Written.
 *            May be the same buffer as x (a row is read completely before it is written).
 *   n_rows   any number of rows >= 0; 0 is an empty input: nothing is launched.
 *   n_cols   row length, 1 .. 2^24.  Rows of up to 16384 elements with n_cols % 8 == 0 stay in
 *            registers between the read and the write; other lengths are read three times.
 *   dtype    rowops_dtype_t of x and y.
 *   stream   hipStream_t to enqueue on (NULL = the default stream).
 *
 * Inputs are assumed finite.  Ownership, asynchrony and alignment as for attn_fwd: the caller owns
 * every buffer, the library allocates nothing and never synchronises, pointers are 16-byte aligned.
 * Returns a rowops_status_t; every check is made before the first HIP call.
 */
int softmax_rows_fwd(const void* x, void* y, long long n_rows, int n_cols, int dtype, void* stream);

/*
 * RMS normalisation over the last dimension (Table 2's rmsnorm row; definition above).
 *
 *   x        DEVICE pointer, [n_rows, d] contiguous (for the paper's shape n_rows = B * n_head *
 *            seq_len and d = d_head), elements of `dtype`.  Read only.
 *   w        DEVICE pointer, [d] weight, elements of `dtype`.  Read only.
 *   y        DEVICE pointer, [n_rows, d] contiguous, elements of `dtype`.  Written.  May be x.
 *   n_rows   >= 0; 0 launches nothing.
 *   d        row length, 1 .. 2^24.  With d % 8 == 0 and d <= 16384 a row stays in registers (several
 *            rows per wavefront when d <= 256); other lengths are read twice.
 *   eps      added to the mean of squares under the root; finite, >= 0.
 *   dtype, stream, ownership, errors: as above.
 */
int rmsnorm_fwd(const void* x, const void* w, void* y, long long n_rows, int d, float eps, int dtype,
                void* stream);

/* Which code path serves rows of this length: 1 = the row stays in registers (one read), 2 = the
 * general path (several reads), 0 = the length or dtype is not accepted.  op: 0 softmax, 1 rmsnorm. */
int rowops_path(int op, int row_len, int dtype);

/* Static, NUL-terminated description of a status code; never NULL. */
const char* rowops_status_str(int status);

#ifdef __cplusplus
}
#endif
#endif
