/*
 * attn.h -- C ABI of the gfx950 fused multi-head attention forward.
 *
 * The operation is the attention kernel class that the paper names first
 * among the specialised LLM kernels (Introduction) and evaluates as one of
 * six kernels (Table 2: B, n_head, seq_len, d_head).  The paper gives no
 * formula; the definition is the standard one:
 *
 *     for every batch b, head h, query row i:
 *         J      = {0..S-1}                     causal == 0
 *                = {0..i}                       causal != 0 (diagonal included)
 *         s_j    = scale * sum_d q[i,d] k[j,d]
 *         lse_i  = ln sum_{j in J} exp(s_j)                 (natural log)
 *         O[i,:] = sum_{j in J} exp(s_j - lse_i) v[j,:]
 *
 * One fixed kernel per (D, dtype, causal) with a hand-set instruction
 * schedule -- the paper's framing of a fixed kernel whose schedule is tuned
 * for throughput (Sections 2.4 and 3.5) -- never visible through this ABI.
 */
#ifndef PAPER_2501_08071_ATTN_H
#define PAPER_2501_08071_ATTN_H

#ifdef __cplusplus
extern "C" {
#endif

/* Element type of q, k and v.  o and lse are always fp32. */
typedef enum { ATTN_F16 = 0, ATTN_BF16 = 1 } attn_dtype_t;

typedef enum {
    ATTN_OK = 0,
    ATTN_ERR_NULL = -1,        /* q, k, v or o is NULL                               */
    ATTN_ERR_SHAPE = -2,       /* B, H, S or D <= 0, or a tensor above 2^40 elements */
    ATTN_ERR_DTYPE = -3,       /* dtype is not an attn_dtype_t                       */
    ATTN_ERR_SCALE = -4,       /* scale is NaN or infinite                           */
    ATTN_ERR_UNSUPPORTED = -5, /* valid request with no kernel instance (D)          */
    ATTN_ERR_LAUNCH = -6,      /* the HIP runtime refused the launch                 */
    ATTN_ERR_ALIGN = -7        /* a pointer is not 16-byte aligned                   */
} attn_status_t;

/*
 * Fused attention forward (the attention row of Table 2; definition above).
 *
 *   q, k, v  DEVICE pointers, [B,H,S,D] contiguous with D fastest, elements of
 *            type `dtype` (IEEE binary16 or bfloat16).  Read only.
 *   o        DEVICE pointer, [B,H,S,D] contiguous fp32.  Written.
 *   lse      DEVICE pointer, [B,H,S] fp32, natural-log logsumexp of the scaled,
 *            masked logits; may be NULL (then it is not written).
 *   B,H,S,D  batch, heads, sequence length (queries == keys), head dimension.
 *            Any S >= 1; D must be 32, 64 or 128.
 *   causal   0: every key visible; non-zero: key j visible to query i iff j <= i.
 *            Masked keys enter the second product with weight 0, so q, k and v must be
 *            finite everywhere: a non-finite row j of v spoils, next to the rows of O
 *            that see key j, the earlier rows of the same block of 64 keys (0 * Inf).
 *   scale    multiplies q.k before the softmax; any finite value.
 *   dtype    attn_dtype_t of q, k, v.
 *   stream   hipStream_t to enqueue on (NULL = the default stream).
 *
 * Ownership: the caller owns every buffer; the library allocates nothing and
 * never synchronises.  Its only state is one flag per device and kernel
 * instance: that the runtime has been told the instance's LDS size (set once,
 * atomically; calls from several host threads are safe).  The call is asynchronous: outputs are valid
 * once `stream` has been synchronised.  o and lse must not alias q, k or v.
 * All pointers must be 16-byte aligned.
 *
 * Errors: returns an attn_status_t and never throws or aborts.  Every argument
 * is checked before the first HIP call, so bad arguments are reported on a
 * machine without a GPU too.
 */
int attn_fwd(const void *q, const void *k, const void *v, float *o, float *lse,
             int B, int H, int S, int D, int causal, float scale, int dtype, void *stream);

/*
 * The same operation with O written in the type of q, k and v (Table 2 gives the kernel's inputs as
 * fp16 tensors; a layer that feeds the next one in half precision wants O that way), rounded to
 * nearest even from the fp32 result (so its error is that of attn_fwd plus one rounding of O: at most
 * 2^-9 |O| for bfloat16, 2^-12 |O| for binary16).  `o` is [B,H,S,D] contiguous in `dtype`; lse stays fp32.  Every
 * other argument, the ownership and error rules are those of attn_fwd; both share one kernel.
 */
int attn_fwd_o16(const void *q, const void *k, const void *v, void *o, float *lse,
                 int B, int H, int S, int D, int causal, float scale, int dtype, void *stream);

/* 1 if attn_fwd has a kernel instance for this request, else 0 (no HIP call). */
int attn_supported(int S, int D, int dtype, int causal);

/* Static, NUL-terminated description of an attn_status_t (never NULL). */
const char *attn_status_str(int status);

/*
 * Name of the kernel attn_fwd launches for this very problem (the symbol a
 * profiler reports; it depends on B and H because small problems take the
 * instance with half the wavefronts, see attn_launch_rows), or NULL if
 * unsupported.  A string constant: no HIP call, safe from any thread.
 */
const char *attn_kernel_name(int B, int H, int S, int D, int dtype, int causal);

/*
 * Query rows per workgroup and keys per inner-loop tile of that kernel
 * (0 if unsupported).  For harnesses that pick tile-edge rows to check.
 */
int attn_tile_rows(int D, int dtype, int causal);
int attn_tile_keys(int D, int dtype, int causal);

/*
 * Query rows per workgroup attn_fwd uses for this very problem: attn_tile_rows, or half of it (the
 * same kernel with half the wavefronts, "..., 4>" in its name) when the problem has so few tiles
 * that the larger ones would leave half of the chip idle.  0 if unsupported.
 */
int attn_launch_rows(int B, int H, int S, int D, int dtype, int causal);

#ifdef __cplusplus
}
#endif
#endif
