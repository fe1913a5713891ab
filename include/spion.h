/*
 * spion.h - C ABI of the MI355X (gfx950) implementation of SPION's layer-wise sparse attention.
 *
 * Paper: "SPION: Layer-Wise Sparse Training of Transformer via Convolutional Flood Filling".
 * The library covers the hot path of the method:
 *   spion_pattern   - Algorithm 3 (generate_pattern): diagonal convolution (Eq. 3), average pooling
 *                     (Eq. 4), flood fill (Algorithm 4) from the first-row and first-column seeds,
 *                     forced diagonal, and the conversion of the pattern to a compressed index
 *                     (Section 4.3; kept at block granularity as BSR plus its transpose BSC, since
 *                     the upsampled pattern P is constant inside each B x B block).
 *   spion_attn_fwd  - Algorithm 5 lines 4-7 / Eq. 5: SDDMM S = scale * Q K^T on the kept blocks, row
 *                     softmax over the kept entries (Algorithm 6), SpMM O = P V; fused in one kernel.
 *   spion_attn_bwd  - the gradient of Eq. 5 with respect to Q, K and V (Section 4.3, "Integration of
 *                     GPU kernels with PyTorch", states that forward and backward kernels exist).
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its comment says HOST.  The caller owns all buffers;
 *     the library never allocates or frees device memory and keeps no state between calls (the one
 *     exception, the built-in scratch array of spion_pattern_static, is described there).
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = the null stream) and
 *     the call returns without synchronising.  Outputs are valid once the stream reaches that point.
 *   - Return value: SPION_OK (0) or a negative spion_status.  Argument errors are detected on the
 *     host before anything is enqueued; nothing is written in that case.
 *   - Tensors Q, K, V, O, dO, dQ, dK, dV are [B, H, L, d] contiguous (d fastest) in the element type
 *     named by `dtype`; LSE is fp32 [B, H, L].  Supported: d == 64, block in {16, 32, 64},
 *     L % block == 0, L / block <= SPION_MAX_NB, and B * H * (L / block) < 2^31 (one workgroup per
 *     block row and head; the backward also needs B * H * (nnzb / 16 + 2 L / block) < 2^31).  A shape
 *     outside these limits is SPION_ERR_SHAPE.
 *   - One pattern (one BSR/BSC index) is shared by all batch items and heads of a layer.
 */
#ifndef SPION_H_
#define SPION_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPION_MAX_NB 1024 /* largest supported number of block rows L / block */
#define SPION_STATIC_MAX_NB 256 /* largest L / block spion_pattern_static accepts */

typedef enum {
    SPION_OK = 0,
    SPION_ERR_NULL = -1,      /* a required pointer is NULL */
    SPION_ERR_SHAPE = -2,     /* unsupported L, d, block, B, H or nnzb */
    SPION_ERR_DTYPE = -3,     /* dtype is not SPION_F32 / SPION_BF16 */
    SPION_ERR_WORKSPACE = -4, /* workspace missing, misaligned (256 B) or too small */
    SPION_ERR_PARAM = -5,     /* even filter, filter too large, quantile outside [0,1], bad flags */
    SPION_ERR_INDEX = -6,     /* malformed block-sparse index (written by spion_index_check only) */
    SPION_ERR_HIP = -7,       /* a HIP runtime call failed (launch error) */
    SPION_ERR_TOO_LARGE = -8  /* spion_pattern_static only: L / block > SPION_STATIC_MAX_NB */
} spion_status;

typedef enum { SPION_F32 = 0, SPION_BF16 = 1 } spion_dtype;

/* How the flood-fill threshold t is derived from pool_out (Section 4.2 uses the alpha% quantile). */
typedef enum {
    SPION_T_ABS = 0,      /* thresh_value is t itself, in pool_out units */
    SPION_T_QUANTILE = 1, /* thresh_value = q in [0,1]: t = sorted(pool_out)[floor(q*(n-1))], n = nb^2 */
    SPION_T_MEAN_KSTD = 2 /* thresh_value = k: t = mean + k * population std of pool_out */
} spion_thresh_mode;

/* spion_pattern_params.flags */
#define SPION_PATTERN_NO_FILL 1u /* SPION-C variant (Section 5): keep every block above t, no flood fill */
/* The two halves of Algorithm 3 on their own.  Eq. 3 and Eq. 4 are linear in A_s and the pooled sums
 * are exact integers, so the pool_sum maps of partial score maps (one per GPU of a sharded batch,
 * say) can be added element by element by the caller and handed to the second half. */
#define SPION_PATTERN_POOL_ONLY 2u /* Eq. 3 + Eq. 4 only: writes pool_sum (required) and nothing else */
#define SPION_PATTERN_FROM_POOL 4u /* threshold, flood fill, compaction from a given pool_sum (required,
                                      read only); A_s is not read and may be NULL */

typedef struct {
    int32_t L;            /* sequence length */
    int32_t block;        /* block size B of pooling / upsampling */
    int32_t filter;       /* diagonal filter size F, odd, (F-1)/2 < block; 1 = no convolution (SPION-F) */
    int32_t thresh_mode;  /* spion_thresh_mode */
    double thresh_value;  /* t, q or k, see spion_thresh_mode */
    uint32_t flags;       /* SPION_PATTERN_* bits, otherwise 0 */
    uint32_t reserved;    /* must be 0 */
} spion_pattern_params;

/* Bytes of device scratch spion_pattern needs for (L, block); 0 if the shape is unsupported. */
size_t spion_pattern_workspace_bytes(int32_t L, int32_t block);

/*
 * Algorithm 3 on the GPU.
 *   A_s       [L, L] fp32 row-major, the head/batch-averaged attention-score map; every entry must be
 *             finite with |a| <= 1 (scores are quantised to 2^-40 fixed point so that the sums of
 *             Eq. 3 and Eq. 4 are exact integers and the == / > tests of Algorithm 4 are exact).
 *   p         HOST pointer to the parameters.
 *   fl_out    [nb, nb] uint8, nb = L / block: the block-level pattern after the diagonal is forced.
 *   row_ptr   [nb + 1], col_idx [capacity nb * nb; the first nnzb entries are written]: BSR index,
 *             block rows in order, block columns ascending inside a row.
 *   col_ptr   [nb + 1], row_idx [nb * nb], bsr_pos [nb * nb]: the transposed index (BSC), columns in
 *             order, rows ascending; bsr_pos[k] is the position in col_idx of the k-th BSC entry.
 *             The three may all be NULL if the caller needs no backward pass.
 *   nnzb      device int32 scalar, number of kept blocks (== row_ptr[nb]).
 *   pool_sum  optional [nb, nb] int64 output: block sums of the convolution output in fixed point,
 *             pool_out = pool_sum / (block^2 * 2^40).  May be NULL unless a SPION_PATTERN_*_POOL flag
 *             is set.  With SPION_PATTERN_POOL_ONLY every other output pointer may be NULL.
 *   workspace at least spion_pattern_workspace_bytes(L, block) bytes, 256-byte aligned.
 */
int spion_pattern(const float *A_s, const spion_pattern_params *p, uint8_t *fl_out, int32_t *row_ptr,
                  int32_t *col_idx, int32_t *col_ptr, int32_t *row_idx, int32_t *bsr_pos,
                  int32_t *nnzb, int64_t *pool_sum, void *workspace, size_t workspace_bytes,
                  void *hip_stream);

/*
 * spion_pattern for callers that cannot allocate device memory or carry a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, outputs and
 * results as spion_pattern without `workspace` / `workspace_bytes`: the scratch (per-block partial
 * sums, pooled sums, cell bits, transposed mask, positions) lives in a 5 MiB array that is part of the library's device
 * image, one copy per GPU, held until the process ends.  The call allocates and frees nothing.
 *   - L / block must not exceed SPION_STATIC_MAX_NB (256; e.g. L = 16384 at block 64), else
 *     SPION_ERR_TOO_LARGE is returned and nothing is enqueued.
 *   - The array's address is looked up on the first call on each device (the device current at the
 *     call, which must be the stream's device); make that first call outside a graph capture.
 *   - All calls on one GPU share the array: the kernels overwrite what they use and rely on nothing a
 *     previous call left there, but two calls that overlap on the same GPU (different streams, or graphs replayed concurrently) race.
 */
int spion_pattern_static(const float *A_s, const spion_pattern_params *p, uint8_t *fl_out,
                         int32_t *row_ptr, int32_t *col_idx, int32_t *col_ptr, int32_t *row_idx,
                         int32_t *bsr_pos, int32_t *nnzb, int64_t *pool_sum, void *hip_stream);

/*
 * Checks a block-sparse index (the compressed form of the pattern, Section 4.3) before it is handed
 * to spion_attn_fwd / spion_attn_bwd, which trust it: an index produced by spion_pattern is always
 * well formed, one built elsewhere may not be, and an entry out of range would be an out-of-bounds
 * access there.  Writes SPION_OK or SPION_ERR_INDEX to the device int32 `status` (read it back after
 * the stream has reached this point).  Checked: row_ptr runs from 0 to nnzb without decreasing; the
 * block columns of every row lie in [0, nb) and ascend strictly; and, when the transposed index is
 * given (col_ptr, row_idx, bsr_pos: all three or none), the same for it, plus bsr_pos[k] naming the
 * position in col_idx of the very block (row_idx[k], column of k).  nb = L / block, nb <= SPION_MAX_NB.
 */
int spion_index_check(const int32_t *row_ptr, const int32_t *col_idx, const int32_t *col_ptr,
                      const int32_t *row_idx, const int32_t *bsr_pos, int32_t nb, int32_t nnzb,
                      int32_t *status, void *hip_stream);

/* spion_attn_params.flags */
#define SPION_ATTN_PAPER_DENOM 1u /* add Algorithm 6's exp(-max) * (L - kept) term to the row sum */
/* spion_attn_bwd only: run one of its two sides on its own (for per-side timing).  The bf16 kernels
 * for block 32 / 64 compute both sides in one launch and either side alone is self-contained; in the
 * other kernels the key side reads what the query side of an earlier call with the same arguments
 * and workspace left there (delta, the key-side work list). */
#define SPION_ATTN_BWD_QUERY_SIDE_ONLY 2u /* delta and dQ only */
#define SPION_ATTN_BWD_KEY_SIDE_ONLY 4u   /* dK and dV only */

typedef struct {
    int32_t B, H, L, d;  /* batch, heads, sequence length, head dimension (64) */
    int32_t block;       /* block size of the pattern: 16, 32 or 64 */
    int32_t dtype;       /* spion_dtype of Q, K, V, O, dO, dQ, dK, dV */
    float scale;         /* score scale; 0 means 1 / sqrt(d) (Eq. 5) */
    uint32_t flags;      /* SPION_ATTN_* bits, otherwise 0 */
} spion_attn_params;

/* Bytes of device scratch for the forward (is_bwd == 0) or backward (is_bwd != 0) call;
 * (size_t)-1 if the parameters are unsupported. */
size_t spion_attn_workspace_bytes(const spion_attn_params *p, int32_t nnzb, int32_t is_bwd);

/*
 * Eq. 5 on the kept blocks: for every (batch, head) and every block row I,
 *   S_IJ = scale * Q_I K_J^T for J in the row's kept columns, P = softmax over the kept entries of
 *   each row, O_I = sum_J P_IJ V_J, LSE_i = log sum_j exp(S_ij).
 * A block row with no kept block gives O = 0 and LSE = -inf.
 *   Q, K, V   inputs [B, H, L, d];  O output [B, H, L, d];  LSE output fp32 [B, H, L].
 *   row_ptr, col_idx, nnzb  BSR index from spion_pattern (nnzb passed by value, as read back by the
 *             caller); 0 <= col_idx < nb and row_ptr must be non-decreasing with row_ptr[nb] == nnzb.
 *   p         HOST pointer.  workspace may be NULL when spion_attn_workspace_bytes(...) is 0.
 */
int spion_attn_fwd(const void *Q, const void *K, const void *V, void *O, float *LSE,
                   const int32_t *row_ptr, const int32_t *col_idx, int32_t nnzb,
                   const spion_attn_params *p, void *workspace, size_t workspace_bytes,
                   void *hip_stream);

/*
 * Gradient of spion_attn_fwd:
 *   delta_i = sum_c dO_ic O_ic;  P = exp(S - LSE);  dV_J += P^T dO_I;  dP = dO_I V_J^T;
 *   dS = P .* (dP - delta);  dQ_I += scale * dS K_J;  dK_J += scale * dS^T Q_I.
 *   Q, K, V, O, dO, LSE  as produced by / passed to spion_attn_fwd with the same index and params.
 *   dQ, dK, dV  outputs [B, H, L, d]; overwritten (not accumulated).  Results are deterministic.
 *   col_ptr, row_idx, bsr_pos  BSC index from spion_pattern (all required).  The kernels walk col_ptr /
 *             row_idx; bsr_pos is not read by them (it is what spion_index_check uses to prove that the
 *             BSC arrays are the transpose of the BSR ones) but must be passed, so that an index cannot be
 *             handed over without its transpose.
 */
int spion_attn_bwd(const void *Q, const void *K, const void *V, const void *O, const void *dO,
                   const float *LSE, void *dQ, void *dK, void *dV, const int32_t *row_ptr,
                   const int32_t *col_idx, const int32_t *col_ptr, const int32_t *row_idx,
                   const int32_t *bsr_pos, int32_t nnzb, const spion_attn_params *p,
                   void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Producers of the pattern input.
 *
 * spion_score_mean: the score maps of the heads (and batch items) of a layer are averaged into the
 * one map that pattern generation works on (Section 3: the heads of a layer show similar patterns).
 *   A_maps  [n_maps, L, L] contiguous, dtype SPION_F32 or SPION_BF16;  A_s output [L, L] fp32:
 *   A_s[i] = (A_maps[0][i] + A_maps[1][i] + ... in that order, fp32) * (1 / n_maps).  L % 8 == 0.
 *
 * spion_frobenius_distance: Eq. 2, distance = | ||A_prev||_F - ||A_cur||_F |, the quantity whose
 * stagnation ends the dense-attention phase (Section 4.1).  fp64 accumulation, fixed summation order.
 *   A_prev, A_cur  fp32 arrays of n elements (16-byte aligned);
 *   out            device double[3]: {distance, ||A_prev||_F, ||A_cur||_F};
 *   workspace      at least spion_frobenius_workspace_bytes() bytes, 256-byte aligned.
 */
int spion_score_mean(const void *A_maps, int32_t n_maps, int32_t L, int32_t dtype, float *A_s,
                     void *hip_stream);
size_t spion_frobenius_workspace_bytes(void);
int spion_frobenius_distance(const float *A_prev, const float *A_cur, int64_t n, double *out,
                             void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Measurement aid (Section 5 reports time and memory; this library reports them against the HBM
 * roofline): copies n_bytes (a positive multiple of 16384; src, dst 16-byte aligned, not overlapping)
 * with the access shapes of the attention kernels - 16 bytes per lane from memory straight into LDS,
 * 16 bytes per lane row stores out - reading and writing every byte exactly once.  A launch of known
 * traffic: what a profiler's memory counters report for it is the scale for their readings of the
 * other kernels in the same run.
 */
int spion_copy_yardstick(const void *src, void *dst, size_t n_bytes, void *hip_stream);

/* Static, NUL-terminated description of a spion_status value. */
const char *spion_strerror(int status);

/* Library version, major * 10000 + minor * 100 + patch. */
int spion_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPION_H_ */
