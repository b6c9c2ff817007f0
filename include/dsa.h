/*
 * dsa.h -- C ABI of the MI355X (gfx950) Dynamic Sparse Attention forward path.
 *
 * The path is the per-layer attention forward of "Transformer Acceleration with Dynamic
 * Sparse Attention" (arXiv 2110.11299):
 *
 *   (a) approximate scores  S~ = Q~ K~^T  from reduced-dimension, int8 query / key
 *       projections (section 3.1, equation 5 and the paragraph after it; "essentially a
 *       low-precision GEMM", section 3.4);
 *   (b) a sparse mask M with the same number of kept keys in every row, found by top-k over
 *       S~ (section 3.1; section 4.2 "keep 10% of the attention weights in each row";
 *       section 5.2 row-wise constraint), at fine-grained or column-vector granularity
 *       (section 5.1, figure 9);
 *   (c) exact attention at the kept positions only: SDDMM  S = Q K^T|_M  (equation 2),
 *       softmax over the kept entries (equation 4: masked entries get weight 0), and
 *       SpMM  Z = A V  (equation 3) -- section 3.4 and section 5.1.
 *
 * Conventions for every entry point
 * ---------------------------------
 *  - Every data pointer is a DEVICE pointer to memory the caller owns (allocated, for
 *    instance, by PyTorch).  The library allocates nothing, frees nothing and never
 *    synchronises: kernels are enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *    the default stream) and the call returns.  Inputs are only read, outputs are fully
 *    overwritten, and no call depends on an earlier one (the library only remembers launch
 *    parameters it has derived for a device).  Pointers must be 16-byte aligned.
 *  - Tensors are contiguous, innermost dimension last:
 *        Q, K, V   [B, H, L, d]   float (DSA_F32) or bfloat16 bit patterns (DSA_BF16)
 *        Qt, Kt    [B, H, L, k]   int8, the quantised projections Q~, K~
 *        idx       [B, H, L/vec, keep]  int32: the mask in ELL form.  Entry (b,h,u,:) lists,
 *                  ascending, the kept key positions of selection unit u: query row u when
 *                  vec = 1, query rows [vec*u, vec*u+vec) when vec = 4 or 8 (they share a list).
 *        S, P      [B, H, L, keep]  float: exact scores / attention weights at the kept
 *                  positions of each query row, in the order of its unit's list
 *        O         [B, H, L, d]   float
 *  - Selection rule (b): unit u keeps the `keep` keys j with the largest score, where the
 *    score is S~[u, j] (vec = 1) or the sum of S~[i, j] over the unit's vec rows (vec = 4, 8),
 *    compared as signed integers; among equal scores the lower j wins.  The result is unique,
 *    so idx is reproducible bit for bit.
 *  - Argument checking happens on the host before anything is launched; a call that returns
 *    an error has launched nothing.  Errors never cross the ABI as exceptions or aborts.
 */
#ifndef DSA_H
#define DSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DSA_OK = 0,
    DSA_ERR_NULL = 1,        /* a required pointer is NULL                                    */
    DSA_ERR_SHAPE = 2,       /* a dimension is out of range (see dsa_shape)                   */
    DSA_ERR_UNSUPPORTED = 3, /* valid in principle, not built: vec, k, d, dtype, size limits  */
    DSA_ERR_ALIGN = 4,       /* a pointer is not 16-byte aligned                              */
    DSA_ERR_WORKSPACE = 5,   /* workspace missing or smaller than dsa_workspace_bytes()       */
    DSA_ERR_HIP = 6          /* the HIP runtime refused a launch                              */
} dsa_status;

typedef enum { DSA_F32 = 0, DSA_BF16 = 1 } dsa_dtype;

/* Problem statement of one attention layer (section 2.1 for B, H, L, d; section 3.1 for k;
 * section 4.2 for keep; section 5.1 for vec). */
typedef struct {
    int32_t B, H;   /* batch, heads: B*H independent problems, each >= 1                      */
    int32_t L;      /* sequence length, L % vec == 0; 1 <= L <= 32768 for the predictor,      */
                    /* L <= 4194304 (2^22) for the attention entry points                     */
    int32_t d;      /* head dimension of Q, K, V: 64 or 128                                   */
    int32_t k;      /* projection dimension of Qt, Kt: a multiple of 16, 16 <= k <= 128       */
    int32_t keep;   /* kept keys per selection unit, 1 <= keep <= L (attention: <= 4096)      */
    int32_t vec;    /* mask granularity in query rows: 1 (fine-grained), 4 or 8 (vector-wise: */
                    /* the 1x4 and 1x8 column vectors of section 5.1, table 3)                */
    int32_t dtype;  /* dsa_dtype of Q, K, V                                                   */
    float scale;    /* factor on the exact scores before softmax; 1/sqrt(d) in equation 2     */
} dsa_shape;

/* Kept count for a keep ratio: floor(ratio*L + 0.5) clamped to [1, L] ("keep 10%",
 * section 4.2).  Host only; no device work. */
int32_t dsa_keep_from_ratio(int32_t L, double ratio);

/* Bytes of device scratch that dsa_predict_mask / dsa_attention_fwd need for this shape
 * (0 is possible).  Returns 0 for an invalid shape. */
size_t dsa_workspace_bytes(const dsa_shape *shape);

/* Steps (a)+(b): approximate scores and top-k mask (section 3.1).  Reads Qt, Kt; writes idx.
 * S~ is never stored.  `ws` / `ws_bytes`: device scratch of at least dsa_workspace_bytes(). */
dsa_status dsa_predict_mask(const dsa_shape *shape, const int8_t *Qt, const int8_t *Kt,
                            int32_t *idx, void *ws, size_t ws_bytes, void *stream);

/* Step (c1), SDDMM (equation 2 at the kept positions; section 3.4):
 * S[b,h,i,t] = scale * sum_c Q[b,h,i,c] * K[b,h,idx[b,h,i/vec,t],c]. */
dsa_status dsa_sddmm(const dsa_shape *shape, const void *Q, const void *K, const int32_t *idx,
                     float *S, void *stream);

/* Step (c2), softmax over the kept entries of each row (equation 4; section 5.1 "Sparse
 * Softmax Computation").  P may alias S. */
dsa_status dsa_sparse_softmax(const dsa_shape *shape, const float *S, float *P, void *stream);

/* Step (c3), SpMM (equation 3; section 3.4):
 * O[b,h,i,:] = sum_t P[b,h,i,t] * V[b,h,idx[b,h,i/vec,t],:]. */
dsa_status dsa_spmm(const dsa_shape *shape, const float *P, const int32_t *idx, const void *V,
                    float *O, void *stream);

/* Steps (c1)-(c3) in one kernel given the mask: S and P stay on chip. */
dsa_status dsa_masked_attention(const dsa_shape *shape, const void *Q, const void *K,
                                const void *V, const int32_t *idx, float *O, void *stream);

/* The whole path (a)-(c) (figure 2(b)): predict the mask, then attend at the kept positions.
 * idx_out may be NULL; if not, it also receives the mask.  When idx_out is NULL the mask
 * lives in `ws`. */
dsa_status dsa_attention_fwd(const dsa_shape *shape, const void *Q, const void *K, const void *V,
                             const int8_t *Qt, const int8_t *Kt, float *O, int32_t *idx_out,
                             void *ws, size_t ws_bytes, void *stream);

/* dsa_attention_fwd for callers that cannot allocate device memory and so cannot bring a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * computation and same kernels as dsa_attention_fwd with idx_out = NULL, but the mask lives in a
 * fixed array inside the library's device image (dsa_noalloc_max_mask_bytes() = 16 MiB per GPU,
 * held until the process ends) instead of a caller workspace.  The call allocates and frees
 * nothing.  The first call on a device resolves the array's address (once per device).
 * A shape whose mask, B*H*(L/vec)*keep*4 bytes rounded up to 256, exceeds the array returns
 * DSA_ERR_WORKSPACE and launches nothing.  Every call on one GPU shares that GPU's array: calls
 * that overlap on one GPU (different streams or threads) race on the mask; calls on one stream
 * are ordered and safe.  Nothing in the array has to start at zero: each call overwrites the
 * part it reads. */
size_t dsa_noalloc_max_mask_bytes(void);
dsa_status dsa_attention_fwd_noalloc(const dsa_shape *shape, const void *Q, const void *K, const void *V,
                                     const int8_t *Qt, const int8_t *Kt, float *O, void *stream);

/* Step (a) alone with the smallest possible consumer, for measuring the int8 contraction:
 * rowmax[b,h,i] = max_j S~[b,h,i,j] (int32 [B,H,L]).  Uses B, H, L, k of the shape only. */
dsa_status dsa_approx_rowmax(const dsa_shape *shape, const int8_t *Qt, const int8_t *Kt,
                             int32_t *rowmax, void *stream);

/* The step in front of (a) (section 3.1, equation 5: the reduced-dimension, low-precision
 * projections), for one tensor X [B,H,L,d] (Q or K; dtype as in the shape) and one projection
 * matrix R [d,k] (float, row-major, device):
 *     Y[r,j] = sum_c X[r,c] R[c,j]   in fp32, as one chain of fused multiply-adds in increasing c,
 *     amax = max |Y| over the whole tensor,  s = 127 / amax  (fp32 division),
 *     Xt[r,j] = clip(rint(Y[r,j] * s), -127, 127)   (rint: halves to even; all zero if amax = 0),
 * so the int8 codes are reproducible bit for bit.  Xt is int8 [B,H,L,k]; amax_out (nullable, device
 * float) receives amax; `ws` is device scratch of at least dsa_project_workspace_bytes(). */
size_t dsa_project_workspace_bytes(const dsa_shape *shape);
dsa_status dsa_project_quantize(const dsa_shape *shape, const void *X, const float *R, int8_t *Xt,
                                float *amax_out, void *ws, size_t ws_bytes, void *stream);

/* Lower prediction precision (section 3.3 sets the prediction precision to INT4; table 2 sweeps
 * INT2 to INT16 and FP32).  `bits` is 8, 4 or 2.  The codes are the integers of magnitude up to
 * qmax = 2^(bits-1) - 1 (127, 7, 1), produced as in dsa_project_quantize with s = qmax / amax, and
 * stored two's complement with 8/bits codes per byte: code j of a row occupies bits
 * [bits * (j mod 8/bits), + bits) of byte j / (8/bits) of that row, rows contiguous
 * ([B,H,L,k*bits/8] bytes).  bits = 8 is dsa_project_quantize / dsa_predict_mask.
 *   dsa_project_quantize_bits: X, R, amax_out, ws as in dsa_project_quantize; Xt receives the
 *     packed codes.
 *   dsa_predict_mask_bits: steps (a)+(b) from packed codes.  gfx950 has no 4-bit or 2-bit integer
 *     matrix instruction, so the codes are widened to int8 in `ws` and the int8 path runs; the
 *     scores, and therefore the mask, are those of the integer codes exactly.  `ws` holds at least
 *     dsa_predict_workspace_bytes_bits(). */
dsa_status dsa_project_quantize_bits(const dsa_shape *shape, int32_t bits, const void *X, const float *R,
                                     void *Xt, float *amax_out, void *ws, size_t ws_bytes, void *stream);
/*   dsa_project_quantize_ternary: the same step with the paper's own projection (equation 5): a sparse random
 *     matrix P in sqrt(3/k) * {-1, 0, 1}^(d x k), so that Y = X P takes additions and subtractions only.  P3
 *     (int8 [d,k], row-major, device) holds the signs -1, 0, 1 (other values: undefined codes); the positive
 *     constant sqrt(3/k) cancels in the quantiser's scale qmax / max|Y| and is left out.  The sums are taken in
 *     fp32 in increasing c, so the codes equal those of dsa_project_quantize_bits with R = the signs as floats,
 *     bit for bit.  X, Xt, bits, amax_out, ws as in dsa_project_quantize_bits. */
dsa_status dsa_project_quantize_ternary(const dsa_shape *shape, int32_t bits, const void *X, const int8_t *P3,
                                        void *Xt, float *amax_out, void *ws, size_t ws_bytes, void *stream);
size_t dsa_predict_workspace_bytes_bits(const dsa_shape *shape, int32_t bits);
dsa_status dsa_predict_mask_bits(const dsa_shape *shape, int32_t bits, const void *Qt, const void *Kt,
                                 int32_t *idx, void *ws, size_t ws_bytes, void *stream);
/*   dsa_attention_fwd_bits: the whole path (a)-(c) as dsa_attention_fwd, from packed codes; `ws` holds
 *     at least dsa_workspace_bytes_bits() (the mask lives there when idx_out is NULL). */
size_t dsa_workspace_bytes_bits(const dsa_shape *shape, int32_t bits);
dsa_status dsa_attention_fwd_bits(const dsa_shape *shape, int32_t bits, const void *Q, const void *K,
                                  const void *V, const void *Qt, const void *Kt, float *O, int32_t *idx_out,
                                  void *ws, size_t ws_bytes, void *stream);

/* Measurement aid for step (a): runs `blocks` workgroups of 4 wavefronts, each issuing 4*iters
 * independent int8 MFMAs (32x32x32) with no memory traffic, i.e. 4*blocks*4*iters*65536 int8
 * operations in all.  Timing it gives the matrix-core rate the chip sustains at its own clocks,
 * to set beside the published peak when judging dsa_approx_rowmax.  `sink` (int32 [blocks*256],
 * device) receives values of no meaning. */
dsa_status dsa_mfma_i8_sustained(int32_t blocks, int32_t iters, int32_t *sink, void *stream);

/* Threshold masks (section 3.1: the mask M may be predicted from S~ "using thresholds" instead of a
 * top-k search; the threshold is a tuned constant).  Steps (a)+(b) with the rule
 *     unit u keeps key j  iff  S~[u, j] >= theta      (signed comparison of the exact integer scores),
 * and a unit that no key satisfies keeps its single best key (largest score, lower index among
 * equals), so that every row has a softmax.  The count per unit varies, so the mask is CSR:
 *     row_ptr int32 [B*H*L/vec + 1], row_ptr[0] = 0;  col int32: unit u keeps col[row_ptr[u] .. row_ptr[u+1]),
 *     ascending.  row_ptr[last] is the number of kept positions in all.
 * `col` has room for col_capacity entries; entries beyond it are not written, and the caller sees
 * from row_ptr[last] > col_capacity that it has to call again with a larger array.  shape->keep is
 * not used (pass 1).  Built for vec = 1, 4 or 8 (the score of a unit is the sum over its vec rows, step
 * (a2)) and k = 16, 32 or 64 (others: DSA_ERR_UNSUPPORTED), and for B*H*L*L <= 2^31 - 1.  `ws`: device scratch of at least dsa_threshold_workspace_bytes(). */
size_t dsa_threshold_workspace_bytes(const dsa_shape *shape);
dsa_status dsa_predict_mask_threshold(const dsa_shape *shape, const int8_t *Qt, const int8_t *Kt, int32_t theta,
                                      int32_t *row_ptr, int32_t *col, int64_t col_capacity, void *ws,
                                      size_t ws_bytes, void *stream);

/* Steps (c1)-(c3) in one kernel for a CSR mask (equations 2, 4, 3 per row over the keys of its unit;
 * any count per unit, a unit without keys gives a zero row).  shape->keep is not used. */
dsa_status dsa_masked_attention_csr(const dsa_shape *shape, const void *Q, const void *K, const void *V,
                                    const int32_t *row_ptr, const int32_t *col, float *O, void *stream);

/* Measurement aid for steps (c1)-(c3): the gathers of the fine-grained attention kernel and nothing
 * else (same launch shape, same key lists, the kept K rows and then the kept V rows of every query
 * row read as 16-byte pieces, no arithmetic).  Timing it gives the rate at which the memory hierarchy
 * serves this access pattern (K and V of a head are L2-resident at the workload sizes), the roof to
 * set beside dsa_masked_attention; the HBM peak is not that roof.  `sink` (uint32 [B*H*L*64], device)
 * receives values of no meaning. */
dsa_status dsa_gather_roof(const dsa_shape *shape, const void *K, const void *V, const int32_t *idx,
                           uint32_t *sink, void *stream);

const char *dsa_status_string(dsa_status status);

/* Library version, "major.minor". */
const char *dsa_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DSA_H */
