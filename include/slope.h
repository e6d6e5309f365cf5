/*
 * slope.h - C ABI of the MI355X (gfx950) double-pruned 2:4 sparse linear layer.
 *
 * The operations are those of SLoPe's sparse pretraining step for one linear layer
 * (paper Sec. 2, Eq. 1-6, Eq. 11 and Algorithm 1):
 *
 *     W in R^{d_out x d_in},  X in R^{b x d_in},  Y, dY in R^{b x d_out},  dX in R^{b x d_in}
 *     W^R      W pruned 2:4 along d_in   (inside each row of W)       forward operand
 *     W^{R,C}  W^R pruned 2:4 once more along d_out (inside each column)  backward operand
 *
 * Conventions common to every call
 *   - All tensor pointers are DEVICE pointers to caller-owned memory, 16-byte aligned,
 *     dense tensors row-major bf16.  The library allocates nothing, keeps no state
 *     between calls and never synchronises: work is queued on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream).
 *   - Return value: SLOPE_OK or a negative slope_status.  Argument errors are found on
 *     the host before anything is launched; nothing is written in that case.
 *     After SLOPE_ERR_HIP, slope_last_hip_error() returns the hipError_t as int.
 *   - Packed 2:4 form of a [rows, cols] matrix pruned along cols (cols % 8 == 0):
 *       vals bf16[rows, cols/2]   vals[r][2g+k] = k-th kept element (ascending column) of
 *                                 the aligned group g = columns 4g..4g+3 of row r
 *       meta u8  [rows, cols/8]   group g sits in bits 4*(g&1)..4*(g&1)+3 of meta[r][g/2]
 *                                 as idx0 | idx1 << 2 with idx0 < idx1 (positions inside
 *                                 the group)
 *     A group with fewer than two kept elements names its lowest free positions as
 *     padding; padded slots hold +0.0.  Only this encoding is produced.
 *   - Bit masks: u8[rows, cols/8], element c of a row is bit (c & 7) of byte c/8.
 *   - Magnitude order: the bf16 bit pattern with the sign cleared, compared as an
 *     integer; on equal magnitude the lower index inside the group wins.  (+0 == -0;
 *     NaN ranks above Inf.)
 *   - Shape limits: d_in % 8 == 0 and d_out % 8 == 0 (slope_prune_rows: any d_out >= 1); b >= 1 is
 *     arbitrary; every extent must stay below 2^31 (SLOPE_ERR_SHAPE otherwise).  The fast kernels
 *     want more (contraction lengths that are multiples of 256, or of 64); other extents are routed to
 *     slower general kernels inside the same calls, never refused.
 *   - Scratch memory ("workspace") is the caller's, 256-byte aligned, and its contents are undefined
 *     after the call.  slope_workspace_bytes tells how much a call wants.  Calls whose names end in
 *     _ws, and the adapter calls, take the buffer's size and return SLOPE_ERR_WORKSPACE when it is too
 *     small; slope_spmm_fwd itself takes the pointer on trust.
 */
#ifndef SLOPE_H
#define SLOPE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SLOPE_OK = 0,
    SLOPE_ERR_NULL = -1,        /* a required pointer is NULL                          */
    SLOPE_ERR_SHAPE = -2,       /* extent <= 0, not a multiple of its quantum, too big */
    SLOPE_ERR_ALIGN = -3,       /* a pointer is not 16-byte aligned                    */
    SLOPE_ERR_UNSUPPORTED = -4, /* N:M other than 2:4, adapter rank not supported      */
    SLOPE_ERR_HIP = -5,         /* a launch failed; see slope_last_hip_error()         */
    SLOPE_ERR_WORKSPACE = -6    /* the scratch buffer is smaller than the call needs   */
} slope_status;

/* Library version (major*100 + minor) and the last hipError_t seen by this thread. */
int slope_version(void);
int slope_last_hip_error(void);
const char* slope_status_string(int status);

/* Byte sizes of the packed form of a [rows, cols] matrix pruned along cols
 * (2 x 16 bits of values and 4 bits of index per group of four; Sec. 2.1 memory analysis,
 * with two 2-bit indices instead of the 3-bit minimum of Eq. 7). 0 on invalid shape. */
size_t slope_packed_vals_bytes(int64_t rows, int64_t cols);
size_t slope_packed_meta_bytes(int64_t rows, int64_t cols);
size_t slope_mask_bytes(int64_t rows, int64_t cols);

/* The calls, as numbered for slope_workspace_bytes (1-5: the five steps of the layer, Algorithm 1). */
typedef enum {
    SLOPE_CALL_PRUNE_ROWS = 1,
    SLOPE_CALL_DOUBLE_PRUNE = 2,
    SLOPE_CALL_SPMM_FWD = 3,
    SLOPE_CALL_SPMM_BWD_X = 4,
    SLOPE_CALL_WGRAD_MASKED = 5,
    SLOPE_CALL_WGRAD_MASKED_WS = 6,
    SLOPE_CALL_SPMM_BWD_X_ADAPTER = 7,
    SLOPE_CALL_WGRAD_ADAPTER = 8,
    SLOPE_CALL_WGRAD_MASKED_T = 9
} slope_call_id;

/* Bytes of scratch memory a call wants for b tokens, a d_out x d_in layer and adapter rank r (0: none);
 * 0 for the calls that take no workspace, for unknown ids and for invalid extents.  The per-call
 * queries below return the same numbers.
 *   slope_spmm_fwd: required when adapters are active (T = X L as bf16[b, r], a K-contiguous copy of L
 *   for many tokens, partial sums); optional otherwise: for a few dozen to about a thousand tokens the
 *   call, given this many bytes, also splits the contraction over d_in and keeps fp32 partial sums
 *   there, which is much faster at those sizes. */
size_t slope_workspace_bytes(int call_id, int64_t b, int64_t d_in, int64_t d_out, int64_t r);
size_t slope_spmm_fwd_workspace_bytes(int64_t b, int64_t d_in, int64_t d_out, int64_t r);

/*
 * slope_prune_rows - magnitude N:M pruning of W along d_in into W^R (Sec. 2.1; the
 * "prune" and "compress" steps of the sparse setup, App. B and App. K).
 *   W        in   bf16[d_out, d_in]
 *   n, m     in   only 2, 4 is implemented (others: SLOPE_ERR_UNSUPPORTED)
 *   Wr_vals  out  bf16[d_out, d_in/2]   packed values of W^R
 *   Wr_meta  out  u8[d_out, d_in/8]     packed indices of W^R
 *   mask_or_null out u8[d_out, d_in/8]  bit mask of the kept positions, or NULL to skip
 * Exactly two positions are kept in every group, zeros included.
 */
slope_status slope_prune_rows(const void* W, int64_t d_out, int64_t d_in, int n, int m,
                              void* Wr_vals, void* Wr_meta, void* mask_or_null, void* stream);

/*
 * slope_double_prune - second 2:4 prune of the already row-pruned weight, taken along
 * d_out, giving W^{R,C} for the backward pass (Sec. 2.1, Eq. 6: transpose the N:M matrix,
 * then impose N:M again).  Only positions named by Wr_meta compete; a group of four along
 * d_out keeps its min(2, #candidates) largest magnitudes.
 *   Wr_vals, Wr_meta  in   packed W^R as written by slope_prune_rows
 *   WrcT_vals  out  bf16[d_in, d_out/2]   packed (W^{R,C})^T: rows = d_in, groups along d_out
 *   WrcT_meta  out  u8[d_in, d_out/8]
 *   maskrc_or_null out u8[d_out, d_in/8]  bit mask of W^{R,C} in W's orientation, or NULL
 * d_out and d_in are multiples of 8 and at most 2^23 each (SLOPE_ERR_SHAPE otherwise).
 */
slope_status slope_double_prune(const void* Wr_vals, const void* Wr_meta, int64_t d_out, int64_t d_in,
                                void* WrcT_vals, void* WrcT_meta, void* maskrc_or_null, void* stream);

/*
 * slope_spmm_fwd - Y = X (W^R)^T, plus (X L) R when adapters are active
 * (Eq. 4; Eq. 11 for the low-rank term with L in R^{d_in x r}, R in R^{r x d_out}).
 *   X   in  bf16[b, d_in]
 *   Wr_vals, Wr_meta in packed W^R
 *   L_or_null in bf16[d_in, r], R_or_null in bf16[r, d_out]; both NULL or r == 0 means no
 *       adapter (the case for all but the last 1 % of pretraining, Sec. 2.2).
 *       r must be a multiple of 32 and at most 512.
 *   Y   out bf16[b, d_out]; fp32 accumulation; X L is rounded to bf16 before it meets R.
 *   workspace: device scratch of slope_workspace_bytes(SLOPE_CALL_SPMM_FWD, ...) bytes, 256-byte
 *       aligned; may be NULL when no adapter is active (if given, it must have that many
 *       bytes all the same).
 * slope_spmm_fwd_ws is the same call with the size of the buffer stated, so that a buffer that is
 * too small is refused (SLOPE_ERR_WORKSPACE) instead of overrun.
 */
slope_status slope_spmm_fwd(const void* X, int64_t b, const void* Wr_vals, const void* Wr_meta,
                            int64_t d_out, int64_t d_in,
                            const void* L_or_null, const void* R_or_null, int64_t r,
                            void* Y, void* workspace, void* stream);
slope_status slope_spmm_fwd_ws(const void* X, int64_t b, const void* Wr_vals, const void* Wr_meta,
                               int64_t d_out, int64_t d_in,
                               const void* L_or_null, const void* R_or_null, int64_t r,
                               void* Y, void* workspace, size_t workspace_bytes, void* stream);

/*
 * slope_spmm_fwd_static - slope_spmm_fwd for callers that cannot allocate device memory or carry a
 * workspace around: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same kernels and bit-identical results, but the scratch memory is a
 * buffer of SLOPE_STATIC_SCRATCH_BYTES inside the library's own device image (every GPU the library
 * runs on holds one copy until the process ends).  The call allocates and frees nothing.
 *   - A shape whose slope_spmm_fwd_workspace_bytes(b, d_in, d_out, r) exceeds SLOPE_STATIC_SCRATCH_BYTES
 *     is rejected with SLOPE_ERR_WORKSPACE before anything is launched; that query is the test.  (Every
 *     token count up to 128 fits for the OPT-66B layers with rank-128 adapters, and so does every
 *     training-size batch of them, whose need is T = X L plus a copy of L, about 10-18 MiB.)
 *   - The buffer is found once per device, on the first call made while that device is current
 *     (make that call outside stream capture); the stream must belong to the current device.
 *   - All calls on one GPU share the buffer: calls that overlap in time on one GPU (different
 *     streams, different threads) race.  Calls queued on one stream are safe.
 */
#define SLOPE_STATIC_SCRATCH_BYTES (72u << 20)
slope_status slope_spmm_fwd_static(const void* X, int64_t b, const void* Wr_vals, const void* Wr_meta,
                                   int64_t d_out, int64_t d_in,
                                   const void* L_or_null, const void* R_or_null, int64_t r,
                                   void* Y, void* stream);

/*
 * slope_spmm_bwd_x - dX = dY W^{R,C}  (Eq. 6; Algorithm 1 line 11).
 *   dY  in  bf16[b, d_out]
 *   WrcT_vals, WrcT_meta in packed (W^{R,C})^T as written by slope_double_prune
 *   dX  out bf16[b, d_in]; fp32 accumulation.
 */
slope_status slope_spmm_bwd_x(const void* dY, int64_t b, const void* WrcT_vals, const void* WrcT_meta,
                              int64_t d_out, int64_t d_in, void* dX, void* stream);

/*
 * slope_wgrad_masked - dW = dY^T X (Eq. 5) evaluated with a dense contraction over the b
 * tokens and written only at the positions W^R keeps, in W^R's packed order
 * (Algorithm 1 lines 12-13: dense product, then prune-and-compress with the weight's mask;
 * App. K: the result is d_out x d_in/2).
 *   dY in bf16[b, d_out], X in bf16[b, d_in], Wr_meta in u8[d_out, d_in/8]
 *   dW_vals out bf16[d_out, d_in/2]; fp32 accumulation.
 * No scratch memory: the operands are read as stored, tokens being their slow index.
 *
 * slope_wgrad_masked_ws - the same result (up to fp32 summation order) through token-contiguous copies
 * of X and dY in the caller's workspace, which is what large layers should use: the product then runs at
 * the rate of the other tile kernels.
 *   workspace  slope_workspace_bytes(SLOPE_CALL_WGRAD_MASKED_WS, b, d_in, d_out, 0) bytes
 *
 * Layers that share an operand (q, k and v share X) need its copy only once:
 *   slope_transpose_tokens  At = token-contiguous copy of A bf16[b, d] (an X or a dY); At has
 *                           slope_token_copy_bytes(b, d) bytes (rows of b rounded up to 64 tokens, zero-filled,
 *                           plus padding of the row pitch; the layout is the library's own)
 *   slope_wgrad_masked_t    the product from two such copies; d_in % 32 == 0 (SLOPE_ERR_SHAPE otherwise).
 *                           workspace_or_null: slope_workspace_bytes(SLOPE_CALL_WGRAD_MASKED_T, b, d_in, d_out, 0)
 *                           bytes of scratch (may be 0), 256-byte aligned.  With it the tiles that a last,
 *                           partly filled round of the chip would hold are cut along the tokens into fp32
 *                           partial sums that a second pass adds in a fixed order (a 9216 x 9216 layer is
 *                           1296 tiles of 256 x 256 on 256 compute units: without the cut its last 16 tiles
 *                           cost a sixth of the call).  NULL: no cut; a buffer that is too small:
 *                           SLOPE_ERR_WORKSPACE.  slope_wgrad_masked_ws's workspace includes this scratch.
 */
slope_status slope_wgrad_masked(const void* dY, const void* X, int64_t b, const void* Wr_meta,
                                int64_t d_out, int64_t d_in, void* dW_vals, void* stream);
size_t slope_wgrad_workspace_bytes(int64_t b, int64_t d_in, int64_t d_out);
slope_status slope_wgrad_masked_ws(const void* dY, const void* X, int64_t b, const void* Wr_meta,
                                   int64_t d_out, int64_t d_in, void* dW_vals,
                                   void* workspace, size_t workspace_bytes, void* stream);
size_t slope_token_copy_bytes(int64_t b, int64_t d);
slope_status slope_transpose_tokens(const void* A, int64_t b, int64_t d, void* At, size_t At_bytes, void* stream);
slope_status slope_wgrad_masked_t(const void* dYt, const void* Xt, int64_t b, const void* Wr_meta,
                                  int64_t d_out, int64_t d_in, void* dW_vals,
                                  void* workspace_or_null, size_t workspace_bytes, void* stream);

/*
 * slope_spmm_bwd_x_adapter - input gradient of a layer with adapters:
 *     dX = dY W^{R,C} + (dY R^T) L^T
 * Eq. 6 plus the derivative of the low-rank term of Eq. 11 with respect to X (Sec. 2.2; the
 * paper leaves it to autograd).  dY R^T is rounded to bf16 before it meets L.
 *   dY, WrcT_vals, WrcT_meta, dX   as for slope_spmm_bwd_x
 *   L   in  bf16[d_in, r]    R  in  bf16[r, d_out]    r % 32 == 0, 32 <= r <= 512
 *   workspace  slope_spmm_bwd_x_adapter_workspace_bytes(b, r) bytes, 256-byte aligned
 */
size_t slope_spmm_bwd_x_adapter_workspace_bytes(int64_t b, int64_t r);
slope_status slope_spmm_bwd_x_adapter(const void* dY, int64_t b, const void* WrcT_vals, const void* WrcT_meta,
                                      int64_t d_out, int64_t d_in, const void* L, const void* R, int64_t r, void* dX,
                                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * slope_wgrad_adapter - all weight gradients of a layer with adapters in one call: the packed,
 * masked dW of slope_wgrad_masked (Eq. 5, Algorithm 1 lines 12-13) and the gradients of the
 * low-rank term of Eq. 11 by the chain rule,
 *     dL = X^T (dY R^T)   bf16[d_in, r]          dR = (X L)^T dY   bf16[r, d_out].
 * The three contractions over the tokens share one pair of token-contiguous copies of X and dY.
 * X L and dY R^T are rounded to bf16 before the second product.
 *   dY, X, Wr_meta, dW_vals   as for slope_wgrad_masked
 *   L, R, r                    as for slope_spmm_fwd (r % 32 == 0, 32 <= r <= 512)
 *   workspace  slope_wgrad_adapter_workspace_bytes(b, d_in, d_out, r) bytes, 256-byte aligned, required
 */
size_t slope_wgrad_adapter_workspace_bytes(int64_t b, int64_t d_in, int64_t d_out, int64_t r);
slope_status slope_wgrad_adapter(const void* dY, const void* X, int64_t b, const void* Wr_meta, int64_t d_out,
                                 int64_t d_in, const void* L, const void* R, int64_t r, void* dW_vals, void* dL,
                                 void* dR, void* workspace, size_t workspace_bytes, void* stream);

/*
 * slope_prune_mask - magnitude N:M pruning for the patterns that have no sparse MFMA (Sec. 2.1:
 * any N:M, e.g. the 1:2 and 2:8 of Lemma 2.1), as a bit mask plus masked dense weights; the
 * products then run on dense MFMA (slope_gemm_tn).  Same magnitude order and tie rule as
 * slope_prune_rows.
 *   W     in   bf16[rows, cols]            cols % 8 == 0
 *   n, m       keep n of every m; m in {2, 4, 8}, 1 <= n <= m (others: SLOPE_ERR_UNSUPPORTED)
 *   axis       0: groups of m consecutive elements inside a row (the row prune, W^R)
 *              1: groups inside a column (the second prune of W^{R,C}); rows % m == 0
 *   candidates_or_null in u8[rows, cols/8]  bit mask; only set positions compete and can be kept
 *              (double pruning: pass the mask of the first prune); NULL = all positions
 *   mask_out   out u8[rows, cols/8]         kept positions (16-byte aligned, like candidates)
 *   masked_out_or_null    out bf16[rows, cols]   W where kept, +0.0 elsewhere
 *   masked_t_out_or_null  out bf16[cols, rows]   the transpose of the same (the backward operand)
 */
slope_status slope_prune_mask(const void* W, int64_t rows, int64_t cols, int n, int m, int axis,
                              const void* candidates_or_null, void* mask_out, void* masked_out_or_null,
                              void* masked_t_out_or_null, void* stream);

/*
 * slope_gemm_tn - C = B A^T on dense MFMA: the forward (Eq. 1 with a masked weight: B = X,
 * A = masked W) and input-gradient (Eq. 3: B = dY, A = transposed masked W) products of the
 * emulated patterns.
 *   B  in  bf16[n, K]    A  in  bf16[m, K]    C  out bf16[n, m]; fp32 accumulation
 *   K % 64 == 0, m % 4 == 0, any n >= 1
 */
slope_status slope_gemm_tn(const void* B, int64_t n, const void* A, int64_t m, int64_t K, void* C, void* stream);

/*
 * slope_sparse_add - out = beta * A + gamma * B on the packed values of two matrices that share
 * one sparsity pattern (App. K, sparse matrix addition).  Algorithm 1 line 15 is the case
 * A = packed masked gradient, beta = 1 / gradient scale, B = packed W^R, gamma = weight decay.
 *   A_vals, B_vals  in   bf16[rows, cols/2]   packed values of two [rows, cols] matrices
 *   rows, cols           logical extents; cols % 8 == 0
 *   out_vals        out  bf16[rows, cols/2]   may be A_vals or B_vals (in place)
 * Each element is fma(beta, a, gamma * b) in fp32, rounded to bf16 (nearest even).  The metadata
 * is not touched: the result has the operands' pattern.
 */
slope_status slope_sparse_add(const void* A_vals, const void* B_vals, int64_t rows, int64_t cols, float beta,
                              float gamma, void* out_vals, void* stream);

/*
 * slope_update_sparse - both sparse copies take the values the optimizer produced for W^R's kept
 * positions (Algorithm 1 lines 17-18; App. K, update sparse matrix).  The masks are static
 * (Sec. 2.1), so no metadata changes: W^R's packed values become Wnew_vals, and every slot of
 * packed (W^{R,C})^T takes the new value of the position it names; slots that name a position
 * outside W^R's mask (padding of groups with fewer than two survivors) stay +0.0.
 * To re-select W^{R,C} by magnitude from the new values instead, call slope_double_prune.
 *   Wnew_vals  in   bf16[d_out, d_in/2]   new packed values, in W^R's pattern
 *   Wr_meta    in   u8[d_out, d_in/8]     metadata of W^R as written by slope_prune_rows
 *   Wr_vals    out  bf16[d_out, d_in/2]   receives a copy of Wnew_vals (no copy if it is Wnew_vals)
 *   WrcT_meta  in   u8[d_in, d_out/8]     metadata of (W^{R,C})^T as written by slope_double_prune
 *   WrcT_vals  out  bf16[d_in, d_out/2]   rewritten completely
 * d_out and d_in are multiples of 8 and at most 2^23 each (SLOPE_ERR_SHAPE otherwise).
 */
slope_status slope_update_sparse(const void* Wnew_vals, const void* Wr_meta, int64_t d_out, int64_t d_in,
                                 void* Wr_vals, const void* WrcT_meta, void* WrcT_vals, void* stream);

/*
 * slope_spmm_fwd_plan - diagnostics, host only (no GPU call): which kernels slope_spmm_fwd (Eq. 4, 11)
 * would launch for a shape.  The choices are cost estimates over the shape alone, so that tests can
 * pin the regimes.  plan: host int32[6]
 *   [0] product: 0 small-batch kernel (one pass over the packed weight), 1 tile kernel with the
 *       contraction split into slabs (needs the workspace), 2 tile kernel, 3 generic kernel
 *       (d_in not a multiple of 256; not a multiple of 64: its form for ragged rows), 4 small-batch
 *       kernel in its row-split form (d_in a multiple of 1024 and enough weight rows, or the
 *       workspace to cut the contraction into slices)
 *   [1], [2] weight rows and tokens per workgroup      [3] slabs or slices (1 = no split)
 *   [4] T = X L: 0 no adapter, 1 split over d_in from L as stored (few tokens),
 *       2 dense tile kernel, 3 dense tile kernel split over d_in, 4 plain arithmetic (d_in % 64 != 0)
 *   [5] chunks of 64 rows of L per workgroup for [4] == 1
 * with_workspace: whether the call would be given its scratch.  Errors as slope_spmm_fwd.
 */
slope_status slope_spmm_fwd_plan(int64_t b, int64_t d_in, int64_t d_out, int64_t r, int with_workspace, int32_t* plan);

/*
 * slope_tile_order - diagnostics, host only (no GPU call): the workgroup -> tile assignment the
 * MFMA tile kernels use for a grid of tiles_m x tiles_n tiles (the XCD-aware order behind the
 * products of Eq. 1, 4-6).  Workgroup w of the launch computes tile (tm[w], tn[w]); -1 in both
 * marks a workgroup that exits at once (ragged chunks).
 *   tm, tn    out  host int32[capacity]
 *   returns the number of workgroups of the launch (entries written), or -1 if capacity is
 *   smaller than that or an extent is not positive.
 */
int64_t slope_tile_order(int64_t tiles_m, int64_t tiles_n, int32_t* tm, int32_t* tn, int64_t capacity);

/*
 * slope_ceiling - diagnostics: micro-benchmarks of what the chip gives the simplest kernel of each kind,
 * so that the rooflines of the products (Eq. 4-6) and of the prune streams (Sec. 2.1) can be quoted
 * against ceilings measured in the same run, next to the published peaks.  One launch per call.
 *   kind   SLOPE_CEILING_SPARSE_MFMA  register-resident loop of v_smfmac_f32_16x16x64_bf16
 *          SLOPE_CEILING_DENSE_MFMA   register-resident loop of v_mfma_f32_16x16x32_bf16
 *          SLOPE_CEILING_SPARSE_MFMA_32, SLOPE_CEILING_DENSE_MFMA_32   the same with the 32 x 32 forms
 *                                     (v_smfmac_f32_32x32x32_bf16, v_mfma_f32_32x32x16_bf16)
 *          SLOPE_CEILING_READ         read-only stream over buf
 *          SLOPE_CEILING_COPY         copy of the first half of buf onto the second half
 *   buf    device memory, 256-byte aligned, at least slope_ceiling_min_bytes() bytes (the MFMA loops take
 *          their operands from its start: fill it with the values the products see); overwritten
 *   iters  iterations of the MFMA loops (16 instructions per wavefront each); ignored by the streams
 *   work   out (host): dense-equivalent flops, or bytes moved, of the launch
 */
typedef enum {
    SLOPE_CEILING_SPARSE_MFMA = 0, SLOPE_CEILING_DENSE_MFMA = 1, SLOPE_CEILING_READ = 2, SLOPE_CEILING_COPY = 3,
    SLOPE_CEILING_SPARSE_MFMA_32 = 4, SLOPE_CEILING_DENSE_MFMA_32 = 5
} slope_ceiling_kind;
size_t slope_ceiling_min_bytes(void);
slope_status slope_ceiling(int kind, void* buf, size_t bytes, int iters, double* work, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SLOPE_H */
