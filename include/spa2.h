/*
 * spa2 — C ABI of the SpargeAttention2 hot path on AMD MI355X (gfx950).
 *
 * Three operations, split at the two seams of the paper's operator
 * O = SpargeAttn2(Q, K, V, k%, p%)  (Sec. 4.3, Alg. 1):
 *
 *   spa2_mask : Alg. 1 steps 2-6.  Mean-pools Q and K per block, forms the
 *               pooled map Pbar = softmax(Qbar Kbar^T * scale) (Sec. 2.2) and
 *               selects, per row, Top-k UNION Top-p (Sec. 4.1 equation).
 *   spa2_fwd  : Alg. 1 steps 7-21.  FlashAttention-style online softmax over
 *               the selected (query block, key block) tiles only (Sec. 2.1).
 *   spa2_bwd  : gradients of spa2_fwd's O w.r.t. Q, K, V over the same tiles
 *               (Sec. 4.3 says a backward pass exists; the mask is constant).
 *
 * Conventions common to every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller.  The
 *     library never allocates or frees device memory and keeps nothing between
 *     calls (the one exception, a fixed scratch array, is described at
 *     spa2_bwd_static).  bf16 tensors are raw 16-bit storage.
 *   - Calls enqueue work on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and return without synchronising.
 *   - Return value: SPA2_OK (0) or a negative SPA2_ERR_* code.  All argument
 *     checks happen before the first launch, so a failed call leaves every
 *     output untouched.  No C++ exception crosses this boundary.
 *   - Block sizes are b_q = 128 query tokens and b_kv = 64 key/value tokens
 *     (App. A).  T_m = ceil(N / 128), T_n = ceil(N / 64); a short last block
 *     is handled (pooled over its valid tokens, padded keys excluded from the
 *     softmax, padded query rows never stored).
 *   - Token tensors (Q, K, V, O, dO, dQ, dK, dV) share one layout given by
 *     spa2_shape: element (b, h, n, c) lives at b*sb + h*sh + n*sn + c, the
 *     head dimension is contiguous, base pointers are 16-byte aligned and
 *     sb, sh, sn are multiples of 8 elements and sn is at most
 *     SPA2_MAX_TOKEN_STRIDE.  [B,H,N,d] and [B,N,H,d] both fit.  Per-row
 *     vectors (LSE) and the pattern arrays are contiguous.
 */
#ifndef SPA2_H
#define SPA2_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPA2_BQ  128
#define SPA2_BKV 64
/* longest row of key blocks the masker sorts in one workgroup (N <= 524288) */
#define SPA2_MAX_TN 8192
/* largest token stride in elements: the kernels reach the 128 rows of a tile
 * with a 32-bit byte offset from the tile's base address */
#define SPA2_MAX_TOKEN_STRIDE (1 << 23)

enum {
  SPA2_OK = 0,
  SPA2_ERR_NULL = -1,         /* a required pointer is NULL */
  SPA2_ERR_SHAPE = -2,        /* B, H, N, d <= 0, or N too long for the masker */
  SPA2_ERR_UNSUPPORTED = -3,  /* d not in {64, 128}, or block sizes other than 128 / 64 */
  SPA2_ERR_ALIGN = -4,        /* pointer not 16-byte aligned or stride not a multiple of 8 */
  SPA2_ERR_RANGE = -5,        /* topk_blocks outside [0, T_n], top_p outside [0, 1], both zero, scale <= 0 */
  SPA2_ERR_WORKSPACE = -6,    /* workspace missing or smaller than spa2_*_workspace_bytes */
  SPA2_ERR_LAUNCH = -7        /* the HIP runtime refused a launch (hipGetLastError) */
};

typedef struct spa2_shape {
  int32_t B, H, N, d;   /* d in {64, 128}; self-attention: Q, K, V all have N tokens */
  int32_t bq, bkv;      /* must be 128 and 64 */
  int64_t sb, sh, sn;   /* element strides of batch, head, token */
} spa2_shape;

/* Block-sparse pattern.  `mask` is the paper's Mbar (Sec. 2.2); the index lists
 * are the same information in the two orders the kernels walk it. */
typedef struct spa2_pattern {
  uint8_t* mask;      /* [B,H,T_m,T_n] 0/1                                          */
  int32_t* row_cnt;   /* [B,H,T_m]      number of selected key blocks of a query block */
  int32_t* row_idx;   /* [B,H,T_m,T_n]  first row_cnt entries valid, ascending j      */
  int32_t* col_cnt;   /* [B,H,T_n]      number of query blocks that selected key block j */
  int32_t* col_idx;   /* [B,H,T_n,T_m]  first col_cnt entries valid, ascending i      */
  /* Optional launch orders (NULL = natural order).  They do not change any result: they only say in which
   * order the attention kernels walk the query blocks (row_order, a permutation of 0..T_m-1 per head) and the
   * key blocks (col_order, a permutation of 0..T_n-1 per head).  col_order is written by spa2_mask /
   * spa2_mask_columns when non-NULL (longest column first, dealt evenly to the XCDs: it balances the
   * dK/dV kernel); row_order is an input only (a caller that knows which query blocks select similar
   * key blocks can place them next to each other), the library never writes it. */
  int32_t* row_order; /* [B,H,T_m] or NULL */
  int32_t* col_order; /* [B,H,T_n] or NULL */
} spa2_pattern;

int spa2_version(void);
const char* spa2_strerror(int code);

/* Host helper: the number of blocks that "the k% largest positions" (Sec. 2.2,
 * Top-k) means for a row of T_n blocks: 0 if k_frac <= 0, otherwise
 * ceil(k_frac * T_n) clamped to [1, T_n].  Case 1 of Sec. 3.2 (Top-20% of ten
 * entries keeps two) fixes the integral case. */
int32_t spa2_topk_blocks(double k_frac, int32_t Tn);

/* Bytes of device scratch spa2_mask / spa2_fwd / spa2_bwd use for this shape (0 = bad shape).
 *   spa2_mask_workspace_bytes      mandatory for spa2_mask and its stages (pooled means).
 *   spa2_fwd_workspace_bytes       optional for spa2_fwd (see there): plan and partial results of split rows.
 *   spa2_bwd_workspace_bytes       full backward workspace: D, then plans and partial results of split rows
 *                                  (dQ) and split columns (dK, dV).
 *   spa2_bwd_workspace_min_bytes   the mandatory leading part of it (D only).  With a buffer between the two
 *                                  sizes the backward kernels split as many lists as the rest of it holds. */
size_t spa2_mask_workspace_bytes(const spa2_shape* shape);
size_t spa2_fwd_workspace_bytes(const spa2_shape* shape);
size_t spa2_bwd_workspace_bytes(const spa2_shape* shape);
size_t spa2_bwd_workspace_min_bytes(const spa2_shape* shape);

/* Alg. 1 steps 2-6 (Sec. 2.2 pooling and pooled map, Sec. 4.1 hybrid rule).
 *   q, k        bf16 token tensors (device).
 *   topk_blocks Top-k block count per row, from spa2_topk_blocks; 0 = Top-p only.
 *   top_p       cumulative-probability threshold in [0, 1]; 0 = Top-k only.
 *   scale       multiplies Qbar Kbar^T (1/sqrt(d) in the paper).
 *   out         all five arrays are written (col_* may be NULL if no backward follows).
 *   pbar_out    optional fp32 [B,H,T_m,T_n]: the pooled map the selection was taken on.
 * Per row: entries are ordered by (Pbar descending, block index ascending);
 * n_p is the shortest prefix whose sum is >= top_p; the first
 * max(1, topk_blocks, n_p) entries are selected.  The prefix sums are exact
 * integer sums of the fp32 Pbar values taken as 62-bit fixed point (each value
 * times 2^62, bits below 2^-62 dropped; top_p converted the same way), so
 * they do not depend on the order of addition and the mask is deterministic.
 * Against a sequential fp64 sum of the same fp32 values the cut can differ
 * only where the cumulative mass lies within rounding (far below 1e-5) of
 * top_p. */
int spa2_mask(const void* q, const void* k, const spa2_shape* shape,
              int32_t topk_blocks, float top_p, float scale,
              spa2_pattern* out, float* pbar_out,
              void* workspace, size_t workspace_bytes, void* stream);

/* The three stages of spa2_mask, callable one by one (spa2_mask is exactly their sequence):
 *   spa2_mask_pool     Sec. 2.2 mean pooling: reads Q and K once, leaves the pooled means in `workspace`;
 *   spa2_mask_select   pooled map, ordering, Top-k UNION Top-p (Sec. 4.1): reads `workspace`, writes
 *                      mask / row_cnt / row_idx (and pbar_out if given);
 *   spa2_mask_columns  lists the same pattern per key block: reads out->mask, writes col_cnt / col_idx.
 * Same argument meaning, ownership and error behaviour as spa2_mask. */
int spa2_mask_pool(const void* q, const void* k, const spa2_shape* shape,
                   void* workspace, size_t workspace_bytes, void* stream);
int spa2_mask_select(const spa2_shape* shape, int32_t topk_blocks, float top_p, float scale,
                     spa2_pattern* out, float* pbar_out,
                     void* workspace, size_t workspace_bytes, void* stream);
int spa2_mask_columns(const spa2_shape* shape, spa2_pattern* out, void* stream);

/* Fills `out` with the all-ones pattern (every tile selected): dense attention
 * through the same kernels, and the sparsity-0 special case. */
int spa2_pattern_full(const spa2_shape* shape, spa2_pattern* out, void* stream);

/* Alg. 1 steps 7-21.  For every query block i, over the key blocks j listed in
 * pattern->row_idx only: S_ij = Q_i K_j^T * scale, running row maximum and sum,
 * O_i accumulated in fp32 and divided by the final sum.
 *   o      bf16 token tensor (written);  lse fp32 [B,H,N] = log sum_j exp(S) per row (written).
 *   o_res  optional (NULL = not wanted) bf16 token tensor, same layout as o: the part of the fp32
 *          result that the rounding of o to bf16 dropped, o_res = bf16(O_fp32 - o).  The backward pass
 *          uses o + o_res for D = rowsum(dO * O); with o alone, the 2^-9 relative rounding of O is the
 *          largest error term of dQ when |K| is large.
 *   workspace  optional (NULL, 0 = none), 16-byte aligned, up to spa2_fwd_workspace_bytes(shape) bytes.  One
 *          workgroup walks one row of the pattern, so a launch cannot end before its longest row has; on layers
 *          with few rows per compute unit the longest rows then set the time.  With a workspace, lists longer than
 *          S = max(16, total tiles / 2048) entries are cut into parts of S that run as workgroups of their own;
 *          the parts' (O, m, l) are combined in part order by a second kernel (Alg. 1 step 18 makes that exact up
 *          to rounding), so results stay deterministic.  On large layers S exceeds every list and nothing changes.
 * Reads pattern->row_cnt / row_idx (and row_order if set). */
int spa2_fwd(const void* q, const void* k, const void* v, const spa2_shape* shape,
             const spa2_pattern* pattern, float scale, void* o, void* o_res, float* lse,
             void* workspace, size_t workspace_bytes, void* stream);

/* Backward of spa2_fwd for upstream gradient d_o, mask held constant.  With
 * P = exp(S - lse) on selected tiles:  dV = P^T dO,  dP = dO V^T,
 * D = rowsum(dO * O),  dS = P * (dP - D),  dQ = dS K * scale,  dK = dS^T Q * scale.
 *   dq, dk, dv  bf16 token tensors (written everywhere, zeros where no tile contributes).
 * Reads row_* (dQ) and col_* (dK, dV) of the pattern.  workspace: at least spa2_bwd_workspace_min_bytes (D);
 * with up to spa2_bwd_workspace_bytes, long rows (dQ) and long columns (dK, dV) are cut into parts as in spa2_fwd
 * and their fp32 partial sums are added in part order. */
int spa2_bwd(const void* q, const void* k, const void* v, const void* o, const void* o_res /* or NULL */,
             const void* d_o, const float* lse, const spa2_shape* shape, const spa2_pattern* pattern,
             float scale, void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes, void* stream);

/* The three stages of spa2_bwd, callable one by one (spa2_bwd is exactly their sequence; a caller
 * that needs only dQ, or only dK and dV, skips the other):
 *   spa2_bwd_delta  D = rowsum(dO * (o + o_res)), fp32 [B,H,N], left in `workspace`;
 *   spa2_bwd_dkdv   dK, dV: one pass per key block over the query blocks listed in col_idx;
 *   spa2_bwd_dq     dQ: one pass per query block over the key blocks listed in row_idx.
 * dkdv and dq read D from `workspace` (written by spa2_bwd_delta for the same o, d_o) and keep their split plans
 * and partial sums in their own sections behind it, so the two may run at the same time on two streams. */
int spa2_bwd_delta(const void* o, const void* o_res /* or NULL */, const void* d_o, const spa2_shape* shape,
                   void* workspace, size_t workspace_bytes, void* stream);
int spa2_bwd_dkdv(const void* q, const void* k, const void* v, const void* d_o, const float* lse,
                  const spa2_shape* shape, const spa2_pattern* pattern, float scale,
                  void* dk, void* dv, void* workspace, size_t workspace_bytes, void* stream);
int spa2_bwd_dq(const void* q, const void* k, const void* v, const void* d_o, const float* lse,
                const spa2_shape* shape, const spa2_pattern* pattern, float scale,
                void* dq, void* workspace, size_t workspace_bytes, void* stream);

/* spa2_bwd for callers that cannot provide or allocate a workspace (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): same arguments, results and error behaviour as spa2_bwd, without the
 * workspace.  D is kept in a fixed array of SPA2_STATIC_MAX_ROWS floats (16 MiB) that the library holds in the
 * memory of every GPU it runs on until the process ends; no allocation happens in this call (the array's device
 * address is looked up on the first call on each device, with the calling thread's current device).
 *   Limit: B * H * N <= SPA2_STATIC_MAX_ROWS, otherwise SPA2_ERR_WORKSPACE and nothing is launched.
 *   Long rows and columns are not split on this path (that needs the larger workspace of spa2_bwd).
 *   All calls on one GPU share that array: two calls whose execution overlaps on one GPU (different streams,
 *   different threads) race on D and give wrong gradients; calls on one stream are safe.  The array keeps the
 *   last call's D; every row a call reads is written by that same call first. */
#define SPA2_STATIC_MAX_ROWS (4 * 1024 * 1024)
int spa2_bwd_static(const void* q, const void* k, const void* v, const void* o, const void* o_res /* or NULL */,
                    const void* d_o, const float* lse, const spa2_shape* shape, const spa2_pattern* pattern,
                    float scale, void* dq, void* dk, void* dv, void* stream);

/* ---- diagnostics: the error of sparse attention and its two parts (Sec. 3.1) ----
 * For every query row, with tau = exp(lse_sparse - lse_dense) the attention mass the mask retains:
 *   o_dense - o_sparse = (o_dense - tau * o_sparse)  +  (tau - 1) * o_sparse
 *                         dropped error                  renormalisation error
 * out, fp64 [B,H,5], per (batch, head) over all rows and channels:
 *   [0] sum |o_dense - o_sparse|   [1] sum |o_dense|   (their ratio is the relative L1 error of Sec. 3.2)
 *   [2] sum |o_dense - tau o_sparse|   [3] sum |(tau - 1) o_sparse|   [4] sum over rows of tau.
 * o_sparse / lse_sparse come from spa2_fwd on the pattern under study, o_dense / lse_dense from spa2_fwd on the
 * pattern spa2_pattern_full writes; the four token tensors share `shape` (bf16; lse fp32 [B,H,N]).  Device
 * pointers, caller-owned; workspace of spa2_error_workspace_bytes(shape) bytes, 16-byte aligned (0 = bad shape).
 * The reduction order is fixed: results are deterministic.  Errors as for spa2_fwd. */
size_t spa2_error_workspace_bytes(const spa2_shape* shape);
int spa2_error_terms(const void* o_sparse, const void* o_dense, const float* lse_sparse, const float* lse_dense,
                     const spa2_shape* shape, double* out, void* workspace, size_t workspace_bytes, void* stream);

/* ---- velocity distillation loss (Sec. 4.2 equation; loss step of Alg. 2) ----
 *   loss = weight * sum over the n elements of (u_sparse - u_full)^2
 *   grad = upstream * 2 * weight * (u_sparse - u_full)        (with respect to u_sparse; the teacher is frozen)
 * The paper's expectation over training samples is weight = 1 / (samples in the batch); 1 / n is the per-element
 * mean.  u_sparse, u_full, grad: device, contiguous, n elements of `dtype` (bf16 or fp32), 16-byte aligned, caller-
 * owned; grad may alias neither input.  loss: device, one fp64.  upstream: device, one fp64 (the derivative of the
 * final objective with respect to loss), or NULL for 1.  The difference is taken in fp32 and the squares are summed
 * in fp64 in a fixed order: the loss is deterministic.  spa2_vd_loss needs a workspace of
 * spa2_vd_loss_workspace_bytes() bytes, 16-byte aligned.  Asynchronous on `stream`.
 * Errors: SPA2_ERR_NULL, _SHAPE (n <= 0), _UNSUPPORTED (dtype), _ALIGN, _RANGE (weight not finite or <= 0),
 * _WORKSPACE, _LAUNCH; checked before anything is launched. */
#define SPA2_DTYPE_BF16 0
#define SPA2_DTYPE_F32  1
size_t spa2_vd_loss_workspace_bytes(void);
int spa2_vd_loss(const void* u_sparse, const void* u_full, int64_t n, int32_t dtype, double weight, double* loss,
                 void* workspace, size_t workspace_bytes, void* stream);
int spa2_vd_loss_grad(const void* u_sparse, const void* u_full, int64_t n, int32_t dtype, double weight,
                      const double* upstream /* or NULL */, void* grad, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SPA2_H */
