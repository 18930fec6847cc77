/*
 * heart.h -- C ABI of the MI355X (gfx950) implementation of the data-parallel hot
 * path of HEART's sparse-attention step for video diffusion transformers.
 *
 * One denoising step of one attention layer calls, in this order (the paper's
 * Temporal Mask Reuse procedure, Alg. 1):
 *     heart_pool_qk  ->  heart_drift  ->  heart_mask_topp  ->  heart_block_sparse_attn
 * (heart_pool_drift does the first two with one launch fewer.)
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller (for instance the
 *     storage of PyTorch-ROCm tensors).  The library allocates nothing, keeps no
 *     state between calls (beyond per-device launch attributes it sets once), reads no
 *     environment variable; an entry point that needs scratch memory takes it as a
 *     workspace argument.  Workspace sizes: heart_workspace_bytes (the hot path),
 *     heart_pool_drift_workspace_bytes, heart_scores_antidiag_workspace_bytes,
 *     heart_ebc_workspace_bytes.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  A call
 *     only enqueues kernels on that stream and returns; it never synchronises.
 *   - Return value: HEART_OK (0) or a negative error code.  After an error
 *     heart_last_error() returns a thread-local message.  Arguments are validated on
 *     the host before anything is launched; a call that fails launches nothing.
 *   - Notation: B batch items (a classifier-free-guidance branch is its own batch
 *     item), H heads, N tokens, D head dimension, `block` tokens per block,
 *     Nb = ceil(N / block); the last block may hold fewer than `block` tokens.
 *   - bf16 tensors are passed as const void* to 2-byte brain-float elements.
 *   - NaN/Inf in inputs is undefined behaviour of the arithmetic (never of memory).
 */
#ifndef HEART_H_
#define HEART_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HEART_OK 0
#define HEART_EINVAL (-1)       /* null pointer, non-positive size, bad flag */
#define HEART_EUNSUPPORTED (-2) /* shape outside what the kernels are built for */
#define HEART_EHIP (-3)         /* the HIP runtime refused a launch */

#define HEART_MAX_NB 1024 /* largest number of blocks per sequence the mask kernel ranks */

/*
 * Shape and memory layout of the Q/K/V/O tensors of one call.
 * Logical shape is [B, H, N, D] with the D axis contiguous (stride 1).  The other
 * three strides are given in ELEMENTS as {batch, head, token}, so both a
 * [B,H,N,D] and a [B,N,H,D] allocation can be passed without a copy.
 * Every base pointer and every stride (in bytes) must be a multiple of 16.
 * Supported: D in {64, 128}; block in {64, 128}.
 */
typedef struct heart_shape {
  int B, H, N, D, block;
  long long q_stride[3];
  long long k_stride[3];
  long long v_stride[3];
  long long o_stride[3];
} heart_shape;

/*
 * Pooling (Alg. 1, step 1; Eq. 4; block granularity of the importance ranking,
 * Sec. 4.2 and the appendix on baseline configurations).
 * One streaming pass over bf16 Q and K yields
 *   qblk, kblk   [B,H,Nb,D] fp32: mean over the real tokens of each block
 *   qmean, kmean [B,H,D]    fp32: mean over all N tokens (token-averaged features
 *                                 of Eq. 4; sum of block sums / N, which differs
 *                                 from the mean of block means when the last
 *                                 block is short)
 * Outputs are contiguous.  Accumulation is fp32 inside a block in a fixed order
 * (results are reproducible run to run) and fp64 across blocks.
 * v_stride / o_stride of `shape` are ignored.
 */
int heart_pool_qk(const heart_shape *shape, const void *q_bf16, const void *k_bf16, float *qblk,
                  float *kblk, float *qmean, float *kmean, void *stream);

/*
 * Mean-pooled drift, reuse rule and layer-level gate (Eq. 4; Sec. 4.2; Alg. 1;
 * gate thresholds in the appendix on HEART configurations).
 *   drift[b,h]   = sum_d |qanchor - qmean| + |kanchor - kmean|   (fp32, fixed halving
 *                  tree over d, so the value is a pure function of the inputs;
 *                  +inf for a head without an anchor)
 *   mark[b,h]    = !has_anchor  ||  drift > delta[h]             (strict, Alg. 1)
 *   gate, per batch item: frac = (#marks)/H in fp32;
 *                  frac < gate_lo : heads that have an anchor reuse, others refresh
 *                  frac > gate_hi : every head refreshes
 *                  otherwise      : refresh = mark
 *                  (gate_lo = 0, gate_hi = 1 disables the gate)
 *   commit != 0  : for refreshed heads qanchor/kanchor <- qmean/kmean and
 *                  has_anchor <- 1; reused heads keep their anchor (Alg. 1).
 * qmean, kmean, qanchor, kanchor: fp32 [B,H,D] contiguous; has_anchor, refresh:
 * uint8 [B,H]; delta: fp32 [H] (device); drift: fp32 [B,H].
 * D must be a power of two, 1 <= D <= 512; H <= 4096.
 */
int heart_drift(int B, int H, int D, const float *qmean, const float *kmean, float *qanchor,
                float *kanchor, unsigned char *has_anchor, const float *delta, float gate_lo,
                float gate_hi, int commit, float *drift, unsigned char *refresh, void *stream);

/*
 * heart_pool_qk and heart_drift in TWO launches instead of three (the paper observes that fixed
 * per-layer cost such as kernel launches caps what mask reuse can gain: Sec. 4.2, last
 * paragraph): the pooling pass, then one launch that computes the token means and, in the
 * workgroup that finishes the last token mean of a batch item, the drift stage.  Arguments and
 * results are those of the two calls: qblk, kblk, qmean, kmean are outputs as in heart_pool_qk
 * (same bits); drift, refresh and the anchor update are what heart_drift gives on those qmean,
 * kmean (same code, same bits).  No workgroup waits for another.
 * workspace: device memory of heart_pool_drift_workspace_bytes(B, H) bytes, 4-byte aligned,
 * holding the completion tickets.  It must be ZERO before the first call that uses it (e.g. one
 * hipMemset after allocating it); every call leaves it zero again, so it can be reused from call
 * to call.  Two calls that run concurrently must not share it.
 * Limits: those of heart_pool_qk and heart_drift (D in {64, 128}, H <= 4096).
 */
int heart_pool_drift(const heart_shape *shape, const void *q_bf16, const void *k_bf16, float *qblk,
                     float *kblk, float *qmean, float *kmean, float *qanchor, float *kanchor,
                     unsigned char *has_anchor, const float *delta, float gate_lo, float gate_hi,
                     int commit, float *drift, unsigned char *refresh, void *workspace,
                     size_t workspace_bytes, void *stream);
size_t heart_pool_drift_workspace_bytes(int B, int H);

/*
 * Block importance and top-p block mask for refreshed heads (top-p rule of
 * Sec. 3.2; minimal set reaching the mass, Eq. 1; scale 1/sqrt(D) of the
 * query-key interaction in the appendix; p = 1 is the dense value).
 *   scores P[i,j] = softmax_j( qblk_i . kblk_j / sqrt(D) )       (dot products on the
 *                   fp64 matrix cores, exponentials fp32)
 *   per row i: rank key blocks by P descending, equal scores by lower index; with
 *   u_j = floor(P_j * 2^30) and T = floor(tau_h * 2^24) keep the shortest prefix
 *   whose  sum(u) * 2^24 >= T * (row total of u);  at least max(1, min_keep)
 *   blocks; tau_h >= 1 keeps all.  The integer mass makes the kept set independent
 *   of summation order.  Then key-block columns j < n_always_kv_blocks are kept in
 *   every row and query rows i < n_dense_q_blocks keep every column.
 * Inputs : qblk, kblk fp32 [B,H,Nb,D] (may both be NULL if scores_in is given);
 *          scores_in fp32 [B,H,Nb,Nb] or NULL: if given, the score stage is skipped
 *          and these scores are ranked instead (each must lie in [0,1]; the kernel
 *          clamps larger values to 1 and counts negative values and NaN as 0, so a
 *          bad table cannot overflow the integer mass);
 *          tau fp32 [H] (device), in (0, 1] for the rule above.  tau lives on the device,
 *          so the host cannot reject a bad value: tau_h <= 0 (or NaN) asks for no mass
 *          and keeps exactly max(1, min_keep) best-ranked blocks per row;
 *          refresh uint8 [B,H] or NULL (= all heads).
 * No workspace: the logits of a row group live in LDS and the selection in registers.
 * Outputs, written only for heads with refresh != 0 (cached masks of reused heads
 * persist, Alg. 1):
 *          mask uint8 [B,H,Nb,Nb] (1 = kept);
 *          kept_idx int32 [B,H,Nb,Nb]: ascending kept key-block indices of each
 *            row in its first kept_count entries (the rest is left untouched);
 *          kept_count int32 [B,H,Nb];
 *          scores_out fp32 [B,H,Nb,Nb] or NULL.
 * Supported: Nb <= HEART_MAX_NB; D a multiple of 16, D <= 128.
 */
int heart_mask_topp(int B, int H, int Nb, int D, const float *qblk, const float *kblk,
                    const float *scores_in, const float *tau, const unsigned char *refresh,
                    int n_always_kv_blocks, int n_dense_q_blocks, int min_keep,
                    unsigned char *mask, int *kept_idx, int *kept_count, float *scores_out,
                    void *stream);

/*
 * heart_mask_topp with a workspace: for D = 64 or 128 (and no scores_in) the dot products of
 * the score stage then run on the int8 matrix cores, which are several times faster than the
 * fp64 ones.  A first small launch writes every block mean of the refreshed heads into the
 * workspace as an exponent and four signed 8-bit slices (the mean rounded to 31 bits below
 * the power of two above its block's largest entry); products of slices and their sums over
 * d are exact integers, and the slice pairs that matter are put together in fp64.  The
 * logits differ from the exact dot products of the fp32 block means by less than 1e-6 of
 * the product of the two blocks' largest entries, like those of the fp64 path they stay far
 * inside the 1e-5 budget of the scores; everything after the logits is the same code.
 * workspace: DEVICE, heart_mask_topp_workspace_bytes(B, H, Nb, D) bytes, 16-byte aligned,
 * contents irrelevant on entry and undefined on return; calls that share it must be
 * stream-ordered.  NULL workspace, scores_in given, or another D: exactly heart_mask_topp.
 */
size_t heart_mask_topp_workspace_bytes(int B, int H, int Nb, int D);
int heart_mask_topp_ws(int B, int H, int Nb, int D, const float *qblk, const float *kblk,
                       const float *scores_in, const float *tau, const unsigned char *refresh,
                       int n_always_kv_blocks, int n_dense_q_blocks, int min_keep,
                       unsigned char *mask, int *kept_idx, int *kept_count, float *scores_out,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * An alternative importance estimator for heart_mask_topp's scores_in argument: block
 * scores from strided antidiagonal sums of Q K^T.  The paper leaves importance ranking to
 * the sparse-attention backbone and names this family by its setting (antidiagonal scoring
 * with stride 16 on blocks of 128 tokens, appendix on baseline configurations) without
 * defining it; what this entry point computes is, with S = stride, block = 8 S,
 * M = ceil(N / S) and tokens past N counted as zero vectors:
 *   L[a,b]     = 1 / (S sqrt(D)) * sum_{r<S} q[S a + S-1-r] . k[S b + r]     (a, b < M)
 *   P[a,:]     = softmax_b L[a,:]
 *   score[I,J] = mean over the reduced queries a of block I of sum_{b in block J} P[a,b]
 * (bf16 products on the matrix cores, fp32 accumulation and exponentials).  Every row of
 * `scores` sums to one up to rounding and every entry lies in [0,1].
 * q, k: bf16 with the strides of `shape` (v/o strides are ignored); refresh: uint8 [B,H]
 * or NULL (= all heads): heads with refresh == 0 are skipped and their part of `scores`
 * is left untouched (pass the same array to heart_mask_topp, which skips them too);
 * scores: fp32 [B,H,Nb,Nb]; workspace: device memory of at least
 * heart_scores_antidiag_workspace_bytes(shape, stride) bytes, 16-byte aligned, contents
 * irrelevant on entry and undefined on return; calls that share a workspace must be
 * stream-ordered.  Supported: block == 8 * stride, Nb <= HEART_MAX_NB, D in {64, 128}.
 */
size_t heart_scores_antidiag_workspace_bytes(const heart_shape *shape, int stride);
int heart_scores_antidiag(const heart_shape *shape, const void *q, const void *k, int stride,
                          const unsigned char *refresh, float *scores, void *workspace,
                          size_t workspace_bytes, void *stream);

/*
 * Block-sparse attention consuming the mask as per-row kept-block lists
 * (the sparse attention the mask is produced for; interaction scale from the
 * appendix on query-key stability).
 *   For head (b,h) and query block i:
 *     out[n,:] = sum_t softmax_t( q_n . k_t * scale ) v_t,   t over the real tokens of
 *     the key blocks kept_idx[b,h,i,0..kept_count[b,h,i])
 *   computed flash-style (online softmax) with bf16 MFMA and fp32 accumulation.
 *   Precision (default): logits from the bf16 matrix cores with fp32 accumulation, scaled
 *   in fp32; exponentials in fp32; the softmax weights are rounded to bf16 for the second
 *   contraction while the row sum adds the unrounded weights; the output is rounded to
 *   bf16.  The error against exact attention on the given bf16 inputs is that of the bf16
 *   rounding of weights and output: within 2e-2 * max(1, max|out| / 2) for any input scale.
 *   With HEART_ATTN_FOLD_SCALE (heart_block_sparse_attn_flags) q is instead multiplied by
 *   scale * log2(e) and rounded to bf16 once, which removes one multiply per logit (about
 *   3 % faster) at the price of one more bf16 rounding of the query: the same bound holds
 *   for q, k of unit scale (logits of a few units; normalised activations), but that error
 *   grows with the cube of the input scale.
 * q, k, v: bf16 with the strides of `shape`; out: bf16 with o_stride; kept_idx /
 * kept_count as written by heart_mask_topp (indices must lie in [0, Nb); order
 * does not matter for the result up to rounding); scale <= 0 means 1/sqrt(D);
 * lse: fp32 [B,H,N] natural-log-sum-exp of the scaled logits over the kept keys,
 * or NULL.  A row with kept_count == 0 yields zeros (lse = -inf).
 * Supported: every (D, block) pair of heart_shape.
 * workspace: device memory of at least heart_attn_workspace_bytes(shape) bytes, 16-byte
 * aligned, or NULL.  With a workspace the call first builds a launch plan in it (whole
 * heads are assigned to the XCDs so that the workgroups of an XCD share one head's K/V
 * in its L2; inside a head the query blocks with the longest kept lists start first;
 * workgroups take items with atomic counters, which levels the load).  The results are
 * the same with and without it.  The contents need not be preserved between calls; two
 * calls that run concurrently must not share a workspace.
 */
int heart_block_sparse_attn(const heart_shape *shape, const void *q_bf16, const void *k_bf16,
                            const void *v_bf16, const int *kept_idx, const int *kept_count,
                            float scale, void *out_bf16, float *lse, void *workspace,
                            size_t workspace_bytes, void *stream);

/* The same call with option flags (0 = heart_block_sparse_attn; unknown bits are an error). */
#define HEART_ATTN_FOLD_SCALE 1u /* fold the softmax scale into q (see Precision above) */
int heart_block_sparse_attn_flags(const heart_shape *shape, const void *q_bf16,
                                  const void *k_bf16, const void *v_bf16, const int *kept_idx,
                                  const int *kept_count, float scale, unsigned flags,
                                  void *out_bf16, float *lse, void *workspace,
                                  size_t workspace_bytes, void *stream);

/*
 * heart_block_sparse_attn_flags for callers that cannot allocate device memory or pass a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The launch plan lives in a static device array of the library
 * (HEART_ATTN_STATIC_PLAN_BYTES on every GPU the library runs on, held until the process
 * ends); the call allocates nothing and otherwise does what heart_block_sparse_attn_flags does
 * with a workspace, with the same results.  It needs heart_workspace_bytes(B, H, Nb, D) <=
 * HEART_ATTN_STATIC_PLAN_BYTES, i.e. B*H*(Nb+2) + 24 <= 262144, and returns HEART_EUNSUPPORTED
 * beyond that.  Every call on a GPU shares that GPU's array (each call rebuilds the plan, so
 * nothing carries over from the previous one): calls that overlap on one GPU -- different
 * streams, or different host threads -- race; keep them stream-ordered.  The first call on a
 * device looks up the array's device address and raises the kernels' LDS limit (two runtime
 * queries, no allocation): make that call once before a stream capture begins.
 */
#define HEART_ATTN_STATIC_PLAN_BYTES (1u << 20)
int heart_block_sparse_attn_static(const heart_shape *shape, const void *q_bf16,
                                   const void *k_bf16, const void *v_bf16, const int *kept_idx,
                                   const int *kept_count, float scale, unsigned flags,
                                   void *out_bf16, float *lse, void *stream);

/*
 * Bytes of workspace the hot path can use for one call: only heart_block_sparse_attn takes one
 * (its launch plan: 24 + B*H*(Nb+2) ints); heart_pool_qk, heart_drift and heart_mask_topp
 * need none.  heart_workspace_bytes takes plain sizes (D does not enter; it is part of the
 * signature so that callers can size by the full shape), heart_attn_workspace_bytes a
 * heart_shape; both return 0 for an invalid shape.
 */
size_t heart_workspace_bytes(int B, int H, int Nb, int D);
size_t heart_attn_workspace_bytes(const heart_shape *shape);

/*
 * Error-guided Budgeted Calibration (Sec. 4.3): offline, not on the serving path.
 *
 * heart_ebc_band_error: the frequency-weighted velocity error of Eq. 6 (bands and weights:
 *   appendix on the frequency-aware velocity error).  err, dense: DEVICE fp32 [C,T,Y,X]
 *   contiguous (sparse-induced error and dense reference; energies are summed over the C
 *   leading entries, the transform axes are T, Y, X, each <= 1024); weights4_host: HOST
 *   array of the four band weights (LL, LH, HL, HH); epsilon >= 0.  out6: DEVICE double[6]
 *   = {weighted error, E_LL, E_LH, E_HL, E_HH, spectral energy of dense}, in the units of an
 *   unnormalised DFT.  workspace: DEVICE, heart_ebc_workspace_bytes(C,T,Y,X), 16-byte
 *   aligned.  Computed without a transform (band projections are circular convolutions
 *   with Dirichlet kernels, in fp64); results are reproducible run to run.
 * heart_ebc_select: the one-candidate-per-head selection of Eq. 5, solved exactly on the
 *   HOST.  error_host, sparsity_host: [n_heads, n_candidates] doubles; minimises the summed
 *   error subject to mean sparsity >= min_mean_sparsity; choice_host: int[n_heads];
 *   total_error_host: double[1].  HEART_EINVAL if the budget cannot be met;
 *   HEART_EUNSUPPORTED if optimality could not be proved within the search limit (the best
 *   selection found is then in choice_host; not observed on tables of 6400 x 8).
 */
int heart_ebc_band_error(long long C, int T, int Y, int X, const float *err, const float *dense,
                         const double *weights4_host, double epsilon, void *workspace,
                         size_t workspace_bytes, double *out6, void *stream);
size_t heart_ebc_workspace_bytes(long long C, int T, int Y, int X);
int heart_ebc_select(int n_heads, int n_candidates, const double *error_host,
                     const double *sparsity_host, double min_mean_sparsity, int *choice_host,
                     double *total_error_host);

/* Thread-local message of the last error returned on this thread ("" if none). */
const char *heart_last_error(void);

/* Library version: major * 10000 + minor * 100 + patch. */
int heart_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HEART_H_ */
