// C ABI of libheart: argument validation and dispatch to the kernel launchers.
// Everything is checked on the host before a kernel is enqueued, so that a bad
// call returns an error code instead of a memory fault on the device.
#include <stdarg.h>
#include <cmath>
#include <stdio.h>

#include "heart_internal.h"

namespace heart {

static thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

void clear_error() { g_err[0] = '\0'; }

int check_launch(const char *what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(HEART_EHIP, "%s: %s", what, hipGetErrorString(e));
  return HEART_OK;
}

static int check_shape(const heart_shape *s, const char *fn) {
  if (!s) return fail(HEART_EINVAL, "%s: shape is NULL", fn);
  if (s->B <= 0 || s->H <= 0 || s->N <= 0)
    return fail(HEART_EINVAL, "%s: B, H, N must be positive (got %d, %d, %d)", fn, s->B, s->H,
                s->N);
  if (s->D != 64 && s->D != 128)
    return fail(HEART_EUNSUPPORTED, "%s: D must be 64 or 128 (got %d)", fn, s->D);
  if (s->block != 64 && s->block != 128)
    return fail(HEART_EUNSUPPORTED, "%s: block must be 64 or 128 (got %d)", fn, s->block);
  long long nb = ((long long)s->N + s->block - 1) / s->block;
  if ((long long)s->B * s->H * nb > 0x7fffffffLL)
    return fail(HEART_EUNSUPPORTED, "%s: B*H*Nb exceeds the 1-D grid limit", fn);
  return HEART_OK;
}

}  // namespace heart

using namespace heart;

extern "C" {

const char *heart_last_error(void) { return g_err; }

int heart_version(void) { return 100; }

int heart_pool_qk(const heart_shape *shape, const void *q, const void *k, float *qblk,
                  float *kblk, float *qmean, float *kmean, void *stream) {
  clear_error();
  if (int rc = check_shape(shape, "heart_pool_qk")) return rc;
  if (!q || !k || !qblk || !kblk || !qmean || !kmean)
    return fail(HEART_EINVAL, "heart_pool_qk: NULL pointer argument");
  if (!aligned16(q) || !aligned16(k) || !aligned16(qblk) || !aligned16(kblk) ||
      !aligned16(qmean) || !aligned16(kmean))
    return fail(HEART_EUNSUPPORTED, "heart_pool_qk: pointers must be 16-byte aligned");
  if (!stride_ok(shape->q_stride) || !stride_ok(shape->k_stride))
    return fail(HEART_EUNSUPPORTED,
                "heart_pool_qk: strides must be multiples of 8 elements, token stride > 0");
  return launch_pool(*shape, q, k, qblk, kblk, qmean, kmean, (hipStream_t)stream);
}

size_t heart_pool_drift_workspace_bytes(int B, int H) {
  if (B <= 0 || H <= 0) return 0;
  (void)H;
  return (size_t)B * sizeof(unsigned);  // one completion ticket per batch item
}

int heart_pool_drift(const heart_shape *shape, const void *q, const void *k, float *qblk,
                     float *kblk, float *qmean, float *kmean, float *qanchor, float *kanchor,
                     unsigned char *has_anchor, const float *delta, float gate_lo, float gate_hi,
                     int commit, float *drift, unsigned char *refresh, void *workspace,
                     size_t workspace_bytes, void *stream) {
  clear_error();
  if (int rc = check_shape(shape, "heart_pool_drift")) return rc;
  if (!q || !k || !qblk || !kblk || !qmean || !kmean || !qanchor || !kanchor || !has_anchor ||
      !delta || !drift || !refresh || !workspace)
    return fail(HEART_EINVAL, "heart_pool_drift: NULL pointer argument");
  if (!aligned16(q) || !aligned16(k) || !aligned16(qblk) || !aligned16(kblk) ||
      !aligned16(qmean) || !aligned16(kmean))
    return fail(HEART_EUNSUPPORTED, "heart_pool_drift: q, k and the pooled outputs must be 16-byte aligned");
  if (!stride_ok(shape->q_stride) || !stride_ok(shape->k_stride))
    return fail(HEART_EUNSUPPORTED,
                "heart_pool_drift: strides must be multiples of 8 elements, token stride > 0");
  if (shape->H > 4096)
    return fail(HEART_EUNSUPPORTED, "heart_pool_drift: H must be <= 4096 (got %d)", shape->H);
  if (!(gate_lo <= gate_hi))
    return fail(HEART_EINVAL, "heart_pool_drift: need gate_lo <= gate_hi (got %g, %g)", gate_lo,
                gate_hi);
  if ((reinterpret_cast<uintptr_t>(workspace) & 3u) != 0)
    return fail(HEART_EUNSUPPORTED, "heart_pool_drift: workspace must be 4-byte aligned");
  if (workspace_bytes < heart_pool_drift_workspace_bytes(shape->B, shape->H))
    return fail(HEART_EINVAL, "heart_pool_drift: workspace of %zu bytes, need %zu", workspace_bytes,
                heart_pool_drift_workspace_bytes(shape->B, shape->H));
  return launch_pool_drift(*shape, q, k, qblk, kblk, qmean, kmean, qanchor, kanchor, has_anchor,
                           delta, gate_lo, gate_hi, commit, drift, refresh, (unsigned *)workspace,
                           (hipStream_t)stream);
}

int heart_drift(int B, int H, int D, const float *qmean, const float *kmean, float *qanchor,
                float *kanchor, unsigned char *has_anchor, const float *delta, float gate_lo,
                float gate_hi, int commit, float *drift, unsigned char *refresh, void *stream) {
  clear_error();
  if (B <= 0 || H <= 0 || D <= 0)
    return fail(HEART_EINVAL, "heart_drift: B, H, D must be positive (got %d, %d, %d)", B, H, D);
  if ((D & (D - 1)) != 0 || D > 512)
    return fail(HEART_EUNSUPPORTED, "heart_drift: D must be a power of two <= 512 (got %d)", D);
  if (H > 4096) return fail(HEART_EUNSUPPORTED, "heart_drift: H must be <= 4096 (got %d)", H);
  if (!qmean || !kmean || !qanchor || !kanchor || !has_anchor || !delta || !drift || !refresh)
    return fail(HEART_EINVAL, "heart_drift: NULL pointer argument");
  if (!(gate_lo <= gate_hi))
    return fail(HEART_EINVAL, "heart_drift: need gate_lo <= gate_hi (got %g, %g)", gate_lo,
                gate_hi);
  return launch_drift(B, H, D, qmean, kmean, qanchor, kanchor, has_anchor, delta, gate_lo,
                      gate_hi, commit, drift, refresh, (hipStream_t)stream);
}

static int mask_topp_checked(int B, int H, int Nb, int D, const float *qblk, const float *kblk,
                             const float *scores_in, const float *tau,
                             const unsigned char *refresh, int n_always_kv_blocks,
                             int n_dense_q_blocks, int min_keep, unsigned char *mask,
                             int *kept_idx, int *kept_count, float *scores_out, void *workspace,
                             size_t workspace_bytes, void *stream) {
  clear_error();
  if (B <= 0 || H <= 0 || Nb <= 0)
    return fail(HEART_EINVAL, "heart_mask_topp: B, H, Nb must be positive (got %d, %d, %d)", B,
                H, Nb);
  if (Nb > HEART_MAX_NB)
    return fail(HEART_EUNSUPPORTED, "heart_mask_topp: Nb = %d exceeds HEART_MAX_NB = %d", Nb,
                HEART_MAX_NB);
  if (!scores_in) {
    if (!qblk || !kblk)
      return fail(HEART_EINVAL, "heart_mask_topp: need qblk and kblk, or scores_in");
    if (D <= 0 || D % 16 != 0 || D > 128)
      return fail(HEART_EUNSUPPORTED,
                  "heart_mask_topp: D must be a positive multiple of 16, <= 128 (got %d)", D);
    if (!aligned16(qblk) || !aligned16(kblk))
      return fail(HEART_EUNSUPPORTED, "heart_mask_topp: qblk/kblk must be 16-byte aligned");
  }
  if (!tau || !mask || !kept_idx || !kept_count)
    return fail(HEART_EINVAL, "heart_mask_topp: NULL pointer argument");
  if (n_always_kv_blocks < 0 || n_dense_q_blocks < 0 || min_keep < 0)
    return fail(HEART_EINVAL, "heart_mask_topp: negative block-count argument");
  if ((long long)B * H * Nb > 0x7fffffffLL)
    return fail(HEART_EUNSUPPORTED, "heart_mask_topp: B*H*Nb exceeds the 1-D grid limit");
  if (workspace) {
    if (!aligned16(workspace))
      return fail(HEART_EUNSUPPORTED, "heart_mask_topp_ws: workspace must be 16-byte aligned");
    const size_t need = mask_topp_workspace_bytes(B, H, Nb, D);
    if (!scores_in && workspace_bytes < need)
      return fail(HEART_EINVAL, "heart_mask_topp_ws: workspace of %zu bytes, need %zu",
                  workspace_bytes, need);
  }
  return launch_mask_topp(B, H, Nb, D, qblk, kblk, scores_in, tau, refresh, n_always_kv_blocks,
                          n_dense_q_blocks, min_keep, mask, kept_idx, kept_count, scores_out,
                          workspace, (hipStream_t)stream);
}

int heart_mask_topp(int B, int H, int Nb, int D, const float *qblk, const float *kblk,
                    const float *scores_in, const float *tau, const unsigned char *refresh,
                    int n_always_kv_blocks, int n_dense_q_blocks, int min_keep,
                    unsigned char *mask, int *kept_idx, int *kept_count, float *scores_out,
                    void *stream) {
  return mask_topp_checked(B, H, Nb, D, qblk, kblk, scores_in, tau, refresh, n_always_kv_blocks,
                           n_dense_q_blocks, min_keep, mask, kept_idx, kept_count, scores_out,
                           nullptr, 0, stream);
}

int heart_mask_topp_ws(int B, int H, int Nb, int D, const float *qblk, const float *kblk,
                       const float *scores_in, const float *tau, const unsigned char *refresh,
                       int n_always_kv_blocks, int n_dense_q_blocks, int min_keep,
                       unsigned char *mask, int *kept_idx, int *kept_count, float *scores_out,
                       void *workspace, size_t workspace_bytes, void *stream) {
  return mask_topp_checked(B, H, Nb, D, qblk, kblk, scores_in, tau, refresh, n_always_kv_blocks,
                           n_dense_q_blocks, min_keep, mask, kept_idx, kept_count, scores_out,
                           workspace, workspace_bytes, stream);
}

size_t heart_mask_topp_workspace_bytes(int B, int H, int Nb, int D) {
  if (B <= 0 || H <= 0 || Nb <= 0 || D <= 0) return 0;
  return mask_topp_workspace_bytes(B, H, Nb, D);
}

static int attn_checked(const heart_shape *shape, const void *q, const void *k, const void *v,
                        const int *kept_idx, const int *kept_count, float scale, unsigned flags,
                        void *out, float *lse, void *workspace, size_t workspace_bytes,
                        void *stream) {
  clear_error();
  if (int rc = check_shape(shape, "heart_block_sparse_attn")) return rc;
  if (flags & ~HEART_ATTN_FOLD_SCALE)
    return fail(HEART_EINVAL, "heart_block_sparse_attn: unknown flag bits 0x%x", flags);
  if (!q || !k || !v || !kept_idx || !kept_count || !out)
    return fail(HEART_EINVAL, "heart_block_sparse_attn: NULL pointer argument");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out))
    return fail(HEART_EUNSUPPORTED,
                "heart_block_sparse_attn: q/k/v/out must be 16-byte aligned");
  if (!stride_ok(shape->q_stride) || !stride_ok(shape->k_stride) ||
      !stride_ok(shape->v_stride) || !stride_ok(shape->o_stride))
    return fail(HEART_EUNSUPPORTED,
                "heart_block_sparse_attn: strides must be multiples of 8 elements, token "
                "stride > 0");
  if (workspace) {
    if (!aligned16(workspace))
      return fail(HEART_EUNSUPPORTED, "heart_block_sparse_attn: workspace must be 16-byte aligned");
    if (workspace_bytes < heart_attn_workspace_bytes(shape))
      return fail(HEART_EINVAL, "heart_block_sparse_attn: workspace of %zu bytes, need %zu",
                  workspace_bytes, heart_attn_workspace_bytes(shape));
  }
  return launch_attn(*shape, q, k, v, kept_idx, kept_count, scale, flags, out, lse,
                     (int *)workspace, (hipStream_t)stream);
}

int heart_block_sparse_attn(const heart_shape *shape, const void *q, const void *k,
                            const void *v, const int *kept_idx, const int *kept_count,
                            float scale, void *out, float *lse, void *workspace,
                            size_t workspace_bytes, void *stream) {
  return attn_checked(shape, q, k, v, kept_idx, kept_count, scale, 0u, out, lse, workspace,
                      workspace_bytes, stream);
}

int heart_block_sparse_attn_flags(const heart_shape *shape, const void *q, const void *k,
                                  const void *v, const int *kept_idx, const int *kept_count,
                                  float scale, unsigned flags, void *out, float *lse,
                                  void *workspace, size_t workspace_bytes, void *stream) {
  return attn_checked(shape, q, k, v, kept_idx, kept_count, scale, flags, out, lse, workspace,
                      workspace_bytes, stream);
}

int heart_block_sparse_attn_static(const heart_shape *shape, const void *q, const void *k,
                                   const void *v, const int *kept_idx, const int *kept_count,
                                   float scale, unsigned flags, void *out, float *lse,
                                   void *stream) {
  clear_error();
  if (int rc = check_shape(shape, "heart_block_sparse_attn_static")) return rc;
  const size_t need = heart_attn_workspace_bytes(shape);
  if (need > HEART_ATTN_STATIC_PLAN_BYTES)
    return fail(HEART_EUNSUPPORTED,
                "heart_block_sparse_attn_static: the launch plan of this shape takes %zu bytes, the "
                "static array holds %u (B*H*(Nb+2) + 24 ints must not exceed %u)",
                need, HEART_ATTN_STATIC_PLAN_BYTES, HEART_ATTN_STATIC_PLAN_BYTES / 4u);
  int *plan = nullptr;
  if (int rc = attn_static_plan(&plan)) return rc;
  return attn_checked(shape, q, k, v, kept_idx, kept_count, scale, flags, out, lse, plan, need,
                      stream);
}

size_t heart_workspace_bytes(int B, int H, int Nb, int D) {
  (void)D;
  if (B <= 0 || H <= 0 || Nb <= 0) return 0;
  // plan header (24 ints) + two entries per head + one entry per (head, query block)
  return ((size_t)B * H * ((size_t)Nb + 2) + 24) * sizeof(int);
}

size_t heart_attn_workspace_bytes(const heart_shape *s) {
  if (!s || s->B <= 0 || s->H <= 0 || s->N <= 0 || s->block <= 0) return 0;
  const long long nb = ((long long)s->N + s->block - 1) / s->block;
  return heart_workspace_bytes(s->B, s->H, (int)nb, s->D);
}

static int check_antidiag(const heart_shape *s, int stride, const char *fn) {
  if (int rc = check_shape(s, fn)) return rc;
  if (stride <= 0 || s->block != 8 * stride)
    return fail(HEART_EUNSUPPORTED, "%s: block must be 8 * stride (got block %d, stride %d)", fn,
                s->block, stride);
  const long long nb = ((long long)s->N + s->block - 1) / s->block;
  if (nb > HEART_MAX_NB)
    return fail(HEART_EUNSUPPORTED, "%s: Nb = %lld exceeds HEART_MAX_NB = %d", fn, nb, HEART_MAX_NB);
  return HEART_OK;
}

size_t heart_scores_antidiag_workspace_bytes(const heart_shape *s, int stride) {
  if (!s || s->B <= 0 || s->H <= 0 || s->N <= 0 || stride <= 0) return 0;
  return antidiag_workspace_bytes(*s, stride);
}

int heart_scores_antidiag(const heart_shape *shape, const void *q, const void *k, int stride,
                          const unsigned char *refresh, float *scores, void *workspace,
                          size_t workspace_bytes, void *stream) {
  clear_error();
  if (int rc = check_antidiag(shape, stride, "heart_scores_antidiag")) return rc;
  if (!q || !k || !scores || !workspace)
    return fail(HEART_EINVAL, "heart_scores_antidiag: NULL pointer argument");
  if (!aligned16(q) || !aligned16(k) || !aligned16(workspace))
    return fail(HEART_EUNSUPPORTED, "heart_scores_antidiag: q, k and workspace must be 16-byte aligned");
  if (!stride_ok(shape->q_stride) || !stride_ok(shape->k_stride))
    return fail(HEART_EUNSUPPORTED,
                "heart_scores_antidiag: strides must be multiples of 8 elements, token stride > 0");
  if (workspace_bytes < heart_scores_antidiag_workspace_bytes(shape, stride))
    return fail(HEART_EINVAL, "heart_scores_antidiag: workspace of %zu bytes, need %zu", workspace_bytes,
                heart_scores_antidiag_workspace_bytes(shape, stride));
  return launch_antidiag(*shape, q, k, stride, refresh, scores, (float *)workspace,
                         (hipStream_t)stream);
}

int heart_ebc_band_error(long long C, int T, int Y, int X, const float *err, const float *dense,
                         const double *weights4_host, double epsilon, void *workspace,
                         size_t workspace_bytes, double *out6, void *stream) {
  clear_error();
  if (C <= 0 || T <= 0 || Y <= 0 || X <= 0)
    return fail(HEART_EINVAL, "heart_ebc_band_error: sizes must be positive");
  if (T > 1024 || Y > 1024 || X > 1024)
    return fail(HEART_EUNSUPPORTED, "heart_ebc_band_error: axes longer than 1024 are not supported");
  if (!err || !dense || !weights4_host || !workspace || !out6)
    return fail(HEART_EINVAL, "heart_ebc_band_error: NULL pointer argument");
  if (!(epsilon >= 0.0)) return fail(HEART_EINVAL, "heart_ebc_band_error: epsilon must be >= 0");
  if (!aligned16(workspace) || workspace_bytes < heart_ebc_workspace_bytes(C, T, Y, X))
    return fail(HEART_EINVAL, "heart_ebc_band_error: workspace of %zu bytes, need %zu (16-byte aligned)",
                workspace_bytes, heart_ebc_workspace_bytes(C, T, Y, X));
  return launch_ebc_band_error(C, T, Y, X, err, dense, weights4_host, epsilon, (double *)workspace,
                               out6, (hipStream_t)stream);
}

size_t heart_ebc_workspace_bytes(long long C, int T, int Y, int X) {
  if (C <= 0 || T <= 0 || Y <= 0 || X <= 0) return 0;
  return ebc_workspace_bytes(C, T, Y, X);
}

int heart_ebc_select(int n_heads, int n_candidates, const double *error_host,
                     const double *sparsity_host, double min_mean_sparsity, int *choice_host,
                     double *total_error_host) {
  clear_error();
  if (n_heads <= 0 || n_candidates <= 0)
    return fail(HEART_EINVAL, "heart_ebc_select: n_heads and n_candidates must be positive");
  if (!error_host || !sparsity_host || !choice_host || !total_error_host)
    return fail(HEART_EINVAL, "heart_ebc_select: NULL pointer argument");
  for (size_t i = 0; i < (size_t)n_heads * n_candidates; ++i)
    if (!std::isfinite(error_host[i]) || !std::isfinite(sparsity_host[i]))
      return fail(HEART_EINVAL, "heart_ebc_select: table entry %zu is not finite", i);
  const int rc = ebc_select_host(n_heads, n_candidates, error_host, sparsity_host,
                                 min_mean_sparsity, choice_host, total_error_host, nullptr);
  if (rc == 1)
    return fail(HEART_EINVAL, "heart_ebc_select: the sparsity budget %g cannot be met",
                min_mean_sparsity);
  if (rc == 2)
    return fail(HEART_EUNSUPPORTED,
                "heart_ebc_select: optimality not proved within the search limit (the best "
                "selection found is in choice_host)");
  return HEART_OK;
}

int heart_ubench_mfma_bf16(const void *a_bf16, const void *b_bf16, int n_workgroups, int iters,
                           float *sink, void *stream) {
  clear_error();
  if (!a_bf16 || !b_bf16 || !sink) return fail(HEART_EINVAL, "heart_ubench_mfma_bf16: NULL pointer argument");
  if (!aligned16(a_bf16) || !aligned16(b_bf16))
    return fail(HEART_EUNSUPPORTED, "heart_ubench_mfma_bf16: operands must be 16-byte aligned");
  if (n_workgroups <= 0 || iters <= 0 || n_workgroups > (1 << 20) || iters > (1 << 24))
    return fail(HEART_EINVAL, "heart_ubench_mfma_bf16: n_workgroups in [1, 2^20], iters in [1, 2^24]");
  return launch_ubench_mfma(a_bf16, b_bf16, n_workgroups, iters, sink, (hipStream_t)stream);
}

int heart_ubench_read(const void *src, size_t bytes, unsigned *sink, void *stream) {
  clear_error();
  if (!src || !sink) return fail(HEART_EINVAL, "heart_ubench_read: NULL pointer argument");
  if (!aligned16(src) || bytes % 16 != 0 || bytes == 0)
    return fail(HEART_EUNSUPPORTED,
                "heart_ubench_read: src 16-byte aligned, bytes a positive multiple of 16");
  return launch_ubench_read(src, bytes, sink, (hipStream_t)stream);
}

int heart_ubench_copy(const void *src, void *dst, size_t bytes, void *stream) {
  clear_error();
  if (!src || !dst) return fail(HEART_EINVAL, "heart_ubench_copy: NULL pointer argument");
  if (!aligned16(src) || !aligned16(dst) || bytes % 16 != 0 || bytes == 0)
    return fail(HEART_EUNSUPPORTED,
                "heart_ubench_copy: pointers 16-byte aligned, bytes a positive multiple of 16");
  return launch_ubench_copy(src, dst, bytes, (hipStream_t)stream);
}

}  // extern "C"
