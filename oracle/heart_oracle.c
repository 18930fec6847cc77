/*
 * CPU oracle for the HEART sparse-attention hot path.  TEST INFRASTRUCTURE ONLY:
 * a plain, slow, obviously-correct statement of what each step computes, used by
 * the tests, the smoke check and the benchmark's CPU-baseline leg.  The product
 * (the HIP library) neither links nor calls anything in this file, and this file
 * shares no code, header, table or helper with it.
 *
 * Arithmetic: inputs are bf16 (exactly representable in fp32/fp64); every sum is
 * accumulated in fp64 and rounded once to fp32 on output, except the drift, whose
 * fp32 summation order is part of its definition here (see oracle_drift).
 *
 * Steps, in the order of the paper's Temporal Mask Reuse procedure (Alg. 1):
 *   oracle_pool       token means (Alg. 1 step 1; mean-pooled drift, Eq. 4) and
 *                     block means (block-level importance, Sec. 4.2 / top-p, Sec. 3.2)
 *   oracle_drift      mean-pooled L1 drift (Eq. 4), reuse rule (Sec. 4.2, Alg. 1),
 *                     layer-level gate (Sec. 4.2 last paragraph; thresholds in the
 *                     appendix on HEART configurations)
 *   oracle_scores     block importance: row softmax of pooled Q.K/sqrt(D)
 *                     (interaction scale from the appendix on query-key stability)
 *   oracle_topp       top-p selection: rank blocks, keep the minimal prefix whose
 *                     cumulative mass reaches tau (Sec. 3.2; minimal set of Eq. 1)
 *   oracle_attn       softmax attention restricted to kept key blocks
 *   oracle_dense_attn unblocked dense attention (brute force, for tests)
 *
 * Readings where the paper is silent that shape this file: ties rank lower key-block index first; "reaches"
 * is >=; cumulative mass is an integer fixed point (floor(P * 2^30)) compared
 * against tau * total so the kept set does not depend on summation order;
 * tau >= 1 keeps every block; drift is summed (not averaged) over D.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline float bf16_to_f32(uint16_t h) {
  uint32_t u = ((uint32_t)h) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return f;
}

/* ---------------------------------------------------------------------------
 * Pooling.  x: bf16 bits, element strides (sb, sh, sn), D contiguous.
 * blk  [B,H,Nb,D]: mean over the n_i real tokens of block i (the last block may be short)
 * mean [B,H,D]   : mean over all N tokens (sum of block sums / N, NOT mean of block means)
 * -------------------------------------------------------------------------*/
void oracle_pool(int B, int H, int N, int D, int block, const uint16_t *x, long long sb,
                 long long sh, long long sn, float *blk, float *mean) {
  int Nb = (N + block - 1) / block;
#pragma omp parallel for collapse(2) schedule(static)
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < H; ++h) {
      double *tot = (double *)calloc((size_t)D, sizeof(double));
      double *acc = (double *)malloc((size_t)D * sizeof(double));
      for (int i = 0; i < Nb; ++i) {
        int n0 = i * block, n1 = n0 + block < N ? n0 + block : N;
        for (int d = 0; d < D; ++d) acc[d] = 0.0;
        for (int n = n0; n < n1; ++n) {
          const uint16_t *row = x + b * sb + h * sh + (long long)n * sn;
          for (int d = 0; d < D; ++d) acc[d] += (double)bf16_to_f32(row[d]);
        }
        float *o = blk + (((size_t)b * H + h) * Nb + i) * D;
        for (int d = 0; d < D; ++d) {
          o[d] = (float)(acc[d] / (double)(n1 - n0));
          tot[d] += acc[d];
        }
      }
      float *m = mean + ((size_t)b * H + h) * D;
      for (int d = 0; d < D; ++d) m[d] = (float)(tot[d] / (double)N);
      free(tot);
      free(acc);
    }
}

/* ---------------------------------------------------------------------------
 * Drift + reuse rule + layer gate + anchor commit.
 * drift_h = sum_d |qa_d - qb_d| + |ka_d - kb_d|, evaluated in fp32 with a fixed
 * halving tree over d (D must be a power of two): a[i] += a[i+s], s = D/2 .. 1.
 * The order is fixed so that a reuse/refresh decision is a well-defined function
 * of the fp32 means.  mark = no anchor, or drift > delta (strict).  Gate (per
 * batch item): frac = marks/H in fp32; frac < gate_lo: every head that has an
 * anchor reuses; frac > gate_hi: every head refreshes; else head-wise marks.
 * With commit != 0 refreshed heads copy the current means into the anchors.
 * Heads without an anchor report drift = +inf.
 * -------------------------------------------------------------------------*/
void oracle_drift(int B, int H, int D, const float *qmean, const float *kmean, float *qanchor,
                  float *kanchor, unsigned char *has_anchor, const float *delta, float gate_lo,
                  float gate_hi, int commit, float *drift, unsigned char *refresh) {
  float *a = (float *)malloc((size_t)D * sizeof(float));
  unsigned char *mark = (unsigned char *)malloc((size_t)H);
  for (int b = 0; b < B; ++b) {
    int n_mark = 0;
    for (int h = 0; h < H; ++h) {
      size_t o = ((size_t)b * H + h) * D;
      if (!has_anchor[b * H + h]) {
        drift[b * H + h] = INFINITY;
        mark[h] = 1;
      } else {
        for (int d = 0; d < D; ++d) {
          float dq = fabsf(qanchor[o + d] - qmean[o + d]);
          float dk = fabsf(kanchor[o + d] - kmean[o + d]);
          a[d] = dq + dk;
        }
        for (int s = D / 2; s >= 1; s /= 2)
          for (int i = 0; i < s; ++i) a[i] = a[i] + a[i + s];
        drift[b * H + h] = a[0];
        mark[h] = a[0] > delta[h] ? 1 : 0;
      }
      n_mark += mark[h];
    }
    float frac = (float)n_mark / (float)H;
    for (int h = 0; h < H; ++h) {
      unsigned char r;
      if (frac < gate_lo)
        r = has_anchor[b * H + h] ? 0 : 1;
      else if (frac > gate_hi)
        r = 1;
      else
        r = mark[h];
      refresh[b * H + h] = r;
      if (r && commit) {
        size_t o = ((size_t)b * H + h) * D;
        memcpy(qanchor + o, qmean + o, (size_t)D * sizeof(float));
        memcpy(kanchor + o, kmean + o, (size_t)D * sizeof(float));
        has_anchor[b * H + h] = 1;
      }
    }
  }
  free(a);
  free(mark);
}

/* ---------------------------------------------------------------------------
 * Block importance: P[i,j] = softmax_j( qblk_i . kblk_j / sqrt(D) ), fp64 inside.
 * scores [B,H,Nb,Nb] fp32.
 * -------------------------------------------------------------------------*/
void oracle_scores(int B, int H, int Nb, int D, const float *qblk, const float *kblk,
                   float *scores) {
  double inv = 1.0 / sqrt((double)D);
#pragma omp parallel for schedule(static)
  for (long long r = 0; r < (long long)B * H * Nb; ++r) {
    long long bh = r / Nb;
    const float *q = qblk + (size_t)r * D;
    double *logit = (double *)malloc((size_t)Nb * sizeof(double));
    double m = -INFINITY;
    for (int j = 0; j < Nb; ++j) {
      const float *k = kblk + ((size_t)bh * Nb + j) * D;
      double s = 0.0;
      for (int d = 0; d < D; ++d) s += (double)q[d] * (double)k[d];
      logit[j] = s * inv;
      if (logit[j] > m) m = logit[j];
    }
    double z = 0.0;
    for (int j = 0; j < Nb; ++j) {
      logit[j] = exp(logit[j] - m);
      z += logit[j];
    }
    float *o = scores + (size_t)r * Nb;
    for (int j = 0; j < Nb; ++j) o[j] = (float)(logit[j] / z);
    free(logit);
  }
}

/* ---------------------------------------------------------------------------
 * Top-p block selection per (b, h, query-block row).
 * Rank key blocks by score descending (equal scores: lower index first).  With
 * u_j = floor(P_j * 2^30) and T = floor(tau * 2^24), keep the shortest prefix of
 * that ranking with  cum(u) * 2^24 >= T * sum(u);  never fewer than
 * max(1, min_keep) blocks; tau >= 1 keeps all.  Afterwards key-block columns
 * j < n_always_kv and all columns of query rows i < n_dense_q are kept as well.
 * Heads with refresh[b,h] == 0 (refresh != NULL) are left untouched.
 * Outputs: mask u8 [B,H,Nb,Nb]; kept_idx i32 [B,H,Nb,Nb] (ascending, first
 * kept_count entries valid, the rest untouched); kept_count i32 [B,H,Nb].
 * -------------------------------------------------------------------------*/
typedef struct {
  float p;
  int j;
} rank_item;

static int rank_cmp(const void *a, const void *b) {
  const rank_item *x = (const rank_item *)a, *y = (const rank_item *)b;
  if (x->p > y->p) return -1;
  if (x->p < y->p) return 1;
  return x->j - y->j;
}

void oracle_topp(int B, int H, int Nb, const float *scores, const float *tau,
                 const unsigned char *refresh, int n_always_kv, int n_dense_q, int min_keep,
                 unsigned char *mask, int *kept_idx, int *kept_count) {
#pragma omp parallel for schedule(static)
  for (long long r = 0; r < (long long)B * H * Nb; ++r) {
    long long bh = r / Nb;
    int h = (int)(bh % H), i = (int)(r % Nb);
    if (refresh && !refresh[bh]) continue;
    const float *p = scores + (size_t)r * Nb;
    unsigned char *m = mask + (size_t)r * Nb;
    rank_item *it = (rank_item *)malloc((size_t)Nb * sizeof(rank_item));
    unsigned __int128 total = 0;
    for (int j = 0; j < Nb; ++j) {
      it[j].p = p[j];
      it[j].j = j;
      total += (uint64_t)floor((double)p[j] * 1073741824.0);
    }
    qsort(it, (size_t)Nb, sizeof(rank_item), rank_cmp);
    int keep;
    if (tau[h] >= 1.0f) {
      keep = Nb;
    } else {
      unsigned __int128 T = (uint64_t)floor((double)tau[h] * 16777216.0);
      unsigned __int128 cum = 0;
      keep = Nb;
      for (int k = 0; k < Nb; ++k) {
        cum += (uint64_t)floor((double)it[k].p * 1073741824.0);
        if (cum * 16777216u >= T * total) {
          keep = k + 1;
          break;
        }
      }
    }
    int floor_keep = min_keep > 1 ? min_keep : 1;
    if (floor_keep > Nb) floor_keep = Nb;
    if (keep < floor_keep) keep = floor_keep;
    memset(m, 0, (size_t)Nb);
    for (int k = 0; k < keep; ++k) m[it[k].j] = 1;
    for (int j = 0; j < Nb; ++j)
      if (j < n_always_kv || i < n_dense_q) m[j] = 1;
    int c = 0;
    int *idx = kept_idx + (size_t)r * Nb;
    for (int j = 0; j < Nb; ++j)
      if (m[j]) idx[c++] = j;
    kept_count[r] = c;
    free(it);
  }
}

/* ---------------------------------------------------------------------------
 * Attention restricted to kept key blocks.  q,k,v: bf16 bits with element
 * strides (sb, sh, sn); out fp32 contiguous [B,H,N,D]; lse (nullable) [B,H,N] is
 * the natural-log-sum-exp of the scaled logits over the kept keys.
 * Only query blocks listed in qblocks[0..n_qblocks) are computed (NULL = all);
 * rows of other query blocks are left untouched.  scale <= 0 means 1/sqrt(D).
 * -------------------------------------------------------------------------*/
void oracle_attn(int B, int H, int N, int D, int block, const uint16_t *q, const uint16_t *k,
                 const uint16_t *v, const long long *qs, const long long *ks,
                 const long long *vs, const int *kept_idx, const int *kept_count, float scale,
                 const int *qblocks, int n_qblocks, float *out, float *lse) {
  int Nb = (N + block - 1) / block;
  double sc = scale > 0.0f ? (double)scale : 1.0 / sqrt((double)D);
  int nq = qblocks ? n_qblocks : Nb;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (long long bh = 0; bh < (long long)B * H; ++bh)
    for (int qi = 0; qi < nq; ++qi) {
      int b = (int)(bh / H), h = (int)(bh % H);
      int i = qblocks ? qblocks[qi] : qi;
      size_t row = ((size_t)bh * Nb + i);
      const int *idx = kept_idx + row * Nb;
      int cnt = kept_count[row];
      int n0 = i * block, n1 = n0 + block < N ? n0 + block : N;
      double *s = (double *)malloc((size_t)cnt * block * sizeof(double));
      double *acc = (double *)malloc((size_t)D * sizeof(double));
      double *qd = (double *)malloc((size_t)D * sizeof(double));
      for (int n = n0; n < n1; ++n) {
        const uint16_t *qr = q + b * qs[0] + h * qs[1] + (long long)n * qs[2];
        for (int d = 0; d < D; ++d) qd[d] = (double)bf16_to_f32(qr[d]);
        double m = -INFINITY;
        int ns = 0;
        for (int c = 0; c < cnt; ++c) {
          int j = idx[c];
          int m0 = j * block, m1 = m0 + block < N ? m0 + block : N;
          for (int t = m0; t < m1; ++t) {
            const uint16_t *kr = k + b * ks[0] + h * ks[1] + (long long)t * ks[2];
            double dot = 0.0;
            for (int d = 0; d < D; ++d) dot += qd[d] * (double)bf16_to_f32(kr[d]);
            dot *= sc;
            s[ns++] = dot;
            if (dot > m) m = dot;
          }
        }
        double z = 0.0;
        for (int d = 0; d < D; ++d) acc[d] = 0.0;
        ns = 0;
        for (int c = 0; c < cnt; ++c) {
          int j = idx[c];
          int m0 = j * block, m1 = m0 + block < N ? m0 + block : N;
          for (int t = m0; t < m1; ++t) {
            const uint16_t *vr = v + b * vs[0] + h * vs[1] + (long long)t * vs[2];
            double p = exp(s[ns++] - m);
            z += p;
            for (int d = 0; d < D; ++d) acc[d] += p * (double)bf16_to_f32(vr[d]);
          }
        }
        float *o = out + ((size_t)bh * N + n) * D;
        for (int d = 0; d < D; ++d) o[d] = (float)(acc[d] / z);
        if (lse) lse[(size_t)bh * N + n] = (float)(m + log(z));
      }
      free(s);
      free(acc);
      free(qd);
    }
}

/* Unblocked dense attention: out[n] = sum_t softmax_t(q_n.k_t * scale) v_t. */
void oracle_dense_attn(int B, int H, int N, int D, const uint16_t *q, const uint16_t *k,
                       const uint16_t *v, const long long *qs, const long long *ks,
                       const long long *vs, float scale, float *out) {
  double sc = scale > 0.0f ? (double)scale : 1.0 / sqrt((double)D);
#pragma omp parallel for schedule(static)
  for (long long r = 0; r < (long long)B * H * N; ++r) {
    long long bh = r / N;
    int b = (int)(bh / H), h = (int)(bh % H), n = (int)(r % N);
    const uint16_t *qr = q + b * qs[0] + h * qs[1] + (long long)n * qs[2];
    double *s = (double *)malloc((size_t)N * sizeof(double));
    double m = -INFINITY;
    for (int t = 0; t < N; ++t) {
      const uint16_t *kr = k + b * ks[0] + h * ks[1] + (long long)t * ks[2];
      double dot = 0.0;
      for (int d = 0; d < D; ++d) dot += (double)bf16_to_f32(qr[d]) * (double)bf16_to_f32(kr[d]);
      s[t] = dot * sc;
      if (s[t] > m) m = s[t];
    }
    double z = 0.0;
    for (int t = 0; t < N; ++t) {
      s[t] = exp(s[t] - m);
      z += s[t];
    }
    float *o = out + (size_t)r * D;
    for (int d = 0; d < D; ++d) {
      double a = 0.0;
      for (int t = 0; t < N; ++t) {
        const uint16_t *vr = v + b * vs[0] + h * vs[1] + (long long)t * vs[2];
        a += s[t] * (double)bf16_to_f32(vr[d]);
      }
      o[d] = (float)(a / z);
    }
    free(s);
  }
}

int oracle_num_threads(void) {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp master
    n = omp_get_num_threads();
  }
#endif
  return n;
}
