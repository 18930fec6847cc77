// heart_mask_topp: block importance from pooled Q/K blocks and top-p block selection
// with a per-head threshold (Sec. 3.2: rank candidate blocks by importance, keep
// them until the accumulated importance reaches tau; Eq. 1: the minimal such set;
// 1/sqrt(D) interaction scale from the appendix on query-key stability).
//
// One workgroup (4 wavefronts) owns R = 8 query-block rows of one head.
//   Phase A  logits[r][j] = qblk_r . kblk_j / sqrt(D): lane <-> key-block column,
//            all R rows per lane, fp64 fused multiply-add (on this chip fp64 FMA
//            issues at the rate of unpacked fp32 FMA, and it takes the dot product
//            out of the error budget of the scores).  The R query rows sit in LDS
//            as fp64 and are read as wave-wide broadcasts.
//   Phase B  row softmax, one wavefront per row, fp32 with the accurate expf.
//   Phase C  top-p selection, one wavefront per row, without sorting: the kept set
//            is "every score above a threshold value v*, plus the lowest-index
//            ties at v*", and v* is found by a 31-step bitwise search on the fp32
//            bit pattern (positive floats order like their bit patterns), each
//            step being one wave-wide integer reduction of the fixed-point mass
//            (DPP / lane-swap reductions on the VALU, no LDS traffic).
//            All mass arithmetic is integer, so the result does not depend on the
//            order of the reduction.  Rank positions for the ascending kept-index
//            list come from wave ballots and population counts.
#include "heart_internal.h"

namespace heart {

constexpr int kRows = 8;  // query-block rows per workgroup

template <int CMAX>  // slots per lane; handles Nb <= 64 * CMAX
__global__ __launch_bounds__(256) void mask_topp_kernel(
    int H, int Nb, int D, const float *__restrict__ qblk, const float *__restrict__ kblk,
    const float *__restrict__ scores_in, const float *__restrict__ tau,
    const unsigned char *__restrict__ refresh, int n_always_kv, int n_dense_q, int min_keep,
    unsigned char *__restrict__ mask, int *__restrict__ kept_idx, int *__restrict__ kept_count,
    float *__restrict__ scores_out) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  constexpr int NBP = 64 * CMAX;
  double *sQ = reinterpret_cast<double *>(smem_raw);                       // [kRows][D]
  float *sP = reinterpret_cast<float *>(smem_raw + (size_t)kRows * D * 8);  // [kRows][NBP]

  const int groups = (Nb + kRows - 1) / kRows;
  const long long bh = blockIdx.x / groups;
  const int i0 = (int)(blockIdx.x % groups) * kRows;
  const int h = (int)(bh % H);
  if (refresh && !refresh[bh]) return;  // reused head: cached mask persists

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  if (!scores_in) {
    // ---- Phase A: logits -------------------------------------------------------
    for (int e = threadIdx.x; e < kRows * D; e += 256) {
      int r = e / D, d = e % D;
      int i = i0 + r;
      sQ[e] = i < Nb ? (double)qblk[((size_t)bh * Nb + i) * D + d] : 0.0;
    }
    __syncthreads();
    const double inv_sqrt_d = 1.0 / sqrt((double)D);
    for (int j = threadIdx.x; j < Nb; j += 256) {
      double acc[kRows];
#pragma unroll
      for (int r = 0; r < kRows; ++r) acc[r] = 0.0;
      const float4 *kp = reinterpret_cast<const float4 *>(kblk + ((size_t)bh * Nb + j) * D);
      for (int d4 = 0; d4 < D / 4; ++d4) {
        float4 kv = kp[d4];
        double k0 = kv.x, k1 = kv.y, k2 = kv.z, k3 = kv.w;
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
          const double *qr = sQ + r * D + d4 * 4;
          acc[r] = fma(k0, qr[0], acc[r]);
          acc[r] = fma(k1, qr[1], acc[r]);
          acc[r] = fma(k2, qr[2], acc[r]);
          acc[r] = fma(k3, qr[3], acc[r]);
        }
      }
#pragma unroll
      for (int r = 0; r < kRows; ++r) sP[r * NBP + j] = (float)(acc[r] * inv_sqrt_d);
    }
    __syncthreads();
  }

  const float tau_h = tau[h];
  const unsigned long long lt_mask = (1ull << lane) - 1ull;

  for (int r = wave; r < kRows; r += 4) {
    const int i = i0 + r;
    if (i >= Nb) break;  // wave-uniform
    const size_t row = (size_t)bh * Nb + i;

    float p[CMAX];
    if (scores_in) {
#pragma unroll
      for (int c = 0; c < CMAX; ++c) {
        int j = lane + 64 * c;
        p[c] = j < Nb ? scores_in[row * Nb + j] : 0.f;
      }
    } else {
      // ---- Phase B: softmax of the row ------------------------------------------
      float m = -__builtin_inff();
#pragma unroll
      for (int c = 0; c < CMAX; ++c) {
        int j = lane + 64 * c;
        p[c] = j < Nb ? sP[r * NBP + j] : -__builtin_inff();
        m = fmaxf(m, p[c]);
      }
      m = wave_max_f32(m);
      float z = 0.f;
#pragma unroll
      for (int c = 0; c < CMAX; ++c) {
        int j = lane + 64 * c;
        p[c] = j < Nb ? expf(p[c] - m) : 0.f;
        z += p[c];
      }
      z = wave_sum_f32(z);
#pragma unroll
      for (int c = 0; c < CMAX; ++c) p[c] = __fdiv_rn(p[c], z);
    }
    if (scores_out) {
#pragma unroll
      for (int c = 0; c < CMAX; ++c) {
        int j = lane + 64 * c;
        if (j < Nb) scores_out[row * Nb + j] = p[c];
      }
    }

    // ---- Phase C: top-p selection ------------------------------------------------
    uint32_t e[CMAX], u[CMAX];
    unsigned long long my_u = 0;
#pragma unroll
    for (int c = 0; c < CMAX; ++c) {
      int j = lane + 64 * c;
      float pc = (j < Nb && p[c] > 0.f) ? p[c] : 0.f;
      e[c] = __float_as_uint(pc);
      u[c] = (uint32_t)floorf(pc * 1073741824.0f);  // exact: power-of-two scaling
      my_u += u[c];
    }
    const unsigned long long U = wave_sum_u64(my_u);
    const bool keep_all = tau_h >= 1.0f;
    uint32_t vf = 0;   // threshold bit pattern
    int cf = 0;        // number of lowest-index ties at vf to keep
    if (!keep_all) {
      const unsigned long long T =
          tau_h > 0.f ? (unsigned long long)floorf(tau_h * 16777216.0f) : 0ull;
      const unsigned long long need = (T * U + 16777215ull) >> 24;
      uint32_t v = 0;
      for (int bit = 30; bit >= 0; --bit) {
        const uint32_t cand = v | (1u << bit);
        unsigned long long s = 0;
#pragma unroll
        for (int c = 0; c < CMAX; ++c) s += e[c] >= cand ? u[c] : 0u;
        s = wave_sum_u64(s);
        if (s >= need) v = cand;
      }
      unsigned long long s_gt = 0;
      int n_gt = 0;
#pragma unroll
      for (int c = 0; c < CMAX; ++c) {
        bool gt = e[c] > v;
        s_gt += gt ? u[c] : 0u;
        n_gt += gt ? 1 : 0;
      }
      s_gt = wave_sum_u64(s_gt);
      n_gt = wave_sum_i32(n_gt);
      int c_m = 0;
      if (need > s_gt) {
        const unsigned long long ustar =
            (unsigned long long)floorf(__uint_as_float(v) * 1073741824.0f);
        c_m = (int)((need - s_gt + ustar - 1ull) / ustar);
      }
      int k_mass = n_gt + c_m;
      int k_min = min(max(1, min_keep), Nb);
      vf = v;
      cf = c_m;
      if (k_mass < k_min) {
        // the floor on the number of kept blocks wins: take the k_min best-ranked
        uint32_t v2 = 0;
        for (int bit = 30; bit >= 0; --bit) {
          const uint32_t cand = v2 | (1u << bit);
          int cnt = 0;
#pragma unroll
          for (int c = 0; c < CMAX; ++c) cnt += e[c] >= cand ? 1 : 0;
          cnt = wave_sum_i32(cnt);
          if (cnt >= k_min) v2 = cand;
        }
        int n_gt2 = 0;
#pragma unroll
        for (int c = 0; c < CMAX; ++c) n_gt2 += (lane + 64 * c < Nb && e[c] > v2) ? 1 : 0;
        n_gt2 = wave_sum_i32(n_gt2);
        vf = v2;
        cf = k_min - n_gt2;
      }
    }

    const bool dense_row = i < n_dense_q;
    int tie_run = 0, out_run = 0;
#pragma unroll
    for (int c = 0; c < CMAX; ++c) {
      const int j = lane + 64 * c;
      const bool valid = j < Nb;
      const bool tie = valid && e[c] == vf;
      const unsigned long long tb = __ballot(tie);
      const int tie_rank = tie_run + __popcll(tb & lt_mask);
      tie_run += __popcll(tb);
      bool keep = valid && (keep_all || dense_row || j < n_always_kv || e[c] > vf ||
                            (tie && tie_rank < cf));
      const unsigned long long kb = __ballot(keep);
      const int pos = out_run + __popcll(kb & lt_mask);
      out_run += __popcll(kb);
      if (valid) mask[row * Nb + j] = keep ? 1 : 0;
      if (keep) kept_idx[row * Nb + pos] = j;
    }
    if (lane == 0) kept_count[row] = out_run;
  }
}

template <int CMAX>
static int launch_cmax(int B, int H, int Nb, int D, const float *qblk, const float *kblk,
                       const float *scores_in, const float *tau, const unsigned char *refresh,
                       int n_always_kv, int n_dense_q, int min_keep, unsigned char *mask,
                       int *kept_idx, int *kept_count, float *scores_out, hipStream_t st) {
  int groups = (Nb + kRows - 1) / kRows;
  size_t lds = scores_in ? 0 : (size_t)kRows * D * 8 + (size_t)kRows * 64 * CMAX * 4;
  long long nwg = (long long)B * H * groups;
  hipLaunchKernelGGL(mask_topp_kernel<CMAX>, dim3((unsigned)nwg), dim3(256), lds, st, H, Nb, D,
                     qblk, kblk, scores_in, tau, refresh, n_always_kv, n_dense_q, min_keep, mask,
                     kept_idx, kept_count, scores_out);
  return check_launch("mask_topp_kernel");
}

int launch_mask_topp(int B, int H, int Nb, int D, const float *qblk, const float *kblk,
                     const float *scores_in, const float *tau, const unsigned char *refresh,
                     int n_always_kv, int n_dense_q, int min_keep, unsigned char *mask,
                     int *kept_idx, int *kept_count, float *scores_out, hipStream_t st) {
#define HEART_TOPP_ARGS                                                                       \
  B, H, Nb, D, qblk, kblk, scores_in, tau, refresh, n_always_kv, n_dense_q, min_keep, mask,   \
      kept_idx, kept_count, scores_out, st
  if (Nb <= 64) return launch_cmax<1>(HEART_TOPP_ARGS);
  if (Nb <= 256) return launch_cmax<4>(HEART_TOPP_ARGS);
  if (Nb <= 512) return launch_cmax<8>(HEART_TOPP_ARGS);
  return launch_cmax<16>(HEART_TOPP_ARGS);
#undef HEART_TOPP_ARGS
}

}  // namespace heart
