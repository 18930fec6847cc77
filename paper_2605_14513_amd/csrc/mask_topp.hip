// heart_mask_topp: block importance from pooled Q/K blocks and top-p block selection
// with a per-head threshold (Sec. 3.2: rank candidate blocks by importance, keep
// them until the accumulated importance reaches tau; Eq. 1: the minimal such set;
// 1/sqrt(D) interaction scale from the appendix on query-key stability).
//
// One workgroup (4 wavefronts) owns R = 8 query-block rows of one head.
//   Phase A  logits[r][j] = qblk_r . kblk_j / sqrt(D): the key blocks stream through
//            LDS in chunks of 32 columns (coalesced loads, next chunk in flight),
//            one (row, column) dot product per lane and chunk in fp64 fused
//            multiply-add (on this chip fp64 FMA issues at the rate of unpacked
//            fp32 FMA, and it takes the dot product out of the error budget of the
//            scores).  The R query rows sit in LDS as fp64.
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

constexpr int kRows = 8;       // query-block rows per workgroup
constexpr int kCols = 32;      // key-block columns staged through LDS at a time (kRows * kCols = 256 lanes)
constexpr int kMaxStage = 4;   // float4 per lane for one staged chunk at D = 128

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
  float *sKt = sP + kRows * NBP;                                            // [kCols][D + 4]

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
    // K blocks travel through LDS in chunks of kCols columns with coalesced 16-byte
    // loads (the next chunk is in flight in registers while this one is consumed);
    // thread (r, c) = (t / kCols, t % kCols) then owns one (query row, key column) dot
    // product per chunk.  Row stride D + 4 floats spreads the columns over the banks.
    const int D4 = D / 4;                      // float4 per K row
    const int per_thread = (kCols * D4 + 255) / 256;
    const int SKT = D + 4;
    const float4 *kg = reinterpret_cast<const float4 *>(kblk + (size_t)bh * Nb * D);
    float4 stage[kMaxStage];
    auto load_chunk = [&](int c0) {
#pragma unroll
      for (int u = 0; u < kMaxStage; ++u) {
        const int e = threadIdx.x + u * 256;
        const int col = e / D4, d4 = e % D4;
        stage[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (u < per_thread && col < kCols && c0 + col < Nb) stage[u] = kg[(size_t)(c0 + col) * D4 + d4];
      }
    };
    auto store_chunk = [&]() {
#pragma unroll
      for (int u = 0; u < kMaxStage; ++u) {
        const int e = threadIdx.x + u * 256;
        const int col = e / D4, d4 = e % D4;
        if (u < per_thread && col < kCols) *reinterpret_cast<float4 *>(sKt + col * SKT + d4 * 4) = stage[u];
      }
    };
    const double inv_sqrt_d = 1.0 / sqrt((double)D);
    const int c = threadIdx.x % kCols, r = threadIdx.x / kCols;
    load_chunk(0);
    for (int c0 = 0; c0 < Nb; c0 += kCols) {
      __syncthreads();  // previous chunk consumed (first pass: sQ written)
      store_chunk();
      __syncthreads();
      if (c0 + kCols < Nb) load_chunk(c0 + kCols);
      // four independent fp64 chains (a single one would be bound by FMA latency)
      double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
      const float *kr = sKt + c * SKT;
      const double *qr = sQ + r * D;
#pragma unroll 4
      for (int d4 = 0; d4 < D4; ++d4) {
        const float4 kv = *reinterpret_cast<const float4 *>(kr + d4 * 4);
        a0 = fma((double)kv.x, qr[d4 * 4 + 0], a0);
        a1 = fma((double)kv.y, qr[d4 * 4 + 1], a1);
        a2 = fma((double)kv.z, qr[d4 * 4 + 2], a2);
        a3 = fma((double)kv.w, qr[d4 * 4 + 3], a3);
      }
      const double acc = (a0 + a1) + (a2 + a3);
      if (c0 + c < Nb) sP[r * NBP + c0 + c] = (float)(acc * inv_sqrt_d);
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
      // v* = largest bit pattern v with mass(scores >= v) >= need, built from the top
      // bit down.  Invariant: mass(>= v) >= need > mass(>= v + 2^(bit+1)); the scores in
      // [v, v + 2^(bit+1)) are undecided.  As soon as a single score is undecided it IS
      // v* (keeping it reaches the mass, dropping it does not), so the loop stops early:
      // typically after about a dozen steps instead of 31.  need == 0 keeps nothing here.
      uint32_t v = need == 0 ? 0x7fffffffu : 0u;
      for (int bit = 30; bit >= 0 && need != 0; --bit) {
        const uint32_t cand = v | (1u << bit);
        unsigned long long s = 0;
#pragma unroll
        for (int c = 0; c < CMAX; ++c) s += e[c] >= cand ? u[c] : 0u;
        s = wave_sum_u64(s);
        if (s >= need) v = cand;
        // undecided scores: [v, v + 2^bit) after this step (wave ballots, scalar counts)
        const uint32_t top = v + (1u << bit);  // exclusive; bit patterns stay below 2^31
        int n_und = 0;
        uint32_t und = 0;
#pragma unroll
        for (int c = 0; c < CMAX; ++c) {
          const bool in = e[c] >= v && e[c] < top;
          n_und += __popcll(__ballot(in));
          und = in ? e[c] : und;
        }
        if (n_und == 1) {
          uint32_t x = und;  // the one lane that holds it has und != 0 unless it is 0
          HEART_WAVE_REDUCE(uint32_t, x, HEART_OP_UMAX);
          v = x > v ? x : v;
          break;
        }
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
  size_t lds = scores_in ? 0
                         : (size_t)kRows * D * 8 + (size_t)kRows * 64 * CMAX * 4 +
                               (size_t)kCols * (D + 4) * 4;
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
