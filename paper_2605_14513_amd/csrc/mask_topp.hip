// heart_mask_topp: block importance from pooled Q/K blocks and top-p block selection
// with a per-head threshold (Sec. 3.2: rank candidate blocks by importance, keep
// them until the accumulated importance reaches tau; Eq. 1: the minimal such set;
// 1/sqrt(D) interaction scale from the appendix on query-key stability).
//
// One workgroup (8 wavefronts) owns R = 16 query-block rows of one head.
//   Phase A  logits[r][j] = qblk_r . kblk_j / sqrt(D) on the fp64 matrix cores
//            (v_mfma_f64_16x16x4_f64: a 16 x 16 tile of logits per wavefront, the
//            contraction over d in steps of 4; fp64 takes the dot product out of the
//            error budget of the scores).  The contraction order over d is free, so
//            lane group g = lane / 16 takes the d range [g D/4, (g+1) D/4): a lane then
//            reads D/4 consecutive floats of one block mean (16-byte loads straight from
//            global memory, no LDS staging) and converts them to fp64 on the way in.
//            The 16 query rows sit in LDS as fp64; the key blocks of the next tile are
//            in flight while the current tile is multiplied.
//            With a caller workspace (kInt8) the same dot products run on the int8 matrix
//            cores instead, which are 6 times faster per tile than the fp64 ones: a small
//            kernel first writes every block mean as an exponent and four signed 8-bit
//            slices (slice_blocks_kernel), products of slices and their sums over d are
//            exact integers (v_mfma_i32_16x16x64_i8), and the slice pairs are put together
//            in fp64.
//   Phase B  row softmax, fp32 with the accurate expf: half a wavefront per row (two rows at
//            a time) when the scores are the kernel's own, one wavefront per row for scores
//            passed in.
//   Phase C  top-p selection, same lanes as phase B, without sorting: the kept set
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

constexpr int kRows = 16;      // query-block rows per workgroup (one MFMA tile high)
constexpr int kMaxF4 = 8;      // float4 per lane and tile at D = 128 (D/16)
constexpr int kWaves = 8;      // wavefronts per workgroup: two rows each per selection pass
typedef __attribute__((ext_vector_type(4))) double f64x4_t;
typedef __attribute__((ext_vector_type(4))) int i32x4_t;

// ---- exact 8-bit slices of the block means ------------------------------------------------
// A block mean x[D] (fp32) becomes an exponent E with |x_d| < 2^E for every d and the
// integers m_d = round(x_d 2^(30-E)), |m_d| <= 2^30, each written as four signed bytes
//   m = b0 2^24 + b1 2^16 + b2 2^8 + b3,   b1..b3 in [-128, 127], b0 in [-64, 64]
// (balanced digits, so that every slice fits the int8 operands of the matrix cores).  The
// rounding moves x_d by at most 2^(E-31), i.e. 2^-31 of the largest entry of its block: far
// inside the 1e-5 budget of the scores (fp32 block means carry 2^-24 themselves).
// Layout: slices [vector][slice t = 0 (b0) .. 3][D] bytes, exponents [vector]; vector =
// (b*H + h) * Nb + block.  Not finite inputs give unspecified (but defined) slices.
constexpr int kSliceThreads = 256;
template <int D>
__global__ __launch_bounds__(kSliceThreads) void slice_blocks_kernel(
    long long n_vec, int Nb, const float *__restrict__ qblk, const float *__restrict__ kblk,
    const unsigned char *__restrict__ refresh, signed char *__restrict__ qs,
    signed char *__restrict__ ks, int *__restrict__ qe, int *__restrict__ ke) {
  constexpr int LPV = D / 4;                   // lanes per vector (a float4 each)
  constexpr int VPW = kSliceThreads / LPV;     // vectors per workgroup
  const int lv = threadIdx.x % LPV;
  const long long vid2 = (long long)blockIdx.x * VPW + threadIdx.x / LPV;  // over q then k
  const bool is_k = vid2 >= n_vec;
  const long long vid = is_k ? vid2 - n_vec : vid2;
  // (lanes of a vector share one wavefront and take the same branch)
  if (vid >= n_vec) return;
  if (refresh && !refresh[vid / Nb]) return;  // reused head: its scores are not computed
  const float4 x = reinterpret_cast<const float4 *>((is_k ? kblk : qblk) + vid * D)[lv];
  float amax = fmaxf(fmaxf(fabsf(x.x), fabsf(x.y)), fmaxf(fabsf(x.z), fabsf(x.w)));
#pragma unroll
  for (int d = 1; d < LPV; d <<= 1) amax = fmaxf(amax, __shfl_xor(amax, d, 64));
  // |x| < 2^E: E = biased exponent - 126 (zeros and denormals: the smallest normal binade)
  const int be = (int)((__float_as_uint(amax) >> 23) & 0xffu);
  const int E = (be > 0 ? be : 1) - 126;
  const float lim = 1073741824.0f;  // 2^30
  const float xs[4] = {x.x, x.y, x.z, x.w};
  uint32_t word[4] = {0u, 0u, 0u, 0u};  // word[t]: slice t of this lane's four d
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float scaled = fminf(fmaxf(rintf(ldexpf(xs[e], 30 - E)), -lim), lim);
    int m = (int)scaled;
#pragma unroll
    for (int t = 3; t >= 0; --t) {
      const int bt = t > 0 ? (int)(signed char)(m & 0xff) : m;  // low byte, signed; the rest for b0
      m = (m - bt) >> 8;
      word[t] |= ((uint32_t)bt & 0xffu) << (8 * e);
    }
  }
  uint32_t *dst = reinterpret_cast<uint32_t *>((is_k ? ks : qs) + vid * 4 * D);
#pragma unroll
  for (int t = 0; t < 4; ++t) dst[t * (D / 4) + lv] = word[t];
  if (lv == 0) (is_k ? ke : qe)[vid] = E;
}

// CMAX: slots per lane; handles Nb <= 64 * CMAX.  NF4T: D / 16 when known at compile time
// (4 or 8), else 0: with it the contraction loop is branch-free, so that the loads of the next
// tile stay in flight under the matrix instructions of the current one.
// kInt8: the score stage reads the slices written by slice_blocks_kernel (NF4T = 4 or 8 only).
struct BlockSlices {
  const signed char *qs, *ks;  // [B*H*Nb][4][D]
  const int *qe, *ke;          // [B*H*Nb]
};
template <int CMAX, int NF4T, bool kInt8>
__global__ __launch_bounds__(64 * kWaves, 4) void mask_topp_kernel(
    int H, int Nb, int D, const float *__restrict__ qblk, const float *__restrict__ kblk,
    const float *__restrict__ scores_in, const float *__restrict__ tau,
    const unsigned char *__restrict__ refresh, int n_always_kv, int n_dense_q, int min_keep,
    unsigned char *__restrict__ mask, int *__restrict__ kept_idx, int *__restrict__ kept_count,
    float *__restrict__ scores_out, BlockSlices sl) {
  static_assert(!kInt8 || NF4T == 4 || NF4T == 8, "slices: D = 64 or 128");
  extern __shared__ __align__(16) unsigned char smem_raw[];
  constexpr int NBP = 64 * CMAX;
  float *sP = reinterpret_cast<float *>(smem_raw);  // [kRows][NBP] logits of the rows
  double *sQ = reinterpret_cast<double *>(smem_raw + (size_t)kRows * NBP * 4);  // [kRows][D + 2]

  if (NF4T) D = 16 * NF4T;  // (a compile-time constant from here on)
  const int groups = (Nb + kRows - 1) / kRows;
  const long long bh = blockIdx.x / groups;
  const int i0 = (int)(blockIdx.x % groups) * kRows;
  const int h = (int)(bh % H);
  if (refresh && !refresh[bh]) return;  // reused head: cached mask persists

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  if constexpr (kInt8) {
    // ---- Phase A on the int8 matrix cores (launched only without scores_in) -------- -----------------------------------------
    // v_mfma_i32_16x16x64_i8: A lane L = (row L%16, 16 bytes of k-group L/16), B lane L =
    // (16 bytes of k-group L/16, column L%16), D lane L register r = (row 4*(L/16) + r,
    // column L%16).  Both operands use the same assignment of d to (k-group, byte): group g
    // holds d = 64 c + 16 g .. + 15 of chunk c.  Slice pairs (ta, tb) carry the weight
    // 2^(48 - 8 (ta + tb)); pairs of equal weight share an accumulator, and the pairs with
    // ta + tb > 3 (weights 2^16 and below against sums of up to 2^69: 2^-23 of the product of
    // the two blocks' largest entries at worst) are left out.
    constexpr int DD = 16 * NF4T, NC = DD / 64;
    const int n16 = lane & 15, g = lane >> 4;
    const size_t vec0 = (size_t)bh * Nb;
    i32x4_t aq[4][NC];
    {
      const int qi = min(i0 + n16, Nb - 1);
      const i32x4_t *qp = reinterpret_cast<const i32x4_t *>(sl.qs + (vec0 + qi) * 4 * DD);
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int c = 0; c < NC; ++c) aq[t][c] = qp[t * (DD / 16) + 4 * c + g];
    }
    int eq[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) eq[r] = sl.qe[vec0 + min(i0 + 4 * g + r, Nb - 1)];
    // (columns past Nb read the last key block instead of branching; their logits are not
    // stored)
    auto load_tile = [&](i32x4_t (&dst)[4][NC], int &ek, int tile) {
      const int j = min(tile * 16 + n16, Nb - 1);
      const i32x4_t *kp = reinterpret_cast<const i32x4_t *>(sl.ks + (vec0 + j) * 4 * DD);
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int c = 0; c < NC; ++c) dst[t][c] = kp[t * (DD / 16) + 4 * c + g];
      ek = sl.ke[vec0 + j];
    };
    const double inv_sqrt_d = 1.0 / sqrt((double)DD);
    const int ntiles = (Nb + 15) / 16;
    i32x4_t kc[4][NC], kn[4][NC];
    int ekc = 0, ekn = 0;
    if (wave < ntiles) load_tile(kc, ekc, wave);
    for (int tile = wave; tile < ntiles; tile += kWaves) {
      if (tile + kWaves < ntiles) load_tile(kn, ekn, tile + kWaves);
      i32x4_t acc[4];
#pragma unroll
      for (int w = 0; w < 4; ++w) acc[w] = i32x4_t{0, 0, 0, 0};
#pragma unroll
      for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int ta = 0; ta < 4; ++ta)
#pragma unroll
          for (int w = ta; w < 4; ++w)  // (accumulators in turn: few back-to-back dependent pairs)
            acc[w] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aq[ta][c], kc[w - ta][c], acc[w], 0, 0, 0);
      const int j = tile * 16 + n16;
      if (j < Nb) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          // exact in fp64: every accumulator is below 2^24 in magnitude
          const double v = (((double)acc[0][r] * 256.0 + (double)acc[1][r]) * 256.0 + (double)acc[2][r]) * 256.0 +
                           (double)acc[3][r];
          // v * 2^24 * 2^(Eq - 30) * 2^(Ek - 30)
          sP[(4 * g + r) * NBP + j] = (float)(ldexp(v, eq[r] + ekc - 36) * inv_sqrt_d);
        }
      }
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int c = 0; c < NC; ++c) kc[t][c] = kn[t][c];
      ekc = ekn;
    }
    __syncthreads();
  } else if (!scores_in) {
    // ---- Phase A: logits -------------------------------------------------------
    // MFMA operand layout (16x16x4 fp64): A lane L = (row L%16, k L/16), B lane L =
    // (k L/16, column L%16), D lane L register r = (row L/16 + 4 r, column L%16).
    const int n16 = lane & 15, g = lane >> 4;
    const int nf4 = NF4T ? NF4T : D / 16;  // float4 per lane: its D/4 consecutive d values
    const float4 *qg = reinterpret_cast<const float4 *>(qblk + (size_t)bh * Nb * D);
    const float4 *kg = reinterpret_cast<const float4 *>(kblk + (size_t)bh * Nb * D);
    const int SQ = D + 2;
    const double *qrow = sQ + n16 * SQ + g * (D / 4);  // this lane's A operands, step by step
    // (columns past Nb read the last key block instead of branching; their logits are not
    // stored)
    auto load_tile = [&](float4 (&dst)[kMaxF4], int tile) {
      const int j = min(tile * 16 + n16, Nb - 1);
#pragma unroll
      for (int u = 0; u < kMaxF4; ++u) {
        if (u < nf4)
          dst[u] = kg[(size_t)j * (D / 4) + g * nf4 + u];
        else
          dst[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      }
    };
    const double inv_sqrt_d = 1.0 / sqrt((double)D);
    const int ntiles = (Nb + 15) / 16;
    float4 kc[kMaxF4], kn[kMaxF4];
    // the 16 query rows as fp64 in LDS (row stride D + 2 doubles: the 16 rows a quarter of
    // the lanes reads fall into distinct banks); keeping them there rather than in 64
    // registers lets more wavefronts share a SIMD, which the latency-bound selection needs
    for (int e = threadIdx.x; e < kRows * (D / 4); e += 64 * kWaves) {
      const int r = e / (D / 4), d4 = e % (D / 4);
      float4 t4 = make_float4(0.f, 0.f, 0.f, 0.f);
      if (i0 + r < Nb) t4 = qg[(size_t)(i0 + r) * (D / 4) + d4];
      double *dst = sQ + r * SQ + d4 * 4;
      dst[0] = (double)t4.x;
      dst[1] = (double)t4.y;
      dst[2] = (double)t4.z;
      dst[3] = (double)t4.w;
    }
    __syncthreads();
    if (wave < ntiles) load_tile(kc, wave);
    for (int tile = wave; tile < ntiles; tile += kWaves) {
      // (compiler barrier: the query operands are re-read from LDS for every tile; hoisted out
      // of the loop they would cost 64 registers and a wavefront per SIMD)
      asm volatile("" ::: "memory");
      if (tile + kWaves < ntiles) load_tile(kn, tile + kWaves);
      f64x4_t acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int u = 0; u < kMaxF4; ++u) {
        if (u < nf4) {  // uniform
          acc = __builtin_amdgcn_mfma_f64_16x16x4f64(qrow[4 * u + 0], (double)kc[u].x, acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f64_16x16x4f64(qrow[4 * u + 1], (double)kc[u].y, acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f64_16x16x4f64(qrow[4 * u + 2], (double)kc[u].z, acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f64_16x16x4f64(qrow[4 * u + 3], (double)kc[u].w, acc, 0, 0, 0);
        }
      }
      const int j = tile * 16 + n16;
      if (j < Nb) {
#pragma unroll
        for (int r = 0; r < 4; ++r) sP[(g + 4 * r) * NBP + j] = (float)(acc[r] * inv_sqrt_d);
      }
#pragma unroll
      for (int u = 0; u < kMaxF4; ++u) kc[u] = kn[u];
    }
    __syncthreads();
  }

  const float tau_h = tau[h];
  const unsigned long long lt_mask = (1ull << lane) - 1ull;

  if (!scores_in) {
    // ---- Phases B and C, two rows per wavefront (scores from phase A) ----------------------
    // Each half of the wavefront (32 lanes) owns one row: the selection is bound by the
    // number of vector instructions, and with 32 lanes per row every search step serves two
    // rows and its reductions take five exchanges instead of six.  The scores of a row sum to
    // one, so every partial sum of the fixed-point masses stays below 2^31: the mass
    // arithmetic is 32-bit here (same integers as in the general path below, hence the same
    // kept sets).  The per-row state (v, top, counts) is replicated over the lanes of a half.
    constexpr int EPL = 2 * CMAX;  // elements per lane: element c is key block l32 + 32 c
    const int l32 = lane & 31, hfw = lane >> 5;
    const uint32_t lt32 = (1u << l32) - 1u;
    static_assert(kRows % (2 * kWaves) == 0, "rows per selection pass");
    for (int rp = 0; rp < kRows / (2 * kWaves); ++rp) {
    const int r = 2 * (wave + rp * kWaves) + hfw;
    const int i = i0 + r;
    const bool row_ok = i < Nb;
    const size_t row = (size_t)bh * Nb + (row_ok ? i : 0);
    float p[EPL];
    {
      float m = -__builtin_inff();
#pragma unroll
      for (int c = 0; c < EPL; ++c) {
        const int j = l32 + 32 * c;
        p[c] = (row_ok && j < Nb) ? sP[r * NBP + j] : -__builtin_inff();
        m = fmaxf(m, p[c]);
      }
      m = half_max_f32(m);
      if (!row_ok) m = 0.f;
      float z = 0.f;
#pragma unroll
      for (int c = 0; c < EPL; ++c) {
        const int j = l32 + 32 * c;
        p[c] = (row_ok && j < Nb) ? expf(p[c] - m) : 0.f;
        z += p[c];
      }
      z = half_sum_f32(z);
      if (!row_ok) z = 1.f;
#pragma unroll
      for (int c = 0; c < EPL; ++c) p[c] = __fdiv_rn(p[c], z);
    }
    if (scores_out && row_ok) {
#pragma unroll
      for (int c = 0; c < EPL; ++c) {
        const int j = l32 + 32 * c;
        if (j < Nb) scores_out[row * Nb + j] = p[c];
      }
    }
    uint32_t e[EPL], u[EPL];
    uint32_t my_u = 0;
#pragma unroll
    for (int c = 0; c < EPL; ++c) {
      const int j = l32 + 32 * c;
      const float pc = (j < Nb && p[c] > 0.f) ? p[c] : 0.f;
      e[c] = __float_as_uint(pc);
      u[c] = (uint32_t)floorf(pc * 1073741824.0f);
      my_u += u[c];
    }
    const uint32_t U = half_sum_u32(my_u);
    const bool keep_all = tau_h >= 1.0f;  // (uniform: one head per workgroup)
    uint32_t vf = 0;
    int cf = 0;
    if (!keep_all) {
      const unsigned long long T =
          tau_h > 0.f ? (unsigned long long)floorf(tau_h * 16777216.0f) : 0ull;
      const uint32_t need = (uint32_t)((T * (unsigned long long)U + 16777215ull) >> 24);
      // The same bitwise search as in the general path, shortened at the top: a score that
      // carries mass is at least 2^-30, so mass(>= 2^-31) is the whole row (>= need) and bits
      // 30..28 of the threshold are known (011); the exponent bits 27..23 are probed on masses
      // alone (a binade holds many scores, the early exit below never fires there); from bit 22
      // on the count of undecided scores is kept incrementally: n_v = #(scores >= v),
      // n_top = #(scores >= top).
      uint32_t v = need == 0 ? 0x7fffffffu : 0x30000000u;
      bool active = need != 0;
      for (int bit = 27; bit >= 23; --bit) {
        if (!__any(active)) break;
        const uint32_t cand = v | (1u << bit);
        uint32_t s = 0;
#pragma unroll
        for (int c = 0; c < EPL; ++c) s += e[c] >= cand ? u[c] : 0u;
        s = half_sum_u32(s);
        if (active && s >= need) v = cand;
      }
      uint32_t n_v = 0, n_top = 0;
      {
        const uint32_t top = v + (1u << 23);
#pragma unroll
        for (int c = 0; c < EPL; ++c) {
          n_v += e[c] >= v ? 1u : 0u;
          n_top += e[c] >= top ? 1u : 0u;
        }
        n_v = half_sum_u32(n_v);
        n_top = half_sum_u32(n_top);
      }
      for (int bit = 22; bit >= 0; --bit) {
        if (!__any(active)) break;
        const uint32_t cand = v | (1u << bit);
        uint32_t s = 0, cn = 0;
#pragma unroll
        for (int c = 0; c < EPL; ++c) {
          const bool ge = e[c] >= cand;
          s += ge ? u[c] : 0u;
          cn += ge ? 1u : 0u;
        }
        s = half_sum_u32(s);
        cn = half_sum_u32(cn);
        if (active) {
          if (s >= need) {
            v = cand;
            n_v = cn;
          } else {
            n_top = cn;
          }
        }
        const bool single = active && (n_v - n_top == 1u);
        if (__any(single)) {
          // the one undecided score of such a row is its threshold
          const uint32_t top = v + (1u << bit);
          uint32_t x = 0;
#pragma unroll
          for (int c = 0; c < EPL; ++c) x = (e[c] >= v && e[c] < top && e[c] > x) ? e[c] : x;
          x = half_max_u32(x);
          if (single) {
            v = x > v ? x : v;
            active = false;
          }
        }
      }
      uint32_t s_gt = 0, n_gt = 0;
#pragma unroll
      for (int c = 0; c < EPL; ++c) {
        const bool gt = e[c] > v;
        s_gt += gt ? u[c] : 0u;
        n_gt += gt ? 1u : 0u;
      }
      s_gt = half_sum_u32(s_gt);
      n_gt = half_sum_u32(n_gt);
      uint32_t c_m = 0;
      if (need > s_gt) {
        const uint32_t ustar = (uint32_t)floorf(__uint_as_float(v) * 1073741824.0f);
        c_m = (need - s_gt + ustar - 1u) / (ustar > 0u ? ustar : 1u);
      }
      const int k_mass = (int)(n_gt + c_m);
      const int k_min = min(max(1, min_keep), Nb);
      vf = v;
      cf = (int)c_m;
      const bool floor_wins = k_mass < k_min;
      if (__any(floor_wins)) {
        // the floor on the number of kept blocks: the k_min best-ranked of such a row
        uint32_t v2 = 0;
        for (int bit = 30; bit >= 0; --bit) {
          const uint32_t cand = v2 | (1u << bit);
          uint32_t cn = 0;
#pragma unroll
          for (int c = 0; c < EPL; ++c) cn += e[c] >= cand ? 1u : 0u;
          cn = half_sum_u32(cn);
          if ((int)cn >= k_min) v2 = cand;
        }
        uint32_t n_gt2 = 0;
#pragma unroll
        for (int c = 0; c < EPL; ++c) n_gt2 += (l32 + 32 * c < Nb && e[c] > v2) ? 1u : 0u;
        n_gt2 = half_sum_u32(n_gt2);
        if (floor_wins) {
          vf = v2;
          cf = k_min - (int)n_gt2;
        }
      }
    }
    const bool dense_row = i < n_dense_q;
    int tie_run = 0, out_run = 0;
#pragma unroll
    for (int c = 0; c < EPL; ++c) {
      const int j = l32 + 32 * c;
      const bool valid = row_ok && j < Nb;
      const bool tie = valid && e[c] == vf;
      const unsigned long long tb = __ballot(tie);
      const uint32_t tbh = hfw ? (uint32_t)(tb >> 32) : (uint32_t)tb;
      const int tie_rank = tie_run + __popc(tbh & lt32);
      tie_run += __popc(tbh);
      const bool keep = valid && (keep_all || dense_row || j < n_always_kv || e[c] > vf ||
                                  (tie && tie_rank < cf));
      const unsigned long long kb = __ballot(keep);
      const uint32_t kbh = hfw ? (uint32_t)(kb >> 32) : (uint32_t)kb;
      const int pos = out_run + __popc(kbh & lt32);
      out_run += __popc(kbh);
      if (valid) mask[row * Nb + j] = keep ? 1 : 0;
      if (keep) kept_idx[row * Nb + pos] = j;
    }
    if (l32 == 0 && row_ok) kept_count[row] = out_run;
    }  // selection passes
    return;
  }

  for (int r = wave; r < kRows; r += kWaves) {
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
      // (scores handed in may be anything: negative values and NaN count as 0, values above
      // 1 as 1, so the fixed-point conversion below cannot overflow)
      float pc = (j < Nb && p[c] > 0.f) ? fminf(p[c], 1.0f) : 0.f;
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
      // (a score that carries mass is at least 2^-30 and none exceeds 1, so bits 30..28 of the
      // threshold are known: 011)
      uint32_t v = need == 0 ? 0x7fffffffu : 0x30000000u;
      for (int bit = 27; bit >= 0 && need != 0; --bit) {
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

template <int CMAX, int NF4T, bool kInt8>
static int launch_cmax_d(int B, int H, int Nb, int D, const float *qblk, const float *kblk,
                       const float *scores_in, const float *tau, const unsigned char *refresh,
                       int n_always_kv, int n_dense_q, int min_keep, unsigned char *mask,
                       int *kept_idx, int *kept_count, float *scores_out, const BlockSlices &sl,
                       hipStream_t st) {
  int groups = (Nb + kRows - 1) / kRows;
  // logits of the row group; the fp64 score stage also keeps its query rows there
  size_t lds = scores_in ? 0 : (size_t)kRows * 64 * CMAX * 4 + (kInt8 ? 0 : (size_t)kRows * (D + 2) * 8);
  long long nwg = (long long)B * H * groups;
  auto kern = mask_topp_kernel<CMAX, NF4T, kInt8>;
  if (lds > 64 * 1024) {
    const int dev = current_device();
    if (dev < 0) return fail(HEART_EHIP, "heart_mask_topp: cannot identify the current device");
    static DeviceFlags attr_set;  // per instantiation: the attribute is per function and device
    if (hipError_t e = set_max_lds_once(attr_set, dev, reinterpret_cast<const void *>(kern), 96 * 1024))
      return fail(HEART_EHIP, "hipFuncSetAttribute(mask kernel LDS): %s", hipGetErrorString(e));
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(64 * kWaves), lds, st, H, Nb, D, qblk, kblk,
                     scores_in, tau, refresh, n_always_kv, n_dense_q, min_keep, mask, kept_idx,
                     kept_count, scores_out, sl);
  return check_launch("mask_topp_kernel");
}

template <int D>
static int launch_slices(int B, int H, int Nb, const float *qblk, const float *kblk,
                         const unsigned char *refresh, signed char *qs, signed char *ks, int *qe,
                         int *ke, hipStream_t st) {
  const long long n_vec = (long long)B * H * Nb;
  constexpr int VPW = kSliceThreads / (D / 4);
  const long long nwg = (2 * n_vec + VPW - 1) / VPW;
  if (nwg > 0x7fffffffLL) return fail(HEART_EUNSUPPORTED, "heart_mask_topp: too many blocks to slice");
  hipLaunchKernelGGL(slice_blocks_kernel<D>, dim3((unsigned)nwg), dim3(kSliceThreads), 0, st, n_vec, Nb,
                     qblk, kblk, refresh, qs, ks, qe, ke);
  return check_launch("slice_blocks_kernel");
}

size_t mask_topp_workspace_bytes(int B, int H, int Nb, int D) {
  // slices of Q and K blocks (4 D bytes each) and their exponents
  return (size_t)B * H * Nb * (2 * (size_t)4 * D + 2 * sizeof(int));
}

template <int CMAX>
static int launch_cmax(int B, int H, int Nb, int D, const float *qblk, const float *kblk,
                       const float *scores_in, const float *tau, const unsigned char *refresh,
                       int n_always_kv, int n_dense_q, int min_keep, unsigned char *mask,
                       int *kept_idx, int *kept_count, float *scores_out, void *workspace,
                       hipStream_t st) {
#define HEART_TOPP_D_ARGS                                                                     \
  B, H, Nb, D, qblk, kblk, scores_in, tau, refresh, n_always_kv, n_dense_q, min_keep, mask,   \
      kept_idx, kept_count, scores_out
  BlockSlices none{nullptr, nullptr, nullptr, nullptr};
  if (!scores_in && workspace && (D == 128 || D == 64)) {
    // score stage on the int8 matrix cores: slices first (one small launch), then the kernel
    const size_t n_vec = (size_t)B * H * Nb;
    signed char *qs = static_cast<signed char *>(workspace);
    signed char *ks = qs + n_vec * 4 * D;
    int *qe = reinterpret_cast<int *>(ks + n_vec * 4 * D);
    int *ke = qe + n_vec;
    const BlockSlices sl{qs, ks, qe, ke};
    if (D == 128) {
      if (int rc = launch_slices<128>(B, H, Nb, qblk, kblk, refresh, qs, ks, qe, ke, st)) return rc;
      return launch_cmax_d<CMAX, 8, true>(HEART_TOPP_D_ARGS, sl, st);
    }
    if (int rc = launch_slices<64>(B, H, Nb, qblk, kblk, refresh, qs, ks, qe, ke, st)) return rc;
    return launch_cmax_d<CMAX, 4, true>(HEART_TOPP_D_ARGS, sl, st);
  }
  // the head dimensions of the attention kernels get a contraction loop of their own
  if (!scores_in && D == 128) return launch_cmax_d<CMAX, 8, false>(HEART_TOPP_D_ARGS, none, st);
  if (!scores_in && D == 64) return launch_cmax_d<CMAX, 4, false>(HEART_TOPP_D_ARGS, none, st);
  return launch_cmax_d<CMAX, 0, false>(HEART_TOPP_D_ARGS, none, st);
#undef HEART_TOPP_D_ARGS
}

int launch_mask_topp(int B, int H, int Nb, int D, const float *qblk, const float *kblk,
                     const float *scores_in, const float *tau, const unsigned char *refresh,
                     int n_always_kv, int n_dense_q, int min_keep, unsigned char *mask,
                     int *kept_idx, int *kept_count, float *scores_out, void *workspace,
                     hipStream_t st) {
#define HEART_TOPP_ARGS                                                                       \
  B, H, Nb, D, qblk, kblk, scores_in, tau, refresh, n_always_kv, n_dense_q, min_keep, mask,   \
      kept_idx, kept_count, scores_out, workspace, st
  // (lane slots in steps of 128 key blocks above 256: unused slots cost selection work)
  if (Nb <= 64) return launch_cmax<1>(HEART_TOPP_ARGS);
  if (Nb <= 256) return launch_cmax<4>(HEART_TOPP_ARGS);
  if (Nb <= 384) return launch_cmax<6>(HEART_TOPP_ARGS);
  if (Nb <= 512) return launch_cmax<8>(HEART_TOPP_ARGS);
  if (Nb <= 640) return launch_cmax<10>(HEART_TOPP_ARGS);
  if (Nb <= 768) return launch_cmax<12>(HEART_TOPP_ARGS);
  if (Nb <= 896) return launch_cmax<14>(HEART_TOPP_ARGS);
  return launch_cmax<16>(HEART_TOPP_ARGS);
#undef HEART_TOPP_ARGS
}

}  // namespace heart
