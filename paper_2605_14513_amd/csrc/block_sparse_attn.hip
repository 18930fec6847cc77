// heart_block_sparse_attn: softmax attention over the tokens of the kept key blocks of
// each query block (the sparse attention that consumes the top-p block mask; logits
// scaled by 1/sqrt(D) as in the appendix on query-key stability).
//
// Work decomposition: one workgroup per (b, h, query block); wavefront w of the
// workgroup owns query rows 32w .. 32w+31 of the block and loops over the kept
// key blocks with an online softmax.  Both contractions run on the bf16 matrix
// cores with v_mfma_f32_32x32x16_bf16, fp32 accumulation.
//
// The kernel computes TRANSPOSED tiles so that no accumulator ever has to move
// between lanes:
//   S^T (keys x queries) = K (keys x d) . Q^T (d x queries)
//   O^T (d x queries)   += V^T (d x keys) . P^T (keys x queries)
// In the 32x32 accumulator layout a lane holds one column (= one query, lane%32)
// and 16 rows (8*(r/4) + 4*(lane/32) + r%4, r = 0..15).  So every softmax
// statistic (running max, running sum, rescale factor) of a query lives in the two
// lanes l and l^32 and is a per-lane scalar, and the exponentiated S^T registers
// are, unchanged, the B operand of the second contraction: a lane must supply 8
// keys of its query per MFMA, and any assignment of keys to the 8 slots is valid
// as long as the A operand (V^T) uses the same one.  The V^T fragments are read
// with that key order from LDS, where V is stored transposed.
//
// LDS: K tile [block][D+8] bf16 (16-byte fragment reads hit 16 distinct bank
// groups per 16 lanes) and V^T tile [D][block+4] bf16 (8-byte fragment reads of 32
// consecutive d rows hit all 64 banks once).  V is transposed in registers on its
// way from global memory (4 keys x 8 d per lane, byte permutes) and written with
// 8-byte stores whose lane->(d-group, key-group) mapping is bank-conflict free.
//
// Workgroup ids are remapped so that the query blocks of one head run on one XCD
// (ids are dealt round-robin to the 8 XCDs, each with its own L2): the kept K/V
// blocks of a head are then re-read from that XCD's L2 instead of from HBM.
#include "heart_internal.h"

namespace heart {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

// Native vector types (not the HIP struct wrappers): loads and stores of these are
// first-class values, so staging arrays of them always live in registers.
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

union Frag8 {
  u32x4_t u;
  bf16x8_t v;
  u32x2_t h[2];
};

__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
  f32x2_t f = {lo, hi};
  bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
  return __builtin_bit_cast(uint32_t, b);
}

// registers that carry one thread's share of a K or V tile from global memory to LDS
template <int n>
struct KStage {
  u32x4_t r[n];
};

constexpr int kNumXcd = 8;

template <int D, int BLK>
__global__ __launch_bounds__(BLK * 2, 2) void attn_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k,
    const uint16_t *__restrict__ v, uint16_t *__restrict__ out, long long qsb, long long qsh,
    long long qsn, long long ksb, long long ksh, long long ksn, long long vsb, long long vsh,
    long long vsn, long long osb, long long osh, long long osn, int H, int BH, int N, int Nb,
    const int *__restrict__ kept_idx, const int *__restrict__ kept_count, float scale_log2e,
    float *__restrict__ lse) {
  constexpr int NT = BLK * 2;       // threads
  constexpr int KT = BLK / 32;      // 32-key tiles per key block
  constexpr int DT = D / 32;        // 32-wide d tiles of the output
  constexpr int KS = D / 16;        // k-steps of the first contraction
  constexpr int SK = D + 8;         // LDS row stride of the K tile (elements)
  constexpr int SV = BLK + 4;       // LDS row stride of the V^T tile (elements)
  constexpr int CPR = D / 8;        // 16-byte chunks per token row
  constexpr int KCH = (BLK * CPR) / NT;  // K chunks per thread
  constexpr int VIT = D / 64;            // V sub-tiles (4 keys x 8 d) per thread
  constexpr int KTH = 2;                 // 32-key tiles per slice of the key block
  constexpr int NH = KT / KTH;           // slices per key block
  constexpr float kRescaleSlack = 8.f;   // log2 units the running reference may lag the max

  extern __shared__ __align__(16) unsigned char smem_raw[];
  uint16_t *sK = reinterpret_cast<uint16_t *>(smem_raw);  // [BLK][SK]; reused for the output
  uint16_t *sVT = sK + BLK * SK;                           // [D][SV]

  // ---- workgroup id -> (head, query block), XCD-aware ------------------------------
  int bh, qb;
  {
    const long long id = blockIdx.x;
    const int full = BH / kNumXcd;
    const long long slot = id / kNumXcd;
    const int xcd = (int)(id % kNumXcd);
    if (slot < (long long)full * Nb) {
      bh = (int)(slot / Nb) * kNumXcd + xcd;
      qb = (int)(slot % Nb);
    } else {
      const long long rem = id - (long long)full * kNumXcd * Nb;
      bh = full * kNumXcd + (int)(rem / Nb);
      qb = (int)(rem % Nb);
    }
  }
  const int b = bh / H, h = bh % H;
  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int l32 = lane & 31, hf = lane >> 5;

  const uint16_t *qbase = q + b * qsb + h * qsh;
  const uint16_t *kbase = k + b * ksb + h * ksh;
  const uint16_t *vbase = v + b * vsb + h * vsh;

  // per-thread constant parts of the staging addresses: K chunk `it` of this thread is
  // row k_r0 + it * (NT / CPR), column k_c; V sub-tile `it` is d-group v_dg, key-group
  // v_kg0 + it * V_KG_STEP (see the file header for why this mapping is conflict free)
  const int k_r0 = t / CPR, k_c = (t % CPR) * 8;
  constexpr int K_R_STEP = NT / CPR;
  const int v_dg = (t & 3) + 4 * ((t >> 5) % (D / 32));
  const int v_kg0 = ((t & 31) >> 2) + 8 * ((t >> 5) / (D / 32));
  constexpr int V_KG_STEP = 8 * ((NT / 32) / (D / 32));

  // Rows past the end of a ragged last block are loaded from the block's last real row
  // instead (always a valid address): their logits are masked to -inf and their
  // softmax weights are exactly 0, so the values never reach the output.
  auto load_k = [&](int kv0, int nvalid) -> KStage<KCH> {
    KStage<KCH> st;
#pragma unroll
    for (int it = 0; it < KCH; ++it) {
      const int r = min(k_r0 + it * K_R_STEP, nvalid - 1);
      st.r[it] = *reinterpret_cast<const u32x4_t *>(kbase + (long long)(kv0 + r) * ksn + k_c);
    }
    return st;
  };
  auto store_k = [&](const KStage<KCH> &st) {
    uint16_t *dst = sK + k_r0 * SK + k_c;
#pragma unroll
    for (int it = 0; it < KCH; ++it)
      *reinterpret_cast<u32x4_t *>(dst + it * K_R_STEP * SK) = st.r[it];
  };
  // V staging is done per 64-key slice `half` of the key block.  With VIT == NH a
  // thread's sub-tile `it` lies in slice `it`; with VIT == 1 its single sub-tile
  // lies in slice v_kg0 / KGH (uniform per wavefront).
  constexpr int KGH = 16;  // key groups (of 4 keys) per slice
  static_assert(VIT == NH || VIT == 1, "V staging layout");
  auto v_mine = [&](int it, int half) -> bool {
    return VIT == NH ? it == half : (v_kg0 / KGH) == half;
  };
  auto load_v = [&](int half, int kv0, int nvalid) -> KStage<4> {
    KStage<4> st;
#pragma unroll
    for (int e = 0; e < 4; ++e) st.r[e] = u32x4_t{0u, 0u, 0u, 0u};
#pragma unroll
    for (int it = 0; it < VIT; ++it)
      if (v_mine(it, half)) {
        const int kg = v_kg0 + it * V_KG_STEP;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = min(kg * 4 + e, nvalid - 1);
          st.r[e] = *reinterpret_cast<const u32x4_t *>(vbase + (long long)(kv0 + r) * vsn + v_dg * 8);
        }
      }
    return st;
  };
  auto store_vt = [&](const KStage<4> &vst, int half) {
    const u32x4_t *vreg = vst.r;
#pragma unroll
    for (int it = 0; it < VIT; ++it)
      if (v_mine(it, half)) {
        const uint32_t w[4][4] = {{vreg[0].x, vreg[0].y, vreg[0].z, vreg[0].w},
                                  {vreg[1].x, vreg[1].y, vreg[1].z, vreg[1].w},
                                  {vreg[2].x, vreg[2].y, vreg[2].z, vreg[2].w},
                                  {vreg[3].x, vreg[3].y, vreg[3].z, vreg[3].w}};
        uint16_t *dst = sVT + (v_dg * 8) * SV + (v_kg0 + it * V_KG_STEP) * 4;
#pragma unroll
        for (int wd = 0; wd < 4; ++wd) {
          // word wd of key e holds d = 2*wd (low half) and d = 2*wd+1 (high half)
          u32x2_t even, odd;
          even.x = __builtin_amdgcn_perm(w[1][wd], w[0][wd], 0x05040100u);  // lo16(k0) | lo16(k1)<<16
          even.y = __builtin_amdgcn_perm(w[3][wd], w[2][wd], 0x05040100u);
          odd.x = __builtin_amdgcn_perm(w[1][wd], w[0][wd], 0x07060302u);   // hi16(k0) | hi16(k1)<<16
          odd.y = __builtin_amdgcn_perm(w[3][wd], w[2][wd], 0x07060302u);
          *reinterpret_cast<u32x2_t *>(dst + (2 * wd) * SV) = even;
          *reinterpret_cast<u32x2_t *>(dst + (2 * wd + 1) * SV) = odd;
        }
      }
  };

  // ---- Q fragments (B operand of S^T = K Q^T), kept in registers ----------------
  // (query rows past N read row N-1; their results are never stored)
  const int qrow = qb * BLK + wave * 32 + l32;
  Frag8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    qf[ks].u = *reinterpret_cast<const u32x4_t *>(qbase + (long long)min(qrow, N - 1) * qsn +
                                                ks * 16 + hf * 8);

  f32x16_t o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  float m_ref = -__builtin_inff();  // reference exponent (log2 domain) of the running sums
  float l_run = 0.f;                // running sum over this lane's keys, relative to m_ref

  const size_t row = (size_t)bh * Nb + qb;
  const int cnt = min(kept_count[row], Nb);
  const int *idx = kept_idx + row * Nb;

  // ---- prologue: first kept block into LDS ---------------------------------------------
  int j_cur = 0, nvalid_cur = 0;
  if (cnt > 0) {
    j_cur = min(max(idx[0], 0), Nb - 1);  // stay in bounds whatever the list holds
    nvalid_cur = min(BLK, N - j_cur * BLK);
    const KStage<KCH> kst = load_k(j_cur * BLK, nvalid_cur);
    store_k(kst);
#pragma unroll
    for (int hh = 0; hh < NH; ++hh) {
      const KStage<4> vst = load_v(hh, j_cur * BLK, nvalid_cur);
      store_vt(vst, hh);
    }
  }
  __syncthreads();

  for (int c = 0; c < cnt; ++c) {
    // After the last kept block the "next" block is the current one again: the staging
    // below then re-stages data nobody reads, which keeps the loop body branch-free.
    const int j_next = min(max(idx[min(c + 1, cnt - 1)], 0), Nb - 1);
    const int nvalid_next = min(BLK, N - j_next * BLK);

    // K of the next kept block travels to registers while the matrix cores work on this one
    const KStage<KCH> kreg = load_k(j_next * BLK, nvalid_next);

    KStage<4> vstage[NH];
    // The key block is processed in NH slices of 64 keys (keeps the S^T and P^T
    // registers to 32 + 16 per lane); each slice is a full online-softmax update.
#pragma unroll
    for (int hh = 0; hh < NH; ++hh) {
      // ---- S^T = K Q^T for keys [64*hh, 64*hh + 64) -------------------------------------
      f32x16_t s[KTH];
#pragma unroll
      for (int kt = 0; kt < KTH; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[kt][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int kt = 0; kt < KTH; ++kt) {
          Frag8 a;
          a.u = *reinterpret_cast<const u32x4_t *>(sK + ((hh * KTH + kt) * 32 + l32) * SK +
                                                 ks * 16 + hf * 8);
          s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, qf[ks].v, s[kt], 0, 0, 0);
        }
      if (hh == NH - 1) {
        // A: every wave is done reading sK and the V^T slices before the last one
        __syncthreads();
        store_k(kreg);
#pragma unroll
        for (int h2 = 0; h2 < NH - 1; ++h2) store_vt(vstage[h2], h2);
      }

      // ---- online softmax (per lane = per query column) -------------------------------
      if (nvalid_cur < BLK) {  // ragged last key block: keys past the end get no weight
#pragma unroll
        for (int kt = 0; kt < KTH; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = (hh * KTH + kt) * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
            if (key >= nvalid_cur) s[kt][r] = -__builtin_inff();
          }
      }
      float m_loc = s[0][0];
#pragma unroll
      for (int kt = 0; kt < KTH; ++kt)
#pragma unroll
        for (int r = 0; r < 16; r += 2) m_loc = fmaxf(fmaxf(m_loc, s[kt][r]), s[kt][r + 1]);
      m_loc = fmaxf(m_loc, __shfl_xor(m_loc, 32, 64));
      const float m_tile = m_loc * scale_log2e;  // scale > 0, so max commutes with scaling
      // The reference exponent only moves when the slice maximum exceeds it by more
      // than the slack: exponentials then stay below 2^slack, and the rescale of the
      // accumulators is skipped for most slices.  (A slice whose keys are all past the
      // end has m_tile = -inf and never bumps.)
      const bool bump = m_tile > m_ref + kRescaleSlack ||
                        (m_ref == -__builtin_inff() && m_tile > -__builtin_inff());
      if (__any(bump)) {
        const float m_new = bump ? m_tile : m_ref;
        const float alpha = bump ? __builtin_amdgcn_exp2f(m_ref - m_new) : 1.f;
        l_run *= alpha;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
        m_ref = m_new;
      }
      // while m_ref is still -inf every logit seen so far was masked: weights are 0
      const float m_sub = m_ref == -__builtin_inff() ? 0.f : m_ref;
      float psum = 0.f;
      Frag8 pf[KTH][2];
#pragma unroll
      for (int kt = 0; kt < KTH; ++kt) {
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          p[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kt][r], scale_log2e, -m_sub));
          psum += p[r];
        }
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          pf[kt][s2].u.x = cvt_pk_bf16(p[8 * s2 + 0], p[8 * s2 + 1]);
          pf[kt][s2].u.y = cvt_pk_bf16(p[8 * s2 + 2], p[8 * s2 + 3]);
          pf[kt][s2].u.z = cvt_pk_bf16(p[8 * s2 + 4], p[8 * s2 + 5]);
          pf[kt][s2].u.w = cvt_pk_bf16(p[8 * s2 + 6], p[8 * s2 + 7]);
        }
      }
      l_run += psum;

      // slice hh of the next V travels to registers during this slice's second contraction
      vstage[hh] = load_v(hh, j_next * BLK, nvalid_next);

      // ---- O^T += V^T P^T ---------------------------------------------------------------
      // slot e of pf[kt][s2] is key (hh*KTH+kt)*32 + 16*s2 + 8*(e/4) + 4*hf + e%4
#pragma unroll
      for (int kt = 0; kt < KTH; ++kt)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) {
            const uint16_t *vp =
                sVT + (dt * 32 + l32) * SV + (hh * KTH + kt) * 32 + 16 * s2 + 4 * hf;
            Frag8 a;
            a.h[0] = *reinterpret_cast<const u32x2_t *>(vp);
            a.h[1] = *reinterpret_cast<const u32x2_t *>(vp + 8);
            o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, pf[kt][s2].v, o[dt], 0, 0, 0);
          }
    }
    // B: every wave is done with the last V^T slice; the new sK and the earlier V^T
    // slices are visible.  The last slice written below is read only after the next A.
    __syncthreads();
    store_vt(vstage[NH - 1], NH - 1);
    j_cur = j_next;
    nvalid_cur = nvalid_next;
  }

  // ---- epilogue: normalise, stage through LDS, coalesced bf16 store -----------------------
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  if (lse && hf == 0 && qrow < N)
    lse[(size_t)bh * N + qrow] =
        l_tot > 0.f ? (m_ref + log2f(l_tot)) * 0.6931471805599453f : -__builtin_inff();
  uint16_t *sO = sK;  // [BLK][SK]; sK is idle after the last barrier
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      u32x2_t pk;
      pk.x = cvt_pk_bf16(o[dt][4 * g + 0] * inv, o[dt][4 * g + 1] * inv);
      pk.y = cvt_pk_bf16(o[dt][4 * g + 2] * inv, o[dt][4 * g + 3] * inv);
      *reinterpret_cast<u32x2_t *>(sO + (wave * 32 + l32) * SK + dt * 32 + 8 * g + 4 * hf) = pk;
    }
  __syncthreads();
  uint16_t *obase = out + b * osb + h * osh;
#pragma unroll
  for (int it = 0; it < KCH; ++it) {
    const int r = k_r0 + it * K_R_STEP;
    const int n = qb * BLK + r;
    if (n < N)
      *reinterpret_cast<u32x4_t *>(obase + (long long)n * osn + k_c) =
          *reinterpret_cast<const u32x4_t *>(sO + r * SK + k_c);
  }
}

template <int D, int BLK>
static int launch_attn_t(const heart_shape &s, const void *q, const void *k, const void *v,
                         const int *kept_idx, const int *kept_count, float scale, void *out,
                         float *lse, hipStream_t st) {
  const int Nb = (s.N + BLK - 1) / BLK;
  const int BH = s.B * s.H;
  const size_t lds = ((size_t)BLK * (D + 8) + (size_t)D * (BLK + 4)) * 2;
  auto kern = attn_kernel<D, BLK>;
  static bool attr_set = false;  // the attribute is per function, set once per process
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess)
      return fail(HEART_EHIP, "hipFuncSetAttribute(max dynamic LDS %zu): %s", lds,
                  hipGetErrorString(e));
    attr_set = true;
  }
  const float sc = scale > 0.f ? scale : 1.0f / sqrtf((float)D);
  const float scale_log2e = sc * 1.4426950408889634f;
  hipLaunchKernelGGL(kern, dim3((unsigned)((long long)BH * Nb)), dim3(BLK * 2), lds, st,
                     (const uint16_t *)q, (const uint16_t *)k, (const uint16_t *)v,
                     (uint16_t *)out, s.q_stride[0], s.q_stride[1], s.q_stride[2], s.k_stride[0],
                     s.k_stride[1], s.k_stride[2], s.v_stride[0], s.v_stride[1], s.v_stride[2],
                     s.o_stride[0], s.o_stride[1], s.o_stride[2], s.H, BH, s.N, Nb, kept_idx,
                     kept_count, scale_log2e, lse);
  return check_launch("attn_kernel");
}

int launch_attn(const heart_shape &s, const void *q, const void *k, const void *v,
                const int *kept_idx, const int *kept_count, float scale, void *out, float *lse,
                hipStream_t st) {
  if (s.D == 128 && s.block == 128)
    return launch_attn_t<128, 128>(s, q, k, v, kept_idx, kept_count, scale, out, lse, st);
  if (s.D == 64 && s.block == 128)
    return launch_attn_t<64, 128>(s, q, k, v, kept_idx, kept_count, scale, out, lse, st);
  if (s.D == 64 && s.block == 64)
    return launch_attn_t<64, 64>(s, q, k, v, kept_idx, kept_count, scale, out, lse, st);
  return fail(HEART_EUNSUPPORTED, "heart_block_sparse_attn: unsupported (D, block) = (%d, %d)",
              s.D, s.block);
}

}  // namespace heart
