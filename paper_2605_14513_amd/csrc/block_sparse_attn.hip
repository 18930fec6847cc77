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

union Frag8 {
  uint4 u;
  bf16x8_t v;
  uint2 h[2];
};

__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
  f32x2_t f = {lo, hi};
  bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
  return __builtin_bit_cast(uint32_t, b);
}

constexpr int kNumXcd = 8;

template <int D, int BLK>
__global__ __launch_bounds__(BLK * 2) void attn_kernel(
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

  // ---- Q fragments (B operand of S^T = K Q^T), kept in registers ----------------
  const int qrow = qb * BLK + wave * 32 + l32;
  Frag8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    qf[ks].u = make_uint4(0u, 0u, 0u, 0u);
    if (qrow < N)
      qf[ks].u = *reinterpret_cast<const uint4 *>(qbase + (long long)qrow * qsn + ks * 16 + hf * 8);
  }

  f32x16_t o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  float m_run = -__builtin_inff();  // running max of the logits, log2 domain
  float l_run = 0.f;                // running sum over this lane's keys

  const size_t row = (size_t)bh * Nb + qb;
  const int cnt = min(kept_count[row], Nb);
  const int *idx = kept_idx + row * Nb;

  for (int c = 0; c < cnt; ++c) {
    int j = idx[c];
    j = min(max(j, 0), Nb - 1);  // stay in bounds whatever the list holds
    const int kv0 = j * BLK;
    const int nvalid = min(BLK, N - kv0);

    __syncthreads();  // every wave is done reading the previous tiles
    // ---- K tile -> LDS ------------------------------------------------------------
#pragma unroll
    for (int it = 0; it < (BLK * CPR) / NT; ++it) {
      const int ch = t + it * NT;
      const int r = ch / CPR, c8 = ch % CPR;
      uint4 g = make_uint4(0u, 0u, 0u, 0u);
      if (r < nvalid)
        g = *reinterpret_cast<const uint4 *>(kbase + (long long)(kv0 + r) * ksn + c8 * 8);
      *reinterpret_cast<uint4 *>(sK + r * SK + c8 * 8) = g;
    }
    // ---- V tile -> registers -> transposed -> LDS ----------------------------------
#pragma unroll
    for (int it = 0; it < D / 64; ++it) {
      const int s = (t >> 5) + (NT / 32) * it;
      const int dg = (t & 3) + 4 * (s % (D / 32));
      const int kg = ((t & 31) >> 2) + 8 * (s / (D / 32));
      uint4 vr[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int r = kg * 4 + e;
        vr[e] = make_uint4(0u, 0u, 0u, 0u);
        if (r < nvalid)
          vr[e] = *reinterpret_cast<const uint4 *>(vbase + (long long)(kv0 + r) * vsn + dg * 8);
      }
      const uint32_t w[4][4] = {{vr[0].x, vr[0].y, vr[0].z, vr[0].w},
                                {vr[1].x, vr[1].y, vr[1].z, vr[1].w},
                                {vr[2].x, vr[2].y, vr[2].z, vr[2].w},
                                {vr[3].x, vr[3].y, vr[3].z, vr[3].w}};
#pragma unroll
      for (int wd = 0; wd < 4; ++wd) {
        // word wd of key e holds d = 2*wd (low half) and 2*wd+1 (high half)
        uint2 even, odd;
        even.x = __builtin_amdgcn_perm(w[1][wd], w[0][wd], 0x05040100u);  // lo16(k0) | lo16(k1)<<16
        even.y = __builtin_amdgcn_perm(w[3][wd], w[2][wd], 0x05040100u);
        odd.x = __builtin_amdgcn_perm(w[1][wd], w[0][wd], 0x07060302u);   // hi16(k0) | hi16(k1)<<16
        odd.y = __builtin_amdgcn_perm(w[3][wd], w[2][wd], 0x07060302u);
        *reinterpret_cast<uint2 *>(sVT + (dg * 8 + 2 * wd) * SV + kg * 4) = even;
        *reinterpret_cast<uint2 *>(sVT + (dg * 8 + 2 * wd + 1) * SV + kg * 4) = odd;
      }
    }
    __syncthreads();

    // ---- S^T = K Q^T ----------------------------------------------------------------
    f32x16_t s[KT];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kt][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        Frag8 a;
        a.u = *reinterpret_cast<const uint4 *>(sK + (kt * 32 + l32) * SK + ks * 16 + hf * 8);
        s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, qf[ks].v, s[kt], 0, 0, 0);
      }
    }

    // ---- online softmax (per lane = per query column) ---------------------------------
    float m_loc = -__builtin_inff();
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float x = s[kt][r] * scale_log2e;
        const int key = kt * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
        if (key >= nvalid) x = -__builtin_inff();
        s[kt][r] = x;
        m_loc = fmaxf(m_loc, x);
      }
    m_loc = fmaxf(m_loc, __shfl_xor(m_loc, 32, 64));
    const float m_new = fmaxf(m_run, m_loc);
    const float m_safe = m_new == -__builtin_inff() ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
    float psum = 0.f;
    Frag8 pf[KT][2];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      float p[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        p[r] = __builtin_amdgcn_exp2f(s[kt][r] - m_safe);
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
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;

    // ---- O^T += V^T P^T -----------------------------------------------------------------
    // slot e of pf[kt][s2] is key kt*32 + 16*s2 + 8*(e/4) + 4*hf + e%4
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const uint16_t *vp = sVT + (dt * 32 + l32) * SV + kt * 32 + 16 * s2 + 4 * hf;
          Frag8 a;
          a.h[0] = *reinterpret_cast<const uint2 *>(vp);
          a.h[1] = *reinterpret_cast<const uint2 *>(vp + 8);
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, pf[kt][s2].v, o[dt], 0, 0, 0);
        }
  }

  // ---- epilogue: normalise, stage through LDS, coalesced bf16 store -----------------------
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  if (lse && hf == 0 && qrow < N)
    lse[(size_t)bh * N + qrow] =
        l_tot > 0.f ? (m_run + log2f(l_tot)) * 0.6931471805599453f : -__builtin_inff();
  __syncthreads();  // all waves finished with sK / sVT
  uint16_t *sO = sK;  // [BLK][SK]
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint2 pk;
      pk.x = cvt_pk_bf16(o[dt][4 * g + 0] * inv, o[dt][4 * g + 1] * inv);
      pk.y = cvt_pk_bf16(o[dt][4 * g + 2] * inv, o[dt][4 * g + 3] * inv);
      *reinterpret_cast<uint2 *>(sO + (wave * 32 + l32) * SK + dt * 32 + 8 * g + 4 * hf) = pk;
    }
  __syncthreads();
  uint16_t *obase = out + b * osb + h * osh;
#pragma unroll
  for (int it = 0; it < (BLK * CPR) / NT; ++it) {
    const int ch = t + it * NT;
    const int r = ch / CPR, c8 = ch % CPR;
    const int n = qb * BLK + r;
    if (n < N)
      *reinterpret_cast<uint4 *>(obase + (long long)n * osn + c8 * 8) =
          *reinterpret_cast<const uint4 *>(sO + r * SK + c8 * 8);
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
