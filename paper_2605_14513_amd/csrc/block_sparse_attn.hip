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
// as long as the A operand (V^T) uses the same one.
//
// LDS holds one K tile [block][D+8] bf16 (16-byte fragment reads of 16 consecutive
// key rows hit 16 distinct 4-bank groups) and one V^T tile [D][block+8] bf16.
// Within every group of 16 keys the V^T tile stores the 4-key chunks in the order
// 0,2,1,3: the 8 keys a lane needs for one MFMA (chunks {0,2} for lanes 0-31,
// {1,3} for lanes 32-63) are then one aligned 16-byte read.  V is transposed in
// registers on its way from global memory (4 keys x 8 d per lane, byte permutes).
//
// Pipeline per kept key block (two workgroup barriers):
//   top      K of the next block -> registers (buffer loads in flight during the MFMAs)
//   slices   the block is consumed in 64-key slices: S^T, online softmax, O^T update
//   barrier A (after the last S^T): K registers -> LDS; V of the next block -> registers
//   barrier B (after the last O^T update): V registers -> transposed -> LDS
// Global loads are buffer loads: rows past the end of the sequence are out of range
// for the descriptor and read as zero, with no branch and no address clamping.
//
// Workgroup ids are remapped (they are dealt round-robin to the 8 XCDs, each with its
// own L2) so that an XCD works on a contiguous eighth of the query blocks of every
// head: balanced across XCDs, and neighbouring query blocks share their kept K/V
// blocks through that XCD's L2.
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
};

__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
  f32x2_t f = {lo, hi};
  bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
  return __builtin_bit_cast(uint32_t, b);
}

// acc + lo + hi of a packed bf16 pair (one v_dot2 against the constant (1, 1))
__device__ __forceinline__ float add_bf16_pair(uint32_t pk, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pk),
                                         __builtin_bit_cast(bf16x2_t, 0x3f803f80u), acc, false);
}

// registers that carry one thread's share of a K or V tile from global memory to LDS
template <int n>
struct Stage {
  u32x4_t r[n];
};

// buffer descriptor over one head's rows: offsets >= bytes read as zero
__device__ __forceinline__ __amdgpu_buffer_rsrc_t head_rsrc(const uint16_t *base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(base), 0, (int)bytes, 0x00020000);
}

constexpr int kNumXcd = 8;

template <int D, int BLK>
__global__ __launch_bounds__(BLK * 2, 2) void attn_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k,
    const uint16_t *__restrict__ v, uint16_t *__restrict__ out, long long qsb, long long qsh,
    long long qsn, long long ksb, long long ksh, long long ksn, long long vsb, long long vsh,
    long long vsn, long long osb, long long osh, long long osn, int H, int BH, int N, int Nb,
    const int *__restrict__ kept_idx, const int *__restrict__ kept_count, float scale_log2e,
    float *__restrict__ lse) {
  constexpr int NT = BLK * 2;            // threads
  constexpr int KT = BLK / 32;           // 32-key tiles per key block
  constexpr int DT = D / 32;             // 32-wide d tiles of the output
  constexpr int KS = D / 16;             // k-steps of the first contraction
  constexpr int SK = D + 8;              // LDS row stride of the K tile (elements)
  constexpr int SV = BLK + 8;            // LDS row stride of the V^T tile (elements)
  constexpr int CPR = D / 8;             // 16-byte chunks per token row
  constexpr int KCH = (BLK * CPR) / NT;  // K chunks per thread
  constexpr int K_R_STEP = NT / CPR;     // rows between a thread's K chunks
  constexpr int VIT = D / 64;            // V sub-tiles (4 keys x 8 d) per thread
  constexpr int V_KG_STEP = 8 * ((NT / 32) / (D / 32));  // key groups between them
  constexpr int KTH = 2;                 // 32-key tiles per slice of the key block
  constexpr int NH = KT / KTH;           // slices per key block
  constexpr float kRescaleSlack = 8.f;   // log2 units the running reference may lag the max

  extern __shared__ __align__(16) unsigned char smem_raw[];
  uint16_t *sK = reinterpret_cast<uint16_t *>(smem_raw);  // [BLK][SK]; reused for the output
  uint16_t *sVT = sK + BLK * SK;                           // [D][SV]

  // ---- workgroup id -> (head, query block), XCD-aware ------------------------------
  // Workgroup ids are dealt round-robin to the 8 XCDs.  XCD x takes the x-th eighth
  // of the query blocks of EVERY head, heads in order: all XCDs then carry the same
  // mix of heads (per-head density differs a lot, so whole heads per XCD would be
  // unbalanced), neighbouring query blocks -- whose kept key blocks overlap -- share
  // an L2, and at any time only one or two heads' K/V are live in the memory-side cache.
  int bh, qb;
  {
    const int per = (Nb + kNumXcd - 1) / kNumXcd;  // query blocks per XCD and head
    const int xcd = (int)(blockIdx.x % kNumXcd);
    const long long slot = blockIdx.x / kNumXcd;
    bh = (int)(slot / per);
    qb = xcd * per + (int)(slot % per);
    if (qb >= Nb) return;  // padding of the last eighth (whole workgroup, before any barrier)
  }
  const int b = bh / H, h = bh % H;
  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int l32 = lane & 31, hf = lane >> 5;

  const __amdgpu_buffer_rsrc_t q_rs = head_rsrc(q + b * qsb + h * qsh, (uint32_t)(N * qsn * 2));
  const __amdgpu_buffer_rsrc_t k_rs = head_rsrc(k + b * ksb + h * ksh, (uint32_t)(N * ksn * 2));
  const __amdgpu_buffer_rsrc_t v_rs = head_rsrc(v + b * vsb + h * vsh, (uint32_t)(N * vsn * 2));
  const uint32_t k_row_bytes = (uint32_t)ksn * 2u, v_row_bytes = (uint32_t)vsn * 2u;

  // K staging: chunk `it` of this thread is row k_r0 + it * K_R_STEP, 16-byte column k_c
  const int k_r0 = t / CPR, k_c = (t % CPR) * 8;
  const uint32_t k_off0 = (uint32_t)k_r0 * k_row_bytes + (uint32_t)k_c * 2u;
  // V staging: sub-tile `it` is d-group v_dg (8 d), key group v_kg0 + it * V_KG_STEP (4 keys);
  // lanes of a half-wave cover 4 d-groups x 8 key groups
  const int v_dg = (t & 3) + 4 * ((t >> 5) % (D / 32));
  const int v_kg0 = ((t & 31) >> 2) + 8 * ((t >> 5) / (D / 32));
  const uint32_t v_off0 = (uint32_t)(v_kg0 * 4) * v_row_bytes + (uint32_t)v_dg * 16u;

  auto load_k = [&](int kv0) -> Stage<KCH> {
    Stage<KCH> st;
    uint32_t off = k_off0 + (uint32_t)kv0 * k_row_bytes;
#pragma unroll
    for (int it = 0; it < KCH; ++it) {
      st.r[it] = __builtin_amdgcn_raw_buffer_load_b128(k_rs, off, 0, 0);
      off += K_R_STEP * k_row_bytes;
    }
    return st;
  };
  auto store_k = [&](const Stage<KCH> &st) {
    uint16_t *dst = sK + k_r0 * SK + k_c;
#pragma unroll
    for (int it = 0; it < KCH; ++it)
      *reinterpret_cast<u32x4_t *>(dst + it * K_R_STEP * SK) = st.r[it];
  };
  auto load_v = [&](int kv0) -> Stage<VIT * 4> {
    Stage<VIT * 4> st;
    uint32_t off = v_off0 + (uint32_t)kv0 * v_row_bytes;
#pragma unroll
    for (int it = 0; it < VIT; ++it) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        st.r[it * 4 + e] = __builtin_amdgcn_raw_buffer_load_b128(v_rs, off + e * v_row_bytes, 0, 0);
      off += V_KG_STEP * 4 * v_row_bytes;
    }
    return st;
  };
  auto store_vt = [&](const Stage<VIT * 4> &st) {
#pragma unroll
    for (int it = 0; it < VIT; ++it) {
      const u32x4_t *vr = st.r + it * 4;
      // 4-key chunk c of a 16-key group is stored at chunk position (0,2,1,3)[c]
      const int kg = v_kg0 + it * V_KG_STEP;
      const int pos = (kg & ~3) | ((kg & 1) << 1) | ((kg >> 1) & 1);
      uint16_t *dst = sVT + (v_dg * 8) * SV + pos * 4;
#pragma unroll
      for (int wd = 0; wd < 4; ++wd) {
        // word wd of key e holds d = 2*wd (low half) and d = 2*wd+1 (high half)
        u32x2_t even, odd;
        even.x = __builtin_amdgcn_perm(vr[1][wd], vr[0][wd], 0x05040100u);  // lo16(k0) | lo16(k1)<<16
        even.y = __builtin_amdgcn_perm(vr[3][wd], vr[2][wd], 0x05040100u);
        odd.x = __builtin_amdgcn_perm(vr[1][wd], vr[0][wd], 0x07060302u);   // hi16(k0) | hi16(k1)<<16
        odd.y = __builtin_amdgcn_perm(vr[3][wd], vr[2][wd], 0x07060302u);
        *reinterpret_cast<u32x2_t *>(dst + (2 * wd) * SV) = even;
        *reinterpret_cast<u32x2_t *>(dst + (2 * wd + 1) * SV) = odd;
      }
    }
  };

  // ---- Q fragments (B operand of S^T = K Q^T), kept in registers ----------------
  const int qrow = qb * BLK + wave * 32 + l32;
  Frag8 qf[KS];
  {
    const uint32_t q_off = (uint32_t)qrow * ((uint32_t)qsn * 2u) + (uint32_t)hf * 16u;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      qf[ks].u = __builtin_amdgcn_raw_buffer_load_b128(q_rs, q_off + ks * 32, 0, 0);
  }

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
  // kept indices are clamped into [0, Nb) so that a bad list cannot leave the tensors
  auto kept = [&](int c) -> int { return min(max(idx[min(c, cnt - 1)], 0), Nb - 1); };

  // ---- prologue: first kept block into LDS ---------------------------------------------
  int j_cur = 0, j_next = 0;
  if (cnt > 0) {
    j_cur = kept(0);
    j_next = kept(1);
    const Stage<KCH> kst = load_k(j_cur * BLK);
    const Stage<VIT * 4> vst = load_v(j_cur * BLK);
    store_k(kst);
    store_vt(vst);
  }
  __syncthreads();

  // LDS read bases of this lane
  const uint16_t *sK_rd = sK + l32 * SK + hf * 8;
  const uint16_t *sV_rd = sVT + l32 * SV + hf * 8;

  for (int c = 0; c < cnt; ++c) {
    // After the last kept block the "next" block is the current one again: the staging
    // below then re-stages data nobody reads, which keeps the loop body branch-free.
    const int j_next2 = kept(c + 2);
    const int nvalid_cur = min(BLK, N - j_cur * BLK);

    // K of the next kept block travels to registers while the matrix cores work on this one
    const Stage<KCH> kreg = load_k(j_next * BLK);
    Stage<VIT * 4> vreg;

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
          a.u = *reinterpret_cast<const u32x4_t *>(sK_rd + (hh * KTH + kt) * 32 * SK + ks * 16);
          s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, qf[ks].v, s[kt], 0, 0, 0);
        }
      if (hh == NH - 1) {
        __syncthreads();  // A: every wave is done reading sK
        store_k(kreg);
        vreg = load_v(j_next * BLK);  // in flight during the rest of this key block
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
      Frag8 pf[KTH][2];
#pragma unroll
      for (int kt = 0; kt < KTH; ++kt) {
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r)
          p[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kt][r], scale_log2e, -m_sub));
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            const uint32_t pk = cvt_pk_bf16(p[8 * s2 + 2 * w], p[8 * s2 + 2 * w + 1]);
            pf[kt][s2].u[w] = pk;
            // the row sum adds the ROUNDED weights, the ones the second contraction uses
            l_run = add_bf16_pair(pk, l_run);
          }
      }

      // ---- O^T += V^T P^T ---------------------------------------------------------------
      // slot e of pf[kt][s2] is key (hh*KTH+kt)*32 + 16*s2 + 8*(e/4) + 4*hf + e%4; in LDS
      // these 8 keys are the 16 bytes at key position (hh*KTH+kt)*32 + 16*s2 + 8*hf
#pragma unroll
      for (int kt = 0; kt < KTH; ++kt)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) {
            Frag8 a;
            a.u = *reinterpret_cast<const u32x4_t *>(sV_rd + dt * 32 * SV +
                                                     (hh * KTH + kt) * 32 + 16 * s2);
            o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, pf[kt][s2].v, o[dt], 0, 0, 0);
          }
    }
    // B: every wave is done reading sVT; the new sK is visible.  The V^T tile written
    // below is read only after the next barrier A.
    __syncthreads();
    store_vt(vreg);
    j_cur = j_next;
    j_next = j_next2;
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
  const size_t lds = ((size_t)BLK * (D + 8) + (size_t)D * (BLK + 8)) * 2;
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
  const long long grid = (long long)BH * ((Nb + kNumXcd - 1) / kNumXcd) * kNumXcd;
  if (grid > 0x7fffffffLL) return fail(HEART_EUNSUPPORTED, "heart_block_sparse_attn: grid too large");
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(BLK * 2), lds, st,
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
  // the kernel addresses one head's rows through 32-bit buffer offsets
  const long long lim = 0xffffffffLL;
  const long long rows = (long long)s.N + 2 * s.block;  // staging may address a few rows past N
  if (rows * s.q_stride[2] * 2 > lim || rows * s.k_stride[2] * 2 > lim ||
      rows * s.v_stride[2] * 2 > lim)
    return fail(HEART_EUNSUPPORTED,
                "heart_block_sparse_attn: (N + 2*block) * token stride * 2 bytes must stay "
                "below 4 GiB");
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
