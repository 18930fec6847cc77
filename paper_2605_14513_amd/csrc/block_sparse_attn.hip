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
  constexpr int DT = D / 32;             // 32-wide d tiles of the output
  constexpr int KS = D / 16;             // k-steps of the first contraction
  constexpr int SK = D + 8;              // LDS row stride of the K tile (elements)
  constexpr int SV = BLK + 8;            // LDS row stride of the V^T tile (elements)
  constexpr int CPR = D / 8;             // 16-byte chunks per token row
  constexpr int KCH = (BLK * CPR) / NT;  // K chunks per thread
  constexpr int K_R_STEP = NT / CPR;     // rows between a thread's K chunks
  constexpr int VIT = D / 64;            // V sub-tiles (4 keys x 8 d) per thread
  constexpr int V_KG_STEP = 8 * ((NT / 32) / (D / 32));  // key groups between them
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

  // Staging is written per operation so that the loop can issue the loads and LDS
  // stores one at a time in the shadow of MFMAs instead of in bursts after a barrier.
  // K: chunk `it` (0 .. KCH-1) of this thread.
  auto load_k1 = [&](Stage<KCH> &st, int it, int kv0) {
    st.r[it] = __builtin_amdgcn_raw_buffer_load_b128(
        k_rs, k_off0 + (uint32_t)(kv0 + it * K_R_STEP) * k_row_bytes, 0, 0);
  };
  auto store_k1 = [&](const Stage<KCH> &st, int it) {
    *reinterpret_cast<u32x4_t *>(sK + (k_r0 + it * K_R_STEP) * SK + k_c) = st.r[it];
  };
  // V: the tile is staged in two halves of BLK/2 keys.  Sub-tile `it` of this thread lies
  // in half (v_kg0 + it * V_KG_STEP) / KGH: with VIT == 2 that is `it`, with VIT == 1 it is
  // uniform per wavefront.  Each sub-tile is 4 loads (keys) and 4 transposed word pairs.
  constexpr int KGH = BLK / 8;  // key groups (of 4 keys) per half
  static_assert(VIT == 1 || (VIT == 2 && V_KG_STEP == KGH), "V staging layout");
  auto v_half_of = [&](int it) -> int { return (v_kg0 + it * V_KG_STEP) / KGH; };
  auto load_v1 = [&](Stage<4> &st, int it, int e, int kv0) {
    st.r[e] = __builtin_amdgcn_raw_buffer_load_b128(
        v_rs, v_off0 + (uint32_t)(kv0 + it * V_KG_STEP * 4 + e) * v_row_bytes, 0, 0);
  };
  // word pair wd (d = 2wd, 2wd+1) of the 4 keys of sub-tile `it`
  auto store_vt1 = [&](const Stage<4> &st, int it, int wd) {
    // 4-key chunk c of a 16-key group is stored at chunk position (0,2,1,3)[c]
    const int kg = v_kg0 + it * V_KG_STEP;
    const int pos = (kg & ~3) | ((kg & 1) << 1) | ((kg >> 1) & 1);
    uint16_t *dst = sVT + (v_dg * 8 + 2 * wd) * SV + pos * 4;
    u32x2_t even, odd;
    even.x = __builtin_amdgcn_perm(st.r[1][wd], st.r[0][wd], 0x05040100u);  // lo16(k0) | lo16(k1)<<16
    even.y = __builtin_amdgcn_perm(st.r[3][wd], st.r[2][wd], 0x05040100u);
    odd.x = __builtin_amdgcn_perm(st.r[1][wd], st.r[0][wd], 0x07060302u);   // hi16(k0) | hi16(k1)<<16
    odd.y = __builtin_amdgcn_perm(st.r[3][wd], st.r[2][wd], 0x07060302u);
    *reinterpret_cast<u32x2_t *>(dst) = even;
    *reinterpret_cast<u32x2_t *>(dst + SV) = odd;
  };
  // Whole-half helpers.  `mine(half)`: does this thread stage anything of that half?
  // (VIT == 2: always, sub-tile it == half; VIT == 1: only if its sub-tile lies there.)
  auto v_it_of = [&](int half) -> int { return VIT == 2 ? half : 0; };
  auto v_mine = [&](int half) -> bool { return VIT == 2 ? true : v_half_of(0) == half; };

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
    Stage<KCH> kst;
#pragma unroll
    for (int it = 0; it < KCH; ++it) load_k1(kst, it, j_cur * BLK);
#pragma unroll
    for (int it = 0; it < KCH; ++it) store_k1(kst, it);
#pragma unroll
    for (int it = 0; it < VIT; ++it) {
      Stage<4> vst;
#pragma unroll
      for (int e = 0; e < 4; ++e) load_v1(vst, it, e, j_cur * BLK);
#pragma unroll
      for (int wd = 0; wd < 4; ++wd) store_vt1(vst, it, wd);
    }
  }
  __syncthreads();

  // LDS read bases of this lane
  const uint16_t *sK_rd = sK + l32 * SK + hf * 8;
  const uint16_t *sV_rd = sVT + l32 * SV + hf * 8;

  // ---- the loop over kept key blocks --------------------------------------------------------
  // A key block is consumed in NSL slices of 32 keys, software-pipelined; the instruction
  // order written here is the intended issue order (fenced with sched_barrier):
  //   B(sl)  MFMAs of S^T(sl+1); after each: one LDS fragment read for a later MFMA, the
  //          exponentials / bf16 rounding / row sum of a few elements of slice sl, and
  //          at most one staging operation                                (MFMA || VALU)
  //   C(sl)  MFMAs of O^T += V^T P^T(sl); after each: one LDS fragment read, part of the
  //          maximum of S^T(sl+1), at most one staging operation          (MFMA || VALU)
  //   then the (rare) move of the reference exponent.
  // Staging of the next key block, spread over these slots:
  //   K loads and V loads of half 0 in B(0); V loads of half 1 in C(NSL-2)
  //   barrier A after B(NSL-2): every wave has read all of sK and V^T half 0
  //   K stores and V^T half-0 stores in C(NSL-2)
  //   barrier B after C(NSL-1): every wave has read V^T half 1; new sK / half 0 visible
  //   V^T half-1 stores in W = S^T(slice 0) of the next block; first read after the next A
  constexpr int NSL = BLK / 32;           // slices per key block
  constexpr int PF = KS < 4 ? KS : 4;     // LDS fragment reads in flight ahead of the MFMAs
  constexpr int EPM = 16 / KS;            // softmax elements handled per S^T MFMA
  constexpr int NPV = 2 * DT;             // MFMAs of one slice's O^T update
  static_assert(16 % KS == 0 && (NSL == 2 || NSL == 4), "slice layout");

  auto kfrag = [&](int sl, int ks) -> u32x4_t {
    return *reinterpret_cast<const u32x4_t *>(sK_rd + sl * 32 * SK + ks * 16);
  };
  // 8 keys of slice sl for MFMA m (s2 = m / DT, d tile m % DT): key positions
  // sl*32 + 16*s2 + 8*hf .. +7 (see header)
  auto vfrag = [&](int sl, int m) -> u32x4_t {
    return *reinterpret_cast<const u32x4_t *>(sV_rd + (m % DT) * 32 * SV + sl * 32 + 16 * (m / DT));
  };

  f32x16_t sacc[2];  // S^T of the slice being exponentiated and of the next one
  Frag8 pf[2];       // P^T of the current slice: [s2] = rows 8*s2 .. 8*s2+7 of the accumulator

  // B: S^T(slice sl) into sacc[sl & 1]; with_exp: interleave the weights of slice sl-1
  // (relative to the reference exponent, rounded to bf16; the row sum adds the ROUNDED
  // weights, the ones the second contraction uses).  extra(slot) injects staging work.
  auto qk_step = [&](int sl, bool with_exp, float m_sub, auto &&extra) {
    f32x16_t acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const f32x16_t &prev = sacc[(sl + 1) & 1];
    Frag8 fa[PF];
#pragma unroll
    for (int j = 0; j < PF; ++j) fa[j].u = kfrag(sl, j);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks % PF].v, qf[ks].v, acc, 0, 0, 0);
      if (ks + PF < KS) fa[ks % PF].u = kfrag(sl, ks + PF);
      if (with_exp) {
#pragma unroll
        for (int e = 0; e < EPM; e += 2) {
          const int r = ks * EPM + e;
          const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(prev[r], scale_log2e, -m_sub));
          const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(prev[r + 1], scale_log2e, -m_sub));
          const uint32_t pk = cvt_pk_bf16(p0, p1);
          pf[r / 8].u[(r % 8) / 2] = pk;
          l_run = add_bf16_pair(pk, l_run);
        }
      }
      extra(ks);
      __builtin_amdgcn_sched_barrier(0);
    }
    sacc[sl & 1] = acc;
  };
  // the weights alone (last slice of a key block: no S^T left to overlap with)
  auto exp_only = [&](int sl, float m_sub) {
    const f32x16_t &cur = sacc[sl & 1];
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
      const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(cur[r], scale_log2e, -m_sub));
      const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(cur[r + 1], scale_log2e, -m_sub));
      const uint32_t pk = cvt_pk_bf16(p0, p1);
      pf[r / 8].u[(r % 8) / 2] = pk;
      l_run = add_bf16_pair(pk, l_run);
    }
  };
  // keys past the end of a ragged last key block get no weight
  auto mask_slice = [&](f32x16_t &x, int sl, int nvalid) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = sl * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
      if (key >= nvalid) x[r] = -__builtin_inff();
    }
  };
  // maximum of one accumulator over this lane's 16 keys, in MAXP partial steps so that
  // it can be spread over MFMA slots; step i folds elements 4i .. 4i+3
  auto max_part = [&](const f32x16_t &x, int i, float m) -> float {
    return fmaxf(fmaxf(fmaxf(m, x[4 * i]), fmaxf(x[4 * i + 1], x[4 * i + 2])), x[4 * i + 3]);
  };
  // Finish the maximum of a slice (combine the two lanes of a query: lane l and l^32 are
  // exchanged with one v_permlane32_swap) and, rarely, move the reference exponent.
  // The reference only moves when the slice maximum exceeds it by more than the slack:
  // exponentials then stay below 2^slack and the accumulator rescale is skipped for
  // most slices.  A slice whose keys are all past the end has maximum -inf and never
  // moves it.  Returns the exponent to subtract (0 while every logit so far was masked).
  auto finish_max = [&](float m_loc) -> float {
    const uint32_t mi = __float_as_uint(m_loc);
    const auto sw = __builtin_amdgcn_permlane32_swap(mi, mi, false, false);
    m_loc = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    const float m_tile = m_loc * scale_log2e;  // scale > 0, so max commutes with scaling
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
    return m_ref == -__builtin_inff() ? 0.f : m_ref;
  };
  // C: O^T += V^T P^T(slice sl); the second half of the MFMA slots also folds the maximum
  // of `nxt` (S^T of the following slice, whose MFMAs were issued before this step and
  // have drained by then).  Returns that lane-local maximum.
  auto pv_step = [&](int sl, bool nxt, auto &&extra) -> float {
    const f32x16_t &nx = sacc[(sl + 1) & 1];
    float m_loc = -__builtin_inff();
    Frag8 fv[PF];
#pragma unroll
    for (int j = 0; j < PF; ++j) fv[j].u = vfrag(sl, j);
#pragma unroll
    for (int m = 0; m < NPV; ++m) {
      o[m % DT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv[m % PF].v, pf[m / DT].v, o[m % DT], 0, 0, 0);
      if (m + PF < NPV) fv[m % PF].u = vfrag(sl, m + PF);
      if (nxt) {
        // 4 partial steps in the last slots
        constexpr int first = NPV >= 4 ? NPV - 4 : 0;
        if (NPV >= 4) {
          if (m >= first) m_loc = max_part(nx, m - first, m_loc);
        } else if (m == NPV - 1) {
#pragma unroll
          for (int i = 0; i < 4; ++i) m_loc = max_part(nx, i, m_loc);
        }
      }
      extra(m);
      __builtin_amdgcn_sched_barrier(0);
    }
    return m_loc;
  };
  auto no_extra = [](int) {};

  float m_sub = 0.f;
  if (cnt > 0) {
    qk_step(0, false, 0.f, no_extra);
    const int nvalid0 = min(BLK, N - j_cur * BLK);
    if (nvalid0 < BLK) mask_slice(sacc[0], 0, nvalid0);
    float m_loc = -__builtin_inff();
#pragma unroll
    for (int i = 0; i < 4; ++i) m_loc = max_part(sacc[0], i, m_loc);
    m_sub = finish_max(m_loc);
  }
  for (int c = 0; c < cnt; ++c) {
    // After the last kept block the "next" block is the current one again: the staging
    // then re-stages data nobody reads, which keeps the loop branch-free.
    const int j_next2 = kept(c + 2);
    const int nvalid_cur = min(BLK, N - j_cur * BLK);
    const int nvalid_next = min(BLK, N - j_next * BLK);
    const int kv_next = j_next * BLK;
    Stage<KCH> kreg;
    Stage<4> v0, v1;  // V sub-tiles of half 0 and half 1 of the next key block
#pragma unroll
    for (int sl = 0; sl < NSL; ++sl) {
      // ---- B(sl) ----
      if (sl + 1 < NSL) {
        qk_step(sl + 1, true, m_sub, [&](int ks) {
          if (sl == 0) {  // K loads and V half-0 loads of the next key block, spread over the slots
#pragma unroll
            for (int it = 0; it < KCH; ++it)
              if (it * KS / KCH == ks) load_k1(kreg, it, kv_next);
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (e * KS / 4 == ks && v_mine(0)) load_v1(v0, v_it_of(0), e, kv_next);
          }
        });
        if (nvalid_cur < BLK) mask_slice(sacc[(sl + 1) & 1], sl + 1, nvalid_cur);
      } else {
        exp_only(sl, m_sub);
      }
      if (sl == NSL - 2) __syncthreads();  // barrier A
      // ---- C(sl) ----
      const float m_loc = pv_step(sl, sl + 1 < NSL, [&](int m) {
        if (sl == NSL - 2) {
          // K stores, spread; V^T half-0 stores (one word pair per slot); V loads, half 1
#pragma unroll
          for (int it = 0; it < KCH; ++it)
            if (it * NPV / KCH == m) store_k1(kreg, it);
          if (m < 4 && v_mine(0)) store_vt1(v0, v_it_of(0), m);
          if (m >= NPV - 4 && v_mine(1)) load_v1(v1, v_it_of(1), m - (NPV - 4), kv_next);
        }
      });
      if (sl + 1 < NSL) m_sub = finish_max(m_loc);
    }
    // barrier B
    __syncthreads();
    // ---- W: S^T(slice 0) of the next key block, with the V^T half-1 stores ----
    qk_step(0, false, 0.f, [&](int ks) {
      if (ks < 4 && v_mine(1)) store_vt1(v1, v_it_of(1), ks);
    });
    if (KS < 4 && v_mine(1)) {
#pragma unroll
      for (int wd = KS; wd < 4; ++wd) store_vt1(v1, v_it_of(1), wd);
    }
    {
      if (nvalid_next < BLK) mask_slice(sacc[0], 0, nvalid_next);
      float m_loc = -__builtin_inff();
#pragma unroll
      for (int i = 0; i < 4; ++i) m_loc = max_part(sacc[0], i, m_loc);
      m_sub = finish_max(m_loc);
    }
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
