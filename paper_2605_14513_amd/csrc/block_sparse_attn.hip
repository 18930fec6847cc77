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
// own L2).  With a work-order list (attn_order_kernel, when the caller passes a
// workspace) the query blocks are launched longest first: kept counts range from 1 to
// Nb per row, and a long row that starts late would otherwise leave most of the chip
// idle at the end.  The order is a stable counting sort on 32 count classes, so rows of
// a class keep their natural order (same head, neighbouring query blocks, which share
// kept K/V blocks), and runs of 8 consecutive list entries go to the same XCD.  Without
// a list an XCD works on a contiguous eighth of the query blocks of every head.
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
constexpr int kOrderRun = 8;      // consecutive work-list entries that go to one XCD
constexpr int kOrderClasses = 32; // count classes of the work-order sort

// Work order for the attention launch: a permutation of the n = B*H*Nb (head, query
// block) items, longest kept list first.  Stable counting sort by count class
// (class 0 = the longest rows) in one workgroup: thread t owns a contiguous segment of
// the items and one column of the class histogram, so that items of a class keep
// their natural order.
__global__ __launch_bounds__(256) void attn_order_kernel(const int *__restrict__ kept_count, int n,
                                                         int Nb, int *__restrict__ order) {
  __shared__ int hist[kOrderClasses][256];
  __shared__ int scan[256];
  const int t = threadIdx.x;
  const int per = (n + 255) / 256;
  const int i0 = min(n, t * per), i1 = min(n, i0 + per);
  auto cls = [&](int c) -> int {
    c = min(max(c, 0), Nb);
    return (kOrderClasses - 1) - (int)(((long long)c * (kOrderClasses - 1)) / Nb);
  };
#pragma unroll
  for (int b = 0; b < kOrderClasses; ++b) hist[b][t] = 0;
  for (int i = i0; i < i1; i += 8) {
    int c[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) c[e] = i + e < i1 ? kept_count[i + e] : 0;
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (i + e < i1) hist[cls(c[e])][t] += 1;
  }
  __syncthreads();
  // exclusive scan over the histogram flattened class-major (index = class * 256 + thread)
  int *flat = &hist[0][0];
  int sum = 0;
  for (int j = 0; j < kOrderClasses; ++j) sum += flat[t * kOrderClasses + j];
  scan[t] = sum;
  __syncthreads();
  for (int d = 1; d < 256; d <<= 1) {
    const int add = t >= d ? scan[t - d] : 0;
    __syncthreads();
    scan[t] += add;
    __syncthreads();
  }
  int run = scan[t] - sum;
  for (int j = 0; j < kOrderClasses; ++j) {
    const int x = flat[t * kOrderClasses + j];
    flat[t * kOrderClasses + j] = run;
    run += x;
  }
  __syncthreads();
  for (int i = i0; i < i1; i += 8) {
    int c[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) c[e] = i + e < i1 ? kept_count[i + e] : 0;
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (i + e < i1) {
        const int b = cls(c[e]);
        const int pos = hist[b][t];
        hist[b][t] = pos + 1;
        order[pos] = i + e;
      }
  }
}
#ifndef HEART_ATTN_PF
#define HEART_ATTN_PF 4
#endif
#ifndef HEART_ATTN_OCC
#define HEART_ATTN_OCC 2  // waves per SIMD the register budget is sized for
#endif

template <int D, int BLK>
__global__ __launch_bounds__(BLK * 2, HEART_ATTN_OCC) void attn_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k,
    const uint16_t *__restrict__ v, uint16_t *__restrict__ out, long long qsb, long long qsh,
    long long qsn, long long ksb, long long ksh, long long ksn, long long vsb, long long vsh,
    long long vsn, long long osb, long long osh, long long osn, int H, int BH, int N, int Nb,
    const int *__restrict__ kept_idx, const int *__restrict__ kept_count, float scale_log2e,
    float *__restrict__ lse, const int *__restrict__ order, int n_items) {
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
  if (order) {
    // list position: runs of kOrderRun consecutive entries per XCD, XCDs interleaved
    const int xcd = (int)(blockIdx.x % kNumXcd);
    const long long slot = blockIdx.x / kNumXcd;
    const long long pos =
        (slot / kOrderRun) * (kNumXcd * kOrderRun) + xcd * kOrderRun + slot % kOrderRun;
    if (pos >= n_items) return;  // padding (whole workgroup, before any barrier)
    const int item = min(max(order[pos], 0), n_items - 1);
    bh = item / Nb;
    qb = item % Nb;
  } else {
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
  // A key block is consumed in NSL slices of 32 keys, software-pipelined.  The MFMAs of one
  // key block form a fixed stream of SEQ instructions:
  //   for sl = 0 .. NSL-1:  B(sl): S^T(sl+1), KS MFMAs on K fragments   (not for the last sl)
  //                         C(sl): O^T += V^T P^T(sl), NPV MFMAs on V^T fragments
  //   W: S^T(slice 0) of the NEXT key block, KS MFMAs
  // Every MFMA takes its A operand from a ring of PF registers filled by 16-byte LDS reads
  // that run PF stream positions ahead, across phase boundaries and across the loop
  // back-edge; only the two barriers (where the LDS contents change) restart the ring.
  // The instruction order written here is the intended issue order (sched_barrier fences).
  // After each MFMA comes a little VALU work that runs in its shadow:
  //   in B(sl): exponentials / bf16 rounding / row sum of a few elements of slice sl
  //   in C(sl): part of the maximum of S^T(sl+1); the rare move of the reference exponent
  //             follows the phase
  // and at most one staging operation for the next key block:
  //   K loads and V loads of half 0 in C(0) (in B(0) when NSL == 2); V loads of half 1 in C(NSL-2)
  //   barrier A before C(NSL-2): every wave has read all of sK and V^T half 0
  //   K stores and V^T half-0 stores in C(NSL-2)
  //   barrier B before W: every wave has read V^T half 1; new sK / half 0 visible
  //   V^T half-1 stores in W; they are first read after the next barrier A
  constexpr int NSL = BLK / 32;           // slices per key block
  constexpr int NPV = 2 * DT;             // MFMAs of one slice's O^T update
  constexpr int STEP = KS + NPV;
  constexpr int G_A = (NSL - 2) * STEP + KS;       // stream position of barrier A: C(NSL-2)
  constexpr int G_W = (NSL - 1) * STEP + NPV;      // stream position of barrier B: W
  constexpr int SEQ = G_W + KS;
  constexpr int PF = HEART_ATTN_PF < KS ? HEART_ATTN_PF : KS;  // LDS reads in flight ahead of the MFMAs
  static_assert(16 % KS == 0 && (NSL == 2 || NSL == 4) && SEQ % PF == 0 && PF <= KS &&
                    PF <= NPV, "stream layout");

  // A-operand fragment of stream position g (g >= SEQ: the next key block's stream)
  auto fetch = [&](int g) -> u32x4_t {
    g %= SEQ;
    const int sl = g / STEP, r = g % STEP;
    if (sl < NSL - 1) {
      if (r < KS)  // B(sl): K fragment of slice sl+1, k-step r
        return *reinterpret_cast<const u32x4_t *>(sK_rd + (sl + 1) * 32 * SK + r * 16);
      // C(sl): 8 keys of slice sl for MFMA m (s2 = m / DT, d tile m % DT): key positions
      // sl*32 + 16*s2 + 8*hf .. +7 (see header)
      const int m = r - KS;
      return *reinterpret_cast<const u32x4_t *>(sV_rd + (m % DT) * 32 * SV + sl * 32 + 16 * (m / DT));
    }
    if (r < NPV)  // C(NSL-1)
      return *reinterpret_cast<const u32x4_t *>(sV_rd + (r % DT) * 32 * SV + sl * 32 + 16 * (r / DT));
    return *reinterpret_cast<const u32x4_t *>(sK_rd + (r - NPV) * 16);  // W: slice 0
  };
  Frag8 ring[PF];
  // after the MFMA at position g: start the read for position g + PF unless a barrier
  // lies in between (then the ring is refilled after that barrier)
  auto prefetch_after = [&](int g) {
    const int t = g + PF;
    const bool crosses = (g < G_A && t >= G_A) || (g < G_W && t >= G_W);
    if (!crosses) ring[t % PF].u = fetch(t);
  };
  auto refill = [&](int g0) {
#pragma unroll
    for (int j = 0; j < PF; ++j) ring[(g0 + j) % PF].u = fetch(g0 + j);
  };

  f32x16_t sacc[2];  // S^T of the slice being exponentiated and of the next one
  Frag8 pf[2];       // P^T of the current slice: [s2] = rows 8*s2 .. 8*s2+7 of the accumulator

  // Weights of one slice relative to the reference exponent, rounded to bf16 for the second
  // contraction (the row sum adds the unrounded fp32 weights).  The work on the 8
  // element pairs of a lane is cut into 32 micro-ops of about 8 VALU cycles each (pair
  // p = u / 4: two FMAs, exponential, exponential, convert + row sum), because only about
  // 24 cycles of a wave's own VALU work hide behind one of its MFMAs and a slot that
  // exceeds that stalls the matrix pipeline: B slots take 3 micro-ops, C slots 2.
  float xt0 = 0.f, xt1 = 0.f;  // the pair in flight
  auto exp_uop = [&](const f32x16_t &x, int u, float m_sub) {
    const int r = 2 * (u >> 2), st = u & 3;
    // (the empty asm statements pin each result to its slot: without them the compiler
    // sinks the whole computation to its first use, out of the MFMA shadow)
    if (st == 0) {
      xt0 = __builtin_fmaf(x[r], scale_log2e, -m_sub);
      xt1 = __builtin_fmaf(x[r + 1], scale_log2e, -m_sub);
      asm volatile("" : "+v"(xt0), "+v"(xt1));
    } else if (st == 1) {
      xt0 = __builtin_amdgcn_exp2f(xt0);
      asm volatile("" : "+v"(xt0));
    } else if (st == 2) {
      xt1 = __builtin_amdgcn_exp2f(xt1);
      asm volatile("" : "+v"(xt1));
    } else {
      // (plain adds for the row sum: they co-issue with MFMAs, dot instructions do not)
      uint32_t pk = cvt_pk_bf16(xt0, xt1);
      l_run += xt0 + xt1;
      asm volatile("" : "+v"(pk), "+v"(l_run));
      pf[r / 8].u[(r % 8) / 2] = pk;
    }
  };
  constexpr int UB = 24 / KS;        // micro-ops per B slot: pairs 0..5 of the slice
  constexpr int UC = 8 / DT;         // micro-ops per C slot m < DT: pairs 6..7
  // B / W: S^T(slice sl) into sacc[sl & 1], stream positions g0 .. g0+KS-1; with_exp:
  // interleave the weights of slice sl-1.  extra(slot) injects staging work.
  auto qk_step = [&](int sl, int g0, bool with_exp, float m_sub, auto &&extra) {
    f32x16_t acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const f32x16_t &prev = sacc[(sl + 1) & 1];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[(g0 + ks) % PF].v, qf[ks].v, acc, 0, 0, 0);
      prefetch_after(g0 + ks);
      if (with_exp) {
#pragma unroll
        for (int u = 0; u < UB; ++u) exp_uop(prev, ks * UB + u, m_sub);
      }
      extra(ks);
      __builtin_amdgcn_sched_barrier(0);
    }
    sacc[sl & 1] = acc;
  };
  // keys past the end of a ragged last key block get no weight
  auto mask_slice = [&](f32x16_t &x, int sl, int nvalid) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = sl * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
      if (key >= nvalid) x[r] = -__builtin_inff();
    }
  };
  // maximum of one accumulator over this lane's 16 keys, in 4 partial steps so that it
  // can be spread over MFMA slots; step i folds elements 4i .. 4i+3
  auto max_part = [&](const f32x16_t &x, int i, float m) -> float {
    m = fmaxf(fmaxf(m, x[4 * i]), x[4 * i + 1]);       // v_max3_f32
    return fmaxf(fmaxf(m, x[4 * i + 2]), x[4 * i + 3]);  // v_max3_f32
  };
  // Finish the maximum of a slice (combine the two lanes of a query: lane l and l^32 are
  // exchanged with one v_permlane32_swap) and, rarely, move the reference exponent.
  // The reference only moves when the slice maximum exceeds it by more than the slack:
  // exponentials then stay below 2^slack and the accumulator rescale is skipped for
  // most slices.  A slice whose keys are all past the end has maximum -inf and never
  // moves it.  Returns the exponent to subtract (0 while every logit so far was masked).
  auto finish_max = [&](float m_loc) -> float {
    uint32_t sw0, sw1;
    swap_halves32(__float_as_uint(m_loc), sw0, sw1);
    m_loc = fmaxf(__uint_as_float(sw0), __uint_as_float(sw1));
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
  // C: O^T += V^T P^T(slice sl), stream positions g0 .. g0+NPV-1.  The first DT slots
  // finish the weights of the slice (pairs 6..7, consumed by the second half of the
  // MFMAs); with_max: the second half of the slots folds the maximum of S^T(sl+1), whose
  // MFMAs were issued before this phase and have drained by then.
  auto pv_step = [&](int sl, int g0, bool with_max, float m_sub, auto &&extra) -> float {
    float m_loc = -__builtin_inff();
    const f32x16_t &nx = sacc[(sl + 1) & 1];
    const f32x16_t &cur = sacc[sl & 1];
#pragma unroll
    for (int m = 0; m < NPV; ++m) {
      o[m % DT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[(g0 + m) % PF].v, pf[m / DT].v, o[m % DT], 0, 0, 0);
      prefetch_after(g0 + m);
      if (m < DT) {
#pragma unroll
        for (int u = 0; u < UC; ++u) exp_uop(cur, 24 + m * UC + u, m_sub);
      }
      if (with_max && m >= DT) {
#pragma unroll
        for (int i = 0; i < 4 / DT; ++i) m_loc = max_part(nx, (m - DT) * (4 / DT) + i, m_loc);
      }
      extra(m);
      __builtin_amdgcn_sched_barrier(0);
    }
    return m_loc;
  };
  auto no_extra = [](int) {};
  // maximum of slice 0 of a key block right after its S^T (prologue and W)
  auto slice0_max = [&](int nvalid) -> float {
    if (nvalid < BLK) mask_slice(sacc[0], 0, nvalid);
    float m_loc = -__builtin_inff();
#pragma unroll
    for (int i = 0; i < 4; ++i) m_loc = max_part(sacc[0], i, m_loc);
    return finish_max(m_loc);
  };

  float m_sub = 0.f;
  if (cnt > 0) {
    refill(G_W);
    qk_step(0, G_W, false, 0.f, no_extra);
    m_sub = slice0_max(min(BLK, N - j_cur * BLK));
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
        qk_step(sl + 1, sl * STEP, true, m_sub, [&](int ks) {
          if (NSL == 2 && sl == 0) {  // short key blocks: C(0) already stores, so load here
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
        // last slice: no S^T left to overlap the first 6 pairs of its weights with
#pragma unroll
        for (int u = 0; u < 24; ++u) exp_uop(sacc[sl & 1], u, m_sub);
      }
      if (sl == NSL - 2) {
        __syncthreads();  // barrier A
        refill(G_A);
      }
      // ---- C(sl) ----
      const int g_c = sl * STEP + (sl + 1 < NSL ? KS : 0);
      const float m_loc = pv_step(sl, g_c, sl + 1 < NSL, m_sub, [&](int m) {
        if (NSL > 2 && sl == 0) {  // K loads and V half-0 loads of the next key block, spread over the slots
#pragma unroll
          for (int it = 0; it < KCH; ++it)
            if (it * NPV / KCH == m) load_k1(kreg, it, kv_next);
          if (m >= NPV - 4 && v_mine(0)) load_v1(v0, v_it_of(0), m - (NPV - 4), kv_next);
        }
        if (sl == NSL - 2) {
          // K stores, spread; V^T half-0 stores (one word pair per slot); V loads, half 1
#pragma unroll
          for (int it = 0; it < KCH; ++it)
            if (it * NPV / KCH == m) store_k1(kreg, it);
          if (m >= NPV - 4 && v_mine(0)) store_vt1(v0, v_it_of(0), m - (NPV - 4));
          if (m >= NPV - 4 && v_mine(1)) load_v1(v1, v_it_of(1), m - (NPV - 4), kv_next);
        }
      });
      if (sl + 1 < NSL) m_sub = finish_max(m_loc);
    }
    // barrier B
    __syncthreads();
    refill(G_W);
    // ---- W: S^T(slice 0) of the next key block, with the V^T half-1 stores ----
    qk_step(0, G_W, false, 0.f, [&](int ks) {
      if (ks < 4 && v_mine(1)) store_vt1(v1, v_it_of(1), ks);
    });
    if (KS < 4 && v_mine(1)) {
#pragma unroll
      for (int wd = KS; wd < 4; ++wd) store_vt1(v1, v_it_of(1), wd);
    }
    m_sub = slice0_max(nvalid_next);
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
                         float *lse, int *order, hipStream_t st) {
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
  const long long n_items = (long long)BH * Nb;
  constexpr long long kGroup = kNumXcd * kOrderRun;
  const long long grid = order ? (n_items + kGroup - 1) / kGroup * kGroup
                               : (long long)BH * ((Nb + kNumXcd - 1) / kNumXcd) * kNumXcd;
  if (grid > 0x7fffffffLL) return fail(HEART_EUNSUPPORTED, "heart_block_sparse_attn: grid too large");
  if (order) {
    hipLaunchKernelGGL(attn_order_kernel, dim3(1), dim3(256), 0, st, kept_count, (int)n_items, Nb,
                       order);
    if (int rc = check_launch("attn_order_kernel")) return rc;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(BLK * 2), lds, st,
                     (const uint16_t *)q, (const uint16_t *)k, (const uint16_t *)v,
                     (uint16_t *)out, s.q_stride[0], s.q_stride[1], s.q_stride[2], s.k_stride[0],
                     s.k_stride[1], s.k_stride[2], s.v_stride[0], s.v_stride[1], s.v_stride[2],
                     s.o_stride[0], s.o_stride[1], s.o_stride[2], s.H, BH, s.N, Nb, kept_idx,
                     kept_count, scale_log2e, lse, (const int *)order, (int)n_items);
  return check_launch("attn_kernel");
}

int launch_attn(const heart_shape &s, const void *q, const void *k, const void *v,
                const int *kept_idx, const int *kept_count, float scale, void *out, float *lse,
                int *order, hipStream_t st) {
  // the kernel addresses one head's rows through 32-bit buffer offsets
  const long long lim = 0xffffffffLL;
  const long long rows = (long long)s.N + 2 * s.block;  // staging may address a few rows past N
  if (rows * s.q_stride[2] * 2 > lim || rows * s.k_stride[2] * 2 > lim ||
      rows * s.v_stride[2] * 2 > lim)
    return fail(HEART_EUNSUPPORTED,
                "heart_block_sparse_attn: (N + 2*block) * token stride * 2 bytes must stay "
                "below 4 GiB");
  if (s.D == 128 && s.block == 128)
    return launch_attn_t<128, 128>(s, q, k, v, kept_idx, kept_count, scale, out, lse, order, st);
  if (s.D == 64 && s.block == 128)
    return launch_attn_t<64, 128>(s, q, k, v, kept_idx, kept_count, scale, out, lse, order, st);
  if (s.D == 64 && s.block == 64)
    return launch_attn_t<64, 64>(s, q, k, v, kept_idx, kept_count, scale, out, lse, order, st);
  return fail(HEART_EUNSUPPORTED, "heart_block_sparse_attn: unsupported (D, block) = (%d, %d)",
              s.D, s.block);
}

}  // namespace heart
