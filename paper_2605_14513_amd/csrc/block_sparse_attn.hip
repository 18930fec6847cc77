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
// K and V never pass through registers on their way in: they are copied from global
// memory straight into LDS by 16-byte LDS-direct buffer loads (rows past the end of the
// sequence are out of range for the buffer descriptor and arrive as zeros, with no
// branch and no address clamping).  Both tiles stay row-major [key][d] and unpadded (a
// direct load fills 1 KB of consecutive LDS); the 16-byte chunk index is XOR-swizzled
// with the row so that fragment reads are bank-conflict free.  K fragments are plain
// 16-byte reads; V^T fragments come from the transposing LDS read ds_read_b64_tr_b16.
//
// The kept key blocks are consumed as one stream of 32-key slices.  K and V arrive in
// double-buffered stages of 64 rows, loaded two slices ahead; V stages are skewed by one
// slice against K stages so that one workgroup barrier per 64 keys retires both (see
// the comment at the loop).  The softmax scale and log2(e) are folded into Q once, and
// the S^T accumulators start from minus the running reference exponent, so an
// accumulator goes into the exponential as it is.
//
// Scheduling.  Kept counts range from 1 to Nb per row and the densities of the heads
// differ a lot, the K/V of one head (16.8 MB at N = 32760, D = 128) is far larger than
// the 4 MB L2 of an XCD, and every query block re-reads its kept K/V blocks.  With a
// caller-provided workspace the launch therefore follows a plan (attn_order_kernel,
// attn_plan_kernel): whole heads are assigned to the 8 XCDs (greedily, heaviest head
// first, by total kept count), each XCD walks through its heads one at a time -- all
// its workgroups then share one head's K/V through that XCD's L2, and only 8 heads are
// in flight in the memory-side cache -- and inside a head the rows with the longest
// kept lists start first (stable counting sort on 32 count classes), so that no long
// row starts late.  A workgroup takes the next item of its XCD's list with an atomic
// counter; when that list is exhausted it takes from another XCD's list, which levels
// whatever imbalance the head assignment left.  Without a workspace an XCD works on a
// contiguous eighth of the query blocks of every head, in index order.
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
typedef __attribute__((ext_vector_type(4))) short s16x4_t;

union Frag8 {
  u32x4_t u;
  bf16x8_t v;
};

__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
  f32x2_t f = {lo, hi};
  bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
  return __builtin_bit_cast(uint32_t, b);
}

// buffer descriptor over one head's rows: offsets >= bytes read as zero
__device__ __forceinline__ __amdgpu_buffer_rsrc_t head_rsrc(const uint16_t *base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(base), 0, (int)bytes, 0x00020000);
}

// the same descriptor as four words in scalar registers, for hand-written buffer instructions
__device__ __forceinline__ u32x4_t head_rsrc_words(const uint16_t *base, uint32_t bytes) {
  const uint64_t a = reinterpret_cast<uint64_t>(base);
  u32x4_t r;
  r.x = __builtin_amdgcn_readfirstlane((uint32_t)a);
  r.y = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32) & 0xffffu);
  r.z = __builtin_amdgcn_readfirstlane(bytes);
  r.w = 0x00020000u;
  return r;
}

constexpr int kNumXcd = 8;
constexpr int kStageRows = 64;    // key rows per K / V stage buffer (two 32-key slices)
constexpr int kOrderClasses = 32;   // count classes of the per-head sort
constexpr int kPlanHdr = 24;        // plan header: 8 cursors, 8 list lengths, 8 list offsets
constexpr int kPlanMaxHeads = 1024; // beyond this heads are dealt to the XCDs round-robin
// Plan layout (ints): [0,8) cursors, [8,16) items per XCD list, [16,24) offset of each
// XCD's heads in the head table, [24, 24+BH) head table (the heads of XCD 0 in the order
// it walks them, then those of XCD 1, ...), [24+BH, 24+2BH) total kept count per head,
// then seq[BH*Nb], head-major: seq[head*Nb + p] = the head's p-th item in launch order
// (item = head * Nb + query block).  Entry i of an XCD's list is item p = i % Nb of its
// (i / Nb)-th head.

// One workgroup, after attn_order_kernel: heads ranked by total kept count, greedy
// assignment of heads (heaviest first) to the least loaded XCD, head table, cursors reset.
__global__ __launch_bounds__(256) void attn_plan_kernel(int BH, int Nb, int *__restrict__ plan) {
  __shared__ int w_head[kPlanMaxHeads];
  __shared__ int sorted[kPlanMaxHeads];
  __shared__ int xcd_of[kPlanMaxHeads], rank_of[kPlanMaxHeads];
  __shared__ int n_heads[kNumXcd], off[kNumXcd];
  const int t = threadIdx.x;
  if (BH <= kPlanMaxHeads) {
    for (int bh = t; bh < BH; bh += 256) w_head[bh] = plan[kPlanHdr + BH + bh];
    __syncthreads();
    // rank by (work descending, index ascending)
    for (int bh = t; bh < BH; bh += 256) {
      const int w = w_head[bh];
      int r = 0;
      for (int j = 0; j < BH; ++j) {
        const int wj = w_head[j];
        r += (wj > w) || (wj == w && j < bh);
      }
      sorted[r] = bh;
    }
    __syncthreads();
    if (t < 64) {
      // greedy on one wavefront: lane x < 8 holds the load of XCD x (scaled to 32 bits;
      // +Nb per head: a row costs about one key block of fixed work); the minimum is a
      // register-only wave reduction, so a step costs no LDS round trips
      int shift = 0;
      while ((((long long)BH * Nb * (Nb + 1)) >> shift) > 0x3fffffffLL) ++shift;
      uint32_t load = t < kNumXcd ? 0u : 0xffffffffu;
      int nh = 0;
      for (int r = 0; r < BH; ++r) {
        const int bh = sorted[r];
        const uint32_t m = wave_min_u32(load);
        const unsigned long long is_min = __ballot(load == m);
        const int best = __ffsll((long long)is_min) - 1;  // least loaded XCD, lowest id on ties
        if (t == best) {
          xcd_of[bh] = best;
          rank_of[bh] = nh++;
          load += (uint32_t)(((long long)w_head[bh] + Nb) >> shift);
        }
      }
      if (t < kNumXcd) n_heads[t] = nh;
    }
  } else {
    if (t < kNumXcd) n_heads[t] = BH / kNumXcd + (t < BH % kNumXcd ? 1 : 0);
  }
  __syncthreads();
  if (t == 0) {
    int run = 0;
    for (int x = 0; x < kNumXcd; ++x) {
      off[x] = run;
      run += n_heads[x];
    }
  }
  __syncthreads();
  if (t < kNumXcd) {
    plan[t] = 0;
    plan[kNumXcd + t] = n_heads[t] * Nb;
    plan[2 * kNumXcd + t] = off[t];
  }
  for (int bh = t; bh < BH; bh += 256) {
    const int x = BH <= kPlanMaxHeads ? xcd_of[bh] : bh % kNumXcd;
    const int r = BH <= kPlanMaxHeads ? rank_of[bh] : bh / kNumXcd;
    plan[kPlanHdr + off[x] + r] = bh;
  }
}

// One workgroup per head: the Nb items of the head, longest kept list first, into the
// head's range of seq, and the head's total kept count.  Stable counting sort by count class (class 0 = the longest
// rows): thread t owns a contiguous segment of the items and one column of the class
// histogram, so that items of a class keep their natural order.  The counts are first
// read once, coalesced and all in flight, and kept as class bytes in LDS when they fit
// (kStaged); otherwise the segments are read from global memory.
constexpr int kOrderStagedMax = 96 * 1024;  // items whose classes fit next to the histogram
template <bool kStaged>
__global__ __launch_bounds__(256) void attn_order_kernel(const int *__restrict__ kept_count, int BH,
                                                         int Nb, uint32_t mult,
                                                         int *__restrict__ plan) {
  const int n = Nb;
  const int item0 = blockIdx.x * Nb;
  kept_count += item0;
  int *order = plan + kPlanHdr + 2 * BH + item0;
  __shared__ int total;
  if (threadIdx.x == 0) total = 0;
  __shared__ int hist[kOrderClasses][256];
  __shared__ int scan[256];
  extern __shared__ unsigned char cls_lds[];  // [n] when kStaged
  const int t = threadIdx.x;
  const int per = (n + 255) / 256;
  const int i0 = min(n, t * per), i1 = min(n, i0 + per);
  // class of a count c in [0, Nb]: (kOrderClasses-1) - floor(c * mult / 2^16) with
  // mult = floor((kOrderClasses-1) * 2^16 / Nb) from the host (no integer division here)
  auto cls = [&](int c) -> int {
    c = min(max(c, 0), Nb);
    return (kOrderClasses - 1) - (int)(((uint32_t)c * mult) >> 16);
  };
  auto cls_of = [&](int i) -> int { return kStaged ? (int)cls_lds[i] : cls(kept_count[i]); };
#pragma unroll
  for (int b = 0; b < kOrderClasses; ++b) hist[b][t] = 0;
  __syncthreads();  // `total` is zero before any wavefront adds to it
  if (kStaged) {
#pragma unroll 16
    for (int i = t; i < n; i += 256) cls_lds[i] = (unsigned char)cls(kept_count[i]);
    __syncthreads();
  }
  for (int i = i0; i < i1; ++i) hist[cls_of(i)][t] += 1;
  {
    int w = 0;
#pragma unroll 4
    for (int i = t; i < n; i += 256) w += min(max(kept_count[i], 0), Nb);
    w = wave_sum_i32(w);
    if ((t & 63) == 0) atomicAdd(&total, w);
  }
  __syncthreads();
  if (t == 0) plan[kPlanHdr + BH + blockIdx.x] = total;
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
  for (int i = i0; i < i1; ++i) {
    const int b = cls_of(i);
    const int pos = hist[b][t];
    hist[b][t] = pos + 1;
    order[pos] = item0 + i;
  }
}

// kExact (the default of the ABI): Q stays as it is and every logit is scaled in fp32 (one more
// multiply per logit); the error is then the bf16 rounding of the weights and of the output
// for any input scale.  !kExact (HEART_ATTN_FOLD_SCALE): the softmax scale is folded into Q
// once (one more bf16 rounding of the query; the error grows with the cube of the input scale,
// inside the budget for inputs of unit scale) and no per-logit multiply is left.
#ifndef HEART_ATTN_PF
#define HEART_ATTN_PF 4  // LDS fragment reads in flight ahead of the MFMAs
#endif
#ifndef HEART_ATTN_OCC
#define HEART_ATTN_OCC 2  // waves per SIMD the register budget is sized for
#endif

template <int D, int BLK, bool kExact>
__global__ __launch_bounds__(BLK * 2, HEART_ATTN_OCC) void attn_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k,
    const uint16_t *__restrict__ v, uint16_t *__restrict__ out, long long qsb, long long qsh,
    long long qsn, long long ksb, long long ksh, long long ksn, long long vsb, long long vsh,
    long long vsn, long long osb, long long osh, long long osn, int H, int BH, int N, int Nb,
    const int *__restrict__ kept_idx, const int *__restrict__ kept_count, float scale_log2e,
    float *__restrict__ lse, int *__restrict__ plan) {
  constexpr int NT = BLK * 2;            // threads
  constexpr int NW = NT / 64;            // wavefronts
  constexpr int DT = D / 32;             // 32-wide d tiles of the output
  constexpr int KS = D / 16;             // k-steps of the first contraction
  constexpr int CPR = D / 8;             // 16-byte chunks per token row
  constexpr int ROWB = D * 2;            // bytes of a token row in LDS (no padding)
  constexpr int RPB = 16 / CPR;          // rows per 256 bytes (one pass over the 64 banks)
  constexpr int TILE_B = kStageRows * ROWB;  // bytes of one K or V stage buffer
  constexpr int RPI = 64 / CPR;          // rows one LDS-direct load instruction covers
  constexpr int IPW = kStageRows / RPI / NW;  // such instructions per wavefront and tile
  constexpr int NSL = BLK / 32;          // 32-key slices per key block
  constexpr int SO = D + 8;              // LDS row stride of the output staging (elements)
  // kExact: S^T comes out of the matrix cores in raw logit units and is multiplied by
  // scale * log2(e) in fp32 as soon as it is complete (in slots of the MFMA stream that have
  // VALU time to spare: where the maximum is folded), so that from there on both variants
  // hold logits in log2 units relative to the reference exponent.  The accumulators start
  // from -m_ref, which kExact therefore converts back to raw units (kInitScale).  The running
  // reference may lag the maximum by 8 log2 units.
  const float kInitScale = kExact ? 1.f / scale_log2e : 1.f;
  constexpr float kRescaleSlack = 8.f;
  static_assert(NW % 2 == 0 && IPW >= 1 && (NSL == 2 || NSL == 4), "tile layout");

  // LDS: [K stage 0][K stage 1][V stage 0][V stage 1], reused for the output at the end
  extern __shared__ __align__(1024) unsigned char smem[];
  const uint32_t smem_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)smem;

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int l32 = lane & 31, hf = lane >> 5;

  // ---- state of the item (head, query block) being processed; set by begin_item ---------
  int bh = 0, qb = 0, b = 0, h = 0, qrow = 0, cnt = 0;
  const int *idx = kept_idx;
  __amdgpu_buffer_rsrc_t q_rs = head_rsrc(q, 0);
  u32x4_t k_rs = head_rsrc_words(k, 0), v_rs = head_rsrc_words(v, 0);
  const uint32_t k_row_bytes = (uint32_t)ksn * 2u, v_row_bytes = (uint32_t)vsn * 2u;

  // ---- per-lane constants of the LDS layout ---------------------------------------------
  // Chunk c (16 bytes) of tile row r is stored at chunk position c ^ f(r):
  //   K: f(r) = (r / RPB) % CPR      -- the 16 rows a quarter-wave reads with one
  //                                     ds_read_b128 (same chunk, consecutive rows) fall
  //                                     into 16 distinct 4-bank groups
  //   V: f(r) = 4 * ((r / RPB) % (CPR/4)) -- the 4 rows x 4 chunks that 32 lanes read with
  //                                     one transposing read fall into distinct groups
  // K fragment of k-step ks (A operand of S^T): row l32 of the slice, chunk 2 ks + hf.
  uint32_t koff[KS];
  {
    const int fk = (l32 / RPB) % CPR;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) koff[ks] = (uint32_t)(l32 * ROWB + (((2 * ks + hf) ^ fk) * 16));
  }
  // V^T fragment (A operand of O^T += V^T P^T) through ds_read_b64_tr_b16: within 16 lanes,
  // lane s supplies the address of 4 consecutive d of one key (key s/4, d chunk s%4) and
  // lane i receives d = i of keys 0..3.  A fragment (8 keys) is two such reads: keys
  // 16 s2 + 4 hf + 0..3 and 16 s2 + 8 + 4 hf + 0..3 of the slice, the order in which the
  // accumulator of S^T holds them.
  uint32_t voff[DT];
  {
    const int s = lane & 15, g16 = (lane >> 4) & 1;
    const int rowv = 4 * hf + (s >> 2);
    const int fv4 = (rowv / RPB) % (CPR / 4);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
      voff[dt] = (uint32_t)(rowv * ROWB + ((4 * (dt ^ fv4) + 2 * g16 + ((s & 3) >> 1)) * 16) +
                            (s & 1) * 8);
  }
  // LDS-direct loads: one instruction moves 16 bytes per lane to 1 KB of consecutive LDS
  // (RPI rows); lane l lands at chunk position l % CPR of row l / CPR and therefore fetches
  // global chunk (l % CPR) ^ f(row).  Wavefront w issues instructions w*IPW .. w*IPW+IPW-1
  // of a tile.  Rows past the end of the sequence are out of range for the descriptor and
  // arrive as zeros.
  uint32_t kdma[IPW], vdma;
  {
    const int drow = lane / CPR, dp = lane % CPR;
#pragma unroll
    for (int ii = 0; ii < IPW; ++ii) {
      const int r = (wave * IPW + ii) * RPI + drow;
      kdma[ii] = (uint32_t)drow * k_row_bytes + (uint32_t)((dp ^ ((r / RPB) % CPR)) * 16);
    }
    vdma = (uint32_t)drow * v_row_bytes + (uint32_t)((dp ^ (4 * ((drow / RPB) % (CPR / 4)))) * 16);
  }
  // tile `buf` of K (is_v = 0) or V (is_v = 1): instruction ii of this wavefront; the
  // first 32 rows of the tile come from key rows key_a.., the last 32 from key_b..
  auto dma = [&](int is_v, int ii, int buf, int key_a, int key_b) __attribute__((always_inline)) {
    const int half = wave / (NW / 2), wi = wave % (NW / 2);
    const int krow = (half ? key_b : key_a) + (wi * IPW + ii) * RPI;
    const uint32_t voffset =
        is_v ? vdma + (uint32_t)krow * v_row_bytes : kdma[ii] + (uint32_t)krow * k_row_bytes;
    const uint32_t dst = smem_lds + (uint32_t)((2 * is_v + buf) * TILE_B + (wave * IPW + ii) * 1024);
    // (the compiler does not see this instruction's LDS write, so it adds no waits of
    // its own: completion is awaited explicitly before the barrier that publishes the tile.
    // The LDS destination travels in M0, which the statement saves and restores: the
    // compiler is free to keep values of its own there)
    uint32_t m0_saved;
    if (is_v)
      asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\t"
                   "buffer_load_dwordx4 %2, %3, 0 offen lds\n\ts_mov_b32 m0, %0"
                   : "=&s"(m0_saved) : "s"(dst), "v"(voffset), "s"(v_rs) : "memory");
    else
      asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\t"
                   "buffer_load_dwordx4 %2, %3, 0 offen lds\n\ts_mov_b32 m0, %0"
                   : "=&s"(m0_saved) : "s"(dst), "v"(voffset), "s"(k_rs) : "memory");
  };

  Frag8 qf[KS];      // Q fragments (B operand of S^T = K Q^T), kept in registers
  f32x16_t o[DT];    // O^T accumulators
  float m_ref = 0.f; // reference exponent (log2 domain) of the running sums
  // S^T accumulators start from -m_ref instead of zero, so they hold logits relative to
  // the reference exponent and go into the exponential as they are
  f32x16_t cinit;
  float l_run = 0.f;  // running sum over this lane's keys, relative to m_ref
  auto begin_item = [&](int item) __attribute__((always_inline)) {
    bh = item / Nb;
    qb = item % Nb;
    b = bh / H;
    h = bh % H;
    q_rs = head_rsrc(q + b * qsb + h * qsh, (uint32_t)(N * qsn * 2));
    k_rs = head_rsrc_words(k + b * ksb + h * ksh, (uint32_t)(N * ksn * 2));
    v_rs = head_rsrc_words(v + b * vsb + h * vsh, (uint32_t)(N * vsn * 2));
    qrow = qb * BLK + wave * 32 + l32;
    const uint32_t q_off = (uint32_t)qrow * ((uint32_t)qsn * 2u) + (uint32_t)hf * 16u;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      qf[ks].u = __builtin_amdgcn_raw_buffer_load_b128(q_rs, q_off + ks * 32, 0, 0);
    if constexpr (!kExact) {
      // fold the softmax scale and log2(e) into Q once: S^T then comes out of the matrix
      // cores in log2 units and no per-logit multiply is left on the VALU
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int w = 0; w < 4; ++w)
          qf[ks].u[w] = cvt_pk_bf16(bf16lo(qf[ks].u[w]) * scale_log2e, bf16hi(qf[ks].u[w]) * scale_log2e);
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
    m_ref = -__builtin_inff();
#pragma unroll
    for (int r = 0; r < 16; ++r) cinit[r] = 0.f;
    l_run = 0.f;
    const size_t row = (size_t)bh * Nb + qb;
    cnt = min(kept_count[row], Nb);
    idx = kept_idx + row * Nb;
  };

  // The kept blocks are consumed as one sequence of 32-key slices.  Kept indices are
  // clamped into [0, Nb) so that a bad list cannot leave the tensors; entries past the
  // end of the list repeat the last one (their data is never used).
  auto kept = [&](int e) -> int { return min(max(idx[min(max(e, 0), cnt - 1)], 0), Nb - 1); };
  // The loop body covers 4 slices starting at slice s0 (list entry eb) and looks ahead up
  // to slice s0+7: the block indices of entries eb .. eb+NE-1 are held in scalar registers
  // and advance by EPB entries per body.  New entries are loaded right before a barrier:
  // a scalar load can only be awaited together with all outstanding LDS reads, and there
  // the pipeline of LDS reads is drained anyway.
  constexpr int EPB = 4 / NSL;      // list entries per loop body
  constexpr int NE = 7 / NSL + 1;   // entries a body can refer to
  int jb[NE];
  // first key row of slice s0 + rel (rel = 0 .. 7) of the current body
  auto key_of = [&](int rel) -> int { return jb[rel / NSL] * BLK + (rel % NSL) * 32; };

  // ---- the stream of MFMAs -----------------------------------------------------------------
  // The kept key blocks are one sequence of 32-key slices sigma = 0, 1, ...  Per slice:
  //   B(sigma): S^T(sigma+1), KS MFMAs on K fragments; in their shadow the exponentials,
  //             bf16 rounding and row sum of slice sigma
  //   C(sigma): O^T += V^T P^T(sigma), NPV MFMAs on V^T fragments; in their shadow the
  //             maximum of S^T(sigma+1); the rare move of the reference exponent follows
  // K and V arrive in stages of 64 rows (two slices), double-buffered, by LDS-direct
  // loads that are issued two slices before their first use.  K stage i holds slices
  // (2i, 2i+1), V stage i holds slices (2i-1, 2i): with this skew the last read of a K
  // stage (in B(2i)) and of a V stage (in C(2i)) are adjacent, ONE barrier per two slices
  // retires both, and every B phase has an S^T to overlap its exponentials with.
  //   ... B(2i) C(2i) | wait for own loads, barrier | B(2i+1) [issue stage i+2] C(2i+1) ...
  // The loop body covers 4 slices (2 stages) so that buffer indices are constants.  Every
  // MFMA takes its A operand from a ring of PF registers filled by LDS reads that run PF
  // stream positions ahead, across phases and the loop back-edge; only the barriers
  // restart the ring.  The instruction order written here is the intended issue order.
  constexpr int NPV = 2 * DT;             // MFMAs of one slice's O^T update
  constexpr int STEP = KS + NPV;
  constexpr int SEQ = 4 * STEP;
  constexpr int G_B0 = STEP, G_B1 = 3 * STEP;  // stream positions right after the barriers
  constexpr int PF = HEART_ATTN_PF < KS ? HEART_ATTN_PF : KS;
  static_assert(16 % KS == 0 && SEQ % PF == 0 && PF <= KS && PF <= NPV, "stream layout");

  // A-operand fragment of stream position g.  Slice q (0..3) of the body: its V and the
  // K of slice q+1 both live in buffer ((q+1)/2)%2, rows ((q+1)%2)*32.
  auto fetch = [&](int g) __attribute__((always_inline)) -> u32x4_t {
    g %= SEQ;
    const int n = g / STEP + 1, r = g % STEP;
    const int buf = (n >> 1) & 1, row0 = (n & 1) * 32;
    if (r < KS)
      return *reinterpret_cast<const u32x4_t *>(smem + buf * TILE_B + row0 * ROWB + koff[r]);
    const int m = r - KS;
    const unsigned char *p = smem + (2 + buf) * TILE_B + (row0 + 16 * (m / DT)) * ROWB + voff[m % DT];
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4_t *)(p));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4_t *)(p + 8 * ROWB));
    const u32x2_t a = __builtin_bit_cast(u32x2_t, lo), c = __builtin_bit_cast(u32x2_t, hi);
    return u32x4_t{a.x, a.y, c.x, c.y};
  };
  Frag8 ring[PF];
  auto prefetch_after = [&](int g) __attribute__((always_inline)) {
    const int t2 = g + PF;
    const bool crosses = (g < G_B0 && t2 >= G_B0) || (g < G_B1 && t2 >= G_B1);
    if (!crosses) ring[t2 % PF].u = fetch(t2);
  };
  auto refill = [&](int g0) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < PF; ++j) ring[(g0 + j) % PF].u = fetch(g0 + j);
  };

  f32x16_t sacc[2];  // S^T of the slice being exponentiated and of the next one
  Frag8 pf[2];       // P^T of the current slice: [s2] = rows 8*s2 .. 8*s2+7 of the accumulator

  // Weights of one slice: exp2 of the accumulator (already relative to the reference
  // exponent), rounded to bf16 for the second contraction; the row sum adds the unrounded
  // fp32 weights.  The 8 element pairs of a lane are 24 micro-ops (exponential,
  // exponential, convert + row sum) that are pinned, a few at a time, behind MFMAs: only
  // about 24 cycles of a wave's own VALU work hide behind one of its MFMAs, and a slot
  // that exceeds that stalls the matrix pipeline.
  float xt0 = 0.f, xt1 = 0.f;  // the pair in flight
  auto exp_uop = [&](const f32x16_t &x, int u) __attribute__((always_inline)) {
    const int r = 2 * (u / 3), st = u % 3;
    // (the empty asm statements pin each result to its slot: without them the compiler
    // sinks the whole computation to its first use, out of the MFMA shadow)
    if (st == 0) {
      xt0 = __builtin_amdgcn_exp2f(x[r]);
      asm volatile("" : "+v"(xt0));
    } else if (st == 1) {
      xt1 = __builtin_amdgcn_exp2f(x[r + 1]);
      asm volatile("" : "+v"(xt1));
    } else {
      // (plain adds for the row sum: they co-issue with MFMAs, dot instructions do not)
      uint32_t pk = cvt_pk_bf16(xt0, xt1);
      l_run += xt0 + xt1;
      asm volatile("" : "+v"(pk), "+v"(l_run));
      pf[r / 8].u[(r % 8) / 2] = pk;
    }
  };
  constexpr int UB = 16 / KS;        // micro-ops per B slot (16 of the 24 in B)
  constexpr int UC = 8 / DT;         // micro-ops per C slot m < DT (the other 8)
  // B: S^T into sacc[dst], stream positions g0 .. g0+KS-1, with the weights of the slice in
  // sacc[dst ^ 1] interleaved.  extra(slot) injects the loads of a later stage.
  auto qk_step = [&](int dst, int g0, auto &&extra) __attribute__((always_inline)) {
    f32x16_t acc;
    const f32x16_t &prev = sacc[dst ^ 1];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[(g0 + ks) % PF].v, qf[ks].v,
                                                    ks == 0 ? cinit : acc, 0, 0, 0);
      prefetch_after(g0 + ks);
#pragma unroll
      for (int u = 0; u < UB; ++u) exp_uop(prev, ks * UB + u);
      extra(ks);
      __builtin_amdgcn_sched_barrier(0);
    }
    sacc[dst] = acc;
  };
  // keys at or past row `nvalid` of the slice (end of a ragged last key block) get no weight
  auto mask_slice = [&](f32x16_t &x, int nvalid) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = 8 * (r >> 2) + 4 * hf + (r & 3);
      if (key >= nvalid) x[r] = -__builtin_inff();
    }
  };
  // maximum of one accumulator over this lane's 16 keys, in 4 partial steps so that it
  // can be spread over MFMA slots; step i folds elements 4i .. 4i+3
  auto max_part = [&](const f32x16_t &x, int i, float m) __attribute__((always_inline)) -> float {
    m = fmaxf(fmaxf(m, x[4 * i]), x[4 * i + 1]);       // v_max3_f32
    return fmaxf(fmaxf(m, x[4 * i + 2]), x[4 * i + 3]);  // v_max3_f32
  };
  // After the maximum m_rel of a slice (over this lane's keys, relative to the reference
  // exponent): the reference only moves when some logit exceeds it by more than the slack,
  // so exponentials stay below 2^slack and almost every slice takes the short path (one
  // compare per lane and a wave-wide vote).  The long path combines the two lanes of each
  // query (lane l and l^32, one v_permlane32_swap), moves the reference of the queries
  // that need it, rescales their sums, makes the not yet exponentiated slice x relative to
  // the new reference, and rewrites the accumulator start values.  A slice whose keys are
  // all past the end has maximum -inf and never moves the reference.
  auto finish_max = [&](float m_rel, f32x16_t &x) __attribute__((always_inline)) {
    const bool first = m_ref == -__builtin_inff();
    if (__any(m_rel > kRescaleSlack || (first && m_rel > -__builtin_inff()))) {
      uint32_t sw0, sw1;
      swap_halves32(__float_as_uint(m_rel), sw0, sw1);
      m_rel = fmaxf(__uint_as_float(sw0), __uint_as_float(sw1));
      const bool bump = m_rel > kRescaleSlack || (first && m_rel > -__builtin_inff());
      const float base = first ? 0.f : m_ref;       // what the accumulators are relative to
      const float delta = bump ? m_rel : 0.f;
      const float m_new = bump ? base + m_rel : m_ref;
      const float alpha = bump ? __builtin_amdgcn_exp2f(m_ref - m_new) : 1.f;  // 0 the first time
      l_run *= alpha;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
#pragma unroll
      for (int r = 0; r < 16; ++r) x[r] -= delta;
      m_ref = m_new;
      const float c0 = m_ref == -__builtin_inff() ? 0.f : -m_ref * kInitScale;
#pragma unroll
      for (int r = 0; r < 16; ++r) cinit[r] = c0;
    }
  };
  // C: O^T += V^T P^T of the slice in sacc[cur], stream positions g0 .. g0+NPV-1.  The first DT slots finish the weights of the slice (consumed by the
  // second half of the MFMAs); the second half of the slots folds the maximum of
  // sacc[cur ^ 1], whose MFMAs were issued before this phase and have drained by then.
  auto pv_step = [&](int cur, int g0) __attribute__((always_inline)) -> float {
    float m_loc = -__builtin_inff();
    f32x16_t &nx = sacc[cur ^ 1];
    const f32x16_t &cx = sacc[cur];
#pragma unroll
    for (int m = 0; m < NPV; ++m) {
      o[m % DT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[(g0 + m) % PF].v, pf[m / DT].v, o[m % DT], 0, 0, 0);
      prefetch_after(g0 + m);
      if (m < DT) {
#pragma unroll
        for (int u = 0; u < UC; ++u) exp_uop(cx, 16 + m * UC + u);
      }
      if (m >= DT) {
#pragma unroll
        for (int i = 0; i < 4 / DT; ++i) {
          const int part = (m - DT) * (4 / DT) + i;
          if constexpr (kExact) {
#pragma unroll
            for (int e = 0; e < 4; ++e) nx[4 * part + e] *= scale_log2e;  // raw logits -> log2 units
          }
          m_loc = max_part(nx, part, m_loc);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    return m_loc;
  };
  auto no_extra = [](int) {};
  auto wait_loads_and_barrier = [&]() __attribute__((always_inline)) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  };

  // ---- work loop --------------------------------------------------------------------------
  // With a plan the workgroups are persistent (two per CU): each takes items from the list
  // of its XCD (workgroup ids are dealt round-robin to the XCDs) with an atomic cursor and,
  // once that list is empty, from the other XCDs' lists.  Without a plan a workgroup
  // processes the one item its id maps to.
  __shared__ int s_item;
  const int x0 = (int)(blockIdx.x % kNumXcd);
  const int len0 = plan ? plan[kNumXcd + x0] : 0;
  const int off0 = plan ? plan[2 * kNumXcd + x0] : 0;
  // (thread 0) entry i of XCD x's list: item p = i % Nb of its (i / Nb)-th head
  const int *head_tbl = plan + kPlanHdr, *seq = plan + kPlanHdr + 2 * BH;
  int cached_r = -1, cached_head = 0;  // the own list's head currently being walked
  auto entry = [&](int x, int off_x, int i) -> int {
    const int r = i / Nb, p = i - r * Nb;
    int head;
    if (x == x0 && r == cached_r) {
      head = cached_head;
    } else {
      head = head_tbl[off_x + r];
      if (x == x0) cached_r = r, cached_head = head;
    }
    return seq[head * Nb + p];
  };
  // (thread 0) item for cursor value i_own of the own list, else from another list, else -1
  auto take = [&](int i_own) -> int {
    if (i_own >= 0 && i_own < len0) return entry(x0, off0, i_own);
    for (int k2 = 1; k2 < kNumXcd; ++k2) {
      const int x = (x0 + k2) % kNumXcd;
      const int len = plan[kNumXcd + x];
      if (len <= 0) continue;
      const int i = atomicAdd(&plan[x], 1);
      if (i < len) return entry(x, plan[2 * kNumXcd + x], i);
    }
    return -1;
  };
  int item = -1;
  if (plan) {
    if (t == 0) s_item = take(len0 > 0 ? atomicAdd(&plan[x0], 1) : -1);
    __syncthreads();
    item = __builtin_amdgcn_readfirstlane(s_item);
  } else {
    // XCD x takes the x-th eighth of the query blocks of every head, heads in order
    const int per = (Nb + kNumXcd - 1) / kNumXcd;  // query blocks per XCD and head
    const long long slot = blockIdx.x / kNumXcd;
    const int qb0 = x0 * per + (int)(slot % per);
    if (qb0 < Nb) item = (int)(slot / per) * Nb + qb0;  // else: padding of the last eighth
  }
  while (item >= 0 && item < BH * Nb) {
  begin_item(item);
  // (thread 0) cursor value and item id of the NEXT item.  The cursor is advanced only in
  // the last loop body, not earlier: items are then started in list order up to about a
  // microsecond, and neighbouring rows of a head, whose kept lists overlap, walk through
  // K/V together (reserving the next item a whole row ahead costs a third of the L2 hits).
  int i_next = -1, item_next = -1;

  if (cnt > 0) {
    // ---- prologue: stages 0 and 1 in flight, S^T and maximum of slice 0 --------------------
    {
#pragma unroll
      for (int e = 0; e < NE; ++e) jb[e] = kept(e);
      const int k0 = key_of(0), k1 = key_of(1), k2 = key_of(2), k3 = key_of(3);
#pragma unroll
      for (int ii = 0; ii < IPW; ++ii) dma(0, ii, 0, k0, k1);
#pragma unroll
      for (int ii = 0; ii < IPW; ++ii) dma(1, ii, 0, k0, k0);
#pragma unroll
      for (int ii = 0; ii < IPW; ++ii) dma(0, ii, 1, k2, k3);
#pragma unroll
      for (int ii = 0; ii < IPW; ++ii) dma(1, ii, 1, k1, k2);
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * IPW) : "memory");  // stage 0 has landed
      __syncthreads();
      f32x16_t acc = cinit;  // zeros: no reference exponent yet
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        Frag8 a;
        a.u = fetch(3 * STEP + ks);  // K of slice 0: buffer 0, rows 0
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, qf[ks].v, acc, 0, 0, 0);
      }
      if constexpr (kExact) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] *= scale_log2e;
      }
      sacc[0] = acc;
      const int nv = N - k0;
      if (nv < 32) mask_slice(sacc[0], nv);
    }
    float m_loc = -__builtin_inff();
#pragma unroll
    for (int i = 0; i < 4; ++i) m_loc = max_part(sacc[0], i, m_loc);
    finish_max(m_loc, sacc[0]);
    refill(0);

    const int T = cnt * NSL / 2;  // stages
    for (int st = 0; st < T; st += 2) {
      // (body: slices s0 = 2 st .. s0+3, list entry eb = s0 / NSL)
      int jn[EPB];
      // ---- slice s0: B, C, then the barrier that retires K stage st and V stage st ----
      qk_step(1, 0, no_extra);
      {
        const int nv = N - key_of(1);
        if (nv < 32) mask_slice(sacc[1], nv);
      }
      m_loc = pv_step(0, KS);
      finish_max(m_loc, sacc[1]);
#pragma unroll
      for (int i = 0; i < EPB; ++i) jn[i] = kept(2 * st / NSL + NE + i);
      wait_loads_and_barrier();
#pragma unroll
      for (int i = 0; i < EPB; ++i) asm volatile("" : "+s"(jn[i]));  // loaded before the barrier
      if (plan && t == 0 && st + 2 >= T && len0 > 0) i_next = atomicAdd(&plan[x0], 1);
      refill(G_B0);
      // ---- slice s0+1; stage st+2 -> buffers 0 ----
      {
        const int ka = key_of(4), kb = key_of(5), va = key_of(3);
        qk_step(0, STEP, [&](int ks) {
#pragma unroll
          for (int ii = 0; ii < 2 * IPW; ++ii)
            if (ii * KS / (2 * IPW) == ks) {
              if (ii < IPW) dma(0, ii, 0, ka, kb);
              else dma(1, ii - IPW, 0, va, ka);
            }
        });
      }
      {
        const int nv = N - key_of(2);
        if (nv < 32) mask_slice(sacc[0], nv);
      }
      m_loc = pv_step(1, STEP + KS);
      finish_max(m_loc, sacc[0]);
      if (NSL == 2 && st + 1 >= T) break;
      // ---- slice s0+2: B, C, barrier retiring K stage st+1 and V stage st+1 ----
      qk_step(1, 2 * STEP, no_extra);
      {
        const int nv = N - key_of(3);
        if (nv < 32) mask_slice(sacc[1], nv);
      }
      m_loc = pv_step(0, 2 * STEP + KS);
      finish_max(m_loc, sacc[1]);
      wait_loads_and_barrier();
      refill(G_B1);
      // ---- slice s0+3; stage st+3 -> buffers 1 ----
      {
        const int ka = key_of(6), kb = key_of(7), va = key_of(5);
        qk_step(0, 3 * STEP, [&](int ks) {
#pragma unroll
          for (int ii = 0; ii < 2 * IPW; ++ii)
            if (ii * KS / (2 * IPW) == ks) {
              if (ii < IPW) dma(0, ii, 1, ka, kb);
              else dma(1, ii - IPW, 1, va, ka);
            }
        });
      }
      {
        const int nv = N - key_of(4);
        if (nv < 32) mask_slice(sacc[0], nv);
      }
      m_loc = pv_step(1, 3 * STEP + KS);
      finish_max(m_loc, sacc[0]);
      // advance the entry window
#pragma unroll
      for (int e = 0; e + EPB < NE; ++e) jb[e] = jb[e + EPB];
#pragma unroll
      for (int i = 0; i < EPB; ++i) jb[NE - EPB + i] = jn[i];
    }
    // loads of stages past the end may still be in flight towards LDS
    wait_loads_and_barrier();
  }
  if (plan && t == 0) {
    if (i_next < 0 && len0 > 0) i_next = atomicAdd(&plan[x0], 1);  // (row without kept blocks)
    if (i_next >= 0 && i_next < len0) item_next = entry(x0, off0, i_next);
  }

  // ---- epilogue: normalise, stage through LDS, coalesced bf16 store -----------------------
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  if (lse && hf == 0 && qrow < N)
    lse[(size_t)bh * N + qrow] =
        l_tot > 0.f ? (m_ref + log2f(l_tot)) * 0.6931471805599453f : -__builtin_inff();
  uint16_t *sO = reinterpret_cast<uint16_t *>(smem);  // [BLK][SO]
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      u32x2_t pk;
      pk.x = cvt_pk_bf16(o[dt][4 * g + 0] * inv, o[dt][4 * g + 1] * inv);
      pk.y = cvt_pk_bf16(o[dt][4 * g + 2] * inv, o[dt][4 * g + 3] * inv);
      *reinterpret_cast<u32x2_t *>(sO + (wave * 32 + l32) * SO + dt * 32 + 8 * g + 4 * hf) = pk;
    }
  __syncthreads();
  uint16_t *obase = out + b * osb + h * osh;
  constexpr int OCH = (BLK * CPR) / NT;  // 16-byte chunks of the output per thread
  constexpr int O_R_STEP = NT / CPR;
  const int o_r0 = t / CPR, o_c = (t % CPR) * 8;
#pragma unroll
  for (int it = 0; it < OCH; ++it) {
    const int r = o_r0 + it * O_R_STEP;
    const int n = qb * BLK + r;
    if (n < N)
      *reinterpret_cast<u32x4_t *>(obase + (long long)n * osn + o_c) =
          *reinterpret_cast<const u32x4_t *>(sO + r * SO + o_c);
  }
  if (!plan) break;
  if (t == 0) s_item = item_next >= 0 ? item_next : take(-1);
  __syncthreads();  // also: everyone has read the output staging before the next item's loads
  item = __builtin_amdgcn_readfirstlane(s_item);
  }  // work loop
}

template <int D, int BLK, bool kExact>
static int launch_attn_t(const heart_shape &s, const void *q, const void *k, const void *v,
                         const int *kept_idx, const int *kept_count, float scale, void *out,
                         float *lse, int *order, hipStream_t st) {
  const int Nb = (s.N + BLK - 1) / BLK;
  const int BH = s.B * s.H;
  const size_t lds = 4 * (size_t)kStageRows * D * 2;  // >= BLK * (D + 8) * 2 of the output staging
  auto kern = attn_kernel<D, BLK, kExact>;
  const int dev = current_device();
  if (dev < 0) return fail(HEART_EHIP, "heart_block_sparse_attn: cannot identify the current device");
  static DeviceFlags attr_set;  // per instantiation: the attribute is per function and device
  if (hipError_t e = set_max_lds_once(attr_set, dev, reinterpret_cast<const void *>(kern), (int)lds))
    return fail(HEART_EHIP, "hipFuncSetAttribute(max dynamic LDS %zu): %s", lds, hipGetErrorString(e));
  const float sc = scale > 0.f ? scale : 1.0f / sqrtf((float)D);
  const float scale_log2e = sc * 1.4426950408889634f;
  const long long n_items = (long long)BH * Nb;
  long long grid = (long long)BH * ((Nb + kNumXcd - 1) / kNumXcd) * kNumXcd;
  if (order) {
    // persistent workgroups: as many as are resident at once (HEART_ATTN_OCC per SIMD, i.e.
    // two workgroups of four wavefronts per CU)
    const int n_cu = cu_count(dev);
    if (n_cu <= 0) return fail(HEART_EHIP, "heart_block_sparse_attn: cannot query the number of CUs");
    const long long resident = (long long)n_cu * HEART_ATTN_OCC * 4 / (BLK / 32);
    grid = n_items < resident ? n_items : resident;
  }
  if (grid > 0x7fffffffLL) return fail(HEART_EUNSUPPORTED, "heart_block_sparse_attn: grid too large");
  if (order) {
    const uint32_t mult = (uint32_t)(((kOrderClasses - 1) << 16) / Nb);
    if (Nb <= kOrderStagedMax) {
      auto okern = attn_order_kernel<true>;
      static DeviceFlags order_attr_set;
      if (hipError_t e = set_max_lds_once(order_attr_set, dev, reinterpret_cast<const void *>(okern),
                                          kOrderStagedMax))
        return fail(HEART_EHIP, "hipFuncSetAttribute(order kernel LDS): %s", hipGetErrorString(e));
      hipLaunchKernelGGL(okern, dim3((unsigned)BH), dim3(256), (size_t)((Nb + 15) / 16 * 16), st,
                         kept_count, BH, Nb, mult, order);
    } else {
      hipLaunchKernelGGL(attn_order_kernel<false>, dim3((unsigned)BH), dim3(256), 0, st, kept_count,
                         BH, Nb, mult, order);
    }
    if (int rc = check_launch("attn_order_kernel")) return rc;
    hipLaunchKernelGGL(attn_plan_kernel, dim3(1), dim3(256), 0, st, BH, Nb, order);
    if (int rc = check_launch("attn_plan_kernel")) return rc;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(BLK * 2), lds, st,
                     (const uint16_t *)q, (const uint16_t *)k, (const uint16_t *)v,
                     (uint16_t *)out, s.q_stride[0], s.q_stride[1], s.q_stride[2], s.k_stride[0],
                     s.k_stride[1], s.k_stride[2], s.v_stride[0], s.v_stride[1], s.v_stride[2],
                     s.o_stride[0], s.o_stride[1], s.o_stride[2], s.H, BH, s.N, Nb, kept_idx,
                     kept_count, scale_log2e, lse, order);
  return check_launch("attn_kernel");
}

template <bool kExact>
static int launch_attn_e(const heart_shape &s, const void *q, const void *k, const void *v,
                         const int *kept_idx, const int *kept_count, float scale, void *out,
                         float *lse, int *order, hipStream_t st) {
  if (s.D == 128 && s.block == 128)
    return launch_attn_t<128, 128, kExact>(s, q, k, v, kept_idx, kept_count, scale, out, lse, order, st);
  if (s.D == 128 && s.block == 64)
    return launch_attn_t<128, 64, kExact>(s, q, k, v, kept_idx, kept_count, scale, out, lse, order, st);
  if (s.D == 64 && s.block == 128)
    return launch_attn_t<64, 128, kExact>(s, q, k, v, kept_idx, kept_count, scale, out, lse, order, st);
  if (s.D == 64 && s.block == 64)
    return launch_attn_t<64, 64, kExact>(s, q, k, v, kept_idx, kept_count, scale, out, lse, order, st);
  return fail(HEART_EUNSUPPORTED, "heart_block_sparse_attn: unsupported (D, block) = (%d, %d)",
              s.D, s.block);
}

int launch_attn(const heart_shape &s, const void *q, const void *k, const void *v,
                const int *kept_idx, const int *kept_count, float scale, unsigned flags, void *out,
                float *lse, int *order, hipStream_t st) {
  // the kernel addresses one head's rows through 32-bit buffer offsets
  const long long lim = 0xffffffffLL;
  const long long rows = (long long)s.N + 2 * s.block;  // staging may address a few rows past N
  if (rows * s.q_stride[2] * 2 > lim || rows * s.k_stride[2] * 2 > lim ||
      rows * s.v_stride[2] * 2 > lim)
    return fail(HEART_EUNSUPPORTED,
                "heart_block_sparse_attn: (N + 2*block) * token stride * 2 bytes must stay "
                "below 4 GiB");
  if (flags & HEART_ATTN_FOLD_SCALE)
    return launch_attn_e<false>(s, q, k, v, kept_idx, kept_count, scale, out, lse, order, st);
  return launch_attn_e<true>(s, q, k, v, kept_idx, kept_count, scale, out, lse, order, st);
}

// ---- launch plan in static device memory, for callers that cannot allocate --------------------
// One array per GPU (every device the library runs on holds its own copy at its own address
// until the process ends).  In host code the array's name is only a stand-in for the symbol:
// the device address is looked up once per device, with that device current, and only that
// pointer is handed to kernels.
static __device__ __align__(256) int g_plan_scratch[HEART_ATTN_STATIC_PLAN_BYTES / sizeof(int)];

int attn_static_plan(int **ptr) {
  const int dev = current_device();
  if (dev < 0)
    return fail(HEART_EHIP, "heart_block_sparse_attn_static: cannot identify the current device");
  static std::atomic<int *> addr[kMaxDevices];
  int *p = addr[dev].load(std::memory_order_acquire);
  if (!p) {
    void *sym = nullptr;
    const hipError_t e = hipGetSymbolAddress(&sym, HIP_SYMBOL(g_plan_scratch));
    if (e != hipSuccess || !sym)
      return fail(HEART_EHIP, "heart_block_sparse_attn_static: hipGetSymbolAddress: %s",
                  hipGetErrorString(e));
    p = static_cast<int *>(sym);
    addr[dev].store(p, std::memory_order_release);  // (threads that race store the same address)
  }
  *ptr = p;
  return HEART_OK;
}

}  // namespace heart
