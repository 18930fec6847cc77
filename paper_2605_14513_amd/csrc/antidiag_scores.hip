// heart_scores_antidiag: an antidiagonal-style block-importance estimator that feeds
// heart_mask_topp through its scores_in argument, as an alternative to the pooled scores.
// The paper leaves importance ranking to the sparse-attention backbone and names this
// family with its setting (antidiagonal scoring, stride 16, blocks of 128 tokens: appendix
// on baseline configurations); the definition implemented here is
//   S = stride, block = 8 S, tokens past N are zero vectors,
//   L[a,b]  = 1/(S sqrt(D)) * sum_{r<S} q[S a + S-1-r] . k[S b + r]   (the antidiagonal of
//             the S x S tile (a,b) of Q K^T), a, b < M = ceil(N/S)
//   P[a,:]  = softmax_b L[a,:]
//   score[I,J] = mean_{a in block I} sum_{b in block J} P[a,b]
//
// L is one bf16 GEMM per head: row a of the left operand is the S token rows of reduced
// query a in reverse order, S*D contiguous-by-row elements, row b of the right operand the
// S token rows of reduced key b in order.  2 M^2 S D FLOP per head on the matrix cores
// (v_mfma_f32_32x32x16_bf16), MFMA-bound.
//
// Kernel 1 (antidiag_tile): one workgroup (8 wavefronts) per 256 x 256 tile of L (128 FLOP
//   per operand byte, which keeps the operand stream from L2 below what it delivers).  The
//   contraction runs in stages of 64 elements (half a token row at D = 128): both operand
//   tiles go from global memory straight into LDS (`buffer_load ... lds`, 16-byte chunks
//   XOR-swizzled by row so that the fragment reads are conflict free), double-buffered
//   (128 KB), one barrier per stage, the loads of the next stage in flight during the MFMAs
//   of the current one; fragments are
//   read one contraction step ahead and the barrier sits in the shadow of the last step's
//   MFMAs.  A wavefront owns 64 reduced queries against 128 reduced keys (S^T layout: keys
//   along the accumulator rows), so a query's maximum over those keys is a per-lane
//   reduction plus one exchange with the partner lane.  The epilogue writes one record per
//   (reduced query, 128 keys): the maximum m and the 16 sums over 8 keys of exp2(L - m).
//   Tiles are independent.
// Kernel 2 (antidiag_combine): one workgroup per query block: global maximum and
//   normaliser of each of its reduced queries from the records, then the mean over the
//   reduced queries of the rescaled key-block sums.
#include "heart_internal.h"

namespace heart {

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t ad_u32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 ad_bf16x8;
typedef __attribute__((ext_vector_type(16))) float ad_f32x16;
union AdFrag {
  ad_u32x4 u;
  ad_bf16x8 v;
};

constexpr int kAdTile = 256;                     // reduced rows per tile side
constexpr int kAdRowB = 128;                     // bytes per tile row and stage (64 bf16)
constexpr int kAdTileB = kAdTile * kAdRowB;      // bytes of one operand tile of one stage
constexpr int kAdKeysPerBlock = 8;               // reduced keys per key block (block = 8 S)
constexpr int kAdLds = 4 * kAdTileB;             // two stages x two operands (128 KB)

// raw buffer descriptor (base, size in bytes) as four words in scalar registers, for the
// hand-written LDS-direct loads; accesses past `bytes` return zeros
__device__ __forceinline__ ad_u32x4 ad_rsrc_words(const uint16_t *base, uint32_t bytes) {
  const uint64_t a = reinterpret_cast<uint64_t>(base);
  ad_u32x4 r;
  r.x = __builtin_amdgcn_readfirstlane((uint32_t)a);
  r.y = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32) & 0xffffu);
  r.z = __builtin_amdgcn_readfirstlane(bytes);
  r.w = 0x00020000u;
  return r;
}

}  // namespace

template <int D>
__global__ __launch_bounds__(512, 2) void antidiag_tile_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, long long qsb, long long qsh,
    long long qsn, long long ksb, long long ksh, long long ksn, int H, int BH, int N, int S, int M,
    int MT2, float scale_log2, const unsigned char *__restrict__ refresh, float *__restrict__ esum,
    float *__restrict__ mref) {
  extern __shared__ __align__(1024) unsigned char smem[];
  // workgroup -> (head, tile): workgroup ids are dealt round-robin to the 8 XCDs; all tiles
  // of a head go to one XCD so that its operand rows are shared through that XCD's L2
  const int tph = MT2 * MT2;
  const long long slot = blockIdx.x / 8;
  const int bh = (int)(blockIdx.x % 8) + 8 * (int)(slot / tph);
  if (bh >= BH) return;
  if (refresh && !refresh[bh]) return;  // reused head: its cached mask persists, no scores needed
  const int tile = (int)(slot % tph);
  const int tq = tile / MT2, tk = tile % MT2;
  const int b = bh / H, h = bh % H;

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int l32 = lane & 31, hf = lane >> 5;
  const int wi = wave >> 2;  // which 128 keys of the tile
  const int wj = wave & 3;   // which 64 queries of the tile

  const ad_u32x4 q_rs = ad_rsrc_words(q + b * qsb + h * qsh, (uint32_t)((long long)N * qsn * 2));
  const ad_u32x4 k_rs = ad_rsrc_words(k + b * ksb + h * ksh, (uint32_t)((long long)N * ksn * 2));
  const uint32_t smem_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)smem;

  // Staging by LDS-direct loads: one instruction moves 16 bytes per lane to 1 KB of consecutive
  // LDS, i.e. 8 tile rows; lane l lands at chunk position l % 8 of row l / 8 and therefore
  // fetches the global chunk (l % 8) ^ f(row) (the XOR swizzle is applied on the global side).
  // Wavefront w issues instructions 4 w .. 4 w + 3 of each operand tile.  The whole byte
  // offset goes through the vector offset, which the descriptor range-checks: rows of tokens
  // >= N are out of range and arrive as zeros.
  constexpr int SPR = D / 64;  // stages per token row
  uint32_t q_dma[4], k_dma[4];
  {
    const int drow = lane >> 3, dp = lane & 7;
#pragma unroll
    for (int ii = 0; ii < 4; ++ii) {
      const int row = 8 * (4 * wave + ii) + drow;
      const uint32_t chunk = (uint32_t)(dp ^ ((row >> 1) & 7));
      // (token index of sub-row 0; the stage adds its sub-row)
      q_dma[ii] = (uint32_t)(S * (kAdTile * tq + row)) * (uint32_t)(qsn * 2) + chunk * 16u;
      k_dma[ii] = (uint32_t)(S * (kAdTile * tk + row)) * (uint32_t)(ksn * 2) + chunk * 16u;
    }
  }
  // (the compiler does not see the LDS write of these instructions: their completion is
  // awaited explicitly before the barrier that publishes the stage)
  auto dma_stage = [&](int st, int buf) __attribute__((always_inline)) {
    const int r = st / SPR, d0 = (st % SPR) * 64;
    const uint32_t qo = (uint32_t)(S - 1 - r) * (uint32_t)(qsn * 2) + (uint32_t)d0 * 2u;
    const uint32_t ko = (uint32_t)r * (uint32_t)(ksn * 2) + (uint32_t)d0 * 2u;
#pragma unroll
    for (int ii = 0; ii < 4; ++ii) {
      const uint32_t dst_a = smem_lds + (uint32_t)(buf * 2 * kAdTileB + (4 * wave + ii) * 1024);
      const uint32_t dst_b = dst_a + (uint32_t)kAdTileB;
      uint32_t m0_saved;  // (M0 carries the LDS destination; saved and restored for the compiler)
      asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\t"
                   "buffer_load_dwordx4 %2, %3, 0 offen lds\n\ts_mov_b32 m0, %0"
                   : "=&s"(m0_saved) : "s"(dst_a), "v"(k_dma[ii] + ko), "s"(k_rs) : "memory");
      asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\t"
                   "buffer_load_dwordx4 %2, %3, 0 offen lds\n\ts_mov_b32 m0, %0"
                   : "=&s"(m0_saved) : "s"(dst_b), "v"(q_dma[ii] + qo), "s"(q_rs) : "memory");
    }
  };
  auto wait_loads_and_barrier = [&]() __attribute__((always_inline)) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  };
  // fragment of contraction step ks (16 elements) of tile row 32 x + l32: chunk 2 ks + hf
  uint32_t foff[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) foff[ks] = (uint32_t)(l32 * kAdRowB + (((2 * ks + hf) ^ ((l32 >> 1) & 7)) * 16));

  ad_f32x16 acc[4][2];
#pragma unroll
  for (int kt = 0; kt < 4; ++kt)
#pragma unroll
    for (int qt = 0; qt < 2; ++qt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[kt][qt][r] = 0.f;

  // the six fragments of one contraction step: 4 of the keys (A operand), 2 of the queries
  struct Frags {
    AdFrag a[4], b[2];
  };
  auto read_frags = [&](Frags &f, int buf, int ks) __attribute__((always_inline)) {
    const unsigned char *A = smem + buf * 2 * kAdTileB + wi * 128 * kAdRowB;
    const unsigned char *B = smem + buf * 2 * kAdTileB + kAdTileB + wj * 64 * kAdRowB;
#pragma unroll
    for (int qt = 0; qt < 2; ++qt)
      f.b[qt].u = *reinterpret_cast<const ad_u32x4 *>(B + qt * 32 * kAdRowB + foff[ks]);
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
      f.a[kt].u = *reinterpret_cast<const ad_u32x4 *>(A + kt * 32 * kAdRowB + foff[ks]);
  };
  auto mfma8 = [&](const Frags &f) __attribute__((always_inline)) {
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
      for (int qt = 0; qt < 2; ++qt)
        acc[kt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[kt].v, f.b[qt].v, acc[kt][qt], 0, 0, 0);
  };

  // Per stage: the fragments of a contraction step are read one step before their MFMAs, and
  // the barrier that hands over the next stage sits between the reads of the stage's last
  // step and its MFMAs, so that the barrier and the first LDS reads of the next stage run in
  // the shadow of eight MFMAs.  By the barrier a wavefront has completed all its reads of the
  // current buffer and its loads of the next stage into the other one; right after it, it
  // issues the loads of the stage after that into the buffer just released.  Loads past the
  // last stage repeat the last stage (into a buffer nobody reads any more).
  const int n_stages = S * SPR;
  const int last = n_stages - 1;
  Frags f0, f1;
  dma_stage(0, 0);
  wait_loads_and_barrier();
  dma_stage(min(1, last), 1);
  read_frags(f0, 0, 0);
  for (int st = 0; st < n_stages; ++st) {
    const int buf = st & 1;
    read_frags(f1, buf, 1);
    mfma8(f0);
    __builtin_amdgcn_sched_barrier(0);
    read_frags(f0, buf, 2);
    mfma8(f1);
    __builtin_amdgcn_sched_barrier(0);
    read_frags(f1, buf, 3);
    mfma8(f0);
    __builtin_amdgcn_sched_barrier(0);
    wait_loads_and_barrier();
    __builtin_amdgcn_sched_barrier(0);
    dma_stage(min(st + 2, last), buf);
    read_frags(f0, buf ^ 1, 0);
    __builtin_amdgcn_sched_barrier(0);
    mfma8(f1);
  }
  // loads of the repeated last stage may still be in flight towards LDS
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  // ---- epilogue: record of (reduced query, 128 keys): maximum and 16 key-block sums ----------
  // accumulator element r of key tile kt: reduced key key0 + 32 kt + 8 (r / 4) + 4 hf + r % 4
  const float ninf = -__builtin_inff();
  const int key0 = kAdTile * tk + 128 * wi;
  const int rec = 2 * tk + wi;  // index of the 128-key record
  const int MT = 2 * MT2, NbP = 16 * MT;
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    float m = ninf;
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = key0 + 32 * kt + 8 * (r >> 2) + 4 * hf + (r & 3);
        const float x = key < M ? acc[kt][qt][r] * scale_log2 : ninf;
        acc[kt][qt][r] = x;
        m = fmaxf(m, x);
      }
    {
      uint32_t s0, s1;
      swap_halves32(__float_as_uint(m), s0, s1);
      m = fmaxf(__uint_as_float(s0), __uint_as_float(s1));
    }
    // (a record whose 128 keys are all past the end has m = -inf and all sums zero)
    const float mm = m == ninf ? 0.f : m;
    float sums[4][4];
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) s += __builtin_amdgcn_exp2f(acc[kt][qt][4 * g + i] - mm);
        uint32_t s0, s1;
        swap_halves32(__float_as_uint(s), s0, s1);
        sums[kt][g] = __uint_as_float(s0) + __uint_as_float(s1);
      }
    const int a = kAdTile * tq + 64 * wj + 32 * qt + l32;
    if (a < M) {
      float *dst = esum + ((size_t)bh * M + a) * NbP + 16 * rec + 8 * hf;
      // lower-half lanes write key blocks 0..7 of the record, upper-half lanes 8..15
      *reinterpret_cast<float4 *>(dst) = hf ? make_float4(sums[2][0], sums[2][1], sums[2][2], sums[2][3])
                                            : make_float4(sums[0][0], sums[0][1], sums[0][2], sums[0][3]);
      *reinterpret_cast<float4 *>(dst + 4) = hf ? make_float4(sums[3][0], sums[3][1], sums[3][2], sums[3][3])
                                                : make_float4(sums[1][0], sums[1][1], sums[1][2], sums[1][3]);
      if (hf == 0) mref[((size_t)bh * M + a) * MT + rec] = m;
    }
  }
}

// One workgroup (4 wavefronts) per (head, query block).  A wavefront normalises two of the
// block's 8 reduced queries on its own (global maximum over the records, normaliser, both
// wave-wide reductions; the loads of both rows are issued before either is reduced), leaves
// the normalised key-block masses in LDS, and after one barrier the workgroup averages the
// 8 rows.  JPL = key blocks per lane (16 MT <= 64 JPL).
template <int JPL>
__global__ __launch_bounds__(256) void antidiag_combine_kernel(int Nb, int M, int MT,
                                                              const unsigned char *__restrict__ refresh,
                                                              const float *__restrict__ esum,
                                                              const float *__restrict__ mref,
                                                              float *__restrict__ scores) {
  constexpr int RQ = kAdKeysPerBlock;       // reduced queries per query block
  extern __shared__ float s_w[];            // [RQ][NbP]
  const int I = blockIdx.x % Nb;
  const long long bh = blockIdx.x / Nb;
  if (refresh && !refresh[bh]) return;
  const int NbP = 16 * MT;
  const int a0 = I * RQ;
  const int na = min(RQ, M - a0);
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  float mr[2], w[2][JPL], mj[2][JPL];
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    const int rr = wave + 4 * x;
    const size_t row = (size_t)bh * M + a0 + (rr < na ? rr : 0);  // (rows past the end: loads of row 0, unused)
    mr[x] = lane < MT ? mref[row * MT + lane] : -__builtin_inff();
#pragma unroll
    for (int u = 0; u < JPL; ++u) {
      const int J = lane + 64 * u;
      w[x][u] = J < NbP ? esum[row * NbP + J] : 0.f;
      mj[x][u] = J < NbP ? mref[row * MT + (J >> 4)] : 0.f;
    }
  }
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    const int rr = wave + 4 * x;
    const float m = wave_max_f32(mr[x]);
    float part = 0.f;
#pragma unroll
    for (int u = 0; u < JPL; ++u) {
      const int J = lane + 64 * u;
      w[x][u] = J < NbP ? w[x][u] * __builtin_amdgcn_exp2f(mj[x][u] - m) : 0.f;
      part += w[x][u];
    }
    const float inv = rr < na ? 1.f / wave_sum_f32(part) : 0.f;
#pragma unroll
    for (int u = 0; u < JPL; ++u) {
      const int J = lane + 64 * u;
      if (J < NbP) s_w[rr * NbP + J] = w[x][u] * inv;
    }
  }
  __syncthreads();
  const float inv_na = 1.f / (float)na;
  for (int J = t; J < Nb; J += 256) {
    float s = 0.f;
#pragma unroll
    for (int rr = 0; rr < RQ; ++rr) s += s_w[rr * NbP + J];
    scores[((size_t)bh * Nb + I) * Nb + J] = s * inv_na;
  }
}

size_t antidiag_workspace_bytes(const heart_shape &s, int stride) {
  const size_t M = ((size_t)s.N + stride - 1) / stride;
  const size_t MT = 2 * ((M + kAdTile - 1) / kAdTile);  // records of 128 keys per reduced query
  return (size_t)s.B * s.H * M * (16 * MT + MT) * sizeof(float);
}

int launch_antidiag(const heart_shape &s, const void *q, const void *k, int stride,
                    const unsigned char *refresh, float *scores, float *workspace, hipStream_t st) {
  const int S = stride;
  const int M = (s.N + S - 1) / S;
  const int MT2 = (M + kAdTile - 1) / kAdTile;
  const int MT = 2 * MT2;
  const int Nb = (s.N + s.block - 1) / s.block;
  const int BH = s.B * s.H;
  if (MT > 64)  // one wavefront reads a reduced query's records in the combine kernel
    return fail(HEART_EUNSUPPORTED, "heart_scores_antidiag: more than 8192 reduced rows");
  // the kernel addresses one head's rows through 32-bit buffer offsets, up to the end of
  // the last tile
  const long long rows = (long long)S * kAdTile * MT2 + S;
  if (rows * s.q_stride[2] * 2 > 0xffffffffLL || rows * s.k_stride[2] * 2 > 0xffffffffLL)
    return fail(HEART_EUNSUPPORTED,
                "heart_scores_antidiag: (N + 257 * stride) * token stride * 2 bytes must stay below 4 GiB");
  const long long grid = (long long)((BH + 7) / 8) * 8 * MT2 * MT2;
  if (grid > 0x7fffffffLL || (long long)BH * Nb > 0x7fffffffLL)
    return fail(HEART_EUNSUPPORTED, "heart_scores_antidiag: grid too large");
  float *esum = workspace;
  float *mref = workspace + (size_t)BH * M * 16 * MT;
  const float scale_log2 = 1.4426950408889634f / ((float)S * sqrtf((float)s.D));
  const int dev = current_device();
  if (dev < 0) return fail(HEART_EHIP, "heart_scores_antidiag: cannot identify the current device");
#define HEART_AD_LAUNCH(DD)                                                                        \
  do {                                                                                             \
    auto kern = antidiag_tile_kernel<DD>;                                                          \
    static DeviceFlags attr_set;                                                                   \
    if (hipError_t e = set_max_lds_once(attr_set, dev, reinterpret_cast<const void *>(kern),       \
                                        kAdLds))                                                   \
      return fail(HEART_EHIP, "hipFuncSetAttribute(antidiagonal tile kernel LDS): %s",             \
                  hipGetErrorString(e));                                                           \
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(512), kAdLds, st, (const uint16_t *)q,     \
                       (const uint16_t *)k, s.q_stride[0], s.q_stride[1], s.q_stride[2],           \
                       s.k_stride[0], s.k_stride[1], s.k_stride[2], s.H, BH, s.N, S, M, MT2,       \
                       scale_log2, refresh, esum, mref);                                           \
  } while (0)
  if (s.D == 128)
    HEART_AD_LAUNCH(128);
  else
    HEART_AD_LAUNCH(64);
#undef HEART_AD_LAUNCH
  if (int rc = check_launch("antidiag_tile_kernel")) return rc;
  const dim3 cgrid((unsigned)((long long)BH * Nb));
  const size_t clds = (size_t)kAdKeysPerBlock * 16 * MT * sizeof(float);
  if (MT <= 16)
    hipLaunchKernelGGL(antidiag_combine_kernel<4>, cgrid, dim3(256), clds, st, Nb, M, MT, refresh, esum,
                       mref, scores);
  else if (MT <= 32)
    hipLaunchKernelGGL(antidiag_combine_kernel<8>, cgrid, dim3(256), clds, st, Nb, M, MT, refresh, esum,
                       mref, scores);
  else
    hipLaunchKernelGGL(antidiag_combine_kernel<16>, cgrid, dim3(256), clds, st, Nb, M, MT, refresh, esum,
                       mref, scores);
  return check_launch("antidiag_combine_kernel");
}

}  // namespace heart
