// heart_pool_qk: block means and token means of bf16 Q and K in one streaming pass
// (Alg. 1 step 1 and Eq. 4 for the token means; the block means feed the
// block-level importance ranking).  heart_pool_drift: the same pass, with the token means,
// the drift, the reuse rule and the layer gate (Eq. 4; Sec. 4.2; Alg. 1) together in ONE
// second launch instead of two -- the paper notes that fixed per-layer cost such as kernel
// launches caps what mask reuse can gain (Sec. 4.2, last paragraph).
//
// Bound by HBM reads: 2*B*H*N*D*2 bytes in, 2*B*H*(Nb+1)*D*4 bytes out.
//
// pool_blocks_kernel: one workgroup of 256 lanes per (tensor, b, h, block).
//   Every lane issues all of its 16-byte loads (8 bf16 each) before it uses any, so
//   a workgroup has its whole 32 KB block in flight; D/8 adjacent lanes cover one
//   token row, i.e. a wavefront reads whole contiguous rows.  Each lane sums its
//   rows in fp32 in row order, the 256/(D/8) row groups are combined through LDS
//   in a fixed order (no atomics on data: results are reproducible), and the block mean
//   is written once.
// Token means (token_mean_workgroup): one workgroup of 1024 lanes per (tensor, b, h) sums
//   block_mean * n_block over the blocks in fp64 in a fixed order and divides by N
//   (the mean of block means would be wrong when the last block is short).
//   heart_pool_qk runs it as a second small kernel (pool_token_mean_kernel).
// token_mean_drift_kernel (heart_pool_drift): the same token-mean workgroups; the one that
//   finishes the last token mean of a batch item -- found with a ticket counter in a caller
//   workspace that is zero on entry and zero again on return -- runs the drift stage for it
//   (drift_workgroup, the code of heart_drift).  No workgroup waits for another.
//   The eight XCDs of the chip have separate L2 caches and a device-wide fence writes back and
//   invalidates a whole L2, so the values that cross workgroups (the token means) move with
//   device-scope atomic stores and loads instead; a workgroup waits for the acknowledgement of
//   its stores before it takes its ticket.
//   (Doing the same in the tail of pool_blocks_kernel, one ticket per block, was measured: a
//   device-wide fence per workgroup took the launch from 0.12 to 3.4 ms, device-scope stores
//   with a ticket per workgroup to 0.23 ms -- under 6 TB/s of reads the store acknowledgement
//   and the atomic's round trip double the lifetime of a workgroup -- so the pooling pass
//   itself stays free of cross-workgroup traffic.)
#include "drift_device.h"
#include "heart_internal.h"

namespace heart {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kPoolThreads = 256;       // pooling pass: lanes per workgroup
constexpr int kMeanThreads = 1024;      // token means (and the drift stage behind them): lanes per workgroup
constexpr int kTokenMeanBatch = 8;      // block means in flight per lane
constexpr int kMeanLdsDoubles = kMeanThreads * 4;  // 32 KB: token-mean slices (fp64); reused for the drift marks

// Device-scope (all XCDs) store of a value that another workgroup of the same launch will read
// (with a device-scope load): coherent across the L2 caches of the XCDs without a cache-wide
// fence.
__device__ __forceinline__ void store_device_scope(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// This wavefront's global stores have been acknowledged (for device-scope stores: at the level
// every XCD sees).
__device__ __forceinline__ void wait_for_own_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Token mean of one (tensor, b, h): src = its block means [Nb][D], dst = [D].  Lanes are
// arranged as D/4 column groups (float4 each) times 1024/(D/4) block slices; each slice adds
// its blocks in increasing block order in fp64, slices are combined in slice order.  Called
// by a whole workgroup of kMeanThreads lanes (contains a barrier); part: LDS, kMeanLdsDoubles
// doubles.
// kAcross: dst is read by another workgroup of this launch (device-scope stores); the
// arithmetic is the same either way.
template <int D, bool kAcross>
__device__ __forceinline__ void token_mean_workgroup(const float *src, int N, int block, int Nb,
                                                     float *dst, double *part) {
  constexpr int CG = D / 4;             // column groups
  constexpr int SL = kMeanThreads / CG; // slices over the blocks
  static_assert(SL * D <= kMeanLdsDoubles, "LDS of the token mean");
  const int cg = threadIdx.x % CG, sl = threadIdx.x / CG;
  const int per = (Nb + SL - 1) / SL;
  const int i0 = sl * per, i1 = min(Nb, i0 + per);
  double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
  // (the loads of kTokenMeanBatch blocks are issued before any is used: the kernel is bound by
  // memory round trips; the order of the additions is the block order either way)
  for (int ib = i0; ib < i1; ib += kTokenMeanBatch) {
    float4 m[kTokenMeanBatch];
#pragma unroll
    for (int u = 0; u < kTokenMeanBatch; ++u) {
      const int i = min(ib + u, i1 - 1);
      m[u] = *reinterpret_cast<const float4 *>(src + (size_t)i * D + cg * 4);
    }
#pragma unroll
    for (int u = 0; u < kTokenMeanBatch; ++u) {
      const int i = ib + u;
      if (i < i1) {
        const double n = (double)min(block, N - i * block);
        a0 += (double)m[u].x * n;
        a1 += (double)m[u].y * n;
        a2 += (double)m[u].z * n;
        a3 += (double)m[u].w * n;
      }
    }
  }
  part[sl * D + cg * 4 + 0] = a0;
  part[sl * D + cg * 4 + 1] = a1;
  part[sl * D + cg * 4 + 2] = a2;
  part[sl * D + cg * 4 + 3] = a3;
  __syncthreads();
  if (threadIdx.x < D) {
    double s = 0.0;
#pragma unroll
    for (int r = 0; r < SL; ++r) s += part[r * D + threadIdx.x];
    if constexpr (kAcross)
      store_device_scope(dst + threadIdx.x, (float)(s / (double)N));
    else
      dst[threadIdx.x] = (float)(s / (double)N);
  }
}

struct PoolDriftArgs {  // what the drift stage needs beyond the token-mean arguments
  float *qanchor, *kanchor;
  unsigned char *has_anchor;
  const float *delta;
  float gate_lo, gate_hi;
  int commit;
  float *drift;
  unsigned char *refresh;
  unsigned *tickets;  // [B]; zero on entry, zero on return
};

template <int D>
__global__ __launch_bounds__(kPoolThreads) void pool_blocks_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, long long qsb, long long qsh,
    long long qsn, long long ksb, long long ksh, long long ksn, int H, int N, int block, int Nb,
    float *__restrict__ qblk, float *__restrict__ kblk) {
  constexpr int LPR = D / 8;               // lanes per token row
  constexpr int RPP = kPoolThreads / LPR;  // rows per pass of the workgroup
  constexpr int MAXP = 128 / RPP;          // passes for the largest block (128 tokens)
  __shared__ float part[RPP * D];

  // blockIdx.x enumerates (b*H+h, tensor, block) with the block index fastest so
  // that consecutive workgroups stream consecutive memory.
  long long wid = blockIdx.x;
  int i = (int)(wid % Nb);
  long long rest = wid / Nb;  // = 2 * (b*H+h) + tensor
  int which = (int)(rest & 1);
  long long bh = rest >> 1;
  int b = (int)(bh / H), h = (int)(bh % H);

  const uint16_t *base = which ? (k + b * ksb + h * ksh) : (q + b * qsb + h * qsh);
  long long sn = which ? ksn : qsn;
  float *outp = (which ? kblk : qblk) + ((size_t)bh * Nb + i) * D;

  int n0 = i * block;
  int nrows = min(block, N - n0);
  int lane_col = (threadIdx.x % LPR) * 8;
  int row0 = threadIdx.x / LPR;

  uint4 v[MAXP];
#pragma unroll
  for (int p = 0; p < MAXP; ++p) {
    int r = row0 + p * RPP;
    v[p] = make_uint4(0u, 0u, 0u, 0u);
    if (r < nrows) {
      // streaming read: every byte is used once by this kernel
      const u32x4 t = __builtin_nontemporal_load(
          reinterpret_cast<const u32x4 *>(base + (long long)(n0 + r) * sn + lane_col));
      v[p] = make_uint4(t.x, t.y, t.z, t.w);
    }
  }
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
  for (int p = 0; p < MAXP; ++p) {
    acc[0] += bf16lo(v[p].x);
    acc[1] += bf16hi(v[p].x);
    acc[2] += bf16lo(v[p].y);
    acc[3] += bf16hi(v[p].y);
    acc[4] += bf16lo(v[p].z);
    acc[5] += bf16hi(v[p].z);
    acc[6] += bf16lo(v[p].w);
    acc[7] += bf16hi(v[p].w);
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[row0 * D + lane_col + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < D) {
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < RPP; ++r) s += part[r * D + threadIdx.x];
    outp[threadIdx.x] = s / (float)nrows;
  }
}

// One workgroup per (tensor, b, h).
template <int D>
__global__ __launch_bounds__(kMeanThreads) void pool_token_mean_kernel(const float *__restrict__ qblk,
                                                                       const float *__restrict__ kblk,
                                                                       int N, int block, int Nb,
                                                                       float *__restrict__ qmean,
                                                                       float *__restrict__ kmean) {
  __shared__ double part[kMeanLdsDoubles];
  const int which = blockIdx.x & 1;
  const long long bh = blockIdx.x >> 1;
  token_mean_workgroup<D, false>((which ? kblk : qblk) + (size_t)bh * Nb * D, N, block, Nb,
                                 (which ? kmean : qmean) + (size_t)bh * D, part);
}

// The same, and the workgroup that completes a batch item runs the drift stage.  A ticket
// (device-scope atomic) is taken after this workgroup's device-scope stores have been
// acknowledged (wait, then barrier, then the atomic of one lane); the workgroup that draws the
// last ticket of its batch item then reads every token mean with device-scope loads.
template <int D>
__global__ __launch_bounds__(kMeanThreads) void token_mean_drift_kernel(
    const float *__restrict__ qblk, const float *__restrict__ kblk, int H, int N, int block, int Nb,
    float *qmean, float *kmean, PoolDriftArgs fa) {
  __shared__ double lds[kMeanLdsDoubles];
  __shared__ int s_last;
  const int which = blockIdx.x & 1;
  const long long bh = blockIdx.x >> 1;
  const int b = (int)(bh / H);
  token_mean_workgroup<D, true>((which ? kblk : qblk) + (size_t)bh * Nb * D, N, block, Nb,
                                (which ? kmean : qmean) + (size_t)bh * D, lds);
  wait_for_own_stores();
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned t = atomicAdd(&fa.tickets[b], 1u);
    s_last = (t == 2u * (unsigned)H - 1u);
    if (s_last) atomicExch(&fa.tickets[b], 0u);  // nobody else touches it any more in this launch
  }
  __syncthreads();
  if (!s_last) return;
  drift_workgroup<true>(b, H, D, qmean, kmean, fa.qanchor, fa.kanchor, fa.has_anchor, fa.delta,
                        fa.gate_lo, fa.gate_hi, fa.commit, fa.drift, fa.refresh,
                        reinterpret_cast<unsigned char *>(lds));
}

template <int D>
static int launch_pool_t(const heart_shape &s, const uint16_t *qp, const uint16_t *kp, float *qblk,
                         float *kblk, float *qmean, float *kmean, const PoolDriftArgs *fused,
                         hipStream_t st) {
  const int Nb = (s.N + s.block - 1) / s.block;
  const long long nwg = 2LL * s.B * s.H * Nb;
  if (nwg > 0x7fffffffLL) return fail(HEART_EUNSUPPORTED, "heart_pool_qk: grid too large");
  const dim3 grid((unsigned)nwg), blk(kPoolThreads), grid2((unsigned)(2 * s.B * s.H)), blk2(kMeanThreads);
  hipLaunchKernelGGL(pool_blocks_kernel<D>, grid, blk, 0, st, qp, kp, s.q_stride[0], s.q_stride[1],
                     s.q_stride[2], s.k_stride[0], s.k_stride[1], s.k_stride[2], s.H, s.N, s.block,
                     Nb, qblk, kblk);
  if (int rc = check_launch("pool_blocks_kernel")) return rc;
  if (fused) {
    hipLaunchKernelGGL(token_mean_drift_kernel<D>, grid2, blk2, 0, st, qblk, kblk, s.H, s.N, s.block,
                       Nb, qmean, kmean, *fused);
    return check_launch("token_mean_drift_kernel");
  }
  hipLaunchKernelGGL(pool_token_mean_kernel<D>, grid2, blk2, 0, st, qblk, kblk, s.N, s.block, Nb,
                     qmean, kmean);
  return check_launch("pool_token_mean_kernel");
}

int launch_pool(const heart_shape &s, const void *q, const void *k, float *qblk, float *kblk,
                float *qmean, float *kmean, hipStream_t st) {
  const uint16_t *qp = (const uint16_t *)q, *kp = (const uint16_t *)k;
  if (s.D == 128) return launch_pool_t<128>(s, qp, kp, qblk, kblk, qmean, kmean, nullptr, st);
  return launch_pool_t<64>(s, qp, kp, qblk, kblk, qmean, kmean, nullptr, st);
}

int launch_pool_drift(const heart_shape &s, const void *q, const void *k, float *qblk, float *kblk,
                      float *qmean, float *kmean, float *qanchor, float *kanchor,
                      unsigned char *has_anchor, const float *delta, float gate_lo, float gate_hi,
                      int commit, float *drift, unsigned char *refresh, unsigned *tickets,
                      hipStream_t st) {
  const uint16_t *qp = (const uint16_t *)q, *kp = (const uint16_t *)k;
  const PoolDriftArgs fa{qanchor, kanchor, has_anchor, delta, gate_lo, gate_hi,
                         commit, drift, refresh, tickets};
  if (s.D == 128) return launch_pool_t<128>(s, qp, kp, qblk, kblk, qmean, kmean, &fa, st);
  return launch_pool_t<64>(s, qp, kp, qblk, kblk, qmean, kmean, &fa, st);
}

}  // namespace heart
