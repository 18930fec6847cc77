// heart_pool_qk: block means and token means of bf16 Q and K in one streaming pass
// (Alg. 1 step 1 and Eq. 4 for the token means; the block means feed the
// block-level importance ranking).
//
// Bound by HBM reads: 2*B*H*N*D*2 bytes in, 2*B*H*(Nb+1)*D*4 bytes out.
//
// Kernel 1 (pool_blocks): one workgroup of 256 lanes per (tensor, b, h, block).
//   Every lane issues all of its 16-byte loads (8 bf16 each) before it uses any, so
//   a workgroup has its whole 32 KB block in flight; D/8 adjacent lanes cover one
//   token row, i.e. a wavefront reads whole contiguous rows.  Each lane sums its
//   rows in fp32 in row order, the 256/(D/8) row groups are combined through LDS
//   in a fixed order (no atomics: results are reproducible), and the block mean is
//   written once.
// Kernel 2 (pool_token_mean): one workgroup of 1024 lanes per (tensor, b, h) sums
//   block_mean * n_block over the blocks in fp64 in a fixed order and divides by N.
//   (mean of block means would be wrong when the last block is short.)
#include "heart_internal.h"

namespace heart {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

template <int D>
__global__ __launch_bounds__(256) void pool_blocks_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, long long qsb, long long qsh,
    long long qsn, long long ksb, long long ksh, long long ksn, int H, int N, int block, int Nb,
    float *__restrict__ qblk, float *__restrict__ kblk) {
  constexpr int LPR = D / 8;     // lanes per token row
  constexpr int RPP = 256 / LPR; // rows per pass of the workgroup
  constexpr int MAXP = 128 / RPP; // passes for the largest block (128 tokens)
  __shared__ float part[RPP][D];

  // blockIdx.x enumerates (tensor, b*H+h, block) with the block index fastest so
  // that consecutive workgroups stream consecutive memory.
  long long wid = blockIdx.x;
  int i = (int)(wid % Nb);
  long long rest = wid / Nb;
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
  for (int e = 0; e < 8; ++e) part[row0][lane_col + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < D) {
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < RPP; ++r) s += part[r][threadIdx.x];
    outp[threadIdx.x] = s / (float)nrows;
  }
}

// One workgroup (1024 lanes) per (tensor, b, h).  Lanes are arranged as D/4 column
// groups (float4 each) times 1024/(D/4) block-slices; each slice adds its blocks in
// increasing block order in fp64 (loads of a slice are independent and issued
// several at a time), slices are combined in slice order.
template <int D>
__global__ __launch_bounds__(1024) void pool_token_mean_kernel(const float *__restrict__ qblk,
                                                               const float *__restrict__ kblk,
                                                               int N, int block, int Nb,
                                                               float *__restrict__ qmean,
                                                               float *__restrict__ kmean) {
  constexpr int CG = D / 4;       // column groups
  constexpr int SL = 1024 / CG;   // slices over the blocks
  __shared__ double part[SL][D];
  int which = blockIdx.x & 1;
  long long bh = blockIdx.x >> 1;
  const float *src = (which ? kblk : qblk) + (size_t)bh * Nb * D;
  float *dst = (which ? kmean : qmean) + (size_t)bh * D;
  int cg = threadIdx.x % CG, sl = threadIdx.x / CG;
  int per = (Nb + SL - 1) / SL;
  int i0 = sl * per, i1 = min(Nb, i0 + per);
  double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
#pragma unroll 8
  for (int i = i0; i < i1; ++i) {
    float4 m = *reinterpret_cast<const float4 *>(src + (size_t)i * D + cg * 4);
    double n = (double)min(block, N - i * block);
    a0 += (double)m.x * n;
    a1 += (double)m.y * n;
    a2 += (double)m.z * n;
    a3 += (double)m.w * n;
  }
  part[sl][cg * 4 + 0] = a0;
  part[sl][cg * 4 + 1] = a1;
  part[sl][cg * 4 + 2] = a2;
  part[sl][cg * 4 + 3] = a3;
  __syncthreads();
  if (threadIdx.x < D) {
    double s = 0.0;
#pragma unroll
    for (int r = 0; r < SL; ++r) s += part[r][threadIdx.x];
    dst[threadIdx.x] = (float)(s / (double)N);
  }
}

int launch_pool(const heart_shape &s, const void *q, const void *k, float *qblk, float *kblk,
                float *qmean, float *kmean, hipStream_t st) {
  int Nb = (s.N + s.block - 1) / s.block;
  long long nwg = 2LL * s.B * s.H * Nb;
  if (nwg > 0x7fffffffLL) return fail(HEART_EUNSUPPORTED, "heart_pool_qk: grid too large");
  const uint16_t *qp = (const uint16_t *)q, *kp = (const uint16_t *)k;
  dim3 grid((unsigned)nwg), blk(256), blk2(1024);
  dim3 grid2((unsigned)(2 * s.B * s.H));
  if (s.D == 128) {
    hipLaunchKernelGGL(pool_blocks_kernel<128>, grid, blk, 0, st, qp, kp, s.q_stride[0],
                       s.q_stride[1], s.q_stride[2], s.k_stride[0], s.k_stride[1], s.k_stride[2],
                       s.H, s.N, s.block, Nb, qblk, kblk);
    if (int rc = check_launch("pool_blocks_kernel")) return rc;
    hipLaunchKernelGGL(pool_token_mean_kernel<128>, grid2, blk2, 0, st, qblk, kblk, s.N, s.block,
                       Nb, qmean, kmean);
  } else {
    hipLaunchKernelGGL(pool_blocks_kernel<64>, grid, blk, 0, st, qp, kp, s.q_stride[0],
                       s.q_stride[1], s.q_stride[2], s.k_stride[0], s.k_stride[1], s.k_stride[2],
                       s.H, s.N, s.block, Nb, qblk, kblk);
    if (int rc = check_launch("pool_blocks_kernel")) return rc;
    hipLaunchKernelGGL(pool_token_mean_kernel<64>, grid2, blk2, 0, st, qblk, kblk, s.N, s.block,
                       Nb, qmean, kmean);
  }
  return check_launch("pool_token_mean_kernel");
}

}  // namespace heart
