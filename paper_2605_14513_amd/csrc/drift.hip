// heart_drift: mean-pooled query-key drift (Eq. 4), the reuse rule of Temporal Mask
// Reuse (Sec. 4.2; Alg. 1), the layer-level gate (Sec. 4.2; thresholds from the
// appendix on HEART configurations) and the anchor update.
//
// The data is tiny (4*B*H*D floats), so this is one launch with one workgroup of 16
// wavefronts per batch item (one head per wavefront and pass): the gate needs the
// count of marked heads of that item, and keeping it inside one workgroup avoids any
// cross-workgroup synchronisation.  The kernel is bound by a few dependent memory
// round trips, not by bandwidth.
//
// drift is summed in fp32 with a fixed halving tree over d:
//   a[d] = |qa[d]-qb[d]| + |ka[d]-kb[d]|;  for s = D/2 .. 1: a[i] += a[i+s] (i < s)
// A wavefront holds element d = lane + 64*c in lane `lane`, slot c; steps with
// s >= 64 combine slots inside a lane, steps with s < 64 are xor-butterflies over
// lanes.  Because fp32 addition is commutative, lane 0 ends with exactly the value
// of the tree above, so the decision is a pure function of the fp32 inputs.
#include "heart_internal.h"

namespace heart {

constexpr int kMaxSlots = 8;   // D <= 512
constexpr int kThreads = 1024; // 16 wavefronts: 16 heads in flight per pass

__global__ __launch_bounds__(kThreads) void drift_kernel(
    int H, int D, const float *__restrict__ qmean, const float *__restrict__ kmean,
    float *__restrict__ qanchor, float *__restrict__ kanchor,
    unsigned char *__restrict__ has_anchor, const float *__restrict__ delta, float gate_lo,
    float gate_hi, int commit, float *__restrict__ drift, unsigned char *__restrict__ refresh) {
  extern __shared__ unsigned char smem[];
  unsigned char *mark = smem;           // [H]
  unsigned char *fin = smem + H;        // [H]
  __shared__ int n_mark_sh;

  const int b = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int slots = D > 64 ? D / 64 : 1;

  for (int h = wave; h < H; h += kThreads / 64) {
    size_t o = ((size_t)b * H + h) * D;
    // all loads are issued unconditionally (the anchor buffers always exist); a head
    // without an anchor ignores the value
    const bool has = has_anchor[(size_t)b * H + h] != 0;
    const float dl = delta[h];
    float a[kMaxSlots];
#pragma unroll
    for (int c = 0; c < kMaxSlots; ++c) {
      a[c] = 0.f;
      int d = lane + 64 * c;
      if (c < slots && d < D) {
        float dq = fabsf(qanchor[o + d] - qmean[o + d]);
        float dk = fabsf(kanchor[o + d] - kmean[o + d]);
        a[c] = dq + dk;
      }
    }
    // steps with s >= 64: a[i] += a[i+s]  <=>  slot c += slot c + s/64
#pragma unroll
    for (int s = kMaxSlots / 2; s >= 1; s >>= 1) {
      if (s < slots) {
#pragma unroll
        for (int c = 0; c < kMaxSlots / 2; ++c)
          if (c < s) a[c] = a[c] + a[c + s];
      }
    }
    float v = a[0];
    // steps with s < 64 (lanes >= D hold +0, adding it is exact)
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) {
      float o2 = __shfl_xor(v, s, 64);
      if (s < D) v = v + o2;
    }
    if (lane == 0) {
      float dv = has ? v : __builtin_inff();
      drift[(size_t)b * H + h] = dv;
      mark[h] = (!has || dv > dl) ? 1 : 0;
    }
  }
  __syncthreads();
  if (wave == 0) {
    uint32_t n = 0;
    for (int h = lane; h < H; h += 64) n += mark[h];
    n = wave_sum_u32(n);
    if (lane == 0) n_mark_sh = (int)n;
  }
  __syncthreads();
  const float frac = __fdiv_rn((float)n_mark_sh, (float)H);
  for (int h = threadIdx.x; h < H; h += blockDim.x) {
    unsigned char r;
    if (frac < gate_lo)
      r = has_anchor[(size_t)b * H + h] ? 0 : 1;
    else if (frac > gate_hi)
      r = 1;
    else
      r = mark[h];
    fin[h] = r;
    refresh[(size_t)b * H + h] = r;
  }
  __syncthreads();
  if (commit) {
    for (int e = threadIdx.x; e < H * D; e += blockDim.x) {
      int h = e / D;
      if (fin[h]) {
        size_t o = (size_t)b * H * D + e;
        qanchor[o] = qmean[o];
        kanchor[o] = kmean[o];
      }
    }
    for (int h = threadIdx.x; h < H; h += blockDim.x)
      if (fin[h]) has_anchor[(size_t)b * H + h] = 1;
  }
}

int launch_drift(int B, int H, int D, const float *qmean, const float *kmean, float *qanchor,
                 float *kanchor, unsigned char *has_anchor, const float *delta, float gate_lo,
                 float gate_hi, int commit, float *drift, unsigned char *refresh,
                 hipStream_t st) {
  hipLaunchKernelGGL(drift_kernel, dim3(B), dim3(kThreads), (size_t)2 * H, st, H, D, qmean,
                     kmean, qanchor, kanchor, has_anchor, delta, gate_lo, gate_hi, commit, drift,
                     refresh);
  return check_launch("drift_kernel");
}

}  // namespace heart
