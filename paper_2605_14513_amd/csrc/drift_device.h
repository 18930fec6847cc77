// drift_workgroup: the mean-pooled drift (Eq. 4), the reuse rule (Sec. 4.2; Alg. 1), the
// layer-level gate (thresholds from the appendix on HEART configurations) and the anchor
// update for ONE batch item, executed by one whole workgroup of any multiple of 64 lanes.
// Called by the standalone drift kernel and by the tail of the fused pooling kernel.
#pragma once

#include "heart_internal.h"

namespace heart {

constexpr int kDriftMaxSlots = 8;  // D <= 512
constexpr int kDriftHeadsPerPass = 4;

// lds: 2 H bytes of LDS (marks, then final decisions).  Every lane of the workgroup must
// call this (it contains workgroup barriers).  kAcross: qmean and kmean were written by other
// workgroups of the same launch, possibly on another XCD, and are read with device-scope
// loads (same values, same arithmetic).
template <bool kAcross = false>
__device__ __forceinline__ void drift_workgroup(
    int b, int H, int D, const float *qmean, const float *kmean, float *qanchor, float *kanchor,
    unsigned char *has_anchor, const float *delta, float gate_lo, float gate_hi, int commit,
    float *drift, unsigned char *refresh, unsigned char *lds) {
  unsigned char *mark = lds;     // [H]
  unsigned char *fin = lds + H;  // [H]
  __shared__ int n_mark_sh;

  auto cur = [](const float *p) -> float {
    if constexpr (kAcross)
      return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else
      return *p;
  };
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n_waves = blockDim.x >> 6;
  const int slots = D > 64 ? D / 64 : 1;

  // A wavefront takes kDriftHeadsPerPass heads at a time and issues the loads of all of them
  // before it reduces any: the stage is bound by dependent memory round trips, not by bandwidth.
  for (int h0 = wave * kDriftHeadsPerPass; h0 < H; h0 += n_waves * kDriftHeadsPerPass) {
    float a[kDriftHeadsPerPass][kDriftMaxSlots];
    bool has[kDriftHeadsPerPass];
    float dl[kDriftHeadsPerPass];
#pragma unroll
    for (int u = 0; u < kDriftHeadsPerPass; ++u) {
      const int h = min(h0 + u, H - 1);  // (a repeated last head is computed and not stored)
      const size_t o = ((size_t)b * H + h) * D;
      // all loads are issued unconditionally (the anchor buffers always exist); a head
      // without an anchor ignores the value
      has[u] = has_anchor[(size_t)b * H + h] != 0;
      dl[u] = delta[h];
#pragma unroll
      for (int c = 0; c < kDriftMaxSlots; ++c) {
        a[u][c] = 0.f;
        const int d = lane + 64 * c;
        if (c < slots && d < D) {
          const float dq = fabsf(qanchor[o + d] - cur(qmean + o + d));
          const float dk = fabsf(kanchor[o + d] - cur(kmean + o + d));
          a[u][c] = dq + dk;
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kDriftHeadsPerPass; ++u) {
      const int h = h0 + u;
      // steps with s >= 64: a[i] += a[i+s]  <=>  slot c += slot c + s/64
#pragma unroll
      for (int s = kDriftMaxSlots / 2; s >= 1; s >>= 1) {
        if (s < slots) {
#pragma unroll
          for (int c = 0; c < kDriftMaxSlots / 2; ++c)
            if (c < s) a[u][c] = a[u][c] + a[u][c + s];
        }
      }
      float v = a[u][0];
      // steps with s < 64 (lanes >= D hold +0, adding it is exact)
#pragma unroll
      for (int s = 32; s >= 1; s >>= 1) {
        float o2 = __shfl_xor(v, s, 64);
        if (s < D) v = v + o2;
      }
      if (lane == 0 && h < H) {
        float dv = has[u] ? v : __builtin_inff();
        drift[(size_t)b * H + h] = dv;
        mark[h] = (!has[u] || dv > dl[u]) ? 1 : 0;
      }
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
    // (a lane loads its elements of a batch of passes before it stores any: the loads are
    // independent round trips, the stores conditional on the head's decision)
    constexpr int kBatch = 4;
    const int n = H * D;
    for (int e0 = threadIdx.x; e0 < n; e0 += kBatch * blockDim.x) {
      float qv[kBatch], kv[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int e = min(e0 + u * (int)blockDim.x, n - 1);
        const size_t o = (size_t)b * n + e;
        qv[u] = cur(qmean + o);
        kv[u] = cur(kmean + o);
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int e = e0 + u * (int)blockDim.x;
        if (e < n && fin[e / D]) {
          const size_t o = (size_t)b * n + e;
          qanchor[o] = qv[u];
          kanchor[o] = kv[u];
        }
      }
    }
    for (int h = threadIdx.x; h < H; h += blockDim.x)
      if (fin[h]) has_anchor[(size_t)b * H + h] = 1;
  }
}

}  // namespace heart
