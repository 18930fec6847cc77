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
// The body lives in drift_device.h (drift_workgroup): the standalone kernel below and the
// tail of the fused pooling kernel run the same code, so both give the same bits.
#include "drift_device.h"

namespace heart {

constexpr int kThreads = 1024; // 16 wavefronts: 16 heads in flight per pass

__global__ __launch_bounds__(kThreads) void drift_kernel(
    int H, int D, const float *__restrict__ qmean, const float *__restrict__ kmean,
    float *__restrict__ qanchor, float *__restrict__ kanchor,
    unsigned char *__restrict__ has_anchor, const float *__restrict__ delta, float gate_lo,
    float gate_hi, int commit, float *__restrict__ drift, unsigned char *__restrict__ refresh) {
  extern __shared__ unsigned char smem[];  // [2 H]: marks, then final decisions
  drift_workgroup(blockIdx.x, H, D, qmean, kmean, qanchor, kanchor, has_anchor, delta, gate_lo,
                  gate_hi, commit, drift, refresh, smem);
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
