// Internal helpers shared by the HIP translation units of libheart (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "heart.h"

namespace heart {

// Records a message for heart_last_error() and returns `code`.
int fail(int code, const char *fmt, ...);
void clear_error();
// Checks hipGetLastError() after a launch; returns HEART_OK or HEART_EHIP.
int check_launch(const char *what);

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool stride_ok(const long long s[3]) {
  // strides are in 2-byte elements; 16-byte granularity = multiples of 8 elements
  return s[0] % 8 == 0 && s[1] % 8 == 0 && s[2] % 8 == 0 && s[2] > 0;
}

// bf16 pair packed in a 32-bit word -> two fp32
__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest even (inputs are finite here)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// launchers implemented per kernel file
int launch_pool(const heart_shape &s, const void *q, const void *k, float *qblk, float *kblk,
                float *qmean, float *kmean, hipStream_t st);
int launch_drift(int B, int H, int D, const float *qmean, const float *kmean, float *qanchor,
                 float *kanchor, unsigned char *has_anchor, const float *delta, float gate_lo,
                 float gate_hi, int commit, float *drift, unsigned char *refresh,
                 hipStream_t st);
int launch_mask_topp(int B, int H, int Nb, int D, const float *qblk, const float *kblk,
                     const float *scores_in, const float *tau, const unsigned char *refresh,
                     int n_always_kv, int n_dense_q, int min_keep, unsigned char *mask,
                     int *kept_idx, int *kept_count, float *scores_out, hipStream_t st);
int launch_attn(const heart_shape &s, const void *q, const void *k, const void *v,
                const int *kept_idx, const int *kept_count, float scale, void *out, float *lse,
                hipStream_t st);

}  // namespace heart
