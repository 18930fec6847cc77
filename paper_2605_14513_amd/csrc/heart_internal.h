// Internal helpers shared by the HIP translation units of libheart (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "heart.h"
#include "heart_diag.h"

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

// Lane exchanges on the VALU.  v_permlane16_swap / v_permlane32_swap exchange the odd
// rows (upper half) of their first operand with the even rows (lower half) of the
// second.  Fed the same value twice they return the pair (r0, r1) with
//   swap16: r0 = rows (0,0,2,2), r1 = rows (1,1,3,3) of v     (a row is 16 lanes)
//   swap32: r0 = halves (lo, lo), r1 = halves (hi, hi) of v
// so OP(r0, r1) combines every lane with its partner row / half, identically on both
// sides.  The second operand goes through an empty asm so that the compiler cannot
// see that both operands are the same value (it would then fold r0 and r1 into one).
__device__ __forceinline__ void swap_rows16(uint32_t v, uint32_t &r0, uint32_t &r1) {
  uint32_t w = v;
  asm volatile("" : "+v"(w));
  const auto r = __builtin_amdgcn_permlane16_swap(v, w, false, false);
  r0 = r[0];
  r1 = r[1];
}
__device__ __forceinline__ void swap_halves32(uint32_t v, uint32_t &r0, uint32_t &r1) {
  uint32_t w = v;
  asm volatile("" : "+v"(w));
  const auto r = __builtin_amdgcn_permlane32_swap(v, w, false, false);
  r0 = r[0];
  r1 = r[1];
}

// Wave-wide reductions that leave the result in every lane, on the VALU only (no LDS
// round trips): xor-1 and xor-2 inside quads and rotations by 4 and 8 inside rows of 16
// lanes as DPP modifiers, then the row and half exchanges above.
#define HEART_WAVE_REDUCE(T, v, OP)                                                      \
  do {                                                                                   \
    v = OP(v, __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(                          \
                  0u, __builtin_bit_cast(uint32_t, v), 0xB1, 0xf, 0xf, false))); /* quad_perm [1,0,3,2] */ \
    v = OP(v, __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(                          \
                  0u, __builtin_bit_cast(uint32_t, v), 0x4E, 0xf, 0xf, false))); /* quad_perm [2,3,0,1] */ \
    v = OP(v, __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(                          \
                  0u, __builtin_bit_cast(uint32_t, v), 0x124, 0xf, 0xf, false))); /* row_ror:4 */ \
    v = OP(v, __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(                          \
                  0u, __builtin_bit_cast(uint32_t, v), 0x128, 0xf, 0xf, false))); /* row_ror:8 */ \
    {                                                                                    \
      uint32_t r0_, r1_;                                                                 \
      swap_rows16(__builtin_bit_cast(uint32_t, v), r0_, r1_);                            \
      v = OP(__builtin_bit_cast(T, r0_), __builtin_bit_cast(T, r1_));                    \
    }                                                                                    \
    {                                                                                    \
      uint32_t r0_, r1_;                                                                 \
      swap_halves32(__builtin_bit_cast(uint32_t, v), r0_, r1_);                          \
      v = OP(__builtin_bit_cast(T, r0_), __builtin_bit_cast(T, r1_));                    \
    }                                                                                    \
  } while (0)
// The same reduction over each half (32 lanes) of the wavefront separately: the result of
// lanes 0..31 in every lane of 0..31, that of lanes 32..63 in every lane of 32..63.
#define HEART_HALF_REDUCE(T, v, OP)                                                      \
  do {                                                                                   \
    v = OP(v, __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(                          \
                  0u, __builtin_bit_cast(uint32_t, v), 0xB1, 0xf, 0xf, false)));          \
    v = OP(v, __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(                          \
                  0u, __builtin_bit_cast(uint32_t, v), 0x4E, 0xf, 0xf, false)));          \
    v = OP(v, __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(                          \
                  0u, __builtin_bit_cast(uint32_t, v), 0x124, 0xf, 0xf, false)));         \
    v = OP(v, __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(                          \
                  0u, __builtin_bit_cast(uint32_t, v), 0x128, 0xf, 0xf, false)));         \
    {                                                                                    \
      uint32_t r0_, r1_;                                                                 \
      swap_rows16(__builtin_bit_cast(uint32_t, v), r0_, r1_);                            \
      v = OP(__builtin_bit_cast(T, r0_), __builtin_bit_cast(T, r1_));                    \
    }                                                                                    \
  } while (0)
// (functions, not expression macros: each argument -- a DPP read -- must be evaluated
// exactly once and with all lanes active)
__device__ __forceinline__ uint32_t heart_op_umax(uint32_t a, uint32_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint32_t heart_op_umin(uint32_t a, uint32_t b) { return a < b ? a : b; }
#define HEART_OP_ADD(a, b) ((a) + (b))
#define HEART_OP_FMAX(a, b) fmaxf((a), (b))
#define HEART_OP_UMAX(a, b) heart_op_umax((a), (b))
#define HEART_OP_UMIN(a, b) heart_op_umin((a), (b))

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
  HEART_WAVE_REDUCE(uint32_t, v, HEART_OP_ADD);
  return v;
}
// Sum of per-lane masses below 2^40: two 32-bit reductions over the low 20 bits and the
// rest (each stays below 2^32 for 64 lanes), recombined exactly.
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
  uint32_t lo = (uint32_t)v & 0xfffffu, hi = (uint32_t)(v >> 20);
  HEART_WAVE_REDUCE(uint32_t, lo, HEART_OP_ADD);
  HEART_WAVE_REDUCE(uint32_t, hi, HEART_OP_ADD);
  return ((unsigned long long)hi << 20) + lo;
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
  HEART_WAVE_REDUCE(uint32_t, v, HEART_OP_UMIN);
  return v;
}
__device__ __forceinline__ int wave_sum_i32(int v) { return (int)wave_sum_u32((uint32_t)v); }
__device__ __forceinline__ uint32_t half_sum_u32(uint32_t v) {
  HEART_HALF_REDUCE(uint32_t, v, HEART_OP_ADD);
  return v;
}
__device__ __forceinline__ uint32_t half_max_u32(uint32_t v) {
  HEART_HALF_REDUCE(uint32_t, v, HEART_OP_UMAX);
  return v;
}
__device__ __forceinline__ float half_max_f32(float v) {
  HEART_HALF_REDUCE(float, v, HEART_OP_FMAX);
  return v;
}
__device__ __forceinline__ float half_sum_f32(float v) {
  HEART_HALF_REDUCE(float, v, HEART_OP_ADD);
  return v;
}
__device__ __forceinline__ float wave_max_f32(float v) {
  HEART_WAVE_REDUCE(float, v, HEART_OP_FMAX);
  return v;
}
__device__ __forceinline__ float wave_sum_f32(float v) {
  HEART_WAVE_REDUCE(float, v, HEART_OP_ADD);
  return v;
}

// Index of the current device, for per-device caches of launch attributes (-1 on error).
constexpr int kMaxDevices = 64;
inline int current_device() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -1;
  return dev;
}

// Per-device "done" flags for set-up that is per function and device (launch attributes,
// device queries).  Host threads may race on the first call: the set-up calls are
// idempotent and the flags are atomic, so the worst case is that two threads both do it.
struct DeviceFlags {
  std::atomic<int> v[kMaxDevices];
};
inline hipError_t set_max_lds_once(DeviceFlags &f, int dev, const void *kern, int bytes) {
  if (f.v[dev].load(std::memory_order_acquire)) return hipSuccess;
  const hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) f.v[dev].store(1, std::memory_order_release);
  return e;
}
// Number of compute units of device `dev` (0 on error), queried once per device.
inline int cu_count(int dev) {
  static DeviceFlags n;
  int v = n.v[dev].load(std::memory_order_acquire);
  if (v > 0) return v;
  if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0)
    return 0;
  n.v[dev].store(v, std::memory_order_release);
  return v;
}

// launchers implemented per kernel file
int launch_pool(const heart_shape &s, const void *q, const void *k, float *qblk, float *kblk,
                float *qmean, float *kmean, hipStream_t st);
int launch_pool_drift(const heart_shape &s, const void *q, const void *k, float *qblk, float *kblk,
                      float *qmean, float *kmean, float *qanchor, float *kanchor,
                      unsigned char *has_anchor, const float *delta, float gate_lo, float gate_hi,
                      int commit, float *drift, unsigned char *refresh, unsigned *tickets,
                      hipStream_t st);
int launch_drift(int B, int H, int D, const float *qmean, const float *kmean, float *qanchor,
                 float *kanchor, unsigned char *has_anchor, const float *delta, float gate_lo,
                 float gate_hi, int commit, float *drift, unsigned char *refresh,
                 hipStream_t st);
int launch_mask_topp(int B, int H, int Nb, int D, const float *qblk, const float *kblk,
                     const float *scores_in, const float *tau, const unsigned char *refresh,
                     int n_always_kv, int n_dense_q, int min_keep, unsigned char *mask,
                     int *kept_idx, int *kept_count, float *scores_out, void *workspace,
                     hipStream_t st);
size_t mask_topp_workspace_bytes(int B, int H, int Nb, int D);
int launch_attn(const heart_shape &s, const void *q, const void *k, const void *v,
                const int *kept_idx, const int *kept_count, float scale, unsigned flags, void *out,
                float *lse, int *order, hipStream_t st);

// Device address, on the current device, of the library's static launch-plan array
// (HEART_ATTN_STATIC_PLAN_BYTES bytes).
int attn_static_plan(int **ptr);

int launch_antidiag(const heart_shape &s, const void *q, const void *k, int stride,
                    const unsigned char *refresh, float *scores, float *workspace, hipStream_t st);
size_t antidiag_workspace_bytes(const heart_shape &s, int stride);

int launch_ebc_band_error(long long C, int T, int Y, int X, const float *err, const float *dense,
                          const double *w, double epsilon, double *ws, double *out,
                          hipStream_t st);
size_t ebc_workspace_bytes(long long C, int T, int Y, int X);
int ebc_select_host(int n, int k, const double *E, const double *S, double s_min, int *choice,
                    double *total_error, long long *nodes);
int launch_ubench_mfma(const void *a, const void *b, int n_wg, int iters, float *sink,
                       hipStream_t st);
int launch_ubench_copy(const void *src, void *dst, size_t bytes, hipStream_t st);
int launch_ubench_read(const void *src, size_t bytes, unsigned *sink, hipStream_t st);

}  // namespace heart
