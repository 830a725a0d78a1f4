// Shared host/device helpers of the Parle library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>

#include "../../include/parle.h"

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef unsigned short us4 __attribute__((ext_vector_type(4)));
typedef unsigned short us8 __attribute__((ext_vector_type(8)));
typedef unsigned short bf16_t;  // raw bfloat16 bits

#define PARLE_WAVE 64

// fp32 -> bf16, round to nearest even; NaN stays a quiet NaN.  gfx950 converts in hardware
// (v_cvt_pk_bf16_f32, two values per instruction).
typedef __bf16 bf16x2_hw __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned short f32_to_bf16(float f) {
  const __bf16 r = (__bf16)f;
  return __builtin_bit_cast(unsigned short, r);
}
// (lo, hi) -> lo in bits 0..15, hi in bits 16..31
__device__ __forceinline__ unsigned int f32x2_to_bf16x2(float lo, float hi) {
  const f2 v = {lo, hi};
  const bf16x2_hw r = __builtin_convertvector(v, bf16x2_hw);
  return __builtin_bit_cast(unsigned int, r);
}
__device__ __forceinline__ us4 f32x4_to_bf16x4(f4 v) {
  typedef unsigned int u2 __attribute__((ext_vector_type(2)));
  const u2 r = {f32x2_to_bf16x2(v.x, v.y), f32x2_to_bf16x2(v.z, v.w)};
  return __builtin_bit_cast(us4, r);
}
__device__ __forceinline__ float bf16_to_f32(unsigned short h) { return __uint_as_float(((unsigned int)h) << 16); }

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = PARLE_WAVE / 2; off > 0; off >>= 1) v += __shfl_down(v, off, PARLE_WAVE);
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = PARLE_WAVE / 2; off > 0; off >>= 1) v += __shfl_down(v, off, PARLE_WAVE);
  return v;
}

// Text behind parle_last_error(NULL) for entry points that have no context (calling thread only).
void parle_internal_set_error(const std::string &msg);

static inline bool aligned_to(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// fp32 -> bf16 (round to nearest even) copy of `count` elements (count % 4 == 0), enqueued on `st`.
parle_status parle_internal_to_bf16(hipStream_t st, const float *src, void *dst, int64_t count);

// Launchers behind the C ABI that also take `coupling_dev`: two floats {g, r} in device memory that
// override the by-value multipliers (a captured launch cannot change its arguments).  NULL = use the
// arguments.
parle_status parle_internal_set_coupling(hipStream_t st, float *coupling_dev, float g, float r);
// The inner-step counter in device memory: set it, add one to it (one-thread kernels).
parle_status parle_internal_set_step(hipStream_t st, long long *step_dev, long long k);
parle_status parle_internal_advance_step(hipStream_t st, long long *step_dev);
parle_status parle_internal_inner_update(hipStream_t st, int32_t n, int64_t n_pad, const float *grad, const float *x,
                                         float *y, float *vy, float *z, void *y_bf16, float eta_inner, float momentum,
                                         float alpha, float weight_decay, float g, const float *coupling_dev);
parle_status parle_internal_elastic_step(hipStream_t st, int32_t n, int64_t n_pad, const float *grad, float *xa,
                                         float *v, float *x_ref, void *xa_bf16, float eta, float eta_ref,
                                         float momentum, float weight_decay, float r, const float *coupling_dev);
