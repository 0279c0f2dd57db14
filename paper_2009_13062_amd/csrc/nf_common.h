// Shared device-side helpers of the merged-operator kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/netfuse.h"

namespace nf {

typedef uint16_t bf16_t;   // bfloat16 bit pattern as stored in HBM

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

constexpr int kWave = 64;          // CDNA wavefront width
constexpr int kNumXcd = 8;         // MI355X: 8 XCDs, workgroups are dealt to them round-robin

__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// Round to nearest even; NaN stays a (quiet) NaN.  gfx950 converts in hardware (v_cvt_pk_bf16_f32).
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
// two floats -> one dword of bf16 (lo in bits 15:0)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Non-temporal 16-byte load for operands that are read once per forward pass (the weights of a matmul): they
// then do not displace the activations that neighbouring operators exchange through the caches.
typedef uint32_t nf_u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ldnt16(const void* p) {
  const nf_u32x4_t v = __builtin_nontemporal_load((const nf_u32x4_t*)p);
  return make_uint4(v.x, v.y, v.z, v.w);
}

template <typename T> __device__ __forceinline__ float load_f32(const T* p);
template <> __device__ __forceinline__ float load_f32<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_f32<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }

template <typename T> __device__ __forceinline__ void store_f32(T* p, float v);
template <> __device__ __forceinline__ void store_f32<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_f32<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16(v); }

// GELU in its erf form, v * Phi(v), with one transcendental: for a = |v|, 1 - Phi(a) = 2^g(a) where
// g(a) = log2(erfc(a / sqrt 2) / 2) is smooth and is replaced by a degree-6 polynomial fitted (weighted
// minimax of the resulting GELU error) on [0, 8]; beyond 8 the tail 2^g is below 1e-15 and a is clamped.
// Phi(v) = 1 - 2^g for v >= 0 and 2^g for v < 0.  Maximum absolute error against the exact function in
// fp32 arithmetic: 6.3e-7 (the rounding of the result itself near |v| = 4); NaN propagates.
__device__ __forceinline__ float gelu_erf(float v) {
  const float a = fminf(fabsf(v), 8.0f);
  float g = fmaf(3.309327075839974e-05f, a, -0.0007692237268202007f);
  g = fmaf(g, a, 0.00808072928339243f);
  g = fmaf(g, a, -0.05341212451457977f);
  g = fmaf(g, a, -0.4587709605693817f);
  g = fmaf(g, a, -1.1512017250061035f);
  g = fmaf(g, a, -0.999993085861206f);
  const float tail = __builtin_amdgcn_exp2f(g);
  return v * (v < 0.f ? tail : 1.0f - tail);
}

__device__ __forceinline__ float apply_act(float v, int act) {
  if (act == NF_ACT_RELU) return v > 0.f ? v : (v != v ? v : 0.f);
  if (act == NF_ACT_GELU) return gelu_erf(v);
  return v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
  return v;
}

// Workgroups are handed to the 8 XCDs round-robin (id % 8), and each XCD has its own L2.  This
// maps the hardware id to a logical id such that consecutive logical ids run on the same XCD, so
// tiles that share operands (the tiles of one model) share an L2.  Bijective for any total.
__device__ __forceinline__ unsigned xcd_remap(unsigned hw_id, unsigned total) {
  const unsigned xcd = hw_id % kNumXcd, local = hw_id / kNumXcd;
  const unsigned base = total / kNumXcd, rem = total % kNumXcd;
  const unsigned start = xcd * base + (xcd < rem ? xcd : rem);
  return start + local;
}

}  // namespace nf
