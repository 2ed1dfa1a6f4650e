// Shared device/host helpers for the gfx950 kernels of the 2BW stage.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace k2bw {

// bf16 is carried as its 16-bit pattern; conversions go through the hardware's
// round-to-nearest-even convert (v_cvt_pk_bf16_f32 on gfx950).
using bf16_t = uint16_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  __bf16 h = static_cast<__bf16>(f);
  return __builtin_bit_cast(uint16_t, h);
}
// two floats -> one 32-bit word holding (lo, hi) bf16
// (one v_cvt_pk_bf16_f32: round to nearest even, as the scalar conversion)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

template <typename T> struct Act;  // activation element type traits
template <> struct Act<float> {
  static constexpr int kVec = 4;  // elements per 16-byte vector
  __device__ static float load(const float* p) { return *p; }
  __device__ static void store(float* p, float v) { *p = v; }
};
template <> struct Act<bf16_t> {
  static constexpr int kVec = 8;
  __device__ static float load(const bf16_t* p) { return bf16_to_f32(*p); }
  __device__ static void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// 8 consecutive activations <-> 8 floats.  Pointers must be 16-byte aligned for bf16 and
// 32-byte aligned for fp32 (every row stride in this library is a multiple of 8 elements).
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p);
  const float4 b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
  v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_t* p, float (&v)[8]) {
  const uint4 a = *reinterpret_cast<const uint4*>(p);
  v[0] = __uint_as_float(a.x << 16); v[1] = __uint_as_float(a.x & 0xffff0000u);
  v[2] = __uint_as_float(a.y << 16); v[3] = __uint_as_float(a.y & 0xffff0000u);
  v[4] = __uint_as_float(a.z << 16); v[5] = __uint_as_float(a.z & 0xffff0000u);
  v[6] = __uint_as_float(a.w << 16); v[7] = __uint_as_float(a.w & 0xffff0000u);
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void store8(bf16_t* p, const float (&v)[8]) {
  uint4 a;
  a.x = pack_bf16x2(v[0], v[1]); a.y = pack_bf16x2(v[2], v[3]);
  a.z = pack_bf16x2(v[4], v[5]); a.w = pack_bf16x2(v[6], v[7]);
  *reinterpret_cast<uint4*>(p) = a;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

// exact GELU and its derivative (erf form)
__device__ __forceinline__ float gelu_f(float u) {
  return 0.5f * u * (1.0f + erff(u * 0.70710678118654752f));
}
__device__ __forceinline__ float gelu_grad_f(float u) {
  const float cdf = 0.5f * (1.0f + erff(u * 0.70710678118654752f));
  const float pdf = 0.39894228040143268f * expf(-0.5f * u * u);
  return cdf + u * pdf;
}

// Versions for the bf16 GEMM epilogues, where GELU is the bulk of the arithmetic (the two
// quarter-rate instructions of an erf through exp and a reciprocal cost as much as the rest).
// Phi(u) = 0.5 + u P(u^2) with u clamped to [-4.5, 4.5]; P has degree 8, fitted (reweighted least
// squares on Chebyshev nodes) to the exact (erf) cdf: |error| < 2.5e-5 over all u, a hundred
// times under the resolution of the bf16 value it is rounded to.  The density term of the
// derivative keeps its exponential.
__device__ __forceinline__ float normal_cdf_fast(float u) {
  const float uc = __builtin_amdgcn_fmed3f(u, -4.5f, 4.5f);
  const float t = uc * uc;
  float p = 3.80569934e-11f;
  p = fmaf(p, t, -4.00232198e-09f);
  p = fmaf(p, t, 1.84616806e-07f);
  p = fmaf(p, t, -4.95974056e-06f);
  p = fmaf(p, t, 8.72766827e-05f);
  p = fmaf(p, t, -1.07673943e-03f);
  p = fmaf(p, t, 9.72949144e-03f);
  p = fmaf(p, t, -6.62404379e-02f);
  p = fmaf(p, t, 3.98866489e-01f);
  return fmaf(uc, p, 0.5f);
}
__device__ __forceinline__ float gelu_fast(float u) { return u * normal_cdf_fast(u); }
__device__ __forceinline__ float gelu_grad_fast(float u) {
  const float e = __builtin_amdgcn_exp2f(-0.72134752044448170f * u * u);   // exp(-u^2/2)
  return fmaf(u * 0.39894228040143268f, e, normal_cdf_fast(u));
}

inline int ceil_div(int64_t a, int64_t b) { return static_cast<int>((a + b - 1) / b); }

}  // namespace k2bw
