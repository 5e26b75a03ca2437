// Shared device helpers for the gfx950 kernels: storage types, vector loads, wave reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace otas {

typedef __bf16 bf16_t;
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

template <typename T> struct Vec;          // 16-byte vector of the storage type
template <> struct Vec<float> {
  static constexpr int N = 4;
  floatx4 v;
  __device__ float get(int i) const { return v[i]; }
  __device__ void set(int i, float f) { v[i] = f; }
};
template <> struct Vec<bf16_t> {
  static constexpr int N = 8;
  bf16x8 v;
  __device__ float get(int i) const { return (float)v[i]; }
  __device__ void set(int i, float f) { v[i] = (bf16_t)f; }   // round to nearest even (v_cvt_pk_bf16_f32)
};

template <typename T> __device__ inline Vec<T> load_vec(const T* p) {
  return *reinterpret_cast<const Vec<T>*>(p);
}
template <typename T> __device__ inline void store_vec(T* p, const Vec<T>& v) {
  *reinterpret_cast<Vec<T>*>(p) = v;
}

__device__ inline float to_float(float x) { return x; }
__device__ inline float to_float(bf16_t x) { return (float)x; }
template <typename T> __device__ inline T from_float(float x);
template <> __device__ inline float from_float<float>(float x) { return x; }
template <> __device__ inline bf16_t from_float<bf16_t>(float x) { return (bf16_t)x; }

// Butterfly reductions over the 64 lanes of a wave: every lane ends with the same value, and the
// order of additions does not depend on which lanes hold data.
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

// Exact GELU: 0.5 x (1 + erf(x / sqrt 2)).
__device__ inline float gelu_exact(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752440f)); }

// The same GELU for results that are rounded to bf16 afterwards: erf by the rational-exponential
// formula 7.1.26 of Abramowitz & Stegun (|error| < 1.5e-7, three orders below half a bf16 unit),
// which costs one exp, one reciprocal and a short polynomial instead of the library erff.
// With z = |x| / sqrt 2, t = 1 / (1 + p z) and erf z = 1 - poly(t) t exp(-z^2):
//   0.5 x (1 + erf(x / sqrt 2)) = max(x, 0) - |x| * (0.5 poly(t)) * t * exp(-x^2 / 2),
// which needs neither the sign transfer nor z itself (the halves are folded into the coefficients).
__device__ inline float gelu_bf16(float x) {
  const float ax = fabsf(x);
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752440f, ax, 1.0f));   // 1 ulp reciprocal
  const float e = __builtin_amdgcn_exp2f(x * x * (-0.5f * 1.44269504088896340736f));
  float p = fmaf(0.5f * 1.061405429f, t, 0.5f * -1.453152027f);
  p = fmaf(p, t, 0.5f * 1.421413741f);
  p = fmaf(p, t, 0.5f * -0.284496736f);
  p = fmaf(p, t, 0.5f * 0.254829592f);
  const float relu = __builtin_amdgcn_fmed3f(x, 0.0f, 3.0e38f);   // max(x, 0) in one instruction
  return fmaf(-ax, p * t * e, relu);
}

}  // namespace otas
