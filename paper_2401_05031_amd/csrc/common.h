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

// The same GELU for results that are rounded to bf16 afterwards, written as
//   0.5 x (1 + erf(x / sqrt 2)) = max(x, 0) - |x| Phi(-|x|),   Phi = the standard normal distribution function.
// log2 Phi(-u) is smooth and close to a parabola: a polynomial of degree 6 in u on [0, 6] (least squares on a
// fine grid, re-weighted until the error of u Phi(-u) is flat) reproduces u Phi(-u) to 5e-8; beyond u = 6 the
// term is below 6e-9 and u is clamped (in the polynomial and in the product).  Evaluated in fp32 the whole function is within 3e-7 of the exact one
// over [-8, 8], four orders below half a bf16 unit of a result of size 1, for six multiply-adds and one exp2 --
// against a reciprocal, an exp2 and eleven other instructions for erf by formula 7.1.26 of Abramowitz & Stegun
// (same accuracy), which this replaces: transcendentals run at quarter rate, and in the GEMM epilogue of the
// MLP's first linear this function is all the ALU work there is.
__device__ inline float gelu_bf16(float x) {
  const float u = fminf(fabsf(x), 6.0f);
  float p = fmaf(3.30306029e-05f, u, -7.68667320e-04f);
  p = fmaf(p, u, 8.07889923e-03f);
  p = fmaf(p, u, -5.34093268e-02f);
  p = fmaf(p, u, -4.58772987e-01f);
  p = fmaf(p, u, -1.15120113e+00f);
  p = fmaf(p, u, -9.99993145e-01f);
  const float relu = __builtin_amdgcn_fmed3f(x, 0.0f, 3.0e38f);   // max(x, 0) in one instruction
  return fmaf(-u, __builtin_amdgcn_exp2f(p), relu);   // u, not |x|: beyond 6 the term stays 6e-9 (also for infinities)
}

}  // namespace otas
