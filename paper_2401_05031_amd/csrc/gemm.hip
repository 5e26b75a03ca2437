// Linear layers of the encoder block (Sec. II-A: per-head Q/K/V projections, the linear after
// the concatenated heads, and the MLP):  Y[M,N] = epilogue(X[M,K] W[N,K]^T + bias[N]).
//
// Two kernels:
//   * gemm_valu_kernel  -- plain fp32 FMA tiles; the true-fp32 path (f32 models) and the fallback
//                          for shapes the MFMA kernel does not take.
//   * gemm_mfma_kernel  -- bf16 MFMA (v_mfma_f32_32x32x16_bf16), fp32 accumulate, LDS-staged
//                          tiles, fused bias / GELU / residual epilogue (bf16 models).
#include "common.h"
#include "kernels.h"

namespace otas {

// Output element type: the residual epilogue writes the float residual stream, the others the
// model's storage type.
template <typename T, int EPI> struct OutType { typedef T type; };
template <typename T> struct OutType<T, EPI_RESIDUAL> { typedef float type; };

template <int EPI>
__device__ inline float epilogue_value(float acc, float bias, const float* res, size_t idx) {
  float v = acc + bias;
  if (EPI == EPI_GELU) v = gelu_exact(v);
  if (EPI == EPI_RESIDUAL) v += res[idx];
  return v;
}

// ------------------------------------------------------------------------------ fp32 FMA tiles
// 64x64 output tile, K step 16, 256 threads, 4x4 outputs per thread, operands converted to fp32
// in LDS ([k][row] layout so that the inner product walks consecutive rows).
template <typename T, int EPI>
__global__ __launch_bounds__(256) void gemm_valu_kernel(const T* __restrict__ A, const T* __restrict__ W,
                                                        const T* __restrict__ bias, const float* res,
                                                        typename OutType<T, EPI>::type* Y, int64_t M, int N,
                                                        int K) {
  typedef typename OutType<T, EPI>::type OT;
  __shared__ float As[16][64 + 4];
  __shared__ float Ws[16][64 + 4];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int64_t m0 = (int64_t)blockIdx.y * 64;
  const int n0 = blockIdx.x * 64;
  const int lr = threadIdx.x >> 2, lk = (threadIdx.x & 3) * 4;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int k0 = 0; k0 < K; k0 += 16) {
    float a[4] = {0.f, 0.f, 0.f, 0.f}, w[4] = {0.f, 0.f, 0.f, 0.f};
    if (m0 + lr < M && k0 + lk < K) {
      const T* p = A + (size_t)(m0 + lr) * K + k0 + lk;
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = to_float(p[i]);
    }
    if (n0 + lr < N && k0 + lk < K) {
      const T* p = W + (size_t)(n0 + lr) * K + k0 + lk;
#pragma unroll
      for (int i = 0; i < 4; ++i) w[i] = to_float(p[i]);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) { As[lk + i][lr] = a[i]; Ws[lk + i][lr] = w[i]; }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float av[4], wv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { av[i] = As[kk][ty * 4 + i]; wv[i] = Ws[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], wv[j], acc[i][j]);
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      const size_t idx = (size_t)m * N + n;
      Y[idx] = from_float<OT>(epilogue_value<EPI>(acc[i][j], to_float(bias[n]), res, idx));
    }
  }
}

template <typename T>
static hipError_t linear_valu(const void* x, const void* w, const void* bias, const float* res, void* y,
                              int64_t M, int N, int K, int epi, hipStream_t s) {
  dim3 grid((N + 63) / 64, (unsigned)((M + 63) / 64)), block(256);
#define OTAS_GEMM(E)                                                                                        \
  gemm_valu_kernel<T, E><<<grid, block, 0, s>>>((const T*)x, (const T*)w, (const T*)bias, res,           \
                                                (typename OutType<T, E>::type*)y, M, N, K)
  if (epi == EPI_NONE) OTAS_GEMM(EPI_NONE);
  else if (epi == EPI_GELU) OTAS_GEMM(EPI_GELU);
  else OTAS_GEMM(EPI_RESIDUAL);
#undef OTAS_GEMM
  return hipGetLastError();
}

hipError_t launch_linear(int dtype, const void* x, const void* w, const void* bias, const float* res, void* y,
                         int64_t M, int N, int K, int epi, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  if (dtype == 0) return linear_valu<float>(x, w, bias, res, y, M, N, K, epi, s);
  return linear_valu<bf16_t>(x, w, bias, res, y, M, N, K, epi, s);
}

}  // namespace otas
