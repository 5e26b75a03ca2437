// Multi-head attention of Sec. II-A over a ragged batch: per query q and head h,
//   O_h = softmax(Q_h K_h^T / sqrt(d_h) [+ ln size_j]) V_h,   heads concatenated into [T, D].
// qkv is the packed [T, 3D] output of the QKV projection (columns Q | K | V, heads contiguous).
//
//   * attention_rows_kernel -- one wave per query row, fp32 arithmetic throughout (f32 models,
//                              and the fallback for head widths the MFMA kernel does not take).
//   * attention_mfma_kernel -- bf16 MFMA with one head's K and V staged in LDS (bf16 models).
#include "common.h"
#include "kernels.h"

namespace otas {

// ------------------------------------------------------------------------------ one wave per row
// grid (ceil(max_n / 4), H, B), 256 threads.  Dynamic LDS: per wave max_n scores + d_h query floats.
template <typename T>
__global__ __launch_bounds__(256) void attention_rows_kernel(const T* __restrict__ qkv,
                                                             const int32_t* __restrict__ sizes,
                                                             const int32_t* __restrict__ off, int D, int H,
                                                             int max_n, float scale, T* __restrict__ o) {
  extern __shared__ float lds[];
  const int dh = D / H;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int q = blockIdx.z, h = blockIdx.y;
  const int base = off[q], n = off[q + 1] - base;
  const int row = blockIdx.x * 4 + wave;
  if (row >= n) return;
  float* sc = lds + (size_t)wave * (max_n + dh);
  float* qv = sc + max_n;
  const size_t ld = (size_t)3 * D;
  const T* qrow = qkv + (size_t)(base + row) * ld + h * dh;
  for (int d = lane; d < dh; d += 64) qv[d] = to_float(qrow[d]);
  __builtin_amdgcn_wave_barrier();
  // logits
  float mx = -INFINITY;
  for (int j = lane; j < n; j += 64) {
    const T* kr = qkv + (size_t)(base + j) * ld + D + h * dh;
    float s = 0.f;
    for (int d = 0; d < dh; d += 4) {
#pragma unroll
      for (int k = 0; k < 4; ++k) s = fmaf(qv[d + k], to_float(kr[d + k]), s);
    }
    s *= scale;
    if (sizes) s += logf((float)sizes[base + j]);
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int j = lane; j < n; j += 64) {
    const float e = expf(sc[j] - mx);
    sc[j] = e;
    sum += e;
  }
  sum = wave_sum(sum);
  __builtin_amdgcn_wave_barrier();
  const float inv = 1.0f / sum;
  for (int d = lane; d < dh; d += 64) {
    const T* vc = qkv + (size_t)base * ld + 2 * D + h * dh + d;
    float acc = 0.f;
    for (int j = 0; j < n; ++j) acc = fmaf(sc[j], to_float(vc[(size_t)j * ld]), acc);
    o[(size_t)(base + row) * D + h * dh + d] = from_float<T>(acc * inv);
  }
}

hipError_t launch_attention(int dtype, const void* qkv, const int32_t* sizes, const int32_t* d_off, int B,
                            int max_n, int D, int H, bool size_bias, void* o, hipStream_t s) {
  if (B <= 0 || max_n <= 0) return hipSuccess;
  const int dh = D / H;
  const float scale = 1.0f / sqrtf((float)dh);
  const int32_t* sz = size_bias ? sizes : nullptr;
  dim3 grid((max_n + 3) / 4, H, B), block(256);
  const size_t lds = (size_t)4 * (max_n + dh) * sizeof(float);
  if (dtype == 0)
    attention_rows_kernel<float><<<grid, block, lds, s>>>((const float*)qkv, sz, d_off, D, H, max_n, scale, (float*)o);
  else
    attention_rows_kernel<bf16_t><<<grid, block, lds, s>>>((const bf16_t*)qkv, sz, d_off, D, H, max_n, scale,
                                                           (bf16_t*)o);
  return hipGetLastError();
}

}  // namespace otas
