// HBM-bound row kernels: integer fill/copy, the prompting module's ragged concatenation
// (Sec. II-B / III-B), LayerNorm (Sec. II-A "normalization"), and the merging module's data
// movement fused with the LayerNorm behind it (Sec. II-C).
#include "common.h"
#include "kernels.h"

namespace otas {

// ---------------------------------------------------------------------------------- fill / copy
__global__ void fill_i32_kernel(int32_t* p, int32_t v, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
__global__ void copy_i32_kernel(const int32_t* __restrict__ a, int32_t* __restrict__ b, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) b[i] = a[i];
}
// One wave that stays busy for `ticks` periods of the constant-rate wall clock (a kernel of known
// duration, used to calibrate what an event pair adds to a launch).  The iteration cap makes the loop end
// whatever the clock does.
__global__ void spin_kernel(int64_t ticks, int32_t* sink) {
  const int64_t t0 = wall_clock64();
  int32_t it = 0;
  while (it < (1 << 22) && wall_clock64() - t0 < ticks) ++it;
  if (threadIdx.x == 0) sink[0] = it;
}
hipError_t launch_spin(int64_t ticks, int32_t* sink, hipStream_t s) {
  spin_kernel<<<dim3(1), dim3(64), 0, s>>>(ticks, sink);
  return hipGetLastError();
}
// One wave that `samples` times sleeps 4 x 8128 shader clocks (s_sleep 127 = 127 x 64 clocks; a sleeping wave
// needs no issue slots, so the waves it shares a SIMD with do not stretch it) and stores how many periods of the
// constant-rate wall clock that took: 4 * 8128 / ticks[s] = shader clocks per wall-clock period while whatever else
// is in flight on the chip runs.  Ends by itself after `samples` samples.
__global__ void clock_probe_kernel(uint32_t* ticks, int32_t samples) {
  for (int32_t s = 0; s < samples; ++s) {
    const uint64_t t0 = wall_clock64();
    asm volatile("s_sleep 127\n s_sleep 127\n s_sleep 127\n s_sleep 127");
    const uint64_t t1 = wall_clock64();
    if (threadIdx.x == 0) ticks[s] = (uint32_t)(t1 - t0);
  }
}
hipError_t launch_clock_probe(uint32_t* ticks, int32_t samples, hipStream_t s) {
  clock_probe_kernel<<<dim3(1), dim3(64), 0, s>>>(ticks, samples);
  return hipGetLastError();
}
hipError_t launch_fill_i32(int32_t* p, int32_t v, int64_t n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  fill_i32_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(p, v, n);
  return hipGetLastError();
}
hipError_t launch_copy_i32(const int32_t* a, int32_t* b, int64_t n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  copy_i32_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(a, b, n);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------- prepend
// One 16-byte chunk per thread.  blockIdx.y = query; blockIdx.x strides over the query's
// (row, chunk) pairs.  Output row i of a query comes from: i < n_lead -> token i;
// i < n_lead + P -> prompt i - n_lead; else token i - P.
template <typename T>
__global__ void prepend_kernel(const T* __restrict__ tokens, const T* __restrict__ prompts,
                               T* __restrict__ out, const int32_t* __restrict__ tok_off,
                               const int32_t* __restrict__ prm_beg, const int32_t* __restrict__ prm_cnt,
                               const int32_t* __restrict__ out_off, int D, int n_lead) {
  constexpr int V = Vec<T>::N;
  const int q = blockIdx.y;
  const int o0 = out_off[q], n_out = out_off[q + 1] - o0;
  const int t0 = tok_off[q], p0 = prm_beg[q], P = prm_cnt[q];   // the query's rows of the prompt tensor
  const int chunks = D / V;
  const int total = n_out * chunks;
  for (int t = blockIdx.x * blockDim.x + threadIdx.x; t < total; t += gridDim.x * blockDim.x) {
    const int i = t / chunks, c = (t - i * chunks) * V;
    const T* src;
    if (i < n_lead) src = tokens + (size_t)(t0 + i) * D;
    else if (i < n_lead + P) src = prompts + (size_t)(p0 + i - n_lead) * D;
    else src = tokens + (size_t)(t0 + i - P) * D;
    store_vec<T>(out + (size_t)(o0 + i) * D + c, load_vec<T>(src + c));
  }
}

hipError_t launch_prepend(int dtype, const void* tokens, const void* prompts, void* out,
                          const int32_t* d_tok_off, const int32_t* d_prm_beg, const int32_t* d_prm_cnt,
                          const int32_t* d_out_off, int B, int max_n_out, int D, int n_lead,
                          hipStream_t s) {
  if (B <= 0 || max_n_out <= 0) return hipSuccess;
  const int V = dtype == 0 ? 4 : 8;
  const int64_t tasks = (int64_t)max_n_out * (D / V);
  unsigned gx = (unsigned)((tasks + 255) / 256);
  if (gx > 64) gx = 64;
  dim3 grid(gx, B), block(256);
  if (dtype == 0)
    prepend_kernel<float><<<grid, block, 0, s>>>((const float*)tokens, (const float*)prompts, (float*)out,
                                                 d_tok_off, d_prm_beg, d_prm_cnt, d_out_off, D, n_lead);
  else
    prepend_kernel<bf16_t><<<grid, block, 0, s>>>((const bf16_t*)tokens, (const bf16_t*)prompts,
                                                  (bf16_t*)out, d_tok_off, d_prm_beg, d_prm_cnt, d_out_off, D, n_lead);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------- per-layer prompting
// The prompting module in front of a layer l >= 1 (Sec. III-B: it sits before the normalisation of
// every layer), on the float residual stream.  grow = false: rows n_lead .. n_lead + P - 1 of every
// query are overwritten with this layer's prompts (x_new == x_old, only those rows are touched).
// grow = true: the P prompts are inserted at row n_lead, the old rows are copied around them into
// x_new (a different buffer; old_off / new_off are the packed offsets before and after).
// 4 floats per thread; blockIdx.y = query.
template <typename T>
__global__ void deep_prompt_kernel(const float* __restrict__ x_old, float* __restrict__ x_new,
                                   const T* __restrict__ prompts, const int32_t* __restrict__ old_off,
                                   const int32_t* __restrict__ new_off, const int32_t* __restrict__ prm_off,
                                   int D, int n_lead, bool grow) {
  const int q = blockIdx.y;
  const int p0 = prm_off[q], P = prm_off[q + 1] - p0;
  const int o0 = new_off[q], n_new = new_off[q + 1] - o0, i0 = old_off[q];
  const int chunks = D / 4;
  const int first = grow ? 0 : n_lead, rows = grow ? n_new : P;   // rows this launch writes
  for (int t = blockIdx.x * blockDim.x + threadIdx.x; t < rows * chunks; t += gridDim.x * blockDim.x) {
    const int i = first + t / chunks, c = (t % chunks) * 4;
    Vec<float> v;
    if (i >= n_lead && i < n_lead + P) {
      const T* src = prompts + (size_t)(p0 + i - n_lead) * D + c;
#pragma unroll
      for (int k = 0; k < 4; ++k) v.set(k, to_float(src[k]));
    } else {
      v = load_vec<float>(x_old + (size_t)(i0 + (i < n_lead ? i : i - P)) * D + c);
    }
    store_vec<float>(x_new + (size_t)(o0 + i) * D + c, v);
  }
}

hipError_t launch_deep_prompt(int dtype, const float* x_old, float* x_new, const void* prompts,
                              const int32_t* d_old_off, const int32_t* d_new_off, const int32_t* d_prm_off, int B,
                              int max_rows, int D, int n_lead, bool grow, hipStream_t s) {
  if (B <= 0 || max_rows <= 0) return hipSuccess;
  if (D % 4 != 0 || (grow && x_old == x_new)) return hipErrorInvalidValue;
  const int64_t tasks = (int64_t)max_rows * (D / 4);
  unsigned gx = (unsigned)((tasks + 255) / 256);
  if (gx > 64) gx = 64;
  dim3 grid(gx, B), block(256);
  if (dtype == 0)
    deep_prompt_kernel<float><<<grid, block, 0, s>>>(x_old, x_new, (const float*)prompts, d_old_off, d_new_off,
                                                     d_prm_off, D, n_lead, grow);
  else
    deep_prompt_kernel<bf16_t><<<grid, block, 0, s>>>(x_old, x_new, (const bf16_t*)prompts, d_old_off, d_new_off,
                                                      d_prm_off, D, n_lead, grow);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------- LayerNorm
// One wave per row, the row held in registers (NCH 16-byte chunks per lane), two-pass statistics
// in fp32 (mean, then the biased variance of the centred values).
// XT = type of the input row (the residual stream is float), T = type of gamma, beta and the output.
// Each lane owns chunks of 8 consecutive columns (two 16-byte loads of a float row).
// xw != nullptr: the row is also written out as floats (16-bit tokens entering the float residual
// stream: the widening copy rides on the first block's LayerNorm).
template <typename XT, typename T, int NCH>
__global__ __launch_bounds__(256) void layer_norm_kernel(const XT* __restrict__ x, const T* __restrict__ g,
                                                         const T* __restrict__ b, T* __restrict__ y,
                                                         int64_t Trows, int D, float eps, float* __restrict__ xw) {
  constexpr int V = 8;
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= Trows) return;
  const int chunks = D / V;
  const XT* xr = x + (size_t)row * D;
  float v[NCH][V];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
    if (c < chunks) {
#pragma unroll
      for (int k0 = 0; k0 < V; k0 += Vec<XT>::N) {
        Vec<XT> t = load_vec<XT>(xr + c * V + k0);
#pragma unroll
        for (int k = 0; k < Vec<XT>::N; ++k) { v[i][k0 + k] = t.get(k); sum += v[i][k0 + k]; }
      }
    } else {
#pragma unroll
      for (int k = 0; k < V; ++k) v[i][k] = 0.f;
    }
  }
  if (xw) {
    float* wr = xw + (size_t)row * D;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = lane + 64 * i;
      if (c < chunks) {
        Vec<float> lo, hi;
#pragma unroll
        for (int k = 0; k < 4; ++k) { lo.set(k, v[i][k]); hi.set(k, v[i][4 + k]); }
        store_vec<float>(wr + c * V, lo);
        store_vec<float>(wr + c * V + 4, hi);
      }
    }
  }
  const float mean = wave_sum(sum) / (float)D;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
    if (c < chunks) {
#pragma unroll
      for (int k = 0; k < V; ++k) { const float d = v[i][k] - mean; sq += d * d; }
    }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)D + eps);
  T* yr = y + (size_t)row * D;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
    if (c < chunks) {
#pragma unroll
      for (int k0 = 0; k0 < V; k0 += Vec<T>::N) {
        Vec<T> gg = load_vec<T>(g + c * V + k0), bb = load_vec<T>(b + c * V + k0), o;
#pragma unroll
        for (int k = 0; k < Vec<T>::N; ++k) o.set(k, (v[i][k0 + k] - mean) * rstd * gg.get(k) + bb.get(k));
        store_vec<T>(yr + c * V + k0, o);
      }
    }
  }
}

template <typename XT, typename T>
static hipError_t layer_norm_dispatch(const void* x, const void* g, const void* b, void* y, int64_t Trows,
                                      int D, float eps, hipStream_t s, float* xw = nullptr) {
  const int chunks = D / 8;
  const int nch = (chunks + 63) / 64;
  dim3 grid((unsigned)((Trows + 3) / 4)), block(256);
#define OTAS_LN(N)                                                                                       \
  layer_norm_kernel<XT, T, N><<<grid, block, 0, s>>>((const XT*)x, (const T*)g, (const T*)b, (T*)y, Trows, D, eps, xw)
  if (nch <= 1) OTAS_LN(1);
  else if (nch <= 2) OTAS_LN(2);
  else if (nch <= 3) OTAS_LN(3);
  else if (nch <= 4) OTAS_LN(4);
  else if (nch <= 8) OTAS_LN(8);
  else return hipErrorInvalidValue;
#undef OTAS_LN
  return hipGetLastError();
}

hipError_t launch_layer_norm(int dtype, bool x_is_float, const void* x, const void* g, const void* b, void* y,
                             int64_t T, int D, float eps, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  if (dtype == 0) return layer_norm_dispatch<float, float>(x, g, b, y, T, D, eps, s);
  return x_is_float ? layer_norm_dispatch<float, bf16_t>(x, g, b, y, T, D, eps, s)
                    : layer_norm_dispatch<bf16_t, bf16_t>(x, g, b, y, T, D, eps, s);
}

hipError_t launch_layer_norm_widen(const void* x_bf16, const void* g, const void* b, void* y, float* x_float,
                                   int64_t T, int D, float eps, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  return layer_norm_dispatch<bf16_t, bf16_t>(x_bf16, g, b, y, T, D, eps, s, x_float);
}

// ---------------------------------------------------------------------------------- merge-apply + LayerNorm
// The merging module's data movement (Sec. II-C: size-weighted average of every surviving token
// with the tokens merged into it, survivors in their original order) fused with the LayerNorm that
// follows it in the block.  One wave per OUTPUT row: it gathers the rows listed for it
// (row_ptr / src_list, the surviving row first, then its sources in ascending position), forms
// sum(size * x) / sum(size) in fp32 in list order, writes the merged residual row and its size,
// and normalises the row it still holds in registers.  Same arithmetic, in the same order, as
// merge_apply_kernel followed by layer_norm_kernel.
template <typename T, int NCH>
__global__ __launch_bounds__(256) void merge_apply_ln_kernel(
    const float* __restrict__ x, const int32_t* __restrict__ sizes, const int32_t* __restrict__ src_list,
    const int32_t* __restrict__ row_ptr, int64_t T_in, int64_t T_out, int D, float* __restrict__ x_out,
    int32_t* __restrict__ sizes_out, const T* __restrict__ g, const T* __restrict__ b, T* __restrict__ y, float eps) {
  constexpr int V = 8;
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= T_out) return;
  const int chunks = D / V;
  const int beg = row_ptr[row];
  const int end = (row + 1 < T_out) ? row_ptr[row + 1] : (int)T_in;
  float v[NCH][V];
#pragma unroll
  for (int i = 0; i < NCH; ++i)
#pragma unroll
    for (int k = 0; k < V; ++k) v[i][k] = 0.f;
  int tot = 0;
  if (end - beg == 1) {   // untouched token: the row itself
    const int srow = src_list[beg];
    tot = sizes ? sizes[srow] : 1;
    const float* xr = x + (size_t)srow * D;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = lane + 64 * i;
      if (c < chunks) {
        const Vec<float> lo = load_vec<float>(xr + c * V), hi = load_vec<float>(xr + c * V + 4);
#pragma unroll
        for (int k = 0; k < 4; ++k) { v[i][k] = lo.get(k); v[i][4 + k] = hi.get(k); }
      }
    }
  } else {
    // Every lane fetches one list entry and its size, so the rows' addresses are in registers before
    // the first row is requested; the rows are then loaded two at a time and accumulated in list order.
    for (int e0 = beg; e0 < end; e0 += 64) {
      const int cnt = min(64, end - e0);
      const int my_src = lane < cnt ? src_list[e0 + lane] : 0;
      const int my_sz = lane < cnt ? (sizes ? sizes[my_src] : 1) : 0;
      for (int e = 0; e < cnt; e += 2) {
        const bool two = e + 1 < cnt;   // the same for the whole wave
        const int s0 = __shfl(my_src, e, kWave), s1 = __shfl(my_src, two ? e + 1 : e, kWave);
        const int z0 = __shfl(my_sz, e, kWave), z1 = __shfl(my_sz, two ? e + 1 : e, kWave);
        const float* x0r = x + (size_t)s0 * D;
        const float* x1r = x + (size_t)s1 * D;
        Vec<float> a[NCH][2], b[NCH][2];
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
          const int c = lane + 64 * i;
          if (c < chunks) {
            a[i][0] = load_vec<float>(x0r + c * V);
            a[i][1] = load_vec<float>(x0r + c * V + 4);
            if (two) {
              b[i][0] = load_vec<float>(x1r + c * V);
              b[i][1] = load_vec<float>(x1r + c * V + 4);
            }
          }
        }
        const float w0 = (float)z0, w1 = (float)z1;
        tot += z0;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
          if (lane + 64 * i < chunks) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              v[i][k] = fmaf(w0, a[i][0].get(k), v[i][k]);
              v[i][4 + k] = fmaf(w0, a[i][1].get(k), v[i][4 + k]);
            }
          }
        }
        if (two) {
          tot += z1;
#pragma unroll
          for (int i = 0; i < NCH; ++i) {
            if (lane + 64 * i < chunks) {
#pragma unroll
              for (int k = 0; k < 4; ++k) {
                v[i][k] = fmaf(w1, b[i][0].get(k), v[i][k]);
                v[i][4 + k] = fmaf(w1, b[i][1].get(k), v[i][4 + k]);
              }
            }
          }
        }
      }
    }
    const float denom = (float)tot;
#pragma unroll
    for (int i = 0; i < NCH; ++i)
#pragma unroll
      for (int k = 0; k < V; ++k) v[i][k] = v[i][k] / denom;
  }
  if (lane == 0) sizes_out[row] = tot;
  float* xo = x_out + (size_t)row * D;
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
    if (c < chunks) {
      Vec<float> lo, hi;
#pragma unroll
      for (int k = 0; k < 4; ++k) { lo.set(k, v[i][k]); hi.set(k, v[i][4 + k]); }
      store_vec<float>(xo + c * V, lo);
      store_vec<float>(xo + c * V + 4, hi);
#pragma unroll
      for (int k = 0; k < V; ++k) sum += v[i][k];
    }
  }
  const float mean = wave_sum(sum) / (float)D;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
    if (c < chunks) {
#pragma unroll
      for (int k = 0; k < V; ++k) { const float d = v[i][k] - mean; sq += d * d; }
    }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)D + eps);
  T* yr = y + (size_t)row * D;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
    if (c < chunks) {
#pragma unroll
      for (int k0 = 0; k0 < V; k0 += Vec<T>::N) {
        Vec<T> gg = load_vec<T>(g + c * V + k0), bb = load_vec<T>(b + c * V + k0), o;
#pragma unroll
        for (int k = 0; k < Vec<T>::N; ++k) o.set(k, (v[i][k0 + k] - mean) * rstd * gg.get(k) + bb.get(k));
        store_vec<T>(yr + c * V + k0, o);
      }
    }
  }
}

template <typename T>
static hipError_t merge_apply_ln_dispatch(const float* x, const int32_t* sizes, const int32_t* src_list,
                                          const int32_t* row_ptr, int64_t T_in, int64_t T_out, int D, float* x_out,
                                          int32_t* sizes_out, const void* g, const void* b, void* y, float eps,
                                          hipStream_t s) {
  const int nch = (D / 8 + 63) / 64;
  dim3 grid((unsigned)((T_out + 3) / 4)), block(256);
#define OTAS_MLN(N)                                                                                               \
  merge_apply_ln_kernel<T, N><<<grid, block, 0, s>>>(x, sizes, src_list, row_ptr, T_in, T_out, D, x_out, sizes_out, \
                                                     (const T*)g, (const T*)b, (T*)y, eps)
  if (nch <= 1) OTAS_MLN(1);
  else if (nch <= 2) OTAS_MLN(2);
  else if (nch <= 3) OTAS_MLN(3);
  else if (nch <= 4) OTAS_MLN(4);
  else if (nch <= 8) OTAS_MLN(8);
  else return hipErrorInvalidValue;
#undef OTAS_MLN
  return hipGetLastError();
}

hipError_t launch_merge_apply_ln(int dtype, const float* x, const int32_t* sizes, const int32_t* src_list,
                                 const int32_t* row_ptr, int64_t T_in, int64_t T_out, int D, float* x_out,
                                 int32_t* sizes_out, const void* g, const void* b, void* y, float eps, hipStream_t s) {
  if (T_out <= 0) return hipSuccess;
  return dtype == 0 ? merge_apply_ln_dispatch<float>(x, sizes, src_list, row_ptr, T_in, T_out, D, x_out, sizes_out, g,
                                                     b, y, eps, s)
                    : merge_apply_ln_dispatch<bf16_t>(x, sizes, src_list, row_ptr, T_in, T_out, D, x_out, sizes_out,
                                                      g, b, y, eps, s);
}

// ---------------------------------------------------------------------------------- split-K reduce + LayerNorm
// Second half of a split-K residual linear: one wave per row adds the S float partial products in
// split order, then the bias and the residual row, writes the new residual row, and (LN) normalises
// the row it still holds in registers with the next block's first LayerNorm.  x_out may be res.
template <int NCH, bool LN>
__global__ __launch_bounds__(256) void splitk_reduce_ln_kernel(const float* __restrict__ part, int S,
                                                               const bf16_t* __restrict__ bias, const float* res,
                                                               float* x_out, int64_t M, int D,
                                                               const bf16_t* __restrict__ g,
                                                               const bf16_t* __restrict__ b, bf16_t* __restrict__ y,
                                                               float eps) {
  constexpr int V = 8;
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;
  const int chunks = D / V;
  const size_t split_stride = (size_t)M * D;
  const float* pr = part + (size_t)row * D;
  const float* rr = res + (size_t)row * D;
  float* xo = x_out + (size_t)row * D;
  float v[NCH][V];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
    if (c < chunks) {
      Vec<float> lo = load_vec<float>(pr + c * V), hi = load_vec<float>(pr + c * V + 4);
      // bias and residual are requested here, with the partial results, and used after them
      const Vec<bf16_t> bv = load_vec<bf16_t>(bias + c * V);
      const Vec<float> rlo = load_vec<float>(rr + c * V), rhi = load_vec<float>(rr + c * V + 4);
#pragma unroll
      for (int k = 0; k < 4; ++k) { v[i][k] = lo.get(k); v[i][4 + k] = hi.get(k); }
      // the other partial results seven at a time (all of them for S <= 8): their loads are in flight together,
      // the additions keep the order sp = 1, 2, ... (S is the same for the whole launch: the tests on it are scalar branches)
      constexpr int UB = 7;
      for (int sp = 1; sp < S; sp += UB) {
        Vec<float> plo[UB], phi[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u)
          if (sp + u < S) {
            const float* p = pr + (size_t)(sp + u) * split_stride + c * V;
            plo[u] = load_vec<float>(p);
            phi[u] = load_vec<float>(p + 4);
          }
#pragma unroll
        for (int u = 0; u < UB; ++u)
          if (sp + u < S) {
#pragma unroll
            for (int k = 0; k < 4; ++k) { v[i][k] += plo[u].get(k); v[i][4 + k] += phi[u].get(k); }
          }
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        v[i][k] = (v[i][k] + bv.get(k)) + rlo.get(k);
        v[i][4 + k] = (v[i][4 + k] + bv.get(4 + k)) + rhi.get(k);
      }
      Vec<float> olo, ohi;
#pragma unroll
      for (int k = 0; k < 4; ++k) { olo.set(k, v[i][k]); ohi.set(k, v[i][4 + k]); }
      store_vec<float>(xo + c * V, olo);
      store_vec<float>(xo + c * V + 4, ohi);
#pragma unroll
      for (int k = 0; k < V; ++k) sum += v[i][k];
    } else {
#pragma unroll
      for (int k = 0; k < V; ++k) v[i][k] = 0.f;
    }
  }
  if (!LN) return;
  const float mean = wave_sum(sum) / (float)D;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
    if (c < chunks) {
#pragma unroll
      for (int k = 0; k < V; ++k) { const float d = v[i][k] - mean; sq += d * d; }
    }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)D + eps);
  bf16_t* yr = y + (size_t)row * D;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
    if (c < chunks) {
      const Vec<bf16_t> gg = load_vec<bf16_t>(g + c * V), bb = load_vec<bf16_t>(b + c * V);
      Vec<bf16_t> o;
#pragma unroll
      for (int k = 0; k < V; ++k) o.set(k, (v[i][k] - mean) * rstd * gg.get(k) + bb.get(k));
      store_vec<bf16_t>(yr + c * V, o);
    }
  }
}

hipError_t launch_splitk_reduce_ln(const float* part, int S, const void* bias, const float* res, float* x_out,
                                   int64_t M, int D, const void* g, const void* b, void* y, float eps,
                                   hipStream_t s) {
  if (M <= 0) return hipSuccess;
  if (S < 1 || D % 8 != 0) return hipErrorInvalidValue;
  const int nch = (D / 8 + 63) / 64;
  dim3 grid((unsigned)((M + 3) / 4)), block(256);
#define OTAS_RED(N)                                                                                              \
  do {                                                                                                           \
    if (y)                                                                                                       \
      splitk_reduce_ln_kernel<N, true><<<grid, block, 0, s>>>(part, S, (const bf16_t*)bias, res, x_out, M, D,    \
                                                              (const bf16_t*)g, (const bf16_t*)b, (bf16_t*)y, eps); \
    else                                                                                                         \
      splitk_reduce_ln_kernel<N, false><<<grid, block, 0, s>>>(part, S, (const bf16_t*)bias, res, x_out, M, D,   \
                                                               nullptr, nullptr, nullptr, eps);                  \
  } while (0)
  if (nch <= 1) OTAS_RED(1);
  else if (nch <= 2) OTAS_RED(2);
  else if (nch <= 3) OTAS_RED(3);
  else if (nch <= 4) OTAS_RED(4);
  else if (nch <= 8) OTAS_RED(8);
  else return hipErrorInvalidValue;
#undef OTAS_RED
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------- model ends
// Front end of the vision transformer (Sec. II-A): the image [C, Hi, Wi] is cut into p x p patches
// (row by row), every patch flattened channel-major into one row of the patch matrix [N, C p p]
// (the layout of a [D, C, p, p] projection weight); the linear projection is the GEMM kernel;
// embed_finish then builds [class token | projected patches] + position embedding.
template <typename T>
__global__ void patchify_kernel(const T* __restrict__ img, T* __restrict__ out, int C, int Hi, int Wi, int p,
                                int64_t total) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= total) return;   // one element per thread: total = B N C p p
  const int nw = Wi / p, nh = Hi / p, kp = C * p * p;
  const int64_t row = t / kp;
  const int k = (int)(t - row * kp);
  const int b = (int)(row / (nh * nw)), pi = (int)(row - (int64_t)b * nh * nw);
  const int py = pi / nw, px = pi - py * nw;
  const int c = k / (p * p), ij = k - c * p * p, i = ij / p, j = ij - i * p;
  out[t] = img[(((size_t)b * C + c) * Hi + (size_t)py * p + i) * Wi + (size_t)px * p + j];
}

template <typename T>
__global__ void embed_finish_kernel(const T* __restrict__ proj, const T* __restrict__ cls, const T* __restrict__ pos,
                                    T* __restrict__ tokens, int N, int D, int n_lead, int64_t total) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= total) return;   // total = B (n_lead + N) D
  const int n = n_lead + N;
  const int64_t row = t / D;
  const int d = (int)(t - row * D);
  const int b = (int)(row / n), i = (int)(row - (int64_t)b * n);
  const float v = i < n_lead ? to_float(cls[d]) : to_float(proj[((size_t)b * N + (i - n_lead)) * D + d]);
  tokens[t] = from_float<T>(v + to_float(pos[(size_t)i * D + d]));
}

hipError_t launch_patchify(int dtype, const void* img, void* out, int B, int C, int Hi, int Wi, int p, hipStream_t s) {
  const int64_t total = (int64_t)B * (Hi / p) * (Wi / p) * C * p * p;
  if (total <= 0) return hipSuccess;
  dim3 grid((unsigned)((total + 255) / 256)), block(256);
  if (dtype == 0) patchify_kernel<float><<<grid, block, 0, s>>>((const float*)img, (float*)out, C, Hi, Wi, p, total);
  else patchify_kernel<bf16_t><<<grid, block, 0, s>>>((const bf16_t*)img, (bf16_t*)out, C, Hi, Wi, p, total);
  return hipGetLastError();
}

hipError_t launch_embed_finish(int dtype, const void* proj, const void* cls, const void* pos, void* tokens, int B,
                               int N, int D, int n_lead, hipStream_t s) {
  const int64_t total = (int64_t)B * (n_lead + N) * D;
  if (total <= 0) return hipSuccess;
  dim3 grid((unsigned)((total + 255) / 256)), block(256);
  if (dtype == 0)
    embed_finish_kernel<float><<<grid, block, 0, s>>>((const float*)proj, (const float*)cls, (const float*)pos,
                                                      (float*)tokens, N, D, n_lead, total);
  else
    embed_finish_kernel<bf16_t><<<grid, block, 0, s>>>((const bf16_t*)proj, (const bf16_t*)cls, (const bf16_t*)pos,
                                                       (bf16_t*)tokens, N, D, n_lead, total);
  return hipGetLastError();
}

// Back end (Sec. III-B: every task has its own head): one workgroup per query normalises the first row
// of the query's output (final LayerNorm, two-pass fp32 statistics, stored in the model's dtype like
// every GEMM operand) and multiplies it with its task's head [K, D]: one class per thread and pass,
// fp32 accumulate in ascending d.  heads: per task {w, b, K}; task[q] picks the head.
template <typename T>
__global__ __launch_bounds__(256) void task_head_kernel(const float* __restrict__ x, const int32_t* __restrict__ off,
                                                        const int32_t* __restrict__ task, const HeadRef* __restrict__ heads,
                                                        const T* __restrict__ g, const T* __restrict__ bta, int D,
                                                        float eps, float* __restrict__ logits, int k_max) {
  extern __shared__ float hrow[];   // [D] normalised row, then 8 floats of reduction scratch
  float* red = hrow + D;
  const int q = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* xr = x + (size_t)off[q] * D;
  float sum = 0.f;
  for (int d = tid; d < D; d += 256) sum += xr[d];
  sum = wave_sum(sum);
  if (lane == 0) red[wave] = sum;
  __syncthreads();
  const float mean = (red[0] + red[1] + red[2] + red[3]) / (float)D;
  __syncthreads();
  float sq = 0.f;
  for (int d = tid; d < D; d += 256) { const float c = xr[d] - mean; sq += c * c; }
  sq = wave_sum(sq);
  if (lane == 0) red[wave] = sq;
  __syncthreads();
  const float rstd = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)D + eps);
  for (int d = tid; d < D; d += 256)
    hrow[d] = to_float(from_float<T>((xr[d] - mean) * rstd * to_float(g[d]) + to_float(bta[d])));
  __syncthreads();
  const HeadRef h = heads[task[q]];
  const T* w = (const T*)h.w;
  const T* b = (const T*)h.b;
  for (int k = tid; k < k_max; k += 256) {
    float acc = 0.f;
    if (k < h.K) {
      const T* wr = w + (size_t)k * D;
      for (int d = 0; d < D; ++d) acc = fmaf(hrow[d], to_float(wr[d]), acc);
      acc += to_float(b[k]);
    }
    logits[(size_t)q * k_max + k] = acc;   // classes beyond the task's count read 0
  }
}

hipError_t launch_task_heads(int dtype, const float* x, const int32_t* d_off, const int32_t* d_task,
                             const void* d_heads, const void* g, const void* b, int B, int D, float eps,
                             float* logits, int k_max, hipStream_t s) {
  if (B <= 0 || k_max <= 0) return hipSuccess;
  const size_t lds = (size_t)(D + 8) * sizeof(float);
  if (dtype == 0)
    task_head_kernel<float><<<dim3(B), dim3(256), lds, s>>>(x, d_off, d_task, (const HeadRef*)d_heads, (const float*)g,
                                                            (const float*)b, D, eps, logits, k_max);
  else
    task_head_kernel<bf16_t><<<dim3(B), dim3(256), lds, s>>>(x, d_off, d_task, (const HeadRef*)d_heads,
                                                             (const bf16_t*)g, (const bf16_t*)b, D, eps, logits, k_max);
  return hipGetLastError();
}

}  // namespace otas
