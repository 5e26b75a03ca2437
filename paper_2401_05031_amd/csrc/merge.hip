// The merging module (Sec. II-C): bipartite matching on cosine similarity, top-r edges, then a
// size-weighted average and an order-preserving compaction.
//
//   merge_plan_kernel  -- one workgroup per query.  It forms the row-normalised metric vectors
//       (head mean of the keys) in LDS and from them computes, in integers, everything the data
//       movement needs: for every surviving token the
//       list of input rows that are averaged into it.  Written as a CSR over the *output* rows of
//       the whole packed batch: row_ptr[j] .. row_ptr[j+1] indexes src_list, whose first entry is
//       the surviving token itself followed by its merged sources in ascending position.
//   merge_apply_kernel -- one 16-byte chunk of one output row per thread: gathers the listed rows,
//       accumulates size * x in fp32 in list order, divides by the summed size.  Reads every input
//       row once and writes every output row once, with no atomics, so results are deterministic.
#include "common.h"
#include "kernels.h"
#include "merge_plan_body.h"

namespace otas {

// Everything but the metric rows.
static inline size_t plan_small_lds_bytes(int max_n) {
  const size_t nA = (max_n + 1) / 2, nB = max_n / 2;
  return sizeof(float) * (3 * nA + nB + 2 * (size_t)max_n + 32 + 8 + 2 * 512);
}
size_t merge_plan_lds_bytes(int max_n, int dm) {
  return sizeof(float) * (size_t)max_n * plan_row_floats(dm) + plan_small_lds_bytes(max_n);
}
size_t merge_plan_rows_bytes(int64_t T, int dm) { return sizeof(float) * (size_t)T * plan_row_floats(dm); }

// One workgroup of 1024 threads per query: merge_plan_body (merge_plan_body.h).
template <typename T, bool ROWS_IN_LDS>
__global__ __launch_bounds__(kPlanThreads) void merge_plan_kernel(
    const T* __restrict__ src, int64_t row_stride, int col_off, int H, int dm, const int32_t* __restrict__ in_off,
    const int32_t* __restrict__ out_off, const int32_t* __restrict__ reff_arr, const int32_t* __restrict__ troff,
    int n_lead, int32_t* __restrict__ src_list, int32_t* __restrict__ row_ptr, int32_t* __restrict__ trace_src,
    int32_t* __restrict__ trace_dst, float* rows) {
  extern __shared__ float lds[];
  merge_plan_body<T, ROWS_IN_LDS>(src, row_stride, col_off, H, dm, in_off, out_off, reff_arr, troff, n_lead, src_list,
                                  row_ptr, trace_src, trace_dst, rows, lds, (int)blockIdx.x, (int)threadIdx.x);
}

hipError_t launch_merge_plan(int dtype, const void* src, int64_t row_stride, int col_off, int H, int dm,
                             const int32_t* d_in_off, const int32_t* d_out_off, const int32_t* d_reff,
                             const int32_t* d_troff, int B, int max_n, int n_lead, int32_t* src_list,
                             int32_t* row_ptr, int32_t* trace_src, int32_t* trace_dst, float* rows, hipStream_t s) {
  if (B <= 0 || max_n <= 0) return hipSuccess;
  if (dm % 4 != 0 || dm > 128 || max_n > kPlanThreads) return hipErrorInvalidValue;
  const bool in_lds = merge_plan_lds_bytes(max_n, dm) <= 160 * 1024;
  if (!in_lds && !rows) return hipErrorInvalidValue;
  const size_t lds = in_lds ? merge_plan_lds_bytes(max_n, dm) : plan_small_lds_bytes(max_n);
#define OTAS_PLAN(TYPE, IN_LDS)                                                                                  \
  do {                                                                                                           \
    auto kern = merge_plan_kernel<TYPE, IN_LDS>;                                                                 \
    hipError_t e = set_max_dynamic_lds((const void*)kern, 160 * 1024);                                           \
    if (e != hipSuccess) return e;                                                                               \
    kern<<<dim3(B), dim3(kPlanThreads), lds, s>>>((const TYPE*)src, row_stride, col_off, H, dm, d_in_off,        \
                                                  d_out_off, d_reff, d_troff, n_lead, src_list, row_ptr,         \
                                                  trace_src, trace_dst, rows);                                   \
  } while (0)
  if (dtype == 0) {
    if (in_lds) OTAS_PLAN(float, true); else OTAS_PLAN(float, false);
  } else {
    if (in_lds) OTAS_PLAN(bf16_t, true); else OTAS_PLAN(bf16_t, false);
  }
#undef OTAS_PLAN
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------ apply
template <typename T>
__global__ __launch_bounds__(256) void merge_apply_kernel(const T* __restrict__ x, const int32_t* __restrict__ sizes,
                                                          const int32_t* __restrict__ src_list,
                                                          const int32_t* __restrict__ row_ptr, int64_t T_in,
                                                          int64_t T_out, int D, T* __restrict__ x_out,
                                                          int32_t* __restrict__ sizes_out) {
  constexpr int V = Vec<T>::N;
  const int chunks = D / V;
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T_out * chunks) return;
  const int64_t j = t / chunks;
  const int c = (int)(t - j * chunks) * V;
  const int beg = row_ptr[j];
  const int end = (j + 1 < T_out) ? row_ptr[j + 1] : (int)T_in;
  const int first = src_list[beg];
  if (end - beg == 1) {  // untouched token: plain copy
    store_vec<T>(x_out + (size_t)j * D + c, load_vec<T>(x + (size_t)first * D + c));
    if (c == 0) sizes_out[j] = sizes ? sizes[first] : 1;
    return;
  }
  float acc[V];
#pragma unroll
  for (int k = 0; k < V; ++k) acc[k] = 0.f;
  int tot = 0;
  for (int e = beg; e < end; ++e) {
    const int srow = src_list[e];
    const int sz = sizes ? sizes[srow] : 1;
    const float w = (float)sz;
    tot += sz;
    const Vec<T> v = load_vec<T>(x + (size_t)srow * D + c);
#pragma unroll
    for (int k = 0; k < V; ++k) acc[k] = fmaf(w, v.get(k), acc[k]);
  }
  const float denom = (float)tot;
  Vec<T> o;
#pragma unroll
  for (int k = 0; k < V; ++k) o.set(k, acc[k] / denom);
  store_vec<T>(x_out + (size_t)j * D + c, o);
  if (c == 0) sizes_out[j] = tot;
}

hipError_t launch_merge_apply(int dtype, const void* x, const int32_t* sizes, const int32_t* src_list,
                              const int32_t* row_ptr, int64_t T_in, int64_t T_out, int D, void* x_out,
                              int32_t* sizes_out, hipStream_t s) {
  if (T_out <= 0) return hipSuccess;
  const int V = dtype == 0 ? 4 : 8;
  const int64_t tasks = T_out * (D / V);
  dim3 grid((unsigned)((tasks + 255) / 256)), block(256);
  if (dtype == 0)
    merge_apply_kernel<float><<<grid, block, 0, s>>>((const float*)x, sizes, src_list, row_ptr, T_in, T_out, D,
                                                     (float*)x_out, sizes_out);
  else
    merge_apply_kernel<bf16_t><<<grid, block, 0, s>>>((const bf16_t*)x, sizes, src_list, row_ptr, T_in, T_out, D,
                                                      (bf16_t*)x_out, sizes_out);
  return hipGetLastError();
}

}  // namespace otas
