// The merging module (Sec. II-C): bipartite matching on cosine similarity, top-r edges, then a
// size-weighted average and an order-preserving compaction.
//
//   merge_plan_kernel  -- one workgroup per query.  From the row-normalised metric vectors it
//       computes, in integers, everything the data movement needs: for every surviving token the
//       list of input rows that are averaged into it.  Written as a CSR over the *output* rows of
//       the whole packed batch: row_ptr[j] .. row_ptr[j+1] indexes src_list, whose first entry is
//       the surviving token itself followed by its merged sources in ascending position.
//   merge_apply_kernel -- one 16-byte chunk of one output row per thread: gathers the listed rows,
//       accumulates size * x in fp32 in list order, divides by the summed size.  Reads every input
//       row once and writes every output row once, with no atomics, so results are deterministic.
#include "common.h"
#include "kernels.h"

namespace otas {

constexpr int kPlanThreads = 256;

// LDS layout of the plan kernel (floats / ints), n = query length, nA = ceil(n/2), nB = floor(n/2):
//   mh   [n][dm+1]  normalised metric rows (padded row stride: lanes walking rows hit distinct banks)
//   best [nA], bcol [nA], part_v [4][nA], part_c [4][nA], merged [nA], cnt [nB], scan [n + 8]
size_t merge_plan_lds_bytes(int max_n, int dm) {
  const size_t nA = (max_n + 1) / 2, nB = max_n / 2;
  return sizeof(float) * ((size_t)max_n * (dm + 1) + nA * 2 + nA * 8 + nA + nB + 2 * (size_t)max_n + 16 + 2 * kPlanThreads);
}

__global__ __launch_bounds__(kPlanThreads) void merge_plan_kernel(
    const float* __restrict__ mhat, int dm, const int32_t* __restrict__ in_off,
    const int32_t* __restrict__ out_off, const int32_t* __restrict__ reff_arr,
    const int32_t* __restrict__ troff, int n_lead, int32_t* __restrict__ src_list,
    int32_t* __restrict__ row_ptr, int32_t* __restrict__ trace_src, int32_t* __restrict__ trace_dst) {
  extern __shared__ float lds[];
  const int q = blockIdx.x, tid = threadIdx.x;
  const int i0 = in_off[q], n = in_off[q + 1] - i0, o0 = out_off[q];
  const int r_eff = reff_arr[q];
  if (n <= 0) return;
  if (r_eff <= 0) {  // nothing merges: every output row is its own single source
    for (int i = tid; i < n; i += kPlanThreads) {
      row_ptr[o0 + i] = i0 + i;
      src_list[i0 + i] = i0 + i;
    }
    return;
  }
  const int nA = (n + 1) >> 1, nB = n >> 1, ldm = dm + 1;
  float* mh = lds;
  float* best = mh + (size_t)n * ldm;
  int* bcol = (int*)(best + nA);
  float* part_v = (float*)(bcol + nA);
  int* part_c = (int*)(part_v + 4 * nA);
  int* merged = part_c + 4 * nA;
  int* cnt = merged + nA;
  int* keep_pos = cnt + nB;      // [n]   exclusive scan of "row survives"
  int* ent_pos = keep_pos + n;   // [n]   exclusive scan of list lengths
  int* wsum = ent_pos + n;       // [2 * kPlanThreads] scan scratch

  for (int t = tid; t < n * dm; t += kPlanThreads) {
    const int i = t / dm, c = t - i * dm;
    mh[i * ldm + c] = mhat[(size_t)(i0 + i) * dm + c];
  }
  __syncthreads();

  // Step 1: every A token picks its most similar B token.  Thread (ax, by): A rows ax, ax+64, ..;
  // B columns by, by+4, ...; strict '>' while walking columns upwards keeps the lowest column of
  // equal maxima.  The dot product always runs c = 0..dm-1 in one fp32 chain.
  const int ax = tid & 63, by = tid >> 6;
  for (int a = ax; a < nA; a += 64) {
    const float* va = mh + (size_t)(2 * a) * ldm;
    float bv = -INFINITY;
    int bc = 0x7fffffff;
    for (int b = by; b < nB; b += 4) {
      const float* vb = mh + (size_t)(2 * b + 1) * ldm;
      float s = 0.f;
      for (int c = 0; c < dm; ++c) s = fmaf(va[c], vb[c], s);
      if (s > bv) { bv = s; bc = b; }
    }
    part_v[by * nA + a] = bv;
    part_c[by * nA + a] = bc;
  }
  __syncthreads();
  for (int a = tid; a < nA; a += kPlanThreads) {
    float bv = part_v[a];
    int bc = part_c[a];
#pragma unroll
    for (int k = 1; k < 4; ++k) {
      const float v = part_v[k * nA + a];
      const int c = part_c[k * nA + a];
      if (v > bv || (v == bv && c < bc)) { bv = v; bc = c; }
    }
    if (2 * a < n_lead) bv = -INFINITY;   // protected leading token: never a merge source
    best[a] = bv;
    bcol[a] = bc;
  }
  __syncthreads();

  // Step 2: keep the r_eff best edges.  rank = number of A tokens that come before this one in
  // (similarity descending, position ascending) order.
  for (int a = tid; a < nA; a += kPlanThreads) {
    const float v = best[a];
    int rank = 0;
    for (int k = 0; k < nA; ++k) {
      const float u = best[k];
      rank += (u > v || (u == v && k < a)) ? 1 : 0;
    }
    const int m = rank < r_eff ? 1 : 0;
    merged[a] = m;
    if (m && trace_src) {
      trace_src[troff[q] + rank] = 2 * a;
      trace_dst[troff[q] + rank] = 2 * bcol[a] + 1;
    }
  }
  __syncthreads();
  for (int b = tid; b < nB; b += kPlanThreads) {
    int c = 0;
    for (int a = 0; a < nA; ++a) c += (merged[a] && bcol[a] == b) ? 1 : 0;
    cnt[b] = c;
  }
  __syncthreads();

  // Step 3: positions.  keep(i) = 1 unless i is a merged A token; entries(i) = keep(i) * (1 +
  // number of sources merged into i).  Exclusive scans of both over i = 0..n-1 (block scan:
  // each thread owns a contiguous run of positions).
  const int per = (n + kPlanThreads - 1) / kPlanThreads;
  const int lo = tid * per, hi = min(n, lo + per);
  int sk = 0, se = 0;
  for (int i = lo; i < hi; ++i) {
    const int k = (i & 1) ? 1 : (merged[i >> 1] ? 0 : 1);
    sk += k;
    se += k ? 1 + ((i & 1) ? cnt[i >> 1] : 0) : 0;
  }
  wsum[tid] = sk;
  wsum[kPlanThreads + tid] = se;
  __syncthreads();
  if (tid == 0) {
    int a = 0, b = 0;
    for (int t = 0; t < kPlanThreads; ++t) {
      const int x = wsum[t], y = wsum[kPlanThreads + t];
      wsum[t] = a;
      wsum[kPlanThreads + t] = b;
      a += x;
      b += y;
    }
  }
  __syncthreads();
  sk = wsum[tid];
  se = wsum[kPlanThreads + tid];
  for (int i = lo; i < hi; ++i) {
    const int k = (i & 1) ? 1 : (merged[i >> 1] ? 0 : 1);
    keep_pos[i] = sk;
    ent_pos[i] = se;
    sk += k;
    se += k ? 1 + ((i & 1) ? cnt[i >> 1] : 0) : 0;
  }
  __syncthreads();

  // Step 4: write the lists.
  for (int i = tid; i < n; i += kPlanThreads) {
    const bool odd = i & 1;
    if (!odd && merged[i >> 1]) continue;
    const int e = i0 + ent_pos[i];
    row_ptr[o0 + keep_pos[i]] = e;
    src_list[e] = i0 + i;
    if (odd && cnt[i >> 1] > 0) {
      const int b = i >> 1;
      int k = 1;
      for (int a = 0; a < nA; ++a)
        if (merged[a] && bcol[a] == b) src_list[e + k++] = i0 + 2 * a;
    }
  }
}

hipError_t launch_merge_plan(const float* mhat, int dm, const int32_t* d_in_off, const int32_t* d_out_off,
                             const int32_t* d_reff, const int32_t* d_troff, int B, int max_n, int n_lead,
                             int32_t* src_list, int32_t* row_ptr, int32_t* trace_src, int32_t* trace_dst,
                             hipStream_t s) {
  if (B <= 0 || max_n <= 0) return hipSuccess;
  const size_t lds = merge_plan_lds_bytes(max_n, dm);
  if (lds > 160 * 1024) return hipErrorInvalidValue;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)merge_plan_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       160 * 1024);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  merge_plan_kernel<<<dim3(B), dim3(kPlanThreads), lds, s>>>(mhat, dm, d_in_off, d_out_off, d_reff, d_troff,
                                                             n_lead, src_list, row_ptr, trace_src, trace_dst);
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
