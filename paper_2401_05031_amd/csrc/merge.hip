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

namespace otas {

constexpr int kPlanThreads = 1024;

template <typename T> struct alignas(4 * sizeof(T)) Quad { T x[4]; };   // 4 consecutive elements, one load

// LDS layout of the plan kernel (4-byte words), n = query length, nA = ceil(n/2), nB = floor(n/2):
//   mh [n][dm+4] normalised metric rows | best [nA] | bcol [nA] | merged [nA] | cnt [nB] |
//   keep_pos [n] | ent_pos [n] | wave_tot [2][16]
size_t merge_plan_lds_bytes(int max_n, int dm) {
  const size_t nA = (max_n + 1) / 2, nB = max_n / 2;
  return sizeof(float) * ((size_t)max_n * (dm + 4) + 3 * nA + nB + 2 * (size_t)max_n + 32 + 8);
}

// Similarity row of one A token against a strided subset of the B tokens.  The A row sits in
// registers (DM4 float4), the B rows are read from LDS as float4 (lanes that share a B row share
// the read).  The dot product always runs c = 0..dm-1 in one fp32 fma chain, whatever the thread
// mapping, so the decision does not depend on the launch shape.
template <int DM4>
__device__ inline void best_of_subset(const float* __restrict__ mh, int ldm, int a, int part, int nB, float& bv,
                                      int& bc) {
  floatx4 av[DM4];
  const float* pa = mh + (size_t)(2 * a) * ldm;
#pragma unroll
  for (int c = 0; c < DM4; ++c) av[c] = *reinterpret_cast<const floatx4*>(pa + 4 * c);
  for (int b = part; b < nB; b += 8) {
    const float* pb = mh + (size_t)(2 * b + 1) * ldm;
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < DM4; ++c) {
      const floatx4 v = *reinterpret_cast<const floatx4*>(pb + 4 * c);
      s = fmaf(av[c][0], v[0], s);
      s = fmaf(av[c][1], v[1], s);
      s = fmaf(av[c][2], v[2], s);
      s = fmaf(av[c][3], v[3], s);
    }
    if (s > bv) { bv = s; bc = b; }   // strict '>' walking upwards: lowest column among equal maxima
  }
}

__device__ inline void best_of_subset_any(const float* __restrict__ mh, int ldm, int dm, int a, int part, int nB,
                                          float& bv, int& bc) {
  const float* pa = mh + (size_t)(2 * a) * ldm;
  for (int b = part; b < nB; b += 8) {
    const float* pb = mh + (size_t)(2 * b + 1) * ldm;
    float s = 0.f;
    for (int c = 0; c < dm; ++c) s = fmaf(pa[c], pb[c], s);
    if (s > bv) { bv = s; bc = b; }
  }
}

// One workgroup of 1024 threads per query.  src: the vectors the similarity is taken on; the metric
// of token i is the mean over H heads of src[(i0 + i) * row_stride + col_off + h * dm + c] (H = 1 for
// a caller-supplied metric, H heads of the attention keys inside the encoder), normalised to unit
// length with fp32 arithmetic.
template <typename T>
__global__ __launch_bounds__(kPlanThreads) void merge_plan_kernel(
    const T* __restrict__ src, int64_t row_stride, int col_off, int H, int dm, const int32_t* __restrict__ in_off,
    const int32_t* __restrict__ out_off, const int32_t* __restrict__ reff_arr, const int32_t* __restrict__ troff,
    int n_lead, int32_t* __restrict__ src_list, int32_t* __restrict__ row_ptr, int32_t* __restrict__ trace_src,
    int32_t* __restrict__ trace_dst) {
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
  const int nA = (n + 1) >> 1, nB = n >> 1, ldm = dm + 4;
  float* mh = lds;
  float* best = mh + (size_t)n * ldm;
  int* bcol = (int*)(best + nA);
  int* merged = bcol + nA;
  int* cnt = merged + nA;
  int* keep_pos = cnt + nB;      // [n] exclusive scan of "row survives"
  int* ent_pos = keep_pos + n;   // [n] exclusive scan of list lengths
  int* wave_tot = ent_pos + n;   // [2][16]

  // Phase 0: head-mean metric rows, 4 columns per thread (one 8- or 16-byte load per head), heads
  // summed in ascending order.
  const int c4n = dm >> 2;
  const float inv_h = 1.0f / (float)H;
  for (int t = tid; t < n * c4n; t += kPlanThreads) {
    const int i = t / c4n, c = (t - i * c4n) * 4;
    const T* p = src + (size_t)(i0 + i) * row_stride + col_off + c;
    float m0 = 0.f, m1 = 0.f, m2 = 0.f, m3 = 0.f;
    for (int h = 0; h < H; ++h) {
      const Quad<T> v = *reinterpret_cast<const Quad<T>*>(p);
      m0 += to_float(v.x[0]); m1 += to_float(v.x[1]); m2 += to_float(v.x[2]); m3 += to_float(v.x[3]);
      p += dm;
    }
    floatx4 o = {m0 * inv_h, m1 * inv_h, m2 * inv_h, m3 * inv_h};
    *reinterpret_cast<floatx4*>(mh + (size_t)i * ldm + c) = o;
  }
  __syncthreads();
  // Phase 1: unit length (one thread per row, columns in ascending order)
  for (int i = tid; i < n; i += kPlanThreads) {
    float* r = mh + (size_t)i * ldm;
    float ss = 0.f;
    for (int c = 0; c < dm; ++c) ss = fmaf(r[c], r[c], ss);
    const float rn = 1.0f / fmaxf(sqrtf(ss), 1e-12f);
    for (int c = 0; c < dm; ++c) r[c] *= rn;
  }
  __syncthreads();

  // Phase 2: every A token picks its most similar B token.  8 consecutive lanes share an A row and
  // split the B columns (b = part, part + 8, ...); their results are combined by shuffles, ties to
  // the lowest column.
  const int part = tid & 7;
  for (int a0 = 0; a0 < nA; a0 += kPlanThreads / 8) {
    const int a = a0 + (tid >> 3);
    float bv = -INFINITY;
    int bc = 0x7fffffff;
    if (a < nA) {
      if (dm == 64) best_of_subset<16>(mh, ldm, a, part, nB, bv, bc);
      else if (dm == 80) best_of_subset<20>(mh, ldm, a, part, nB, bv, bc);
      else best_of_subset_any(mh, ldm, dm, a, part, nB, bv, bc);
    }
#pragma unroll
    for (int o = 4; o > 0; o >>= 1) {
      const float v = __shfl_xor(bv, o, kWave);
      const int c = __shfl_xor(bc, o, kWave);
      if (v > bv || (v == bv && c < bc)) { bv = v; bc = c; }
    }
    if (a < nA && part == 0) {
      best[a] = (2 * a < n_lead) ? -INFINITY : bv;   // protected leading token: never a merge source
      bcol[a] = bc;
    }
  }
  __syncthreads();

  // Phase 3: keep the r_eff best edges.  rank = number of A tokens that come before this one in
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

  // Phase 4: positions.  keep(i) = 1 unless i is a merged A token; entries(i) = keep(i) * (1 +
  // number of sources merged into i).  Exclusive scans of both over i = 0..n-1, one position per
  // thread (n <= 1024): wave scan by shuffles, then the wave totals.
  {
    const int i = tid, lane = tid & 63, w = tid >> 6;
    int k = 0, e = 0;
    if (i < n) {
      k = (i & 1) ? 1 : (merged[i >> 1] ? 0 : 1);
      e = k ? 1 + ((i & 1) ? cnt[i >> 1] : 0) : 0;
    }
    int sk = k, se = e;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int tk = __shfl_up(sk, o, kWave), te = __shfl_up(se, o, kWave);
      if (lane >= o) { sk += tk; se += te; }
    }
    if (lane == 63) { wave_tot[w] = sk; wave_tot[16 + w] = se; }
    __syncthreads();
    int ok = 0, oe = 0;
    for (int j = 0; j < w; ++j) { ok += wave_tot[j]; oe += wave_tot[16 + j]; }
    if (i < n) {
      keep_pos[i] = ok + sk - k;
      ent_pos[i] = oe + se - e;
    }
  }
  __syncthreads();

  // Phase 5: write the lists.
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

hipError_t launch_merge_plan(int dtype, const void* src, int64_t row_stride, int col_off, int H, int dm,
                             const int32_t* d_in_off, const int32_t* d_out_off, const int32_t* d_reff,
                             const int32_t* d_troff, int B, int max_n, int n_lead, int32_t* src_list,
                             int32_t* row_ptr, int32_t* trace_src, int32_t* trace_dst, hipStream_t s) {
  if (B <= 0 || max_n <= 0) return hipSuccess;
  if (dm % 4 != 0 || dm > 128 || max_n > kPlanThreads) return hipErrorInvalidValue;
  const size_t lds = merge_plan_lds_bytes(max_n, dm);
  if (lds > 160 * 1024) return hipErrorInvalidValue;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)merge_plan_kernel<float>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void*)merge_plan_kernel<bf16_t>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              160 * 1024);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  if (dtype == 0)
    merge_plan_kernel<float><<<dim3(B), dim3(kPlanThreads), lds, s>>>(
        (const float*)src, row_stride, col_off, H, dm, d_in_off, d_out_off, d_reff, d_troff, n_lead, src_list, row_ptr,
        trace_src, trace_dst);
  else
    merge_plan_kernel<bf16_t><<<dim3(B), dim3(kPlanThreads), lds, s>>>(
        (const bf16_t*)src, row_stride, col_off, H, dm, d_in_off, d_out_off, d_reff, d_troff, n_lead, src_list,
        row_ptr, trace_src, trace_dst);
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
