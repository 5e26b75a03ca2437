// The plan of the merging module (Sec. II-C) for one query, as device functions that a workgroup executes:
//   merge_plan_select  phases 0-2: head-mean metric, unit length, every A token's most similar B token
//                      (NT threads, a multiple of 64: kPlanThreads on its own, fewer beside attention)
//   merge_plan_lists   phases 3-5: the r best edges, list slots, scans, the lists (any multiple of 64 threads)
//   merge_plan_body    both, one after the other
// Used by merge_plan_kernel (one workgroup per query runs the whole plan), by the kernel that runs the selection
// beside attention in one launch, and by the GEMM kernels that run the list phases beside the projection.
#ifndef OTAS_MERGE_PLAN_BODY_H_
#define OTAS_MERGE_PLAN_BODY_H_

#include "common.h"

namespace otas {

constexpr int kPlanThreads = 1024;

template <typename T> struct alignas(4 * sizeof(T)) Quad { T x[4]; };   // 4 consecutive elements, one load
template <typename T> struct alignas(8 * sizeof(T)) Oct { T x[8]; };    // 8 consecutive elements, one load

// LDS layout of the plan kernel (4-byte words), n = query length, nA = ceil(n/2), nB = floor(n/2):
//   mh [n][dm+4] normalised metric rows | best [nA] | bcol [nA] | merged [nA] | cnt [nB] |
//   keep_pos [n] | ent_pos [n] | wave_tot [2][16] | part_v [512] | part_c [512]
// (the list phases on their own use the part from best on, without part_v / part_c).
// Floats per metric row in LDS: the even and the odd columns each padded to a multiple of 4, plus 4.
__host__ __device__ static inline int plan_row_floats(int dm) { return 2 * (((dm >> 1) + 3) & ~3) + 4; }
// Bytes of LDS the list phases need for a query of up to max_n tokens, and that for the longest query there is.
static inline size_t plan_lists_lds_bytes(int max_n) {
  const size_t nA = (max_n + 1) / 2, nB = max_n / 2;
  return 4 * (3 * nA + nB + 2 * (size_t)max_n + 32);
}
constexpr size_t kPlanListsLdsMax = 4 * (3 * 512 + 512 + 2 * 1024 + 32);

// One workgroup of NT threads per query (q; tid = thread index in the workgroup; lds: its dynamic LDS).
// src: the vectors the similarity is taken on; the metric of token i is the mean over H heads of src[(i0 + i) * row_stride + col_off + h * dm + c] (H = 1 for
// a caller-supplied metric, H heads of the attention keys inside the encoder), normalised to unit
// length with fp32 arithmetic.
// ROWS_IN_LDS = false: the metric rows of the query live in global memory (rows + i0 * ldm: the
// query's own rows of a [T][ldm] float buffer; written and read by this workgroup only, between its
// barriers) instead of LDS, for queries whose rows do not fit the 160 KB; same arithmetic, same order.
// TO_GLOBAL = false: the result (best[a] = similarity of A token a's best match, -inf for a protected leading
// token; bcol[a] = that B token) stays in LDS behind the metric rows, valid for every thread on return.
// TO_GLOBAL = true: it goes to g_best[i0 + a], g_bcol[i0 + a] (a < nA) for merge_plan_lists in a later launch.
// Queries with nothing to merge return at once.
// part / parts: the A tokens are dealt to `parts` workgroups in blocks of 32 (block k goes to workgroup k % parts);
// this one is number `part` and computes the rows it needs -- all B tokens and its own A tokens -- and the result
// of its A tokens only (parts > 1 needs TO_GLOBAL).  Every row and every similarity is computed by the same
// arithmetic in the same order whatever `parts` is.
template <typename T, bool ROWS_IN_LDS, bool TO_GLOBAL, int NT = kPlanThreads>
__device__ __forceinline__ void merge_plan_select(
    const T* __restrict__ src, int64_t row_stride, int col_off, int H, int dm, const int32_t* __restrict__ in_off,
    const int32_t* __restrict__ reff_arr, int n_lead, float* rows, float* lds, float* __restrict__ g_best,
    int32_t* __restrict__ g_bcol, const int q, const int tid, const int part = 0, const int parts = 1) {
  const int i0 = in_off[q], n = in_off[q + 1] - i0;
  if (n <= 0 || reff_arr[q] <= 0) return;
  const int half = dm >> 1, hp = (half + 3) & ~3;   // columns per parity, and their padded count
  const int nA = (n + 1) >> 1, nB = n >> 1, ldm = 2 * hp + 4;
  const int nAb = (nA + 31) >> 5, nBb = (nB + 31) >> 5;
  const int nAl = (nAb - part + parts - 1) / parts;   // A blocks of this workgroup: part, part + parts, ...
  if (nAl <= 0) return;
  // The rows this workgroup needs, numbered u = 0 .. n_need - 1: the nB B tokens, then its A blocks (the last
  // block may run past nA: -1).
  const int n_need = nB + nAl * 32;
  auto token_of = [&](int u) {
    if (u < nB) return 2 * u + 1;
    const int v = u - nB, a = (part + parts * (v >> 5)) * 32 + (v & 31);
    return a < nA ? 2 * a : -1;
  };
  // Metric rows in LDS: the A tokens (even positions) first, then the B tokens, one row of ldm
  // floats per token, so that consecutive tokens of one set are ldm = dm + 4 floats apart (16 lanes
  // reading 16 bytes each from 16 consecutive rows then fall on all 64 banks once).  Inside a row the
  // columns are stored even ones first, then odd ones (each group zero-padded to a multiple of 4):
  // column c sits at (c & 1) * hp + c / 2, so
  // the two halves of a wave (which feed the even and the odd k of every fp32 MFMA) each read
  // consecutive floats.
  float* mh;
  float* best;
  if constexpr (ROWS_IN_LDS) {
    mh = lds;
    best = mh + (size_t)n * ldm;
  } else {
    mh = rows + (size_t)i0 * ldm;
    best = lds;
  }
  int* bcol = (int*)(best + nA);
  int* wave_tot = bcol + 2 * nA + nB + 2 * n;   // behind merged, cnt, keep_pos, ent_pos of the list phases
  auto row_of = [&](int i) { return mh + (size_t)((i & 1) ? nA + (i >> 1) : (i >> 1)) * ldm; };

  // Phase 0: head-mean metric rows, heads summed in ascending order.  A thread takes 8 columns of a token when the
  // source is 16-bit and 16-byte aligned with dm % 8 == 0 (one 16-byte load per head, two 16-byte LDS stores: this phase is bound by
  // instruction issue on the one CU that runs the query), else 4 columns.
  const float inv_h = 1.0f / (float)H;
  if (sizeof(T) == 2 && (dm & 7) == 0 && (row_stride & 7) == 0 && (col_off & 7) == 0 &&
      (reinterpret_cast<uintptr_t>(src) & 15) == 0) {
    const int c8n = dm >> 3;
    for (int t = tid; t < n_need * c8n; t += NT) {
      const int u = t / c8n, c = (t - u * c8n) * 8, i = token_of(u);
      if (i < 0) continue;
      const T* p = src + (size_t)(i0 + i) * row_stride + col_off + c;
      float m[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) m[e] = 0.f;
#pragma unroll 4
      for (int h = 0; h < H; ++h) {
        const Oct<T> v = *reinterpret_cast<const Oct<T>*>(p);
#pragma unroll
        for (int e = 0; e < 8; ++e) m[e] += to_float(v.x[e]);
        p += dm;
      }
      float* r = row_of(i);
      const int ce = c >> 1;   // columns c, c+2, c+4, c+6 are even ones, the others odd ones
      *reinterpret_cast<floatx4*>(r + ce) = floatx4{m[0] * inv_h, m[2] * inv_h, m[4] * inv_h, m[6] * inv_h};
      *reinterpret_cast<floatx4*>(r + hp + ce) = floatx4{m[1] * inv_h, m[3] * inv_h, m[5] * inv_h, m[7] * inv_h};
    }
  } else {
    const int c4n = dm >> 2;
    for (int t = tid; t < n_need * c4n; t += NT) {
      const int u = t / c4n, c = (t - u * c4n) * 4, i = token_of(u);
      if (i < 0) continue;
      const T* p = src + (size_t)(i0 + i) * row_stride + col_off + c;
      float m0 = 0.f, m1 = 0.f, m2 = 0.f, m3 = 0.f;
#pragma unroll 4
      for (int h = 0; h < H; ++h) {
        const Quad<T> v = *reinterpret_cast<const Quad<T>*>(p);
        m0 += to_float(v.x[0]); m1 += to_float(v.x[1]); m2 += to_float(v.x[2]); m3 += to_float(v.x[3]);
        p += dm;
      }
      float* r = row_of(i);
      const int ce = c >> 1;   // columns c, c+2 are even ones, c+1, c+3 odd ones
      r[ce] = m0 * inv_h;
      r[ce + 1] = m2 * inv_h;
      r[hp + ce] = m1 * inv_h;
      r[hp + ce + 1] = m3 * inv_h;
    }
  }
  if (hp != half)   // the padding columns take part in the contraction: zero
    for (int t = tid; t < n_need * 2 * (hp - half); t += NT) {
      const int u = t / (2 * (hp - half)), c = t - u * (2 * (hp - half)), i = token_of(u);
      if (i >= 0) row_of(i)[(c & 1) * hp + half + (c >> 1)] = 0.f;
    }
  __syncthreads();
  // Phase 1: unit length.  16 consecutive lanes share a row of 2 hp floats (the zero padding adds nothing): lane j
  // sums the squares of the 16-byte pieces j, j + 16, ... in ascending order, the sixteen partial sums are added by
  // a fixed butterfly, and every lane scales its own pieces.
  {
    const int q4 = (2 * hp) >> 2;   // 16-byte pieces per row
    for (int u0 = 0; u0 < n_need; u0 += NT / 16) {
      const int u = u0 + (tid >> 4), j = tid & 15;
      const int i = u < n_need ? token_of(u) : -1;
      float* r = row_of(i >= 0 ? i : 1);   // n >= 2 here: token 1 exists
      float ss = 0.f;
      for (int m = j; m < q4; m += 16) {
        const floatx4 v = *reinterpret_cast<const floatx4*>(r + 4 * m);
        ss = fmaf(v[0], v[0], ss); ss = fmaf(v[1], v[1], ss); ss = fmaf(v[2], v[2], ss); ss = fmaf(v[3], v[3], ss);
      }
      ss += __shfl_xor(ss, 1, kWave);
      ss += __shfl_xor(ss, 2, kWave);
      ss += __shfl_xor(ss, 4, kWave);
      ss += __shfl_xor(ss, 8, kWave);
      const float rn = 1.0f / fmaxf(sqrtf(ss), 1e-12f);
      if (i >= 0)
        for (int m = j; m < q4; m += 16) {
          floatx4 v = *reinterpret_cast<const floatx4*>(r + 4 * m);
          v[0] *= rn; v[1] *= rn; v[2] *= rn; v[3] *= rn;
          *reinterpret_cast<floatx4*>(r + 4 * m) = v;
        }
    }
  }
  __syncthreads();

  // Phase 2: every A token picks its most similar B token.  The similarity matrix is a dense
  // contraction over the metric width, done on the matrix cores in true fp32
  // (v_mfma_f32_32x32x2_f32), transposed: B tokens are the first operand (rows), A tokens the second
  // (columns), so a lane owns ONE A token and holds 16 of a 32-token B block's similarities in its
  // accumulator (rows 8 (e / 4) + 4 (lane >> 5) + (e & 3)): its arg-max is a scan of its own registers
  // in ascending B order plus one exchange with lane ^ 32.  Wave w owns the workgroup's A block w % nAl and every
  // G-th B block; the G partial results per A token are combined through LDS.  Ties go to the
  // lowest B position at every step.
  constexpr int NWV = NT / 64;
  const int G = max(1, NWV / nAl);
  int* part_c = wave_tot + 32;
  float* part_v = reinterpret_cast<float*>(part_c + 512);
  {
    const int lane = tid & 63, w = tid >> 6;
    const int fr = lane & 31, fk = lane >> 5;
    // nAl <= NWV: one (A block, B group) per wave, groups beyond G idle; more A blocks than waves: one group, the
    // waves take the blocks in turn
    const bool wide = nAl > NWV;
    const int grp = wide ? 0 : w / nAl;
    for (int al = wide ? w : w % nAl; al < nAl && grp < G; al += wide ? NWV : nAl) {
      const int a = (part + parts * al) * 32 + fr;
      const float* pa = mh + (size_t)min(a, nA - 1) * ldm + fk * hp;
      float bv = -INFINITY;
      int bc = 0x7fffffff;
      for (int bb = grp; bb < nBb; bb += G) {
        const float* pb = mh + (size_t)(nA + min(bb * 32 + fr, nB - 1)) * ldm + fk * hp;
        floatx16 acc;
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[e] = 0.f;
        // MFMA u contracts over columns 2u (lanes 0..31) and 2u + 1 (lanes 32..63): with the even /
        // odd column split a lane's operands of four consecutive MFMAs are one 16-byte read
        for (int k0 = 0; k0 < hp; k0 += 8) {   // 8 MFMAs per batch, their operand reads issued first
          const floatx4 ra0 = *reinterpret_cast<const floatx4*>(pa + k0);
          const floatx4 rb0 = *reinterpret_cast<const floatx4*>(pb + k0);
          floatx4 ra1 = ra0, rb1 = rb0;
          if (k0 + 4 < hp) {
            ra1 = *reinterpret_cast<const floatx4*>(pa + k0 + 4);
            rb1 = *reinterpret_cast<const floatx4*>(pb + k0 + 4);
          }
#pragma unroll
          for (int u = 0; u < 4; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(rb0[u], ra0[u], acc, 0, 0, 0);
          if (k0 + 4 < hp) {
#pragma unroll
            for (int u = 0; u < 4; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(rb1[u], ra1[u], acc, 0, 0, 0);
          }
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int b = bb * 32 + 8 * (e >> 2) + 4 * fk + (e & 3);
          if (b < nB && acc[e] > bv) { bv = acc[e]; bc = b; }
        }
      }
      const float ov = __shfl_xor(bv, 32, kWave);
      const int oc = __shfl_xor(bc, 32, kWave);
      if (ov > bv || (ov == bv && oc < bc)) { bv = ov; bc = oc; }
      if (fk == 0) {
        part_v[grp * (nAl * 32) + al * 32 + fr] = bv;
        part_c[grp * (nAl * 32) + al * 32 + fr] = bc;
      }
    }
  }
  __syncthreads();
  for (int t = tid; t < nAl * 32; t += NT) {
    const int a = (part + parts * (t >> 5)) * 32 + (t & 31);
    if (a >= nA) continue;
    float bv = part_v[t];
    int bc = part_c[t];
    for (int g = 1; g < G; ++g) {
      const float v = part_v[g * (nAl * 32) + t];
      const int c = part_c[g * (nAl * 32) + t];
      if (v > bv || (v == bv && c < bc)) { bv = v; bc = c; }
    }
    const float v = (2 * a < n_lead) ? -INFINITY : bv;   // protected leading token: never a merge source
    if constexpr (TO_GLOBAL) {
      g_best[i0 + a] = v;
      g_bcol[i0 + a] = bc;
    } else {
      best[a] = v;
      bcol[a] = bc;
    }
  }
  if constexpr (!TO_GLOBAL) __syncthreads();
}

// The list phases for query q by a workgroup of NT threads (a multiple of 64, at most 1024).  small: LDS for
// best [nA] | bcol [nA] | merged [nA] | cnt [nB] | keep_pos [n] | ent_pos [n] | wave_tot [32] (4-byte words).
// FROM_GLOBAL = false: best / bcol are already there (merge_plan_select in the same workgroup);
// true: they are read from g_best / g_bcol [i0 + a].  Integer work only, apart from comparisons of the
// similarities: the result does not depend on NT.
template <int NT, bool FROM_GLOBAL>
__device__ __forceinline__ void merge_plan_lists(
    float* small, const float* __restrict__ g_best, const int32_t* __restrict__ g_bcol,
    const int32_t* __restrict__ in_off, const int32_t* __restrict__ out_off, const int32_t* __restrict__ reff_arr,
    const int32_t* __restrict__ troff, int32_t* __restrict__ src_list, int32_t* __restrict__ row_ptr,
    int32_t* __restrict__ trace_src, int32_t* __restrict__ trace_dst, const int q, const int tid) {
  const int i0 = in_off[q], n = in_off[q + 1] - i0, o0 = out_off[q];
  const int r_eff = reff_arr[q];
  if (n <= 0) return;
  if (r_eff <= 0) {  // nothing merges: every output row is its own single source
    for (int i = tid; i < n; i += NT) {
      row_ptr[o0 + i] = i0 + i;
      src_list[i0 + i] = i0 + i;
    }
    return;
  }
  const int nA = (n + 1) >> 1, nB = n >> 1;
  float* best = small;
  int* bcol = (int*)(best + nA);
  int* merged = bcol + nA;
  int* cnt = merged + nA;
  int* keep_pos = cnt + nB;      // [n] exclusive scan of "row survives"
  int* ent_pos = keep_pos + n;   // [n] exclusive scan of list lengths
  int* wave_tot = ent_pos + n;   // [2][16]
  if constexpr (FROM_GLOBAL) {
    for (int a = tid; a < nA; a += NT) {
      best[a] = g_best[i0 + a];
      bcol[a] = g_bcol[i0 + a];
    }
    __syncthreads();
  }

  // Phase 3: keep the r_eff best edges.  rank = number of A tokens that come before this one in
  // (similarity descending, position ascending) order; 8 consecutive lanes share an A token and
  // split the tokens it is compared with.  slot = number of kept edges with the same destination
  // and a lower source position (the order of a destination's source list).
  for (int b = tid; b < nB; b += NT) cnt[b] = 0;
  for (int a0 = 0; a0 < nA; a0 += NT / 8) {
    const int a = min(a0 + (tid >> 3), nA - 1), part = tid & 7;
    const float v = best[a];
    int rank = 0;
    for (int k = part; k < nA; k += 8) {
      const float u = best[k];
      rank += (u > v || (u == v && k < a)) ? 1 : 0;
    }
    rank += __shfl_xor(rank, 1, kWave);
    rank += __shfl_xor(rank, 2, kWave);
    rank += __shfl_xor(rank, 4, kWave);
    if (part == 0 && a0 + (tid >> 3) < nA) merged[a] = rank < r_eff ? 1 : 0;
    if (part == 0 && a0 + (tid >> 3) < nA && rank < r_eff && trace_src) {
      trace_src[troff[q] + rank] = 2 * a;
      trace_dst[troff[q] + rank] = 2 * bcol[a] + 1;
    }
  }
  __syncthreads();
  for (int a0 = 0; a0 < nA; a0 += NT / 8) {
    const int a = min(a0 + (tid >> 3), nA - 1), part = tid & 7;
    const int dst = bcol[a];
    int slot = 0;
    for (int k = part; k < a; k += 8) slot += (merged[k] && bcol[k] == dst) ? 1 : 0;
    slot += __shfl_xor(slot, 1, kWave);
    slot += __shfl_xor(slot, 2, kWave);
    slot += __shfl_xor(slot, 4, kWave);
    if (part == 0 && a0 + (tid >> 3) < nA && merged[a]) {
      atomicAdd(&cnt[dst], 1);      // integer count: the result does not depend on the order
      best[a] = __int_as_float(slot);   // best is dead from here on: reuse it for the slot
    }
  }
  __syncthreads();

  // Phase 4: positions.  keep(i) = 1 unless i is a merged A token; entries(i) = keep(i) * (1 +
  // number of sources merged into i).  Exclusive scans of both over i = 0..n-1: every thread takes
  // ceil(n / NT) consecutive positions (one when n <= NT), wave scan of the thread sums by shuffles,
  // then the wave totals.
  {
    const int C = (n + NT - 1) / NT;
    const int lane = tid & 63, w = tid >> 6;
    auto keep_of = [&](int i) { return (i & 1) ? 1 : (merged[i >> 1] ? 0 : 1); };
    auto ent_of = [&](int i, int k) { return k ? 1 + ((i & 1) ? cnt[i >> 1] : 0) : 0; };
    int k_sum = 0, e_sum = 0;
    for (int c = 0; c < C; ++c) {
      const int i = tid * C + c;
      if (i < n) {
        const int k = keep_of(i);
        k_sum += k;
        e_sum += ent_of(i, k);
      }
    }
    int sk = k_sum, se = e_sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int tk = __shfl_up(sk, o, kWave), te = __shfl_up(se, o, kWave);
      if (lane >= o) { sk += tk; se += te; }
    }
    if (lane == 63) { wave_tot[w] = sk; wave_tot[16 + w] = se; }
    __syncthreads();
    int pk = sk - k_sum, pe = se - e_sum;
    for (int j = 0; j < w; ++j) { pk += wave_tot[j]; pe += wave_tot[16 + j]; }
    for (int c = 0; c < C; ++c) {
      const int i = tid * C + c;
      if (i < n) {
        const int k = keep_of(i), e = ent_of(i, k);
        keep_pos[i] = pk;
        ent_pos[i] = pe;
        pk += k;
        pe += e;
      }
    }
  }
  __syncthreads();

  // Phase 5: write the lists: every surviving row opens its list with itself, every merged A token
  // enters its destination's list at its slot.
  for (int i = tid; i < n; i += NT) {
    const bool odd = i & 1;
    if (!odd && merged[i >> 1]) {
      const int a = i >> 1, d = 2 * bcol[a] + 1;
      src_list[i0 + ent_pos[d] + 1 + __float_as_int(best[a])] = i0 + i;
    } else {
      const int e = i0 + ent_pos[i];
      row_ptr[o0 + keep_pos[i]] = e;
      src_list[e] = i0 + i;
    }
  }
}

// The whole plan of query q by one workgroup of NT threads (a multiple of 64; tid = thread index; lds: its dynamic LDS).
template <typename T, bool ROWS_IN_LDS, int NT = kPlanThreads>
__device__ __forceinline__ void merge_plan_body(
    const T* __restrict__ src, int64_t row_stride, int col_off, int H, int dm, const int32_t* __restrict__ in_off,
    const int32_t* __restrict__ out_off, const int32_t* __restrict__ reff_arr, const int32_t* __restrict__ troff,
    int n_lead, int32_t* __restrict__ src_list, int32_t* __restrict__ row_ptr, int32_t* __restrict__ trace_src,
    int32_t* __restrict__ trace_dst, float* rows, float* lds, const int q, const int tid) {
  merge_plan_select<T, ROWS_IN_LDS, false, NT>(src, row_stride, col_off, H, dm, in_off, reff_arr, n_lead, rows, lds,
                                               nullptr, nullptr, q, tid);
  const int n = in_off[q + 1] - in_off[q];
  float* small = ROWS_IN_LDS ? lds + (size_t)max(n, 0) * plan_row_floats(dm) : lds;
  merge_plan_lists<NT, false>(small, nullptr, nullptr, in_off, out_off, reff_arr, troff, src_list, row_ptr, trace_src,
                              trace_dst, q, tid);
}

}  // namespace otas
#endif  // OTAS_MERGE_PLAN_BODY_H_
