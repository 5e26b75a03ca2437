// Multi-head attention of Sec. II-A over a ragged batch: per query q and head h,
//   O_h = softmax(Q_h K_h^T / sqrt(d_h) [+ ln size_j]) V_h,   heads concatenated into [T, D].
// qkv is the packed [T, 3D] output of the QKV projection (columns Q | K | V, heads contiguous).
//
//   * attention_rows_kernel -- one wave per query row, fp32 arithmetic throughout (f32 models,
//                              and the fallback for head widths the MFMA kernel does not take).
//   * attention_mfma_kernel -- bf16 MFMA with one head's K and V staged in LDS (bf16 models).
#include <algorithm>
#include <cstdlib>

#include "common.h"
#include "kernels.h"
#include "merge_plan_body.h"

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


// ------------------------------------------------------------------------------ bf16 MFMA
// grid (ceil(max_n / (32 NW)), H, B), NW waves (4 or 8): each wave owns 32 query rows of one (query, head).
// The keys and values of the head are staged in LDS in chunks of up to KC rows (rows padded
// by 16 bytes so that the 16 lanes served per clock fall on distinct banks); every wave then walks
// the chunk in blocks of 32 keys with an online softmax (running row maximum and sum, fp32).
//
// Both products are computed transposed, so that a lane always owns ONE query row:
//   S^T[key, row] = K[key, :] . Q[row, :]     A operand = K rows (LDS), B operand = Q rows (registers)
//   O^T[d, row]  += V^T[d, key] P^T[key, row] A operand = V^T (LDS, transposing read), B = P^T
// With the 32x32 accumulator layout a lane (row = lane & 31, half = lane >> 5) holds, of a 32-key
// block, the keys 8 (e / 4) + 4 half + (e & 3), e = 0..15: row maxima and sums are reductions over a
// lane's own registers plus one exchange with lane ^ 32, and the probabilities feed the second MFMA
// straight from registers: its k-slot i of half h is defined to be key 16 kk + 8 (i / 4) + 4 h +
// (i & 3), which is exactly what accumulator registers 8 kk .. 8 kk + 7 hold.  V^T is read with the
// same key order by ds_read_b64_tr_b16 (gfx950): in every group of 16 lanes, lane s supplies the
// address of V[k0 + s / 4][d0 + 4 (s & 3) ..+3] and lane i receives V[k0 + 0..3][d0 + i].
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef short short8_t __attribute__((ext_vector_type(8)));

// One (query q, head h, block xblk of 32 NW query rows) on NW waves: tid = thread index among those 64 NW
// threads, smem = their LDS region.  Every __syncthreads() below is reached by all threads of the workgroup
// that share q and xblk (the trip counts depend on the query's length and xblk only), so a workgroup may run
// several heads of one query side by side, each on its own NW waves and LDS region.
template <int DH, bool BIAS, int KC, int NW>
__device__ __forceinline__ void attention_mfma_body(const bf16_t* __restrict__ qkv, const int32_t* __restrict__ sizes,
                                                    const int32_t* __restrict__ off, int D, float scale,
                                                    bf16_t* __restrict__ o, const int q, const int h, const int xblk,
                                                    unsigned char* smem, const int tid) {
  constexpr int KS = DH / 16;             // k-steps of Q K^T
  constexpr int DT = (DH + 31) / 32;      // 32-row tiles of O^T
  constexpr int LD = DH + 8;              // LDS row stride in elements (16 bytes of padding)
  constexpr int VROWS = KC + 4;           // V^T reads of the last d tile may run past DH: keep them in bounds
  bf16_t* Ks = reinterpret_cast<bf16_t*>(smem);           // [KC][LD]
  bf16_t* Vs = Ks + KC * LD;                              // [VROWS][LD]
  float* lnsz = reinterpret_cast<float*>(Vs + VROWS * LD);  // [KC] log2(size) of the chunk's keys

  const int lane = tid & 63, wave = tid >> 6;
  const int base = off[q], n = off[q + 1] - base;
  constexpr int NT = 64 * NW;             // threads: NW waves of 32 query rows each
  const int row0 = xblk * (32 * NW);
  if (row0 >= n) return;
  const size_t ld = (size_t)3 * D;
  const int fr = lane & 31, fk = lane >> 5;
  const int my_row = row0 + wave * 32 + fr;
  const bool wave_active = row0 + wave * 32 < n;

  // Q fragments (B operand): lane (row, half) holds Q[row][16 ks + 8 half .. +7]
  bf16x8 qf[KS];
  {
    const bf16_t* qrow = qkv + (size_t)(base + (my_row < n ? my_row : n - 1)) * ld + h * DH + fk * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qrow + ks * 16);
  }

  floatx16 oacc[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[t][e] = 0.f;
  float m_run = -INFINITY, l_part = 0.f;
  const float scale2 = scale * 1.44269504088896340736f;   // logits are kept in units of ln 2

  for (int c0 = 0; c0 < n; c0 += KC) {
    const int nc = min(KC, n - c0);
    const int nc_pad = (nc + 31) & ~31;
    if (c0 > 0) __syncthreads();   // everyone is done with the previous chunk
    // stage K and V rows c0 .. c0 + nc_pad - 1 (zero beyond n)
    constexpr int CPR = DH / 8;    // 16-byte chunks per row
    // batches of 4 chunk pairs per thread: all eight loads of a batch are issued before the first
    // LDS store waits for them, so their latencies overlap
    const int n_chunks = nc_pad * CPR;
    for (int t0 = 0; t0 < n_chunks; t0 += 4 * NT) {
      bf16x8 kv[4], vv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int t = t0 + u * NT + tid;
        const int r = t / CPR, c = (t - r * CPR) * 8;
        const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
        kv[u] = zero;
        vv[u] = zero;
        if (t < n_chunks && r < nc) {
          const bf16_t* src = qkv + (size_t)(base + c0 + r) * ld + D + h * DH + c;
          kv[u] = *reinterpret_cast<const bf16x8*>(src);
          vv[u] = *reinterpret_cast<const bf16x8*>(src + D);
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int t = t0 + u * NT + tid;
        const int r = t / CPR, c = (t - r * CPR) * 8;
        if (t < n_chunks) {
          *reinterpret_cast<bf16x8*>(Ks + r * LD + c) = kv[u];
          *reinterpret_cast<bf16x8*>(Vs + r * LD + c) = vv[u];
        }
      }
    }
    if (BIAS) {
      for (int t = tid; t < nc_pad; t += NT) lnsz[t] = t < nc ? log2f((float)sizes[base + c0 + t]) : 0.f;
    }
    __syncthreads();
    if (!wave_active) continue;

    // The key blocks are software-pipelined inside the wave: the MFMA chain of block b + 1's logits is
    // issued before the softmax arithmetic of block b starts, so the matrix pipe works under the VALU
    // instructions of the same wave (the kernel runs at two to four waves per SIMD and is bound by
    // these dependency waits, not by VALU or MFMA throughput).
    auto s_block = [&](floatx16& sacc, int kb) {   // S^T block: logits of keys kb .. kb + 31
#pragma unroll
      for (int e = 0; e < 16; ++e) sacc[e] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(Ks + (kb + fr) * LD + ks * 16 + fk * 8);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sacc, 0, 0, 0);
      }
    };
    auto softmax_pv = [&](floatx16& sacc, int kb) {
      // Logits in base-2 units, t = s * (scale * log2 e) [+ log2(size)], so that exp(s - m) is one
      // v_exp_f32.  Without the size bias the scaling is folded into the exponent's argument,
      // exp2(fma(s, scale2, -m)): the maximum is taken over the raw products (scale2 > 0) and scaled
      // once per row.  Only the chunk's last block can hold keys past the end.
      float mx = -INFINITY;
      if (BIAS) {
#pragma unroll
        for (int e = 0; e < 16; ++e)
          sacc[e] = sacc[e] * scale2 + lnsz[kb + 8 * (e >> 2) + 4 * fk + (e & 3)];
      }
      if (kb + 32 > nc) {   // wave-uniform: keys past the end of the sequence
#pragma unroll
        for (int e = 0; e < 16; ++e)
          sacc[e] = (kb + 8 * (e >> 2) + 4 * fk + (e & 3)) < nc ? sacc[e] : -INFINITY;
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sacc[e]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
      if (!BIAS) mx *= scale2;
      if (__any(mx > m_run)) {   // some row's maximum moved: rescale what has been accumulated
        const float m_new = fmaxf(m_run, mx);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);   // 0 on the first block (m_run = -inf)
        m_run = m_new;
        l_part *= alpha;
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
          for (int e = 0; e < 16; ++e) oacc[t][e] *= alpha;
      }
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float pv = BIAS ? __builtin_amdgcn_exp2f(sacc[e] - m_run)
                              : __builtin_amdgcn_exp2f(fmaf(sacc[e], scale2, -m_run));
        sacc[e] = pv;
        psum += pv;
      }
      l_part += psum;
      // O^T += V^T P^T, two k-steps of 16 keys
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        bf16x8 pf;
#pragma unroll
        for (int i = 0; i < 8; ++i) pf[i] = (bf16_t)sacc[8 * kk + i];
        // transposing reads: lane s of each 16-lane group points at V[k0 + s/4][d0 + 4 (s & 3)]
        const int s16 = lane & 15;
        const int d0 = ((lane >> 4) & 1) * 16;
        const int k0 = kb + 16 * kk + 4 * fk;
#pragma unroll
        for (int t = 0; t < DT; ++t) {
          const bf16_t* vp = Vs + (k0 + (s16 >> 2)) * LD + t * 32 + d0 + 4 * (s16 & 3);
          const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) short4_t*)(vp));
          const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) short4_t*)(vp + 8 * LD));
          const short8_t both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
          bf16x8 vf;
          __builtin_memcpy(&vf, &both, 16);
          oacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, oacc[t], 0, 0, 0);
        }
      }
    };
    const int nblk = nc_pad >> 5;
    floatx16 s_even, s_odd;
    s_block(s_even, 0);
    for (int b = 0; b < nblk; b += 2) {
      if (b + 1 < nblk) s_block(s_odd, (b + 1) * 32);
      __builtin_amdgcn_sched_barrier(0);
      softmax_pv(s_even, b * 32);
      if (b + 1 < nblk) {
        if (b + 2 < nblk) s_block(s_even, (b + 2) * 32);
        __builtin_amdgcn_sched_barrier(0);
        softmax_pv(s_odd, (b + 1) * 32);
      }
    }
  }
  if (!wave_active) return;
  const float l_tot = l_part + __shfl_xor(l_part, 32, kWave);
  if (my_row < n) {
    const float inv = 1.0f / l_tot;
    bf16_t* orow = o + (size_t)(base + my_row) * D + h * DH;
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int d = t * 32 + g * 8 + fk * 4;
        if (d < DH) {
          bf16x4 ov = {(bf16_t)(oacc[t][g * 4 + 0] * inv), (bf16_t)(oacc[t][g * 4 + 1] * inv),
                       (bf16_t)(oacc[t][g * 4 + 2] * inv), (bf16_t)(oacc[t][g * 4 + 3] * inv)};
          *reinterpret_cast<bf16x4*>(orow + d) = ov;
        }
      }
  }
}

template <int DH, bool BIAS, int KC, int NW>
__global__ __launch_bounds__(64 * NW, DH <= 64 ? 4 : 2) void attention_mfma_kernel(const bf16_t* __restrict__ qkv,
                                                             const int32_t* __restrict__ sizes,
                                                             const int32_t* __restrict__ off, int D, float scale,
                                                             bf16_t* __restrict__ o) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  attention_mfma_body<DH, BIAS, KC, NW>(qkv, sizes, off, D, scale, o, (int)blockIdx.z, (int)blockIdx.y, (int)blockIdx.x,
                                        smem, (int)threadIdx.x);
}

// Attention and the merge plan of a layer in ONE launch (both only read the layer's QKV projection, and
// kernels of one stream do not overlap): the first workgroups run the plan -- workgroup q the whole plan of query q
// (merge_plan_body), or, when sel_best is given, `parts` workgroups per query only its selection
// (merge_plan_select: the lists are then written beside the next launch) -- the others run attention, each on
// 8 / NW heads of one (query, row block) side by side.  The plan workgroups come first in dispatch order, so their
// long serial chains start at once and the attention workgroups fill the other CUs.  Workgroups of 512 threads:
// attention then has the shape of the stand-alone kernel (one head of eight waves, or two of four: heads in one
// workgroup share its barriers, and four heads in lock-step in 1024-thread workgroups cost attention a fifth of its
// speed), and a plan workgroup shares its CU with an attention workgroup instead of taking the CU.  Head width 64
// only (four waves per SIMD leave 128 registers per lane).
// grid.x = B * parts + xblks * (H / G) * B with G = 8 / NW (parts = plan workgroups per query, 1 for the whole plan).
constexpr int kFusedThreads = 512;
template <bool BIAS, int KC, int NW>
__global__ __launch_bounds__(kFusedThreads, 4) void attention_plan_kernel(
    const bf16_t* __restrict__ qkv, const int32_t* __restrict__ sizes, const int32_t* __restrict__ off, int D, int H,
    float scale, bf16_t* __restrict__ o, int B, int xblks, const int32_t* __restrict__ out_off,
    const int32_t* __restrict__ reff_arr, const int32_t* __restrict__ troff, int n_lead,
    int32_t* __restrict__ src_list, int32_t* __restrict__ row_ptr, int32_t* __restrict__ trace_src,
    int32_t* __restrict__ trace_dst, float* __restrict__ sel_best, int32_t* __restrict__ sel_bcol, int parts,
    int unit_lds) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int DH = 64, WT = kFusedThreads, G = WT / 64 / NW;
  if ((int)blockIdx.x < B * parts) {   // workgroup-uniform
    if (sel_best)   // the selection only, `parts` workgroups per query: the lists are written beside the output projection
      merge_plan_select<bf16_t, true, true, WT>(qkv, 3 * (int64_t)D, D, H, DH, off, reff_arr, n_lead, nullptr,
                                                reinterpret_cast<float*>(smem), sel_best, sel_bcol,
                                                (int)blockIdx.x / parts, (int)threadIdx.x, (int)blockIdx.x % parts,
                                                parts);
    else
      merge_plan_body<bf16_t, true, WT>(qkv, 3 * (int64_t)D, D, H, DH, off, out_off, reff_arr, troff, n_lead, src_list,
                                        row_ptr, trace_src, trace_dst, nullptr, reinterpret_cast<float*>(smem),
                                        (int)blockIdx.x, (int)threadIdx.x);
    return;
  }
  int id = (int)blockIdx.x - B * parts;
  const int hg = H / G;
  const int xblk = id % xblks;
  id /= xblks;
  const int hgrp = id % hg, q = id / hg;
  const int unit = (int)threadIdx.x / (64 * NW), tid = (int)threadIdx.x % (64 * NW);
  attention_mfma_body<DH, BIAS, KC, NW>(qkv, sizes, off, D, scale, o, q, hgrp * G + unit, xblk, smem + (size_t)unit * unit_lds,
                                        tid);
}

template <int DH, bool BIAS>
static hipError_t attention_mfma_b(const void* qkv, const int32_t* sz, const int32_t* d_off, int B, int max_n, int D,
                                 int H, float scale, void* o, hipStream_t s) {
  constexpr int LD = DH + 8;
  // Sequences of up to 128 rows (and those beyond 256): four waves per workgroup, keys and values
  // staged 128 at a time ((128 + 132) rows of DH + 8 bf16 = 37 KB at DH = 64, so four workgroups share
  // a CU and cover each other's MFMA-dependency and barrier waits).  Sequences of 129 .. 256 rows: one
  // workgroup of eight waves per (query, head) instead of two of four, with the head's keys and values
  // staged once and in one piece (75 KB at DH = 64, two workgroups per CU): one load phase per
  // workgroup instead of two (measured on MI355X, batch 64, 12 heads: 26.3 us against 27.2 at n = 197,
  // 18.2 against 20.6 at n = 133).
#define OTAS_ATTN(KC, NWV)                                                                                        \
  do {                                                                                                            \
    const size_t lds = (size_t)(KC + KC + 4) * LD * sizeof(bf16_t) + KC * sizeof(float);                          \
    auto kern = attention_mfma_kernel<DH, BIAS, KC, NWV>;                                                         \
    hipError_t e = set_max_dynamic_lds((const void*)kern, (int)lds);                                              \
    if (e != hipSuccess) return e;                                                                                \
    dim3 grid((max_n + 32 * NWV - 1) / (32 * NWV), H, B), block(64 * NWV);                                        \
    kern<<<grid, block, lds, s>>>((const bf16_t*)qkv, sz, d_off, D, scale, (bf16_t*)o);                           \
  } while (0)
  if (max_n > 128 && max_n <= 256) OTAS_ATTN((DH <= 64 ? 256 : 128), 8);   // wider heads: two pieces, as before
  else OTAS_ATTN(128, 4);
#undef OTAS_ATTN
  return hipGetLastError();
}

template <int DH>
static hipError_t attention_mfma(const void* qkv, const int32_t* sz, const int32_t* d_off, int B, int max_n, int D,
                                 int H, float scale, void* o, hipStream_t s) {
  return sz ? attention_mfma_b<DH, true>(qkv, sz, d_off, B, max_n, D, H, scale, o, s)
            : attention_mfma_b<DH, false>(qkv, sz, d_off, B, max_n, D, H, scale, o, s);
}

// Whether launch_attention_plan takes this case (pure host).
bool attention_plan_takes(int dtype, int max_n, int D, int H) {
  if (dtype == 0 || H <= 0 || D != 64 * H || max_n <= 0 || max_n > kPlanThreads) return false;
  if (merge_plan_lds_bytes(max_n, 64) > 160 * 1024) return false;
  const int G = (max_n > 128 && max_n <= 256) ? 1 : 2;   // heads per workgroup: 8 waves / (8 or 4 waves per head)
  return H % G == 0;
}

// Attention of a layer together with the layer's merge plan (bf16, head width 64, H a multiple of the heads a
// workgroup takes, every query's metric rows in LDS); hipErrorInvalidValue otherwise -- the caller then launches
// the two kernels one after the other.
hipError_t launch_attention_plan(const void* qkv, const int32_t* sizes, const int32_t* d_off, const int32_t* d_out_off,
                                 const int32_t* d_reff, const int32_t* d_troff, int B, int max_n, int D, int H,
                                 bool size_bias, int n_lead, void* o, int32_t* src_list, int32_t* row_ptr,
                                 int32_t* trace_src, int32_t* trace_dst, float* sel_best, int32_t* sel_bcol,
                                 hipStream_t s) {
  if (B <= 0 || max_n <= 0) return hipSuccess;
  if (H <= 0 || D != 64 * H || max_n > kPlanThreads || (sel_best == nullptr) != (sel_bcol == nullptr))
    return hipErrorInvalidValue;
  const size_t plan_lds = merge_plan_lds_bytes(max_n, 64);
  if (plan_lds > 160 * 1024) return hipErrorInvalidValue;
  const float scale = 1.0f / sqrtf(64.0f);
  const int32_t* sz = size_bias ? sizes : nullptr;
  constexpr int LD = 64 + 8;
  // Workgroups per query for the selection: a small batch leaves most CUs idle, and the selection's chain (load the
  // keys, unit length, similarities: each proportional to the A tokens a workgroup owns, plus all B tokens) is what
  // the launch then waits for.  Up to 64 plan workgroups in all, and no more per query than it has blocks of 32 A tokens.
  int parts = 1;
  if (sel_best) parts = std::max(1, std::min(std::min(4, 64 / B), (max_n / 2 + 31) / 32));
#define OTAS_FUSED(BIASV, KC, NWV)                                                                                \
  do {                                                                                                            \
    constexpr int G = kFusedThreads / 64 / NWV;                                                                   \
    if (H % G != 0) return hipErrorInvalidValue;                                                                  \
    const size_t unit = ((size_t)(KC + KC + 4) * LD * sizeof(bf16_t) + KC * sizeof(float) + 15) & ~(size_t)15;    \
    const size_t lds = unit * G > plan_lds ? unit * G : plan_lds;                                                 \
    if (lds > 160 * 1024) return hipErrorInvalidValue;                                                            \
    auto kern = attention_plan_kernel<BIASV, KC, NWV>;                                                            \
    hipError_t e = set_max_dynamic_lds((const void*)kern, 160 * 1024);                                            \
    if (e != hipSuccess) return e;                                                                                \
    const int xblks = (max_n + 32 * NWV - 1) / (32 * NWV);                                                        \
    dim3 grid((unsigned)(B * parts + xblks * (H / G) * B)), block(kFusedThreads);                                 \
    kern<<<grid, block, lds, s>>>((const bf16_t*)qkv, sz, d_off, D, H, scale, (bf16_t*)o, B, xblks, d_out_off,    \
                                  d_reff, d_troff, n_lead, src_list, row_ptr, trace_src, trace_dst, sel_best,     \
                                  sel_bcol, parts, (int)unit);                                                    \
  } while (0)
  if (max_n > 128 && max_n <= 256) {
    if (sz) OTAS_FUSED(true, 256, 8); else OTAS_FUSED(false, 256, 8);
  } else {
    if (sz) OTAS_FUSED(true, 128, 4); else OTAS_FUSED(false, 128, 4);
  }
#undef OTAS_FUSED
  return hipGetLastError();
}

hipError_t launch_attention(int dtype, const void* qkv, const int32_t* sizes, const int32_t* d_off, int B,
                            int max_n, int D, int H, bool size_bias, void* o, hipStream_t s) {
  if (B <= 0 || max_n <= 0) return hipSuccess;
  const int dh = D / H;
  const float scale = 1.0f / sqrtf((float)dh);
  const int32_t* sz = size_bias ? sizes : nullptr;
  dim3 grid((max_n + 3) / 4, H, B), block(256);
  const size_t lds = (size_t)4 * (max_n + dh) * sizeof(float);
  if (dtype != 0) {
    if (dh == 64) return attention_mfma<64>(qkv, sz, d_off, B, max_n, D, H, scale, o, s);
    if (dh == 80) return attention_mfma<80>(qkv, sz, d_off, B, max_n, D, H, scale, o, s);
    if (dh == 96) return attention_mfma<96>(qkv, sz, d_off, B, max_n, D, H, scale, o, s);
    if (dh == 128) return attention_mfma<128>(qkv, sz, d_off, B, max_n, D, H, scale, o, s);
  }
  if (dtype == 0)
    attention_rows_kernel<float><<<grid, block, lds, s>>>((const float*)qkv, sz, d_off, D, H, max_n, scale, (float*)o);
  else
    attention_rows_kernel<bf16_t><<<grid, block, lds, s>>>((const bf16_t*)qkv, sz, d_off, D, H, max_n, scale,
                                                           (bf16_t*)o);
  return hipGetLastError();
}

}  // namespace otas
