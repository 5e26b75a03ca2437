// Linear layers of the encoder block (Sec. II-A: per-head Q/K/V projections, the linear after
// the concatenated heads, and the MLP):  Y[M,N] = epilogue(X[M,K] W[N,K]^T + bias[N]).
//
// Kernels:
//   * gemm_valu_kernel  -- plain fp32 FMA tiles; the true-fp32 path (f32 models) and the fallback
//                          for shapes the MFMA kernels do not take.
//   * bf16 MFMA (v_mfma_f32_32x32x16_bf16), fp32 accumulate, operand tiles loaded straight into
//     swizzled LDS stages, fused bias / GELU / residual epilogue (bf16 models):
//       gemm_mfma_k32_kernel     128 x 128, K step 32, three workgroups per CU (also split-K)
//       gemm_mfma128k64_kernel   128 x 128, K step 64, two per CU (also split-K: the form split launches run)
//       gemm_mfma256w8_kernel    192 / 256 / 320 x 256, eight waves, one per CU
//       gemm_mfma64_kernel       64 x 64, K step 32, for products of very few rows
//     pick_mfma_kernel chooses among them with a cost model fitted to measured launch times; splitk_factor
//     decides with the same model whether the MLP's second linear is split over K.
//     Each kernel has a PLAN form for the attention output projection, whose first workgroups write the lists
//     of the layer's merge plan (merge_plan_lists) instead of computing a tile.
#include <algorithm>
#include <cmath>
#include <cstdlib>

#include "common.h"
#include "kernels.h"
#include "merge_plan_body.h"

namespace otas {

// Output element type: the residual epilogue writes the float residual stream, the others the
// model's storage type.
template <typename T, int EPI> struct OutType { typedef T type; };
template <typename T> struct OutType<T, EPI_RESIDUAL> { typedef float type; };
template <typename T> struct OutType<T, EPI_PARTIAL> { typedef float type; };

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



// Epilogue shared by the MFMA kernels.  A lane's accumulators belong to ONE output row and to
// scattered 4-column groups, so storing them directly would touch 32 rows with 16-byte pieces per
// instruction.  Instead every wave transposes its tile through its own LDS region, 32 rows at a
// time: it writes acc[i][j][e] (row = lane & 31, columns 32 j + 8 (e / 4) + 4 (lane >> 5) + (e & 3))
// as floats into a [32][WN + 4] slab, reads the slab back row-major (16 bytes per lane, WN / 4
// lanes per row) and applies bias / GELU / residual there, where the bias and residual loads and the
// output stores are contiguous runs of a full row segment.  stage: this wave's region of
// 32 * (32 TN + 4) floats, no longer used by anyone else (barrier before the call).
template <int EPI, int TM, int TN>
__device__ inline void mfma_epilogue(const floatx16 (&acc)[TM][TN], float* stage, const bf16_t* __restrict__ bias,
                                     const float* res, typename OutType<bf16_t, EPI>::type* Y, int64_t M, int N,
                                     int64_t m_wave, int n_wave, int lane) {
  constexpr int WN = 32 * TN, LDR = WN + 4;
  constexpr int LPR = WN / 4;      // lanes per row when reading back
  constexpr int RPI = 64 / LPR;    // rows per read-back instruction
  constexpr int NIT = 32 / RPI;
  const int fr = lane & 31, fk = lane >> 5;
  const int rrow = lane / LPR, rcol = (lane % LPR) * 4;
  const int n = n_wave + rcol;
  const bool n_ok = n < N;         // N % 8 == 0: a 4-column group is inside or outside as a whole
  bf16x4 bb = {(bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f};
  if (EPI != EPI_PARTIAL) bb = *reinterpret_cast<const bf16x4*>(bias + (n_ok ? n : 0));
  // The residual rows of slab i + 1 are requested before slab i goes through LDS, so their latency
  // is covered by a whole slab's work instead of being waited for once per slab.
  floatx4 rr[2][NIT];
  auto load_res = [&](int i) {
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int64_t m = m_wave + i * 32 + it * RPI + rrow;
      rr[i & 1][it] = *reinterpret_cast<const floatx4*>(res + (size_t)(m < M ? m : M - 1) * N + (n_ok ? n : 0));
    }
  };
  if (EPI == EPI_RESIDUAL) load_res(0);
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int64_t m_slab = m_wave + i * 32;
    if (EPI == EPI_RESIDUAL && i + 1 < TM) load_res(i + 1);
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const floatx4 v = {acc[i][j][g * 4 + 0], acc[i][j][g * 4 + 1], acc[i][j][g * 4 + 2], acc[i][j][g * 4 + 3]};
        *reinterpret_cast<floatx4*>(stage + fr * LDR + j * 32 + g * 8 + fk * 4) = v;
      }
    // the slab is read back four rows per lane at a time before anything is stored: one LDS wait per group
    // instead of one per store
    constexpr int GRP = NIT < 4 ? NIT : 4;
    floatx4 ag[GRP];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int row = it * RPI + rrow;
      if (it % GRP == 0) {
#pragma unroll
        for (int u = 0; u < GRP; ++u)
          ag[u] = *reinterpret_cast<const floatx4*>(stage + ((it + u) * RPI + rrow) * LDR + rcol);
      }
      const floatx4 a = ag[it % GRP];
      float v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = EPI == EPI_PARTIAL ? a[e] : a[e] + (float)bb[e];
      if (EPI == EPI_GELU) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = gelu_bf16(v[e]);
      }
      const int64_t m = m_slab + row;
      if (m < M && n_ok) {
        const size_t idx = (size_t)m * N + n;
        if (EPI == EPI_RESIDUAL) {
          floatx4 o = {v[0] + rr[i & 1][it][0], v[1] + rr[i & 1][it][1], v[2] + rr[i & 1][it][2], v[3] + rr[i & 1][it][3]};
          *reinterpret_cast<floatx4*>(reinterpret_cast<float*>(Y) + idx) = o;
        } else if (EPI == EPI_PARTIAL) {
          floatx4 o = {v[0], v[1], v[2], v[3]};
          *reinterpret_cast<floatx4*>(reinterpret_cast<float*>(Y) + idx) = o;
        } else {
          bf16x4 o = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
          *reinterpret_cast<bf16x4*>(reinterpret_cast<bf16_t*>(Y) + idx) = o;
        }
      }
    }
  }
}

// Epilogue for the 16-bit outputs (no residual).  Bias and GELU are applied to the accumulators in
// registers (a lane owns runs of 4 consecutive columns of one row), the results are rounded to bf16
// and only then transposed through the wave's LDS slab, [32][WN + 8] bf16: half the LDS traffic of the
// float slab, and the read-back hands every lane 8 consecutive columns, so the global stores are
// 16 bytes per lane and a row segment of 2 WN bytes goes out in one instruction.
template <int EPI, int TM, int TN>
__device__ inline void mfma_epilogue_bf16(const floatx16 (&acc)[TM][TN], bf16_t* stage, const bf16_t* __restrict__ bias,
                                          bf16_t* Y, int64_t M, int N, int64_t m_wave, int n_wave, int lane) {
  constexpr int WN = 32 * TN, LDR = WN + 8;
  constexpr int LPR = WN / 8;      // lanes per row when reading back
  constexpr int RPI = 64 / LPR;    // rows per read-back instruction
  constexpr int NIT = 32 / RPI;
  const int fr = lane & 31, fk = lane >> 5;
  const int rrow = lane / LPR, rcol = (lane % LPR) * 8;
  const int n_out = n_wave + rcol;
  const bool n_ok = n_out < N;     // N % 8 == 0: an 8-column group is inside or outside as a whole
  bf16x4 bb[TN][4];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int n = n_wave + 32 * j + 8 * g + 4 * fk;
      bb[j][g] = *reinterpret_cast<const bf16x4*>(bias + (n < N ? n : 0));
    }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int64_t m_slab = m_wave + i * 32;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          v[e] = acc[i][j][g * 4 + e] + (float)bb[j][g][e];
          if (EPI == EPI_GELU) v[e] = gelu_bf16(v[e]);
        }
        const bf16x4 o = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
        *reinterpret_cast<bf16x4*>(stage + fr * LDR + j * 32 + g * 8 + fk * 4) = o;
      }
    // all of the slab's rows are read back before the first is stored: one LDS wait per slab instead of one per
    // store, and one address computation (the rows of a lane are RPI * N elements apart)
    bf16x8 a[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) a[it] = *reinterpret_cast<const bf16x8*>(stage + (it * RPI + rrow) * LDR + rcol);
    bf16_t* yp = Y + (size_t)(m_slab + rrow) * N + n_out;
#pragma unroll
    for (int it = 0; it < NIT; ++it)
      if (m_slab + it * RPI + rrow < M && n_ok) *reinterpret_cast<bf16x8*>(yp + (size_t)it * RPI * N) = a[it];
  }
}

// ------------------------------------------------------------------------------ bf16 MFMA tiles
// All MFMA kernels compute the transposed tile (W rows as the first operand, X rows as the second): a
// lane then holds, for one output row m, runs of 4 consecutive output columns n, which makes the
// epilogue's loads and stores 8- or 16-byte vectors along the row.

// Tile order.  Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2, and inside
// an XCD the ~32 resident workgroups are consecutive in that XCD's sequence.  Give XCD x the
// sequence positions s = id / 8 of one contiguous band of tiles, and inside the band walk groups of
// GM tile rows column by column, so that the tiles in flight on one XCD form a compact block that
// shares activation and weight panels through that L2.
__device__ inline void tile_of_block(int bid, int tiles_m, int tiles_n, int& tile_m, int& tile_n) {
  constexpr int GM = 8;
  const int nblk = tiles_m * tiles_n;
  const int per = nblk >> 3;
  int t = bid;
  if (bid < per * 8) t = (bid & 7) * per + (bid >> 3);   // full bands; the remainder keeps its id
  const int group = GM * tiles_n;
  const int g = t / group, idx = t - g * group;
  const int rows = min(GM, tiles_m - g * GM);            // the last group may be shorter
  tile_n = idx / rows;
  tile_m = g * GM + (idx - tile_n * rows);
}

// ------------------------------------------------------------------------------ direct-to-LDS kernels
// Operand tiles go from global memory straight into LDS (global_load_lds_dwordx4: 16 bytes per lane,
// each wave instruction fills 1 KB of consecutive LDS; no staging registers, no ds_write) through a
// ring of stages of K step 32.  Loads complete in issue order, so "at most n still in flight"
// (s_waitcnt vmcnt(n)) means everything but the n youngest has landed; a wave waits for its own
// loads, then a raw s_barrier makes every wave's loads visible.  The compiler is kept from moving
// LDS accesses across these points by empty asm memory clobbers.
// Stage layout: rows of 64 B (32 bf16); 16-byte chunk c of row r sits at chunk c ^ ((r >> 2) & 3).
// The DMA writes are linear; a fragment read is served 16 lanes per clock and its 16 consecutive
// rows of one chunk column fall on 16 different (row mod 4, chunk position) pairs, i.e. on all 64
// banks once.  Lane i of a DMA instruction writes LDS row base + i/4, chunk position i%4, so it must
// fetch logical chunk (i%4) ^ ((row >> 2) & 3) of that row.
#define OTAS_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (7 << 4) | (15 << 8) | (((n) >> 4) << 14))
// vmcnt(0) and lgkmcnt(0): this wave's loads have landed AND its LDS reads have returned.
#define OTAS_WAIT_LOADS_AND_LDS() __builtin_amdgcn_s_waitcnt(7 << 4)
#define OTAS_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define OTAS_LPTR(p) ((__attribute__((address_space(3))) void*)(p))


// The list phases of the merge plan inside a GEMM launch (PLAN variants of the kernels below): the launch's first
// pt.B workgroups each write the lists of one query and leave; the others compute tiles as if those did not exist.
// The attention output projection runs this way: the lists depend on the selection made beside attention one
// launch earlier, and the projection leaves CUs idle at the batch sizes this matters for.
template <int NT>
__device__ __forceinline__ void plan_tail_run(const PlanTail& pt, unsigned char* smem, int q, int tid) {
  merge_plan_lists<NT, true>(reinterpret_cast<float*>(smem), pt.best, pt.bcol, pt.in_off, pt.out_off, pt.reff, pt.troff,
                             pt.src_list, pt.row_ptr, pt.trace_src, pt.trace_dst, q, tid);
}
#define OTAS_PLAN_TAIL_OR_TILE(NT)                          \
  int bid = (int)blockIdx.x;                                \
  if constexpr (PLAN) {                                     \
    if (bid < pt.B) {                                       \
      plan_tail_run<NT>(pt, smem, bid, (int)threadIdx.x);   \
      return;                                               \
    }                                                       \
    bid -= pt.B;                                            \
  }

// ------------------------------------------------------------------------------ (64 TM) x 128, K step 32
// Four waves in a 2 x 2 arrangement, each owning (32 TM) x 64 outputs; block tile (64 TM) x 128.  The
// library runs TM = 2 (128 rows, three workgroups per CU); TM = 3 and 4 (192 / 256 rows, two per CU)
// were measured on MI355X and lose to the 256-wide kernels on every large shape (60 us against 50 us
// for 12608 x 2304 x 768) and win by less than 10 % on a handful of mid-size ones, so they are not
// dispatched.  K step 32, operand tiles loaded straight into a ring of NS = 3 LDS stages by
// global_load_lds_dwordx4 (deeper rings, NS = 4 .. 8, change nothing: a lone workgroup is bound by what
// one CU can stream from L2, about 50 GB/s, not by load latency).  Several workgroups share a CU:
// while one waits at its barrier or for its fragments, or runs its epilogue (bias, GELU, the residual
// traffic), the others keep the matrix pipe busy.
//   iteration t: wait for this wave's loads of tile t, barrier, start the loads of tile t+NS-1 into
//                the stage tile t-1 used, then the two k-steps of tile t (fragment reads of the
//                second step are issued between the MFMAs of the first).
template <int EPI, int NS, int TM, bool PLAN = false>
__global__ __launch_bounds__(256, TM == 2 ? 3 : 2) void gemm_mfma_k32_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, const bf16_t* __restrict__ bias, const float* res,
    typename OutType<bf16_t, EPI>::type* Y, int64_t M, int N, int K, int k_len, int tiles_m, int tiles_n,
    PlanTail pt) {
  // K is the row length of A and W; this workgroup contracts over k_len of it, starting at
  // blockIdx.y * k_len (split-K launches write one float partial result [M, N] per blockIdx.y).
  constexpr int WM = 32 * TM, BM = 2 * WM, BN = 128, BK = 32, WN = 64, TN = 2;
  constexpr int STAGE_A = BM * BK, STAGE_W = BN * BK;   // elements per stage
  constexpr int NM = TM * TN, NF = TM + TN, ND = TM + 2;   // MFMAs / fragment reads per k-step, loads per tile
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* As = reinterpret_cast<bf16_t*>(smem);   // [NS][BM][32]
  bf16_t* Ws = As + NS * STAGE_A;                 // [NS][128][32]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: LDS addresses of the DMA stay scalar
  const int wm = wave >> 1, wn = wave & 1;
  int tile_m, tile_n;
  OTAS_PLAN_TAIL_OR_TILE(256)
  tile_of_block(bid, tiles_m, tiles_n, tile_m, tile_n);
  const int64_t m0 = (int64_t)tile_m * BM;
  const int n0 = tile_n * BN;

  // DMA addressing: 16 rows of 64 B per instruction; wave w owns rows w*16*TM .. of the A tile and rows
  // w*32 .. of the W tile.  Global addresses: uniform base (tile origin + this split's k range + k)
  // plus a constant per-lane 32-bit byte offset.
  uint32_t a_off[TM], w_off[2];
#pragma unroll
  for (int j = 0; j < TM; ++j) {
    const int row = wave * (16 * TM) + j * 16 + (lane >> 2);
    const int c = (lane & 3) ^ ((row >> 2) & 3);
    const int64_t a_last = M - 1 - m0;                // rows past the end repeat the last row
    const uint32_t ra = (uint32_t)(row < a_last ? row : a_last);
    a_off[j] = (ra * (uint32_t)K + (uint32_t)c * 8u) * (uint32_t)sizeof(bf16_t);
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int row = wave * 32 + j * 16 + (lane >> 2);
    const int c = (lane & 3) ^ ((row >> 2) & 3);
    const int w_last = N - 1 - n0;
    const uint32_t rw = (uint32_t)(row < w_last ? row : w_last);
    w_off[j] = (rw * (uint32_t)K + (uint32_t)c * 8u) * (uint32_t)sizeof(bf16_t);
  }
  const char* a_base = reinterpret_cast<const char*>(A + (size_t)m0 * K + (size_t)blockIdx.y * k_len);
  const char* w_base = reinterpret_cast<const char*>(W + (size_t)n0 * K + (size_t)blockIdx.y * k_len);
  if (EPI == EPI_PARTIAL) Y += (size_t)blockIdx.y * M * N;
  const int KT = k_len / BK;
  auto dma_one = [&](int kt, int st, int d) {   // d = 0..TM-1: A rows; TM, TM+1: W rows
    const size_t kb = (size_t)((kt < KT ? kt : KT - 1) * BK) * sizeof(bf16_t);
    if (d < TM)
      __builtin_amdgcn_global_load_lds(OTAS_GPTR(a_base + kb + a_off[d]),
                                       OTAS_LPTR(As + st * STAGE_A + (wave * (16 * TM) + d * 16) * BK), 16, 0, 0);
    else
      __builtin_amdgcn_global_load_lds(OTAS_GPTR(w_base + kb + w_off[d - TM]),
                                       OTAS_LPTR(Ws + st * STAGE_W + (wave * 32 + (d - TM) * 16) * BK), 16, 0, 0);
  };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int fr = lane & 31, fk = lane >> 5;
  const int frag_row = fr * BK, sw = (fr >> 2) & 3;
  bf16x8 af[2][TM], wf[2][TN];
  auto read_frag = [&](int st, int ks, int slot, int f) {   // f = 0..TM-1: A tiles; then the W tiles
    const int c = (((ks << 1) + fk) ^ sw) * 8;
    if (f < TM)
      af[slot][f] = *reinterpret_cast<const bf16x8*>(As + st * STAGE_A + (wm * WM + f * 32) * BK + frag_row + c);
    else
      wf[slot][f - TM] =
          *reinterpret_cast<const bf16x8*>(Ws + st * STAGE_W + (wn * WN + (f - TM) * 32) * BK + frag_row + c);
  };
  auto mfma_one = [&](int slot, int t) {
    const int i = t / TN, j = t % TN;
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[slot][j], af[slot][i], acc[i][j], 0, 0, 0);
  };

  // Prologue: tiles 0 .. NS-2.  Loads complete in issue order: "at most n in flight" = all but the n
  // youngest have landed.
#pragma unroll
  for (int t = 0; t < NS - 1; ++t)
#pragma unroll
    for (int d = 0; d < ND; ++d) dma_one(t, t, d);

  int st = 0, st_new = NS - 1;
  for (int kt = 0; kt < KT; ++kt) {
    OTAS_VMCNT(ND * (NS - 2));   // tile kt landed; tiles kt+1 .. kt+NS-2 may still be in flight
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int f = 0; f < NF; ++f) read_frag(st, 0, 0, f);
#pragma unroll
    for (int d = 0; d < ND; ++d) dma_one(kt + NS - 1, st_new, d);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < NM; ++t) {
      mfma_one(0, t);
      if (t < NF) read_frag(st, 1, 1, t);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int t = 0; t < NM; ++t) mfma_one(1, t);
    st = st + 1 == NS ? 0 : st + 1;
    st_new = st_new + 1 == NS ? 0 : st_new + 1;
  }
  OTAS_VMCNT(0);      // every load of this wave has landed ...
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();   // ... and of every other wave: the stages become the epilogue's staging area
  asm volatile("" ::: "memory");
  if constexpr (EPI == EPI_NONE || EPI == EPI_GELU)
    mfma_epilogue_bf16<EPI, TM, TN>(acc, reinterpret_cast<bf16_t*>(smem) + wave * 32 * (WN + 8), bias, Y, M, N,
                                    m0 + wm * WM, n0 + wn * WN, lane);
  else
    mfma_epilogue<EPI, TM, TN>(acc, reinterpret_cast<float*>(smem) + wave * 32 * (WN + 4), bias, res, Y, M, N,
                               m0 + wm * WM, n0 + wn * WN, lane);
}

template <int NS, int TM>
static hipError_t linear_mfma_k32(const void* x, const void* w, const void* bias, const float* res, void* y,
                                  int64_t M, int N, int K, int epi, hipStream_t s, int splits = 1,
                                  const PlanTail* pt = nullptr) {
  constexpr int BM = 64 * TM;
  const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (N + 127) / 128;
  const size_t lds = (size_t)NS * (BM + 128) * 32 * sizeof(bf16_t);
  static_assert(4 * 32 * (64 + 4) * sizeof(float) <= (size_t)NS * (BM + 128) * 32 * sizeof(bf16_t), "epilogue slab");
  static_assert(kPlanListsLdsMax <= (size_t)NS * (BM + 128) * 32 * sizeof(bf16_t), "plan lists");
  dim3 grid((unsigned)(tiles_m * tiles_n + (pt ? pt->B : 0)), (unsigned)splits), block(256);
  const int k_len = K / splits;
#define OTAS_MFMA(E, ...)                                                                                         \
  do {                                                                                                            \
    auto kern = gemm_mfma_k32_kernel<E, NS, TM, ##__VA_ARGS__>;                                                   \
    hipError_t e = set_max_dynamic_lds((const void*)kern, (int)lds);                                              \
    if (e != hipSuccess) return e;                                                                                \
    kern<<<grid, block, lds, s>>>((const bf16_t*)x, (const bf16_t*)w, (const bf16_t*)bias, res,                   \
                                  (typename OutType<bf16_t, E>::type*)y, M, N, K, k_len, tiles_m, tiles_n,        \
                                  pt ? *pt : PlanTail{});                                                         \
  } while (0)
  if (pt) {
    if (epi != EPI_RESIDUAL || splits != 1) return hipErrorInvalidValue;
    OTAS_MFMA(EPI_RESIDUAL, true);
  } else if (epi == EPI_NONE) OTAS_MFMA(EPI_NONE);
  else if (epi == EPI_GELU) OTAS_MFMA(EPI_GELU);
  else if (epi == EPI_PARTIAL) OTAS_MFMA(EPI_PARTIAL);
  else OTAS_MFMA(EPI_RESIDUAL);
#undef OTAS_MFMA
  return hipGetLastError();
}

// ------------------------------------------------------------------------------ 64 x 64, K step 32
// For products of so few rows that 128 x 128 tiles leave most CUs without a workgroup (small serving batches: a
// ViT-B query is 197 rows): block tile 64 x 64, four waves of 32 x 32 in a 2 x 2 arrangement, the same
// direct-to-LDS ring as gemm_mfma_k32_kernel with NS = 4 stages of 8 KB (up to five workgroups per CU).  Four times
// the workgroups of the 128 x 128 tiling at twice the operand bytes per FLOP: it wins while the launch is bound by
// the serial k-loop of a lone workgroup per CU, not by what the CUs can load.
template <int EPI, bool PLAN = false>
__global__ __launch_bounds__(256, 4) void gemm_mfma64_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W,
                                                             const bf16_t* __restrict__ bias, const float* res,
                                                             typename OutType<bf16_t, EPI>::type* Y, int64_t M, int N,
                                                             int K, int tiles_m, int tiles_n, PlanTail pt) {
  constexpr int BM = 64, BN = 64, BK = 32, NS = 4, ND = 2;
  constexpr int STAGE_A = BM * BK, STAGE_W = BN * BK;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* As = reinterpret_cast<bf16_t*>(smem);   // [NS][64][32]
  bf16_t* Ws = As + NS * STAGE_A;                 // [NS][64][32]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  int tile_m, tile_n;
  OTAS_PLAN_TAIL_OR_TILE(256)
  tile_of_block(bid, tiles_m, tiles_n, tile_m, tile_n);
  const int64_t m0 = (int64_t)tile_m * BM;
  const int n0 = tile_n * BN;
  // DMA: 16 rows of 64 B per instruction; wave w loads rows 16 w .. of the A tile and of the W tile
  uint32_t a_off, w_off;
  {
    const int row = wave * 16 + (lane >> 2);
    const int c = (lane & 3) ^ ((row >> 2) & 3);
    const int64_t a_last = M - 1 - m0;
    const int w_last = N - 1 - n0;
    const uint32_t ra = (uint32_t)(row < a_last ? row : a_last), rw = (uint32_t)(row < w_last ? row : w_last);
    a_off = (ra * (uint32_t)K + (uint32_t)c * 8u) * (uint32_t)sizeof(bf16_t);
    w_off = (rw * (uint32_t)K + (uint32_t)c * 8u) * (uint32_t)sizeof(bf16_t);
  }
  const char* a_base = reinterpret_cast<const char*>(A + (size_t)m0 * K);
  const char* w_base = reinterpret_cast<const char*>(W + (size_t)n0 * K);
  const int KT = K / BK;
  auto dma = [&](int kt, int st) {
    const size_t kb = (size_t)((kt < KT ? kt : KT - 1) * BK) * sizeof(bf16_t);
    __builtin_amdgcn_global_load_lds(OTAS_GPTR(a_base + kb + a_off), OTAS_LPTR(As + st * STAGE_A + wave * 16 * BK), 16, 0, 0);
    __builtin_amdgcn_global_load_lds(OTAS_GPTR(w_base + kb + w_off), OTAS_LPTR(Ws + st * STAGE_W + wave * 16 * BK), 16, 0, 0);
  };
  floatx16 acc[1][1];
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[0][0][e] = 0.f;
  const int fr = lane & 31, fk = lane >> 5;
  const int frag_row = fr * BK, sw = (fr >> 2) & 3;
#pragma unroll
  for (int t = 0; t < NS - 1; ++t) dma(t, t);
  int st = 0, st_new = NS - 1;
  for (int kt = 0; kt < KT; ++kt) {
    OTAS_VMCNT(ND * (NS - 2));
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    bf16x8 af[2], wf[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const int c = (((ks << 1) + fk) ^ sw) * 8;
      af[ks] = *reinterpret_cast<const bf16x8*>(As + st * STAGE_A + (wm * 32) * BK + frag_row + c);
      wf[ks] = *reinterpret_cast<const bf16x8*>(Ws + st * STAGE_W + (wn * 32) * BK + frag_row + c);
    }
    dma(kt + NS - 1, st_new);
    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[0], af[0], acc[0][0], 0, 0, 0);
    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[1], af[1], acc[0][0], 0, 0, 0);
    st = st + 1 == NS ? 0 : st + 1;
    st_new = st_new + 1 == NS ? 0 : st_new + 1;
  }
  OTAS_VMCNT(0);
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  if constexpr (EPI == EPI_NONE || EPI == EPI_GELU)
    mfma_epilogue_bf16<EPI, 1, 1>(acc, reinterpret_cast<bf16_t*>(smem) + wave * 32 * (32 + 8), bias, Y, M, N,
                                  m0 + wm * 32, n0 + wn * 32, lane);
  else
    mfma_epilogue<EPI, 1, 1>(acc, reinterpret_cast<float*>(smem) + wave * 32 * (32 + 4), bias, res, Y, M, N,
                             m0 + wm * 32, n0 + wn * 32, lane);
}

static hipError_t linear_mfma64(const void* x, const void* w, const void* bias, const float* res, void* y, int64_t M,
                                int N, int K, int epi, hipStream_t s, const PlanTail* pt = nullptr) {
  const int tiles_m = (int)((M + 63) / 64), tiles_n = (N + 63) / 64;
  const size_t lds = (size_t)4 * (64 + 64) * 32 * sizeof(bf16_t);
  static_assert(4 * 32 * (32 + 4) * sizeof(float) <= (size_t)4 * (64 + 64) * 32 * sizeof(bf16_t), "epilogue slab");
  static_assert(kPlanListsLdsMax <= (size_t)4 * (64 + 64) * 32 * sizeof(bf16_t), "plan lists");
  dim3 grid((unsigned)(tiles_m * tiles_n + (pt ? pt->B : 0))), block(256);
#define OTAS_MFMA(E, ...)                                                                                         \
  do {                                                                                                            \
    gemm_mfma64_kernel<E, ##__VA_ARGS__><<<grid, block, lds, s>>>(                                                \
        (const bf16_t*)x, (const bf16_t*)w, (const bf16_t*)bias, res, (typename OutType<bf16_t, E>::type*)y, M,   \
        N, K, tiles_m, tiles_n, pt ? *pt : PlanTail{});                                                           \
  } while (0)
  if (pt) {
    if (epi != EPI_RESIDUAL) return hipErrorInvalidValue;
    OTAS_MFMA(EPI_RESIDUAL, true);
  } else if (epi == EPI_NONE) OTAS_MFMA(EPI_NONE);
  else if (epi == EPI_GELU) OTAS_MFMA(EPI_GELU);
  else OTAS_MFMA(EPI_RESIDUAL);
#undef OTAS_MFMA
  return hipGetLastError();
}

// ------------------------------------------------------------------------------ 256x256, 8 waves
// The large-shape kernel: block tile 256 x 256, 8 waves of 128 x 64 (2 x 4 arrangement), two LDS
// stages of K step 64 (128 KB; rows of 128 B, i.e. whole cache lines per row and k-tile: streaming
// 64-byte row pieces reaches ~13 TB/s from L2 on MI355X, 128-byte pieces 15-16).  128 accumulator registers per lane let two waves share each SIMD, so one
// wave's barrier / LDS waits are covered by the other's MFMAs, while the L2 traffic per MFMA is half
// that of the 128 x 128 tiling (which is bound by L2 -> LDS bandwidth: streaming operand tiles into
// LDS tops out near 13 TB/s chip-wide on MI355X).
// After each MFMA one piece of later work is issued (a fragment read for the next k-step / next
// tile, or a load instruction of the tile after next), so that this issue overlaps the MFMA's cycles
// in the matrix pipe.  A load is in flight for one whole 64-wide tile before it is needed.
// Stage layout: 16-byte chunk c of row r sits at chunk c ^ ((r >> 1) & 7) (conflict-free for the
// linear DMA writes and for the 16-lanes-per-clock fragment reads).
// The tile height is a template parameter: BM = 64 TM rows (TM = 3, 4, 5: 192, 256, 320) by 256
// columns.  Whole rounds of one workgroup per CU are what this kernel costs, so the launcher picks
// the height whose tile count wastes the least of the last round.
template <int EPI, int TM, bool PLAN = false>
__global__ __launch_bounds__(512, 1) void gemm_mfma256w8_kernel(const bf16_t* __restrict__ A,
                                                                const bf16_t* __restrict__ W,
                                                                const bf16_t* __restrict__ bias, const float* res,
                                                                typename OutType<bf16_t, EPI>::type* Y, int64_t M,
                                                                int N, int K, int tiles_m, int tiles_n, PlanTail pt) {
  constexpr int WM = 32 * TM, BM = 2 * WM, BN = 256, BK = 64, WN = 64, TN = 2, NS = 2;
  constexpr int STAGE_A = BM * BK, STAGE_W = BN * BK;
  constexpr int NA = BM / 64;   // DMA instructions per wave for the A tile (8 rows each), 4 for W
  constexpr int NM = TM * TN, NF = TM + TN, ND = NA + 4;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* As = reinterpret_cast<bf16_t*>(smem);   // [NS][BM][64]
  bf16_t* Ws = As + NS * STAGE_A;                 // [NS][256][64]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: LDS addresses of the DMA stay scalar
  const int wm = wave >> 2, wn = wave & 3;
  int tile_m, tile_n;
  OTAS_PLAN_TAIL_OR_TILE(512)
  tile_of_block(bid, tiles_m, tiles_n, tile_m, tile_n);
  const int64_t m0 = (int64_t)tile_m * BM;
  const int n0 = tile_n * BN;

  // DMA addressing: rows of 128 B (a whole cache line of K per row and k-tile), 8 lanes per row, 8 rows
  // per instruction; wave w owns rows w*8*NA .. of the A tile and rows w*32 .. of the W tile.
  // Lane i writes LDS row base + i/8, chunk position i%8, so it fetches logical chunk
  // (i%8) ^ ((row >> 1) & 7) of that row.
  // Global addresses are a uniform base (tile origin + k, scalar registers) plus a per-lane 32-bit
  // byte offset that never changes, so issuing a load costs no vector arithmetic.
  uint32_t a_off[NA], w_off[4];
#pragma unroll
  for (int j = 0; j < NA; ++j) {
    const int row = wave * (8 * NA) + j * 8 + (lane >> 3);
    const int c = (lane & 7) ^ ((row >> 1) & 7);
    const int64_t last = M - 1 - m0;                  // rows past the end repeat the last row
    const uint32_t r = (uint32_t)(row < last ? row : last);
    a_off[j] = (r * (uint32_t)K + (uint32_t)c * 8u) * (uint32_t)sizeof(bf16_t);
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int row = wave * 32 + j * 8 + (lane >> 3);
    const int c = (lane & 7) ^ ((row >> 1) & 7);
    const int last = N - 1 - n0;
    const uint32_t r = (uint32_t)(row < last ? row : last);
    w_off[j] = (r * (uint32_t)K + (uint32_t)c * 8u) * (uint32_t)sizeof(bf16_t);
  }
  const char* a_base = reinterpret_cast<const char*>(A + (size_t)m0 * K);
  const char* w_base = reinterpret_cast<const char*>(W + (size_t)n0 * K);
  const int KT = K / BK;
  auto dma_one = [&](int kt, int st, int d) {   // d = 0..NA-1: A rows; NA..NA+3: W rows
    const size_t kb = (size_t)((kt < KT ? kt : KT - 1) * BK) * sizeof(bf16_t);
    if (d < NA)
      __builtin_amdgcn_global_load_lds(OTAS_GPTR(a_base + kb + a_off[d]),
                                       OTAS_LPTR(As + st * STAGE_A + (wave * (8 * NA) + d * 8) * BK), 16, 0, 0);
    else
      __builtin_amdgcn_global_load_lds(OTAS_GPTR(w_base + kb + w_off[d - NA]),
                                       OTAS_LPTR(Ws + st * STAGE_W + (wave * 32 + (d - NA) * 8) * BK), 16, 0, 0);
  };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int fr = lane & 31, fk = lane >> 5;
  const int frag_row = fr * BK, sw = (fr >> 1) & 7;
  bf16x8 af[2][TM], wf[2][TN];
  auto read_frag = [&](int st, int ks, int slot, int f) {   // f = 0..TM-1: A tiles; then the W tiles
    const int c = (((ks << 1) + fk) ^ sw) * 8;
    if (f < TM)
      af[slot][f] = *reinterpret_cast<const bf16x8*>(As + st * STAGE_A + (wm * WM + f * 32) * BK + frag_row + c);
    else
      wf[slot][f - TM] =
          *reinterpret_cast<const bf16x8*>(Ws + st * STAGE_W + (wn * WN + (f - TM) * 32) * BK + frag_row + c);
  };
  auto mfma_one = [&](int slot, int t) {
    const int i = t / TN, j = t % TN;
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[slot][j], af[slot][i], acc[i][j], 0, 0, 0);
  };
  // one k-step: NM MFMAs, each of the first NF followed by one fragment read of the next k-step
  auto kstep = [&](int slot, int st_next, int ks_next) {
#pragma unroll
    for (int t = 0; t < NM; ++t) {
      mfma_one(slot, t);
      if (t < NF) read_frag(st_next, ks_next, slot ^ 1, t);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Two stages.  Per tile t (stage t & 1): k-steps 0..2 (the fragments of k-step 3 are read
  // during k-step 2), then wait for this wave's loads of tile t+1, barrier -- after it nobody reads
  // stage t & 1 any more and tile t+1 is visible --, then k-step 3 while the loads of tile t+2 are
  // issued into stage t & 1 and the first fragments of tile t+1 are read.
#pragma unroll
  for (int d = 0; d < ND; ++d) dma_one(0, 0, d);
#pragma unroll
  for (int d = 0; d < ND; ++d) dma_one(1, 1, d);
  OTAS_VMCNT(ND);    // tile 0 landed (this wave's part)
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
#pragma unroll
  for (int f = 0; f < NF; ++f) read_frag(0, 0, 0, f);

  for (int kt = 0; kt < KT; ++kt) {
    const int st = kt & 1;
    kstep(0, st, 1);
    kstep(1, st, 2);
    kstep(0, st, 3);
    // tile kt+1 landed, and the fragments of k-step 3 (read from stage st above, used below) are in
    // registers: after the barrier other waves start overwriting stage st
    OTAS_WAIT_LOADS_AND_LDS();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    // k-step 3: fragments of (tile kt+1, k-step 0) and the ND load instructions of tile kt+2,
    // spread over the MFMAs
#pragma unroll
    for (int t = 0; t < NM; ++t) {
      mfma_one(1, t);
      if (t < NF) read_frag(st ^ 1, 0, 0, t);
#pragma unroll
      for (int d = t * ND / NM; d < (t + 1) * ND / NM; ++d) dma_one(kt + 2, st, d);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  OTAS_VMCNT(0);
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  if constexpr (EPI == EPI_NONE || EPI == EPI_GELU)
    mfma_epilogue_bf16<EPI, TM, TN>(acc, reinterpret_cast<bf16_t*>(smem) + wave * 32 * (WN + 8), bias, Y, M, N,
                                    m0 + wm * WM, n0 + wn * WN, lane);
  else
    mfma_epilogue<EPI, TM, TN>(acc, reinterpret_cast<float*>(smem) + wave * 32 * (WN + 4), bias, res, Y, M, N,
                               m0 + wm * WM, n0 + wn * WN, lane);
}

template <int TM>
static hipError_t linear_mfma256w8(const void* x, const void* w, const void* bias, const float* res, void* y,
                                   int64_t M, int N, int K, int epi, hipStream_t s, const PlanTail* pt = nullptr) {
  constexpr int BM = 64 * TM;
  const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (N + 255) / 256;
  const size_t lds = (size_t)2 * (BM + 256) * 64 * sizeof(bf16_t);
  dim3 grid((unsigned)(tiles_m * tiles_n + (pt ? pt->B : 0))), block(512);
#define OTAS_MFMA(E, ...)                                                                                         \
  do {                                                                                                            \
    auto kern = gemm_mfma256w8_kernel<E, TM, ##__VA_ARGS__>;                                                      \
    hipError_t e = set_max_dynamic_lds((const void*)kern, (int)lds);                                              \
    if (e != hipSuccess) return e;                                                                                \
    kern<<<grid, block, lds, s>>>((const bf16_t*)x, (const bf16_t*)w, (const bf16_t*)bias, res,                   \
                                  (typename OutType<bf16_t, E>::type*)y, M, N, K, tiles_m, tiles_n,               \
                                  pt ? *pt : PlanTail{});                                                         \
  } while (0)
  if (pt) {
    if (epi != EPI_RESIDUAL) return hipErrorInvalidValue;
    OTAS_MFMA(EPI_RESIDUAL, true);
  } else if (epi == EPI_NONE) OTAS_MFMA(EPI_NONE);
  else if (epi == EPI_GELU) OTAS_MFMA(EPI_GELU);
  else OTAS_MFMA(EPI_RESIDUAL);
#undef OTAS_MFMA
  return hipGetLastError();
}

// ------------------------------------------------------------------------------ 128x128, K step 64
// Block tile 128 x 128, 4 waves of 64 x 64, two LDS stages of K step 64 (rows of 128 B = whole cache
// lines, 64 KB in all, two workgroups per CU).  Same per-tile protocol as gemm_mfma256w8_kernel:
// k-steps 0..2, wait for the next tile + barrier, k-step 3 while the loads of the tile after next
// are issued into the stage just freed.
template <int EPI, bool PLAN = false>
__global__ __launch_bounds__(256, 2) void gemm_mfma128k64_kernel(const bf16_t* __restrict__ A,
                                                                 const bf16_t* __restrict__ W,
                                                                 const bf16_t* __restrict__ bias, const float* res,
                                                                 typename OutType<bf16_t, EPI>::type* Y, int64_t M,
                                                                 int N, int K, int k_len, int tiles_m, int tiles_n,
                                                                 PlanTail pt) {
  constexpr int BM = 128, BN = 128, BK = 64, WM = 64, WN = 64, TM = 2, TN = 2;
  constexpr int STAGE = BM * BK;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* As = reinterpret_cast<bf16_t*>(smem);   // [2][128][64]
  bf16_t* Ws = As + 2 * STAGE;                    // [2][128][64]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: LDS addresses of the DMA stay scalar
  const int wm = wave >> 1, wn = wave & 1;
  int tile_m, tile_n;
  OTAS_PLAN_TAIL_OR_TILE(256)
  tile_of_block(bid, tiles_m, tiles_n, tile_m, tile_n);
  const int64_t m0 = (int64_t)tile_m * BM;
  const int n0 = tile_n * BN;

  // wave w owns rows w*32 .. w*32+31 of each operand tile, 8 rows (of 128 B) per instruction.
  // Global addresses: uniform base (tile origin + k) plus a constant per-lane 32-bit byte offset.
  uint32_t a_off[4], w_off[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int row = wave * 32 + j * 8 + (lane >> 3);
    const int c = (lane & 7) ^ ((row >> 1) & 7);
    const int64_t a_last = M - 1 - m0;                // rows past the end repeat the last row
    const int w_last = N - 1 - n0;
    const uint32_t ra = (uint32_t)(row < a_last ? row : a_last), rw = (uint32_t)(row < w_last ? row : w_last);
    a_off[j] = (ra * (uint32_t)K + (uint32_t)c * 8u) * (uint32_t)sizeof(bf16_t);
    w_off[j] = (rw * (uint32_t)K + (uint32_t)c * 8u) * (uint32_t)sizeof(bf16_t);
  }
  // split-K launches: workgroup row blockIdx.y contracts over k_len columns from blockIdx.y * k_len and writes the
  // float partial result [M, N] number blockIdx.y
  const char* a_base = reinterpret_cast<const char*>(A + (size_t)m0 * K + (size_t)blockIdx.y * k_len);
  const char* w_base = reinterpret_cast<const char*>(W + (size_t)n0 * K + (size_t)blockIdx.y * k_len);
  if (EPI == EPI_PARTIAL) Y += (size_t)blockIdx.y * M * N;
  const int KT = k_len / BK;
  auto dma_one = [&](int kt, int st, int d) {   // d = 0..7
    const size_t kb = (size_t)((kt < KT ? kt : KT - 1) * BK) * sizeof(bf16_t);
    const int j = d >> 1;
    if ((d & 1) == 0)
      __builtin_amdgcn_global_load_lds(OTAS_GPTR(a_base + kb + a_off[j]),
                                       OTAS_LPTR(As + st * STAGE + (wave * 32 + j * 8) * BK), 16, 0, 0);
    else
      __builtin_amdgcn_global_load_lds(OTAS_GPTR(w_base + kb + w_off[j]),
                                       OTAS_LPTR(Ws + st * STAGE + (wave * 32 + j * 8) * BK), 16, 0, 0);
  };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int fr = lane & 31, fk = lane >> 5;
  const int frag_row = fr * BK, sw = (fr >> 1) & 7;
  bf16x8 af[2][TM], wf[2][TN];
  auto read_frag = [&](int st, int ks, int slot, int f) {   // f = 0,1: A tiles; 2,3: W tiles
    const int c = (((ks << 1) + fk) ^ sw) * 8;
    if (f < TM)
      af[slot][f] = *reinterpret_cast<const bf16x8*>(As + st * STAGE + (wm * WM + f * 32) * BK + frag_row + c);
    else
      wf[slot][f - TM] =
          *reinterpret_cast<const bf16x8*>(Ws + st * STAGE + (wn * WN + (f - TM) * 32) * BK + frag_row + c);
  };
  auto mfma_one = [&](int slot, int t) {
    const int i = t / TN, j = t % TN;
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[slot][j], af[slot][i], acc[i][j], 0, 0, 0);
  };
  auto kstep = [&](int slot, int st_next, int ks_next) {   // 4 MFMAs, the next k-step's 4 fragments in between
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      mfma_one(slot, t);
      read_frag(st_next, ks_next, slot ^ 1, t);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

#pragma unroll
  for (int d = 0; d < 8; ++d) dma_one(0, 0, d);
#pragma unroll
  for (int d = 0; d < 8; ++d) dma_one(1, 1, d);
  OTAS_VMCNT(8);
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
#pragma unroll
  for (int f = 0; f < TM + TN; ++f) read_frag(0, 0, 0, f);

  for (int kt = 0; kt < KT; ++kt) {
    const int st = kt & 1;
    kstep(0, st, 1);
    kstep(1, st, 2);
    kstep(0, st, 3);
    // tile kt+1 landed, and the fragments of k-step 3 (read from stage st above, used below) are in
    // registers: after the barrier other waves start overwriting stage st
    OTAS_WAIT_LOADS_AND_LDS();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int t = 0; t < 4; ++t) {   // k-step 3: first fragments of tile kt+1, loads of tile kt+2
      mfma_one(1, t);
      read_frag(st ^ 1, 0, 0, t);
      dma_one(kt + 2, st, 2 * t);
      dma_one(kt + 2, st, 2 * t + 1);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  OTAS_VMCNT(0);
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  if constexpr (EPI == EPI_NONE || EPI == EPI_GELU)
    mfma_epilogue_bf16<EPI, TM, TN>(acc, reinterpret_cast<bf16_t*>(smem) + wave * 32 * (WN + 8), bias, Y, M, N,
                                    m0 + wm * WM, n0 + wn * WN, lane);
  else
    mfma_epilogue<EPI, TM, TN>(acc, reinterpret_cast<float*>(smem) + wave * 32 * (WN + 4), bias, res, Y, M, N,
                               m0 + wm * WM, n0 + wn * WN, lane);
}

static hipError_t linear_mfma128k64(const void* x, const void* w, const void* bias, const float* res, void* y,
                                    int64_t M, int N, int K, int epi, hipStream_t s, int splits = 1,
                                    const PlanTail* pt = nullptr) {
  const int tiles_m = (int)((M + 127) / 128), tiles_n = (N + 127) / 128;
  const size_t lds = (size_t)2 * 2 * 128 * 64 * sizeof(bf16_t);
  dim3 grid((unsigned)(tiles_m * tiles_n + (pt ? pt->B : 0)), (unsigned)splits), block(256);
  const int k_len = K / splits;
#define OTAS_MFMA(E, ...)                                                                                         \
  do {                                                                                                            \
    auto kern = gemm_mfma128k64_kernel<E, ##__VA_ARGS__>;                                                         \
    hipError_t e = set_max_dynamic_lds((const void*)kern, (int)lds);                                              \
    if (e != hipSuccess) return e;                                                                                \
    kern<<<grid, block, lds, s>>>((const bf16_t*)x, (const bf16_t*)w, (const bf16_t*)bias, res,                   \
                                  (typename OutType<bf16_t, E>::type*)y, M, N, K, k_len, tiles_m, tiles_n,        \
                                  pt ? *pt : PlanTail{});                                                         \
  } while (0)
  if (pt) {
    if (epi != EPI_RESIDUAL || splits != 1) return hipErrorInvalidValue;
    OTAS_MFMA(EPI_RESIDUAL, true);
  } else if (epi == EPI_NONE) OTAS_MFMA(EPI_NONE);
  else if (epi == EPI_GELU) OTAS_MFMA(EPI_GELU);
  else if (epi == EPI_PARTIAL) OTAS_MFMA(EPI_PARTIAL);
  else OTAS_MFMA(EPI_RESIDUAL);
#undef OTAS_MFMA
  return hipGetLastError();
}

// Runs one named kernel (gemm_kernel_id in kernels.h); hipErrorInvalidValue if it does not take the shape.
static hipError_t linear_mfma_kernel(int kernel, const void* x, const void* w, const void* bias, const float* res,
                                     void* y, int64_t M, int N, int K, int epi, hipStream_t s,
                                     const PlanTail* pt = nullptr) {
  const bool k32 = K % 32 == 0 && K >= 64, k64 = K % 64 == 0 && K >= 128;
  switch (kernel) {
    case GK_128_K32: return k32 ? linear_mfma_k32<3, 2>(x, w, bias, res, y, M, N, K, epi, s, 1, pt) : hipErrorInvalidValue;
    case GK_128_K64: return k64 ? linear_mfma128k64(x, w, bias, res, y, M, N, K, epi, s, 1, pt) : hipErrorInvalidValue;
    case GK_192X256: return k64 ? linear_mfma256w8<3>(x, w, bias, res, y, M, N, K, epi, s, pt) : hipErrorInvalidValue;
    case GK_256X256: return k64 ? linear_mfma256w8<4>(x, w, bias, res, y, M, N, K, epi, s, pt) : hipErrorInvalidValue;
    case GK_320X256: return k64 ? linear_mfma256w8<5>(x, w, bias, res, y, M, N, K, epi, s, pt) : hipErrorInvalidValue;
    case GK_64X64: return k32 ? linear_mfma64(x, w, bias, res, y, M, N, K, epi, s, pt) : hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
  }
}

// Kernel choice by a cost model fitted to per-launch times measured on MI355X inside the encoder
// (ViT-B shapes, all three epilogues, every kernel forced in turn).  A kernel with tile bm x bn and S
// workgroup slots on the chip (256 CUs x workgroups per CU) takes
//     (alpha[epilogue] + beta K) * G(tiles),   G = full rounds + p + (1 - p) * (last round's fill),
// i.e. whole rounds of S tiles, a partly filled last round costing p of a round plus its share.
// The choice depends on the shape only, so a shape always runs the same kernel.
static double rounds_cost(double tiles, int slots, double p) {
  const double full = std::floor(tiles / slots), frac = tiles / slots - full;
  return full + (frac > 0 ? p + (1.0 - p) * frac : 0.0);
}

static int pick_mfma_kernel(int64_t M, int N, int K, int epi, double* cost_us = nullptr) {
  if (cost_us) *cost_us = 0.0;
  // So few outputs that even 64 x 64 tiles do not fill the chip twice: the small-tile kernel (measured on MI355X
  // at K = 768: 197 x 2304 8.3 -> 5.9 us, 788 x 768 9.6 -> 6.4, 2368 x 768 12.1 -> 9.8; from ~470 tiles on it loses,
  // 788 x 3072 11.1 -> 12.9, 3392 x 768 13.2 -> 14.6: it loads twice the operand bytes per FLOP)
  if (((M + 63) / 64) * ((N + 63) / 64) <= 450 && !cost_us) return GK_64X64;
  if (K % 64 != 0 || K < 128) return GK_128_K32;
  struct Cand { int id, bm, bn, slots; double alpha[3], beta, p; };
  static const Cand cands[] = {
      {GK_128_K32, 128, 128, 768, {4.06, 7.04, 13.0}, 0.0278, 0.27},
      {GK_128_K64, 128, 128, 512, {3.17, 6.37, 8.75}, 0.0161, 0.58},
      {GK_192X256, 192, 256, 256, {4.36, 10.8, 11.9}, 0.0215, 0.72},
      {GK_256X256, 256, 256, 256, {5.85, 14.9, 12.7}, 0.0252, 0.72},
      {GK_320X256, 320, 256, 256, {8.34, 19.2, 14.7}, 0.0284, 0.74},
  };
  double best = 1e30;
  int kernel = GK_128_K32;
  for (const Cand& c : cands) {
    const double tiles = (double)((M + c.bm - 1) / c.bm) * ((N + c.bn - 1) / c.bn);
    const double cost =
        (c.alpha[epi == EPI_RESIDUAL ? 2 : epi == EPI_GELU ? 1 : 0] + c.beta * K) * rounds_cost(tiles, c.slots, c.p);
    if (cost < best) { best = cost; kernel = c.id; }
  }
  if (cost_us) *cost_us = best;
  return kernel;
}

// Split-K for few-tile, long-K products (the MLP's second linear once merging has shrunk the
// batch): with M * N / 128^2 tiles below the 512 workgroups the chip holds, one workgroup per
// tile walks the whole K alone and the launch is bound by that serial chain.  S workgroups per tile
// each contract over K / S and write a float partial result; a second kernel adds the partial
// results in split order (a fixed order: results are reproducible), the bias and the residual, and
// applies the LayerNorm that follows -- so the split costs S + 1 more float passes over the
// output than the one-kernel form followed by its LayerNorm.  S minimises the same cost model as
// above (partial-output form of the 128 x 128 K-step-64 kernel, fitted to launches of 704 ... 7488
// rows at N = 768, K = 3072 with S = 2 ... 12, 9 % rms) plus those passes at the rate the reduce
// kernel reaches inside the encoder.  S never exceeds max_split.
int splitk_factor(int dtype, int64_t M, int N, int K, int max_split) {
  if (dtype == 0 || K < 2048 || K % 64 != 0 || N % 8 != 0 || M <= 0) return 1;
  const double pass_us = (double)M * N * 4.0 / 6.0e6;   // one float pass over the output at 6 TB/s
  double unsplit;
  pick_mfma_kernel(M, N, K, EPI_RESIDUAL, &unsplit);
  double best = unsplit + 1.5 * pass_us;                // + the LayerNorm pass: float in, 16-bit out
  int S = 1;
  const double tiles = (double)((M + 127) / 128) * ((N + 127) / 128);
  static const int cand[] = {2, 3, 4, 6, 8};
  for (int c : cand) {
    if (c > max_split || K % (c * 64) != 0 || K / c < 128) continue;
    const double cost = (6.5 + 0.0153 * (K / c)) * rounds_cost(tiles * c, 512, 0.556) + (c + 2.5) * pass_us;
    if (cost < best) { best = cost; S = c; }
  }
  return S;
}

hipError_t launch_linear_splitk(const void* x, const void* w, float* part, int64_t M, int N, int K, int S,
                                hipStream_t s) {
  if (M <= 0) return hipSuccess;
  if (S < 1 || K % (S * 32) != 0 || K / S < 64 || N % 8 != 0) return hipErrorInvalidValue;
  if (K % (S * 64) == 0 && K / S >= 128) return linear_mfma128k64(x, w, nullptr, nullptr, part, M, N, K, EPI_PARTIAL, s, S);
  return linear_mfma_k32<3, 2>(x, w, nullptr, nullptr, part, M, N, K, EPI_PARTIAL, s, S);
}

hipError_t launch_linear(int dtype, const void* x, const void* w, const void* bias, const float* res, void* y,
                         int64_t M, int N, int K, int epi, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  if (dtype == 0) return linear_valu<float>(x, w, bias, res, y, M, N, K, epi, s);
  if (K % 32 == 0 && K >= 64 && N % 8 == 0)
    return linear_mfma_kernel(pick_mfma_kernel(M, N, K, epi), x, w, bias, res, y, M, N, K, epi, s);
  return linear_valu<bf16_t>(x, w, bias, res, y, M, N, K, epi, s);
}

// Whether the projection's launch has workgroup slots to spare for B list workgroups: they take a slot each (a
// launch's dynamic LDS is the same for all its workgroups), so beside a launch that fills its last round they would
// cost a round of their own (measured: + 5 us on such launches, what the selection-only plan saves beside attention).
bool linear_plan_tail_fits(int64_t M, int N, int K, int B) {
  if (M <= 0 || B <= 0 || !(K % 32 == 0 && K >= 64 && N % 8 == 0)) return false;
  int bm = 128, bn = 128, slots = 768;
  switch (pick_mfma_kernel(M, N, K, EPI_RESIDUAL)) {
    case GK_128_K64: slots = 512; break;
    case GK_192X256: bm = 192; bn = 256; slots = 256; break;
    case GK_256X256: bm = 256; bn = 256; slots = 256; break;
    case GK_320X256: bm = 320; bn = 256; slots = 256; break;
    case GK_64X64: bm = 64; bn = 64; slots = 1024; break;
    default: break;
  }
  const int64_t tiles = ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
  return tiles % slots + B <= slots && tiles % slots != 0;
}

hipError_t launch_linear_plan_tail(const void* x, const void* w, const void* bias, const float* res, void* y,
                                   int64_t M, int N, int K, const PlanTail& tail, int max_n, hipStream_t s) {
  if (M <= 0 || tail.B <= 0 || max_n > kPlanThreads || plan_lists_lds_bytes(max_n) > kPlanListsLdsMax ||
      !(K % 32 == 0 && K >= 64 && N % 8 == 0))
    return hipErrorInvalidValue;
  return linear_mfma_kernel(pick_mfma_kernel(M, N, K, EPI_RESIDUAL), x, w, bias, res, y, M, N, K, EPI_RESIDUAL, s, &tail);
}

int linear_kernel_choice(int dtype, int64_t M, int N, int K, int epi) {
  if (dtype == 0) return GK_FMA;
  if (K % 32 == 0 && K >= 64 && N % 8 == 0) return pick_mfma_kernel(M, N, K, epi);
  return GK_FMA;
}

hipError_t launch_linear_kernel(int kernel, int dtype, const void* x, const void* w, const void* bias,
                                const float* res, void* y, int64_t M, int N, int K, int epi, hipStream_t s) {
  if (kernel == GK_AUTO) return launch_linear(dtype, x, w, bias, res, y, M, N, K, epi, s);
  if (M <= 0) return hipSuccess;
  if (kernel == GK_FMA)
    return dtype == 0 ? linear_valu<float>(x, w, bias, res, y, M, N, K, epi, s)
                      : linear_valu<bf16_t>(x, w, bias, res, y, M, N, K, epi, s);
  if (dtype == 0 || N % 8 != 0) return hipErrorInvalidValue;
  return linear_mfma_kernel(kernel, x, w, bias, res, y, M, N, K, epi, s);
}

}  // namespace otas
#undef OTAS_PLAN_TAIL_OR_TILE
