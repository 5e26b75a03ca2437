// Host-side launchers of the gfx950 kernels.  Internal to the library: the public surface is the
// C ABI in include/otas.h.  dtype is an otas_dtype value; every pointer is a device pointer.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace otas {

enum Epilogue { EPI_NONE = 0, EPI_GELU = 1, EPI_RESIDUAL = 2, EPI_PARTIAL = 3 /* internal: raw float sums */ };

// Sets hipFuncAttributeMaxDynamicSharedMemorySize once per (kernel, device); thread-safe.
hipError_t set_max_dynamic_lds(const void* kernel, int bytes);

// One wave busy for `ticks` wall-clock periods (hipDeviceAttributeWallClockRate); sink: one int.
hipError_t launch_spin(int64_t ticks, int32_t* sink, hipStream_t s);
// One wave sampling the shader clock against the wall clock; ticks: device [samples]; shader clocks per sample: kClockProbeClocks.
constexpr int kClockProbeClocks = 4 * 127 * 64;
hipError_t launch_clock_probe(uint32_t* ticks, int32_t samples, hipStream_t s);
hipError_t launch_fill_i32(int32_t* p, int32_t v, int64_t n, hipStream_t s);
hipError_t launch_copy_i32(const int32_t* src, int32_t* dst, int64_t n, hipStream_t s);

// Query q takes rows d_prm_beg[q] .. + d_prm_cnt[q] - 1 of the prompt tensor.
hipError_t launch_prepend(int dtype, const void* tokens, const void* prompts, void* out,
                          const int32_t* d_tok_off, const int32_t* d_prm_beg, const int32_t* d_prm_cnt,
                          const int32_t* d_out_off, int B, int max_n_out, int D, int n_lead,
                          hipStream_t s);

// Prompting module in front of a layer l >= 1 on the float residual stream: overwrite the P prompt
// rows of every query in place (grow = false, x_new == x_old) or insert P rows at n_lead while
// copying into another buffer (grow = true).  prompts: this layer's rows, model dtype.  max_rows:
// the largest number of rows one query writes (P, or its new length).
hipError_t launch_deep_prompt(int dtype, const float* x_old, float* x_new, const void* prompts,
                              const int32_t* d_old_off, const int32_t* d_new_off, const int32_t* d_prm_off, int B,
                              int max_rows, int D, int n_lead, bool grow, hipStream_t s);

// Model ends.  patchify: images [B, C, Hi, Wi] -> patch matrix [B N, C p p] (patches row by row,
// flattened channel-major).  embed_finish: tokens [B, n_lead + N, D] = [cls | proj rows] + pos.
// task_heads: logits[q, :K_task] = W_task LN_final(x[off[q]]) + b_task; d_heads is a device array of
// {const void* w, const void* b, int K} records (16-byte stride + padding as laid out by the host).
struct HeadRef { const void* w; const void* b; int32_t K; int32_t pad; };   // 24 bytes, 8-byte aligned
hipError_t launch_patchify(int dtype, const void* img, void* out, int B, int C, int Hi, int Wi, int p, hipStream_t s);
hipError_t launch_embed_finish(int dtype, const void* proj, const void* cls, const void* pos, void* tokens, int B,
                               int N, int D, int n_lead, hipStream_t s);
hipError_t launch_task_heads(int dtype, const float* x, const int32_t* d_off, const int32_t* d_task,
                             const void* d_heads, const void* g, const void* b, int B, int D, float eps,
                             float* logits, int k_max, hipStream_t s);

// x_is_float: the input rows are float (the residual stream) even when dtype is bf16.
hipError_t launch_layer_norm(int dtype, bool x_is_float, const void* x, const void* g, const void* b,
                             void* y, int64_t T, int D, float eps, hipStream_t s);
// LayerNorm of bf16 rows that also writes the rows out as floats (x_float [T, D]).
hipError_t launch_layer_norm_widen(const void* x_bf16, const void* g, const void* b, void* y, float* x_float,
                                   int64_t T, int D, float eps, hipStream_t s);

// EPI_RESIDUAL: res and y are float (the residual stream) for every dtype; otherwise y has the
// model's dtype.
hipError_t launch_linear(int dtype, const void* x, const void* w, const void* bias,
                         const float* res, void* y, int64_t M, int N, int K, int epi,
                         hipStream_t s);

// The same with the kernel named by the caller (tests and profiling exercise every kernel at every
// shape this way): GK_AUTO = launch_linear's own choice, GK_FMA = the plain-FMA kernel (any dtype),
// the others bf16 MFMA kernels named by block tile (rows x columns) and K step.  Returns
// hipErrorInvalidValue if the kernel does not take the shape (K % 32 / K % 64, N % 8).
enum gemm_kernel_id {
  GK_AUTO = 0, GK_FMA = 1, GK_128_K32 = 2, GK_128_K64 = 3, GK_192X256 = 4, GK_256X256 = 5, GK_320X256 = 6,
  GK_64X64 = 7, GK_COUNT = 8
};
int linear_kernel_choice(int dtype, int64_t M, int N, int K, int epi);   // the id launch_linear runs for this shape
hipError_t launch_linear_kernel(int kernel, int dtype, const void* x, const void* w, const void* bias,
                                const float* res, void* y, int64_t M, int N, int K, int epi, hipStream_t s);

// Split-K form of the residual linear for bf16 models: splitk_factor picks S (1 = do not split);
// launch_linear_splitk writes S float partial products part[S][M][N] of x W^T, each over K / S;
// launch_splitk_reduce_ln then forms x_out = res + bias + sum_s part[s] (s ascending) and, when
// y != nullptr, y = LayerNorm(x_out) with gamma g, beta b in bf16 (the next block's first norm).
int splitk_factor(int dtype, int64_t M, int N, int K, int max_split = 8);
hipError_t launch_linear_splitk(const void* x, const void* w, float* part, int64_t M, int N, int K, int S,
                                hipStream_t s);
hipError_t launch_splitk_reduce_ln(const float* part, int S, const void* bias, const float* res, float* x_out,
                                   int64_t M, int D, const void* g, const void* b, void* y, float eps,
                                   hipStream_t s);

hipError_t launch_attention(int dtype, const void* qkv, const int32_t* sizes,
                            const int32_t* d_off, int B, int max_n, int D, int H, bool size_bias,
                            void* o, hipStream_t s);

// Attention and the merge plan of one layer in a single launch (bf16 models of head width 64 whose queries all
// fit the plan's LDS form; the plan's metric is the head mean of the keys in qkv).  Returns
// hipErrorInvalidValue, having launched nothing, for every other case.
// With sel_best / sel_bcol (device, one entry per packed token row) the launch runs only the plan's selection
// (every A token's best match) and leaves it there; the lists are then written by the first B workgroups of
// launch_linear_plan_tail, beside the attention output projection.  With both NULL it runs the whole plan.
bool attention_plan_takes(int dtype, int max_n, int D, int H);
hipError_t launch_attention_plan(const void* qkv, const int32_t* sizes, const int32_t* d_off, const int32_t* d_out_off,
                                 const int32_t* d_reff, const int32_t* d_troff, int B, int max_n, int D, int H,
                                 bool size_bias, int n_lead, void* o, int32_t* src_list, int32_t* row_ptr,
                                 int32_t* trace_src, int32_t* trace_dst, float* sel_best, int32_t* sel_bcol,
                                 hipStream_t s);

// What the list phases of the merge plan (merge_plan_lists) need when they run inside another kernel's launch.
struct PlanTail {
  const int32_t *in_off, *out_off, *reff, *troff;   // device: per-query offsets in / out, r_eff, trace offsets
  int32_t *src_list, *row_ptr, *trace_src, *trace_dst;
  const float* best;                                // the selection's result, one entry per packed token row
  const int32_t* bcol;
  int B;                                            // queries = leading workgroups that run the lists
};
// y = x W^T + bias + res (bf16 operands, float residual in and out) as launch_linear with EPI_RESIDUAL, and in
// the same launch the list phases of the merge plan for tail.B queries of at most max_n tokens.
// hipErrorInvalidValue, having launched nothing, when no MFMA kernel takes the shape.  linear_plan_tail_fits: whether
// the launch's last round has B workgroup slots to spare (pure host); if not, the lists are better written elsewhere.
bool linear_plan_tail_fits(int64_t M, int N, int K, int B);
hipError_t launch_linear_plan_tail(const void* x, const void* w, const void* bias, const float* res, void* y,
                                   int64_t M, int N, int K, const PlanTail& tail, int max_n, hipStream_t s);

// The metric of token i is the mean over H heads of src[i * row_stride + col_off + h * dm + c]
// (dtype = type of src), normalised to unit length inside the kernel.  The kernel keeps a query's unit
// metric rows in LDS when merge_plan_lds_bytes(max_n, dm) <= 160 KB; otherwise in `rows`, a device
// buffer of merge_plan_rows_bytes(T, dm) bytes for the T packed tokens (16-byte aligned; may be NULL
// when every query fits LDS, else the launch fails with hipErrorInvalidValue).
hipError_t launch_merge_plan(int dtype, const void* src, int64_t row_stride, int col_off, int H, int dm,
                             const int32_t* d_in_off, const int32_t* d_out_off, const int32_t* d_reff,
                             const int32_t* d_troff, int B, int max_n, int n_lead, int32_t* src_list,
                             int32_t* row_ptr, int32_t* trace_src, int32_t* trace_dst, float* rows, hipStream_t s);
size_t merge_plan_lds_bytes(int max_n, int dm);
size_t merge_plan_rows_bytes(int64_t T, int dm);

// dtype: type of x and x_out (0 = float, 1 = bf16).
hipError_t launch_merge_apply(int dtype, const void* x, const int32_t* sizes,
                              const int32_t* src_list, const int32_t* row_ptr, int64_t T_in,
                              int64_t T_out, int D, void* x_out, int32_t* sizes_out,
                              hipStream_t s);

// merge-apply on the float residual stream fused with the following LayerNorm: writes the merged
// rows x_out (float), their sizes, and y = LN(x_out) in the model's dtype (gamma, beta of that dtype).
hipError_t launch_merge_apply_ln(int dtype, const float* x, const int32_t* sizes, const int32_t* src_list,
                                 const int32_t* row_ptr, int64_t T_in, int64_t T_out, int D, float* x_out,
                                 int32_t* sizes_out, const void* g, const void* b, void* y, float eps,
                                 hipStream_t s);

}  // namespace otas
