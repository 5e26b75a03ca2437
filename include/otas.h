/*
 * otas.h -- C ABI of the token-adapted transformer encoder for AMD MI355X (gfx950).
 *
 * The operations are those of the OTAS paper (arXiv 2401.05031): a pre-norm transformer encoder
 * (Sec. II-A) with a prompting module that prepends trained prompt tokens (Sec. II-B, Sec. III-B)
 * and a merging module that, in every layer between attention and the MLP, removes the r most
 * redundant tokens by bipartite similarity matching and a weighted average (Sec. II-C,
 * Sec. III-B).  The paper's one signed number gamma per batch is split here into two
 * non-negative per-query numbers: P prompt tokens added once, r tokens removed per layer.
 *
 * General conventions
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are ordinary host memory.
 *   - Token tensors are packed row-major [T, D]: query q owns rows offsets[q] .. offsets[q+1]-1.
 *     Element type is the model's dtype (float or bf16, 2 bytes, upper half of an IEEE float)
 *     unless a parameter says "float": inside the encoder the residual stream is always float
 *     (bf16 is used for the GEMM and attention operands), and the encoder returns it as float.
 *   - The caller owns every buffer.  The library allocates device memory only in otas_create
 *     (a small plan buffer) and, if the optional benchmark probe otas_clock_probe_start is used, at its
 *     first call (256 KB of samples), and frees both in otas_destroy.
 *   - All device work is enqueued on the HIP stream given to otas_create and the calls return
 *     without waiting for it.  Host outputs (offsets_out) are complete on return, because every
 *     sequence length is a function of (n, r, layer) alone and is computed on the host.
 *   - Host arrays are read during the call and never retained.
 *   - Every argument check happens on the host before any launch: a call that fails with
 *     EINVAL / ESHAPE / ENOMEM / EUNSUPPORTED has enqueued nothing.  A HIP runtime failure in the
 *     middle of a call (EDEVICE) leaves the call's outputs undefined; the library waits for the
 *     streams it owns before returning it.  Errors are returned as otas_status, never thrown.
 *   - Calls on one context must not overlap in time from different host threads.
 */
#ifndef OTAS_H_
#define OTAS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { OTAS_F32 = 0, OTAS_BF16 = 1 } otas_dtype;

typedef enum {
  OTAS_OK = 0,
  OTAS_EINVAL = 1,       /* NULL pointer, negative count, malformed offsets               */
  OTAS_ESHAPE = 2,       /* shapes that contradict the model description                  */
  OTAS_ENOMEM = 3,       /* workspace or plan buffer too small                            */
  OTAS_EDEVICE = 4,      /* a HIP runtime call failed                                     */
  OTAS_EUNSUPPORTED = 5  /* a size outside what the kernels are built for (see limits)    */
} otas_status;

enum {
  OTAS_FLAG_SIZE_BIAS = 1u << 0, /* add ln(size_j) to the attention logits of key j.  Not part of
                                    the paper's definition of attention (Sec. II-A); off by default. */
  OTAS_FLAG_TRACE = 1u << 1      /* write every layer's merge edges to trace_src / trace_dst */
};

/* Limits of this build: D % H == 0, head width d_h in {64, 80, 96, 128} for bf16 and any
 * multiple of 4 up to 128 for f32, D % 8 == 0, F % 8 == 0, sequence length per query <= 1024,
 * n_lead in {0, 1}.  The plan kernel keeps the unit metric vector of every token of a query in LDS
 * while 4 (n (d_m + 8) + 1064) <= 163840 bytes (n <= 554 at metric width d_m = 64, 453 at 80, 293 at
 * 128); longer merging queries keep them in the workspace (same arithmetic and order, slower).  Only
 * otas_token_merge_static, which has no workspace, refuses such a batch with OTAS_EUNSUPPORTED; the
 * encoder needs F * sizeof(element) >= 4 (d_h + 8) for them (it borrows the MLP's hidden buffer). */
#define OTAS_MAX_SEQ 1024

typedef struct {
  int32_t L;        /* encoder blocks                                                     */
  int32_t D;        /* model width                                                        */
  int32_t H;        /* attention heads (Sec. II-A)                                        */
  int32_t F;        /* MLP hidden width                                                   */
  int32_t dtype;    /* otas_dtype: type of tokens, weights and all arithmetic inputs      */
  float ln_eps;     /* LayerNorm epsilon                                                  */
  int32_t n_lead;   /* leading tokens that are never merged away (1 = class token, or 0)  */
} otas_model_desc;

/* Device pointers to one block's parameters, all of the model's dtype.  Linear weights are
 * [out, in] row-major (y = x W^T + b).  w_qkv is [3D, D] with rows ordered Q | K | V and the H
 * heads contiguous inside each third (Sec. II-A per-head projections).  The pointers are kept,
 * not copied: the memory must stay valid until otas_destroy. */
typedef struct {
  const void *ln1_g, *ln1_b;   /* [D]            */
  const void *w_qkv, *b_qkv;   /* [3D, D], [3D]  */
  const void *w_proj, *b_proj; /* [D, D], [D]    */
  const void *ln2_g, *ln2_b;   /* [D]            */
  const void *w_fc1, *b_fc1;   /* [F, D], [F]    */
  const void *w_fc2, *b_fc2;   /* [D, F], [D]    */
} otas_layer_weights;

typedef struct otas_ctx otas_ctx;

/* Create a context for one model.  layers: host array of L structs holding dev pointers.
 * hip_stream: a hipStream_t (NULL = the default stream).  The device current at the time of the
 * call is the one the context works on.  Returns EINVAL/ESHAPE/EUNSUPPORTED on bad descriptions,
 * EDEVICE if the plan buffer cannot be allocated. */
otas_status otas_create(otas_ctx **ctx, const otas_model_desc *desc,
                        const otas_layer_weights *layers, void *hip_stream);
otas_status otas_destroy(otas_ctx *ctx);

/* Length schedule of one query (pure host; Sec. III-B shape laws).  n0 tokens, P prompts added
 * once, then in each of the L layers r_eff = min(r, floor((n - n_lead) / 2)) tokens removed.
 * len_out[L+1]: length entering layer 0..L-1, then the output length. */
otas_status otas_schedule(int32_t n0, int32_t P, int32_t r, int32_t n_lead, int32_t L,
                          int32_t *len_out);

/* Split factor the encoder uses for the MLP's second linear (y = x W^T, x [M, K], W [N, K]) of a
 * bf16 model: 1 = one kernel with the residual epilogue; S > 1 = S partial products over K / S
 * each, added in split order by a second kernel that also applies the next block's first
 * LayerNorm (so that block launches no LayerNorm kernel of its own).  S is one of 1, 2, 3, 4, 6, 8
 * and never above max_split; the encoder passes max_split = otas_splitk_room(ctx, T0, M), the room
 * the workspace of a single-lane call that entered with T0 token rows has for partial products of M
 * rows (two float rows per token row, up to eight for batches of at most 1024 token rows).  Pure
 * host functions; they let a caller account for which kernels a forward pass launches. */
int32_t otas_splitk_factor(const otas_ctx *ctx, int64_t M, int32_t N, int32_t K, int32_t max_split);
int32_t otas_splitk_room(const otas_ctx *ctx, int64_t T0, int64_t M);

/* Lanes.  otas_encoder_forward and otas_encoder_layers may cut the batch into up to 8 lanes,
 * contiguous query ranges with about equal token counts, and run them side by side: lane 0 on
 * the context's stream, the others on streams the context owns (default priority), forked from
 * the context's stream at the start of the call and joined into it before the call returns, so
 * the caller sees ordinary stream order.  Lane g of G ends with the first query at whose end the
 * running token count reaches floor(T0 (g + 1) / G) (every lane keeps at least one query).
 * Queries are independent (Sec. III-B: a batch is a set of queries, each with its own strategy) and
 * a lane's kernels are chosen from the lane's own row counts, so a lane's rows are, bit for bit,
 * what a call on that lane's queries alone returns (given the same room for split-K partial
 * products per token row, which the whole batch's size sets: always so for lanes of more than 4096
 * token rows); against another lane count they agree bit for bit where no launch is split over K
 * (otas_splitk_factor) and to rounding otherwise.  lanes = 0
 * (the default) lets the library choose from the batch size (today: 1); 1 runs the whole batch as
 * one sequence of launches.
 * Environment: the library reads one variable, OTAS_DEBUG (any value: name failing HIP calls on
 * stderr).  No environment variable changes which kernel runs for a shape. */
otas_status otas_set_lanes(otas_ctx *ctx, int32_t lanes);

/* Bytes of device workspace otas_encoder_forward needs for B queries with T0 packed tokens in
 * total (pure host).  Returns 0 on invalid arguments. */
size_t otas_workspace_bytes(const otas_ctx *ctx, int32_t B, int64_t T0);
/* Same for otas_token_merge: the plan arrays, plus 528 bytes per token once T > 293 (room for the unit metric
 * rows of queries too long for the plan kernel's LDS, at the widest metric). */
size_t otas_merge_workspace_bytes(int32_t B, int64_t T);

/* Prompting module (Sec. II-B, Sec. III-B): for every query, put its P_q prompt rows in front of
 * its input tokens, after the n_lead leading tokens:  [lead | prompts | remaining tokens].
 *   tokens  dev [T_in, D], tok_offsets host [B+1]
 *   prompts dev [sum P, D] (may be NULL if sum P == 0), prompt_offsets host [B+1]
 *   out     dev [T_in + sum P, D]; must not alias the inputs
 *   out_offsets host [B+1], filled on return.
 * A query shorter than n_lead tokens is EINVAL. */
otas_status otas_prompt_prepend(otas_ctx *ctx, const void *tokens, const int32_t *tok_offsets,
                                const void *prompts, const int32_t *prompt_offsets, int32_t B,
                                void *out, int32_t *out_offsets);

/* The same with the prompts taken from a prompt repository (Sec. III-B: the trained prompts of every
 * task are kept in a repository and a query takes those of its task): query q takes rows
 * prompt_first[q] .. prompt_first[q] + prompt_count[q] - 1 of pool, dev [pool_rows, D]; several queries
 * may take the same rows.  prompt_first / prompt_count host [B]; a range outside the pool is EINVAL. */
otas_status otas_prompt_prepend_pool(otas_ctx *ctx, const void *tokens, const int32_t *tok_offsets,
                                     const void *pool, int64_t pool_rows, const int32_t *prompt_first,
                                     const int32_t *prompt_count, int32_t B, void *out,
                                     int32_t *out_offsets);

/* Merging module (Sec. II-C) applied once to every query of a packed batch.
 * Tokens at even positions of a query form set A, odd positions set B.  Every A token picks the
 * B token whose metric vector has the highest cosine similarity (ties: lowest position); the
 * r_eff = min(r_q, floor((n_q - n_lead)/2)) A tokens with the highest such similarity (ties:
 * lower position first) are merged into their picks by an average weighted with the token
 * sizes; sizes add; the surviving rows keep their order.
 *   x       dev [T, D]      tokens
 *   metric  dev [T, dm]     vectors the similarity is taken on (model dtype), dm % 4 == 0, dm <= 128
 *   sizes   dev [T] int32   tokens each row stands for; NULL = all 1
 *   offsets host [B+1], r host [B]
 *   workspace dev, >= otas_merge_workspace_bytes(B, T) bytes, 256-byte aligned
 *   x_out   dev [T', D], sizes_out dev [T'] with T' = sum (n_q - r_eff_q); no aliasing of inputs
 *   offsets_out host [B+1], filled on return
 *   trace_src / trace_dst dev [sum r_eff] int32 or both NULL: per query (in batch order) the
 *     merged edges in rank order, as positions inside the query's input sequence. */
otas_status otas_token_merge(otas_ctx *ctx, const void *x, const void *metric, int32_t dm,
                             const int32_t *sizes, const int32_t *offsets, const int32_t *r,
                             int32_t B, void *workspace, size_t workspace_bytes, void *x_out,
                             int32_t *sizes_out, int32_t *offsets_out, int32_t *trace_src,
                             int32_t *trace_dst);

/* otas_token_merge for callers that cannot allocate device memory or hand over a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same arguments,
 * same kernels and bit-identical results, without the workspace: the merge lists live in a static
 * device array of the library (one copy per GPU, about 0.5 MB, held until the process ends), and the
 * call itself allocates nothing on the device or the host.
 * Limits: B <= OTAS_STATIC_MERGE_MAX_QUERIES and offsets[B] <= OTAS_STATIC_MERGE_MAX_ROWS, else
 * OTAS_ENOMEM before any launch.  All calls on one GPU share the one array: calls that overlap in time
 * on the same GPU (different contexts or streams) race on it; calls in stream order on one context
 * are safe, and nothing from an earlier call is read (every list entry a call reads it has written).
 * Launches of this entry point are not recorded by otas_timing_*. */
#define OTAS_STATIC_MERGE_MAX_ROWS 65536
#define OTAS_STATIC_MERGE_MAX_QUERIES 1024
otas_status otas_token_merge_static(otas_ctx *ctx, const void *x, const void *metric, int32_t dm,
                                    const int32_t *sizes, const int32_t *offsets, const int32_t *r,
                                    int32_t B, void *x_out, int32_t *sizes_out, int32_t *offsets_out,
                                    int32_t *trace_src, int32_t *trace_dst);

/* Token-adapted encoder forward (Sec. III-B unified model; the ServeModel.forward of Sec. IV
 * without the task heads).  Per layer and query:
 *   x += Proj(Attention(LN1(x)));  merge r_eff tokens using the cosine similarity of the
 *   head-averaged attention keys;  x += FC2(GELU(FC1(LN2(x)))).
 *   x0      dev [T0, D]  tokens with prompts already prepended (otas_prompt_prepend)
 *   offsets host [B+1], r host [B] removal count per layer for each query
 *   flags   OTAS_FLAG_*
 *   workspace dev, >= otas_workspace_bytes(ctx, B, T0) bytes, 256-byte aligned
 *   x_out   dev float [T_L, D] (the residual stream after the last block, for every dtype),
 *           sizes_out dev [T_L] int32, offsets_out host [B+1] (filled on return)
 *   trace_src / trace_dst dev int32 [sum over layers and queries of r_eff], required with
 *     OTAS_FLAG_TRACE, ignored otherwise.  Layout: layer-major, then query, then rank order;
 *     values are positions inside the query's sequence as it enters that layer's merge.
 * x_out must not alias x0 or the workspace. */
otas_status otas_encoder_forward(otas_ctx *ctx, const void *x0, const int32_t *offsets,
                                 const int32_t *r, int32_t B, uint32_t flags, void *workspace,
                                 size_t workspace_bytes, void *x_out, int32_t *sizes_out,
                                 int32_t *offsets_out, int32_t *trace_src, int32_t *trace_dst);

/* The same for a contiguous range of blocks [layer_begin, layer_end) starting from a given state:
 * x0 is the residual stream entering block layer_begin, dev float [T0, D] for every dtype (what a
 * previous stage returned in x_out), and sizes_in (dev int32 [T0], NULL = all 1) the number of
 * original tokens each row stands for.  otas_encoder_forward is
 * otas_encoder_layers(0, L, sizes_in = NULL).  The trace covers the blocks of the range only.
 * Use: running the encoder in stages, and per-layer parity checks. */
otas_status otas_encoder_layers(otas_ctx *ctx, int32_t layer_begin, int32_t layer_end,
                                const void *x0, const int32_t *sizes_in, const int32_t *offsets,
                                const int32_t *r, int32_t B, uint32_t flags, void *workspace,
                                size_t workspace_bytes, void *x_out, int32_t *sizes_out,
                                int32_t *offsets_out, int32_t *trace_src, int32_t *trace_dst);

/* Per-layer prompting (Sec. III-B: the prompting module sits in front of the normalisation of
 * EVERY layer; Sec. II-B: prompts "added per layer").  Two readings, both for batches that do not
 * merge (Sec. III-B: a model performs either prompting or reduction during inference):
 *   OTAS_PROMPT_REPLACE  before the normalisation of every layer l >= 1 the P_q prompt rows of query
 *                        q (rows n_lead .. n_lead + P_q - 1) are overwritten with layer l's prompts;
 *                        lengths stay n_q.
 *   OTAS_PROMPT_GROW     before the normalisation of every layer l >= 1 P_q new prompt rows are
 *                        inserted at row n_lead; query q enters layer l with n_q + l P_q rows.
 *   x0      dev [T0, D]  tokens with layer 0's prompts already prepended (otas_prompt_prepend)
 *   offsets host [B+1]   of x0;  prompt_offsets host [B+1]: P_q = difference, P = prompt_offsets[B]
 *   prompts dev [L, P, D] model dtype: prompts[l] holds every query's rows for layer l in batch
 *           order (prompts[0] is not read); may be NULL if P == 0
 *   workspace dev >= otas_workspace_bytes(ctx, B, T_L), T_L = T0 (replace) or T0 + (L - 1) P (grow)
 *   x_out   dev float [T_L, D], sizes_out dev [T_L] (all 1), offsets_out host [B+1]
 * A query needs n_q >= n_lead + P_q; every length must stay <= OTAS_MAX_SEQ (EUNSUPPORTED). */
enum { OTAS_PROMPT_REPLACE = 1, OTAS_PROMPT_GROW = 2 };
otas_status otas_encoder_forward_deep(otas_ctx *ctx, const void *x0, const int32_t *offsets, int32_t B,
                                      int32_t mode, const void *prompts,
                                      const int32_t *prompt_offsets, void *workspace,
                                      size_t workspace_bytes, void *x_out, int32_t *sizes_out,
                                      int32_t *offsets_out);

/* Model ends (Sec. II-A: the image is split into fixed-size patches, projected linearly and added
 * to the position embedding; Sec. III-B / IV: every task has its own head parameters and a query is
 * forwarded to the head of its task).
 * otas_patch_embed: images dev [B, C, Hi, Wi] (model dtype) -> tokens dev [B (n_lead + N), D],
 *   N = (Hi / patch)(Wi / patch) patches taken row by row, each flattened channel-major (the layout
 *   of a [D, C, patch, patch] projection weight w_patch, bias b_patch [D]); the class token cls [D]
 *   goes in front when n_lead = 1 (NULL allowed when n_lead = 0); pos [n_lead + N, D] is added to
 *   every row.  tok_offsets host [B+1] is filled.  workspace dev >=
 *   otas_patch_embed_workspace_bytes (patch matrix + projection).  Hi, Wi multiples of patch
 *   (EINVAL), C patch^2 % 8 == 0 and n_lead + N <= OTAS_MAX_SEQ (EUNSUPPORTED).
 * otas_task_heads: logits[q, k] = W_t LN_final(x[offsets[q]]) + b_t for t = task[q], k < classes_t,
 *   0 for classes_t <= k < k_max.  x dev float [T, D] (the encoder's output), offsets / task host,
 *   heads host [n_tasks] of dev pointers (w [classes, D], b [classes], model dtype), lnf_g / lnf_b
 *   dev [D], logits dev float [B, k_max]. */
typedef struct {
  const void *w;
  const void *b;
  int32_t classes;
} otas_task_head;
size_t otas_patch_embed_workspace_bytes(const otas_ctx *ctx, int32_t B, int32_t C, int32_t Hi,
                                        int32_t Wi, int32_t patch);
otas_status otas_patch_embed(otas_ctx *ctx, const void *images, int32_t B, int32_t C, int32_t Hi,
                             int32_t Wi, int32_t patch, const void *w_patch, const void *b_patch,
                             const void *cls, const void *pos, void *workspace,
                             size_t workspace_bytes, void *tokens, int32_t *tok_offsets);
otas_status otas_task_heads(otas_ctx *ctx, const float *x, const int32_t *offsets,
                            const int32_t *task, int32_t B, const otas_task_head *heads,
                            int32_t n_tasks, const void *lnf_g, const void *lnf_b, float *logits,
                            int32_t k_max);

/* Individual steps of the path, exposed for parity tests and profiling.  All pointers dev,
 * model dtype, enqueued on the context's stream.
 *   otas_layer_norm: y[T,D] = LN(x[T,D]) with biased variance and the context's eps.
 *   otas_linear:     y[T,N] = epilogue(x[T,K] W[N,K]^T + b[N]);  epilogue 0 = none, 1 = exact
 *                    GELU, 2 = add residual res[T,N]; with epilogue 2, res and y are float (the
 *                    residual stream) and res may equal y.
 *   otas_attention:  o[T,D] = concat_h softmax(Q_h K_h^T / sqrt(d_h) [+ ln size_j]) V_h from
 *                    qkv[T,3D]; sizes dev int32 [T] or NULL; offsets host [B+1]. */
otas_status otas_layer_norm(otas_ctx *ctx, const void *x, const void *g, const void *b,
                            int64_t T, void *y);
otas_status otas_linear(otas_ctx *ctx, const void *x, const void *w, const void *b,
                        const void *res, int64_t T, int32_t N, int32_t K, int32_t epilogue,
                        void *y);
otas_status otas_attention(otas_ctx *ctx, const void *qkv, const int32_t *sizes,
                           const int32_t *offsets, int32_t B, uint32_t flags, void *o);

/* otas_linear with the kernel named by the caller, so that tests and profiles can run every GEMM
 * kernel of the library at every shape (otas_linear and the encoder choose by shape alone).
 * kernel: 0 the library's own choice, 1 plain fp32-FMA tiles (any dtype), and for bf16 models the
 * MFMA kernels named by block tile (rows x columns) and K step: 2 128x128 k32, 3 128x128 k64,
 * 4 192x256 k64, 5 256x256 k64, 6 320x256 k64, 7 64x64 k32.
 * OTAS_EUNSUPPORTED if the kernel does not take the shape (k32 kernels need K % 32 == 0 and K >= 64,
 * k64 kernels K % 64 == 0 and K >= 128) or the dtype. */
#define OTAS_LINEAR_KERNELS 8
/* The kernel (numbering above, never 0) that otas_linear and the encoder run for this shape; pure host
 * function, -1 on invalid arguments.  Lets a benchmark report tiles and rounds per launch. */
int32_t otas_linear_choice(const otas_ctx *ctx, int64_t T, int32_t N, int32_t K, int32_t epilogue);
otas_status otas_linear_kernel(otas_ctx *ctx, int32_t kernel, const void *x, const void *w,
                               const void *b, const void *res, int64_t T, int32_t N, int32_t K,
                               int32_t epilogue, void *y);

/* Per-launch timing for benchmarks (callers that want the time of each kernel kind measured with
 * HIP events on the context's stream).  otas_timing_enable(ctx, 1) waits for the stream, then makes
 * every later launch of this context record an event before and after itself;
 * otas_timing_read waits for the stream, returns for each kind 0 .. otas_timing_kinds()-1 the summed
 * milliseconds and the number of launches since the last read, and clears the records.
 * Enabling also measures what an event pair adds to the launch it brackets -- the median reading of
 * pairs around a one-wave kernel that spins for 10 us / 30 us of the device's wall clock, less the
 * spin and less 1 us for the dispatch's own ramp (otas_timing_overhead_ms; 0 when the calibration
 * is not self-consistent) -- and every record is reported net of it.
 * A launch has one kind, named for its main work: where the encoder runs the merge plan (or its
 * selection phases) inside the attention launch and the plan's list-writing phases inside the
 * output projection's launch (bf16 models of head width 64), those records are "attention" and
 * "gemm_proj", and "merge_plan" counts only the plans that had a launch of their own.
 * total_ms / launches: host arrays of otas_timing_kinds() entries.  Off by default. */
otas_status otas_timing_enable(otas_ctx *ctx, int32_t on);
int32_t otas_timing_kinds(void);
const char *otas_timing_kind_name(int32_t kind);
otas_status otas_timing_read(otas_ctx *ctx, double *total_ms, int64_t *launches);
float otas_timing_overhead_ms(const otas_ctx *ctx);
/* The same records one by one, in launch order, without clearing them: kind and milliseconds of up
 * to cap launches into the host arrays; returns the number of records held (-1 on error). */
int32_t otas_timing_read_launches(otas_ctx *ctx, int32_t cap, int32_t *kinds, float *ms);

/* Shader clock under load, for benchmarks (MI355X lowers its clock under sustained matrix work, by an amount that
 * depends on the operand data; a roofline fraction against the data-sheet peak therefore needs the clock that the
 * measured kernels actually ran at).  otas_clock_probe_start enqueues, on a stream of the context's own (created at
 * first use, default priority, with a sample buffer that otas_destroy frees), one wave that `samples` times sleeps
 * 32512 shader clocks and stores how many periods of the device's constant-rate wall clock that took; it returns
 * at once, and whatever the caller launches next runs beside the probe.  A sample lasts 13.5 us at 2.4 GHz.
 * otas_clock_probe_read waits for the probe to end and writes the shader clock of each sample in MHz, in
 * order, into mhz[0 .. *n), *n = min(samples, cap); *n = 0 if no probe was started since the last read.
 * samples: 1 .. OTAS_CLOCK_PROBE_MAX_SAMPLES, else OTAS_EINVAL.  One probe at a time per context: a second start
 * waits for the first to end and discards its samples. */
#define OTAS_CLOCK_PROBE_MAX_SAMPLES 65536
otas_status otas_clock_probe_start(otas_ctx *ctx, int32_t samples);
otas_status otas_clock_probe_read(otas_ctx *ctx, float *mhz /* host [cap] */, int32_t cap, int32_t *n);

const char *otas_strerror(otas_status s);

#ifdef __cplusplus
}
#endif
#endif /* OTAS_H_ */
