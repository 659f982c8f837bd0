/*
 * lemix_stage.h - C ABI of the MI355X pipeline-stage library.
 *
 * One *stage* is a run of consecutive decoder blocks of a GPT- or Llama-family
 * model resident on one GPU (paper: System Model and Terminology, Table 1;
 * model families and sizes: Evaluation, Table 2).  The co-located system the
 * paper schedules issues two kinds of task against a stage (Table 1; Runtime
 * Memory-Aware Scheduling, Algorithm 2: Forward(task, s), Backward(task)):
 *   - inference tasks, forward only: a prefill, then KV-cached decode steps
 *     that extend the prefilled context (Autoregressive Generation,
 *     Algorithm 3 and the text after it);
 *   - training tasks: forward plus backward over a micro-batch.
 * The entry points below are those calls.  The paper gives no block
 * arithmetic; the textbook pre-LayerNorm GPT block and the RMSNorm + RoPE +
 * SwiGLU LLaMA block are used (see the block definitions further down).
 *
 * General conventions
 *   - Every pointer marked [dev] is device memory owned by the caller; [host]
 *     is host memory owned by the caller.  The library allocates device memory
 *     only inside ls_create (RoPE table, 16-bit operand copy of the weights)
 *     and frees it in ls_destroy.  It keeps the pointer given to
 *     ls_bind_params (borrowed, read-only).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work on it and return without synchronising, except
 *     stage_probe_interference, which measures time and therefore waits.
 *   - All tensors are dense row-major.
 *   - Errors: every call returns an ls_status; nothing throws or aborts
 *     across the ABI.  Arguments are validated on the host before any launch;
 *     ls_last_error() returns a thread-local description of the last failure.
 *   - Calls on one ls_stage from several host threads are allowed when they
 *     use different workspaces (the stage itself is read-only after
 *     ls_bind_params).
 */
#ifndef LEMIX_STAGE_H
#define LEMIX_STAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ls_stage ls_stage; /* opaque */

typedef enum {
  LS_OK = 0,
  LS_EINVAL = -1, /* bad argument (null pointer, non-positive size, shape mismatch, page overflow) */
  LS_ENOMEM = -2, /* device or host allocation failed in ls_create */
  LS_EHIP = -3,   /* a HIP runtime call or launch failed */
  LS_ESTATE = -4  /* call order violated (e.g. no parameters bound) */
} ls_status;

typedef enum { LS_BLOCK_GPT_PRELN = 0, LS_BLOCK_LLAMA = 1 } ls_block;
typedef enum { LS_F32 = 0, LS_BF16 = 1, LS_F16 = 2 } ls_dtype;
typedef enum { LS_ACT_GELU_TANH = 0, LS_ACT_GELU_ERF = 1, LS_ACT_SWIGLU = 2 } ls_act;

/*
 * Stage description.
 *   dtype      storage type of the parameter vector: LS_F32 or LS_BF16.
 *   io_dtype   element type of X, Y, dY, dX: LS_F32 or LS_BF16 (LS_F32 only
 *              when dtype is LS_F32).  The residual stream is kept in fp32
 *              inside the stage whatever this is.
 *   mma_dtype  format of the matrix-core operands, of every activation the
 *              stage stores between kernels, and of the KV pool:
 *              LS_F32 when dtype is LS_F32 (no matrix cores, plain fp32 FMA);
 *              LS_BF16 or LS_F16 when dtype is LS_BF16.  With LS_F16 the
 *              library keeps an fp16 copy of the bf16 weights (exact for
 *              |w| >= 2^-14, absolute error <= 2^-25 below); accumulation is
 *              fp32 in every mode.
 *   act        LS_ACT_GELU_* for GPT blocks, LS_ACT_SWIGLU for LLaMA blocks.
 *   head_dim   32, 64 or 128; d_model == n_heads * head_dim; d_ff % 8 == 0.
 *   max_pos    largest absolute token position + 1 (RoPE table rows).
 */
typedef struct {
  int32_t block, dtype, io_dtype, mma_dtype, act;
  int32_t n_layers, d_model, n_heads, head_dim, d_ff;
  float norm_eps, rope_theta;
  int32_t page_size; /* tokens per KV page, power of two, 8..64 */
  int32_t max_pos;
} ls_config;

/*
 * Block definitions (x is one token row of the fp32 residual stream).
 *  GPT pre-LN:  h1 = LN(x; g1,b1); [q|k|v] = h1 Wqkv^T + bqkv;
 *               o = causal softmax(q k^T / sqrt(head_dim)) v per head;
 *               x1 = x + o Wo^T + bo; h2 = LN(x1; g2,b2);
 *               y = x1 + GELU(h2 W1^T + b1) W2^T + b2.
 *  LLaMA:       h1 = RMSNorm(x; g1); [q|k|v] = h1 Wqkv^T; q,k <- RoPE(pos)
 *               (half-split pairs (i, i + head_dim/2), angle pos*theta^(-2i/head_dim));
 *               o as above; x1 = x + o Wo^T; h2 = RMSNorm(x1; g2);
 *               y = x1 + (SiLU(h2 Wg^T) * (h2 Wu^T)) Wd^T.
 *  LN uses the biased variance, eps inside the square root; RMSNorm divides
 *  by sqrt(mean(x^2) + eps).  Masked scores are excluded from the softmax.
 *
 * Parameter vector (elements of `dtype`, blocks concatenated in order; every
 * linear is [out, in] row-major):
 *  GPT  : ln1_g[d] ln1_b[d] W_qkv[3d,d] b_qkv[3d] W_o[d,d] b_o[d]
 *         ln2_g[d] ln2_b[d] W_1[F,d] b_1[F] W_2[d,F] b_2[d]
 *  LLaMA: g1[d] W_qkv[3d,d] W_o[d,d] g2[d] W_gu[2F,d] (gate rows, then up rows) W_d[d,F]
 * Parameter gradients use the same order, always fp32.
 */

ls_status ls_create(const ls_config* cfg, ls_stage** out);
void ls_destroy(ls_stage* s);

/* Copies the configuration the stage was created with. */
ls_status ls_get_config(const ls_stage* s, ls_config* out);

/* Number of parameter elements of the whole stage. */
size_t ls_param_count(const ls_stage* s);

/* Bind the parameter vector [dev].  Enqueues (on `stream`) the conversion of
 * the weights to the matrix-core operand format when that differs from
 * `dtype`; call again after the caller changes the weights. */
ls_status ls_bind_params(ls_stage* s, const void* params, void* stream);

/* Bytes of scratch a call needs for at most max_tokens rows (training: B*L;
 * prefill: total chunk tokens; decode: batch) — one workspace per concurrent call. */
size_t ls_workspace_bytes(const ls_stage* s, int max_tokens);

/* Bytes of activations stage_train_fwd keeps for stage_train_bwd. */
size_t ls_saved_bytes(const ls_stage* s, int B, int L);

/*
 * Paged KV cache, owned by the caller, one pool per stage.
 *   k_pool, v_pool [dev]  [n_layers][n_pages][n_heads][page_size][head_dim],
 *                         elements of mma_dtype (K is stored after RoPE).
 *   block_table    [dev]  [B][max_pages_per_req] int32 physical page ids;
 *                         entry j covers tokens j*page_size .. (j+1)*page_size-1.
 *   ctx_len        [dev]  [B] int32, tokens already cached per request.
 *   ctx_len_host   [host] the same values; used for argument validation and
 *                         launch sizing only.
 * A call appends the K/V rows of its new tokens at positions ctx_len[b].. and
 * does not change ctx_len: the caller advances it afterwards.  The pools need
 * no initialisation: slots beyond a request's context (the tail of its last
 * page, spare pages) may hold any bit pattern, NaN and infinity included, and
 * never reach a result.
 */
typedef struct {
  void* k_pool;
  void* v_pool;
  const int32_t* block_table;
  const int32_t* ctx_len;
  const int32_t* ctx_len_host;
  int32_t n_pages, max_pages_per_req;
} ls_kv;

/*
 * Inference forward over prompt chunks (paper: Autoregressive Generation —
 * each incoming request is a prefilling workload).  Request b contributes
 * chunk_len[b] consecutive rows of X; its rows sit at absolute positions
 * ctx_len[b] .. ctx_len[b]+chunk_len[b]-1 and attend to the request's cached
 * keys plus the causal part of the chunk.
 *   X [dev] [sum(chunk_len), d] io_dtype;  chunk_len [host] [B], B <= 32;
 *   Y [dev] same shape as X.
 * LS_EINVAL if a request would need more than max_pages_per_req pages or a
 * position >= max_pos.
 */
ls_status stage_prefill(ls_stage* s, const void* X, const int32_t* chunk_len, int B,
                        const ls_kv* kv, void* Y, void* workspace, void* stream);

/*
 * One decode step for B requests (decoding extends a prefilled context):
 * X [dev] [B, d] holds one new token per request at position ctx_len[b];
 * it attends over ctx_len[b]+1 keys.  Y [dev] [B, d].
 */
ls_status stage_decode(ls_stage* s, const void* X, int B, const ls_kv* kv, void* Y,
                       void* workspace, void* stream);

/*
 * Training forward on a micro-batch of B sequences of L tokens, each from
 * position 0 (a training task's forward is an inference forward that also
 * keeps activations).  X, Y [dev] [B, L, d] io_dtype; saved [dev]
 * ls_saved_bytes(B, L) bytes, consumed by stage_train_bwd with the same B, L.
 */
ls_status stage_train_fwd(ls_stage* s, const void* X, int B, int L, void* Y, void* saved,
                          void* workspace, void* stream);

/*
 * Training backward.  dY [dev] [B, L, d] io_dtype -> dX [dev] same shape, and
 * dParams [dev] fp32[ls_param_count], gradient summed over all B*L tokens.
 * accumulate = 0 overwrites dParams, 1 adds to it (micro-batches of one task).
 */
ls_status stage_train_bwd(ls_stage* s, const void* dY, int B, int L, const void* saved,
                          void* dX, float* dParams, int accumulate, void* workspace,
                          void* stream);

/*
 * One forward over a hybrid iteration-level mini-batch (Continuous Batching:
 * a mini-batch holds the ongoing decodes together with newly admitted prompt
 * chunks; Algorithm 3 forms it, this call executes it on the stage).  Requests
 * 0 .. n_decode-1 contribute one row each (a decode step at position
 * ctx_len[b]); requests n_decode .. n_decode+n_prefill-1 contribute
 * chunk_len[b - n_decode] rows each (positions ctx_len[b] ..), in that order:
 *   X, Y [dev] [n_decode + sum(chunk_len), d] io_dtype;  chunk_len [host];
 *   kv describes all n_decode + n_prefill requests (block_table rows and
 *   ctx_len in the same order).
 * The projections and FFN run once over all rows, so the decode rows share
 * the weight traffic of the prompt chunks; attention runs the decode kernel
 * on the first n_decode rows and the prompt-chunk kernel on the rest.  Row
 * results equal those of separate stage_decode / stage_prefill calls up to
 * rounding order.  n_prefill <= 32; errors as stage_prefill.
 */
ls_status stage_step(ls_stage* s, const void* X, int n_decode, const int32_t* chunk_len,
                     int n_prefill, const ls_kv* kv, void* Y, void* workspace, void* stream);

/*
 * Model update after training tasks (Model Update Synchronization: every
 * co-located instance applies its own local updates, and the inference tasks
 * that follow on the same stage are served from the updated weights).  The
 * paper names no optimizer; the two textbook rules are offered:
 *   LS_OPT_SGD    g' = g + wd w;  b <- momentum b + g';  w <- w - lr b
 *   LS_OPT_ADAMW  m <- beta1 m + (1 - beta1) g;  v <- beta2 v + (1 - beta2) g^2;
 *                 w <- w - lr (m / (1 - beta1^step) / (sqrt(v / (1 - beta2^step)) + eps) + wd w)
 * where g = grad_scale * dParams (e.g. one over the number of accumulated
 * micro-batches) and the decay wd applies to the weight matrices only, not to
 * normalisation gains or biases.  step counts updates from 1.
 */
typedef enum { LS_OPT_SGD = 0, LS_OPT_ADAMW = 1 } ls_opt_kind;
typedef struct {
  int32_t kind;
  float lr, beta1, beta2, eps, weight_decay, momentum, grad_scale;
  int32_t step;
} ls_optim;

/*
 * One fused bandwidth-bound pass over the stage's parameters, enqueued on
 * `stream`.  All vectors are device memory of ls_param_count(s) elements in
 * boundary order, caller-owned:
 *   params   the vector bound with ls_bind_params (cfg.dtype), rewritten as
 *            the rounded master weights; the library's operand-format copy is
 *            rewritten in the same pass, so stage_* calls enqueued afterwards
 *            on the same stream compute with the new weights;
 *   master   fp32 weights (may be `params` itself for an fp32 stage), updated;
 *   m, v     fp32 optimizer state (m = momentum buffer for SGD, v unused and
 *            may be null), updated;
 *   dParams  fp32 gradients from stage_train_bwd, read only.
 * fp32 vectors must be 16-byte aligned.  LS_EINVAL on null arguments, an
 * unknown kind, step < 1 or a `params` that is not the bound vector.
 */
ls_status stage_optimizer_step(ls_stage* s, const ls_optim* opt, void* params, float* master,
                               float* m, float* v, const float* dParams, void* stream);

/*
 * Interference probe (the co-location effect the paper measures: training
 * and inference contending for one GPU).  Runs `iters` repetitions of
 *   A: one stage_decode(dec_X, dec_B, kv, dec_Y, ws_a) on stream_a,
 *   B: one stage_train_fwd + stage_train_bwd(trn_*, ws_b) on stream_b,
 * first A alone, then B alone, then both launched together, and writes
 * average milliseconds per repetition to out_ms[6] [host]:
 *   {A alone, B alone, A together, B together, wall time together, 0}.
 * KV rows written by the decode step land at the same positions every
 * repetition (ctx_len is not advanced).  Synchronises both streams.
 */
ls_status stage_probe_interference(ls_stage* s, const void* dec_X, int dec_B, const ls_kv* kv,
                                   void* dec_Y, void* ws_a, const void* trn_X, int trn_B,
                                   int trn_L, void* trn_Y, void* trn_saved, const void* trn_dY,
                                   void* trn_dX, float* trn_dParams, void* ws_b, void* stream_a,
                                   void* stream_b, int iters, float* out_ms);

/* Thread-local text for the last non-OK status returned on this thread. */
const char* ls_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LEMIX_STAGE_H */
