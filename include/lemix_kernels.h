/*
 * lemix_kernels.h - kernel-level entry points of the stage library.
 *
 * These are the individual steps stage_prefill / stage_decode /
 * stage_train_fwd / stage_train_bwd are built from, exported so that each can
 * be checked against the CPU definition and timed on its own.  All pointers
 * are device memory owned by the caller unless marked [host]; `stream` is a
 * hipStream_t passed as void*; every call enqueues and returns.
 * dtype arguments take ls_dtype values (LS_F32 / LS_BF16 / LS_F16).
 */
#ifndef LEMIX_KERNELS_H
#define LEMIX_KERNELS_H

#include "lemix_stage.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * The block's linear maps and their gradients (forward Y = X W^T + b, input
 * gradient dX = dY W, weight gradient dW = dY^T X):
 *   C[M,N] = (accumulate ? C : 0) + (resid ? resid : 0) + sum_k A(m,k) B(n,k) + bias[n]
 * A(m,k) is at A[m*lda + k] when a_kmajor, else at A[k*lda + m]; likewise B(n,k).
 * op_dtype LS_BF16 / LS_F16: MFMA path, fp32 accumulation; the contiguous
 * extent of each operand, lda and ldb must be multiples of 8 elements and the
 * bases 16-byte aligned.  op_dtype LS_F32: plain FMA path, no constraints.
 * c_dtype is LS_F32 or op_dtype; resid is fp32 [M, ldr]; accumulate needs
 * c_dtype LS_F32.  bias has N elements of bias_dtype.
 */
ls_status lsk_gemm(int op_dtype, int M, int N, int K, const void* A, long lda, int a_kmajor,
                   const void* B, long ldb, int b_kmajor, void* C, long ldc, int c_dtype,
                   const void* bias, int bias_dtype, const float* resid, long ldr,
                   int accumulate, void* stream);

/* dst[i] = (dst_dtype) src[i], i < n. */
ls_status lsk_convert(const void* src, int src_dtype, void* dst, int dst_dtype, size_t n,
                      void* stream);

/*
 * Row normalisation of the fp32 residual stream x[T,d] -> h[T,d] (h_dtype).
 * kind 0: LayerNorm (x-mean)*rstd*gamma+beta, biased variance; kind 1:
 * RMSNorm x*rstd*gamma.  eps is added inside the square root.  mean (kind 0)
 * and rstd are written as fp32[T] when non-null.  gamma/beta have p_dtype.
 */
ls_status lsk_norm_fwd(int kind, const float* x, int T, int d, const void* gamma,
                       const void* beta, int p_dtype, float eps, void* h, int h_dtype,
                       float* mean, float* rstd, void* stream);

/*
 * Backward of lsk_norm_fwd fused with the residual-gradient add:
 *   dx = dres + norm_bwd(dh)   (fp32 [T,d]; dres may be null = 0)
 * and optionally a copy of dx in dx16_dtype (the next GEMM's operand).
 * dgamma (and dbeta for kind 0) = column sums over the T rows, fp32[d],
 * overwritten or accumulated.  partial: fp32 scratch of
 * lsk_norm_bwd_partial_floats(T, d) elements.
 */
size_t lsk_norm_bwd_partial_floats(int T, int d);
ls_status lsk_norm_bwd(int kind, const void* dh, int dh_dtype, const float* x,
                       const float* mean, const float* rstd, const void* gamma, int p_dtype,
                       int T, int d, const float* dres, float* dx, void* dx16, int dx16_dtype,
                       float* dgamma, float* dbeta, int accumulate, float* partial,
                       void* stream);

/*
 * Half-split rotary embedding in place on the q and k parts of qkv[T, 3d]
 * (columns [0,d) and [d,2d), heads of head_dim): pair (i, i+head_dim/2) of
 * row t is rotated by sign * pos[t] * theta^(-2i/head_dim); cos/sin come from
 * table[pos][i] = {cos, sin} (fp32 pairs, head_dim/2 per position).
 */
ls_status lsk_rope(void* qkv, int dtype, int T, int n_heads, int head_dim, const int32_t* pos,
                   const float* table, float sign, void* stream);

/* GELU forward g = GELU(u) and backward du = dg * GELU'(u); kind = ls_act. */
ls_status lsk_gelu_fwd(const void* u, void* g, int dtype, size_t n, int kind, void* stream);
ls_status lsk_gelu_bwd(const void* dg, const void* u, void* du, int dtype, size_t n, int kind,
                       void* stream);
/* SwiGLU on gu[T, 2F] (gate columns then up columns): a = SiLU(gate)*up, and
 * its backward dgu = [da*up*SiLU'(gate) | da*SiLU(gate)]. */
ls_status lsk_swiglu_fwd(const void* gu, void* a, int dtype, int T, int F, void* stream);
ls_status lsk_swiglu_bwd(const void* da, const void* gu, void* dgu, int dtype, int T, int F,
                         void* stream);

/* out[n] (+)= sum_t x[t*ld + n] (bias gradients); partial: fp32 scratch of
 * lsk_colsum_partial_floats(T, N) elements. */
size_t lsk_colsum_partial_floats(int T, int N);
ls_status lsk_colsum(const void* x, int dtype, int T, int N, long ld, float* out,
                     int accumulate, float* partial, void* stream);

/*
 * Causal attention over contiguous sequences (training): qkv[B*L, 3d] holds
 * q | k | v per row; o[B*L, d]; lse[B*L, n_heads] = log-sum-exp of the scaled
 * scores of each (row, head) (fp32, may be null).  impl 0 = plain kernel,
 * 1 = MFMA kernel (16-bit only).
 */
ls_status lsk_attn_fwd(int impl, const void* qkv, int dtype, int B, int L, int n_heads,
                       int head_dim, void* o, float* lse, void* stream);
/* Backward of the above: dqkv[B*L, 3d] from dO[B*L, d], the forward's qkv, o
 * and lse.  dvec: fp32 scratch of lsk_attn_bwd_scratch_floats(B, L, n_heads)
 * floats (rowsum(dO*O) per (row, head), then per-workgroup and global max|dO|,
 * then the log-sum-exp in base 2 per (row, head) for the head_dim-128 kernels). */
size_t lsk_attn_bwd_scratch_floats(int B, int L, int n_heads);
ls_status lsk_attn_bwd(int impl, const void* qkv, const void* o, const void* dO,
                       const float* lse, int dtype, int B, int L, int n_heads, int head_dim,
                       void* dqkv, float* dvec, void* stream);

/*
 * lsk_attn_bwd followed by the backward of the rotary embedding on the dq and
 * dk parts of dqkv (each pair rotated by minus its position's angle: the
 * rotation is orthogonal, so its transpose is the inverse rotation; RoFormer
 * section 3.4.2 as used by the LLaMA block of Model Architecture).  pos[t]
 * (device, int32[B*L]) must equal t mod L; table is the device
 * [max_pos][head_dim/2][cos, sin] fp32 table, max_pos >= L.  The matrix-core
 * kernels rotate in their stores; otherwise lsk_rope runs afterwards.
 */
ls_status lsk_attn_bwd_rope(int impl, const void* qkv, const void* o, const void* dO,
                            const float* lse, int dtype, int B, int L, int n_heads,
                            int head_dim, void* dqkv, float* dvec, const int32_t* pos,
                            const float* table, void* stream);

/*
 * Offload and reload of one request's paged K/V (Algorithm 2, memory-aware
 * execution: after waiting T_max a task's KV cache is moved to host memory and
 * the task resumes from that copy).  The packed form holds whole pages,
 * ceil(n_tokens / page_size) of them, for all layers:
 *   packed[layer][0 = K, 1 = V][j][head][slot][head_dim]
 *       = pool[layer][block_table[request][j]][head][slot][:]
 * lsk_kv_packed_bytes gives its size.  lsk_kv_offload enqueues a gather into
 * `staging` (device, that many bytes) and one copy to `host`; lsk_kv_reload
 * enqueues the copy back and a scatter into the pages that kv->block_table
 * assigns to the request at that time (they may differ from the pages it was
 * offloaded from).  `host` should be pinned memory for the copy to be
 * asynchronous; both buffers are the caller's and must stay untouched until
 * the stream has passed the call.  Bit-exact.  cfg is the stage's
 * configuration (layout of the pool).  LS_EINVAL when the request needs more
 * pages than a block-table row holds.
 * lsk_memory_available: used + need_bytes <= threshold_bytes, with used =
 * total - free device memory as the driver reports it (Algorithm 2's
 * MemoryAvailable test against M_threshold); *used_bytes (nullable) gets used.
 */
size_t lsk_kv_packed_bytes(const ls_config* cfg, int n_tokens);
ls_status lsk_kv_offload(const ls_config* cfg, const ls_kv* kv, int request, int n_tokens,
                         void* staging, void* host, void* stream);
ls_status lsk_kv_reload(const ls_config* cfg, const ls_kv* kv, int request, int n_tokens,
                        const void* host, void* staging, void* stream);
ls_status lsk_memory_available(size_t need_bytes, size_t threshold_bytes, int* available,
                               size_t* used_bytes);

/*
 * The update of one parameter tensor of n elements (see stage_optimizer_step
 * for the rules): kind 0 = SGD with momentum, 1 = AdamW; step >= 1.  grad, m,
 * v (AdamW only), master are fp32 device vectors; params is the tensor in its
 * storage type param_dtype (LS_F32, in which case it may be `master` itself,
 * or LS_BF16), rewritten as round(master); params_op (nullable) is the
 * matrix-core operand copy in op_dtype (LS_F16 / LS_BF16), rewritten as the
 * conversion of the stored parameter.  Algorithmic bytes per element: 16 read,
 * 12 written, plus 2 per 16-bit copy.
 */
ls_status lsk_optimizer(int kind, float lr, float beta1, float beta2, float eps, float weight_decay,
                        float momentum, float grad_scale, int step, size_t n, const float* grad,
                        float* m, float* v, float* master, void* params, int param_dtype,
                        void* params_op, int op_dtype, void* stream);

/*
 * The forward-layout product of a decoder block's linear maps (Model
 * Architecture): C[M, N] = X[M, K] W[N, K]^T + bias + resid, as lsk_gemm with
 * both operands k-major, plus a caller workspace `scratch` (device, fp32,
 * scratch_floats elements, may be null).  When M x N gives fewer than about
 * 200 tiles of 128 x 128 (prompt chunks of a few hundred tokens) the
 * contraction is split over up to 8 workgroups per tile; their fp32 partial
 * results go through `scratch` and are added in a fixed order, so the result
 * is deterministic.  Shapes that do not need it, or a workspace smaller than
 * 2 * M * N floats, take the lsk_gemm path.  Errors as lsk_gemm.
 */
ls_status lsk_gemm_ws(int op_dtype, int M, int N, int K, const void* X, long ldx, const void* W,
                      long ldw, void* C, long ldc, int c_dtype, const void* bias,
                      int bias_dtype, const float* resid, long ldr, float* scratch,
                      size_t scratch_floats, void* stream);

/*
 * The LLaMA block's QKV projection with its rotary embedding (Model
 * Architecture: attention sub-layer with rotary positions): qkv[T, 3d] =
 * H[T, d] Wqkv[3d, d]^T in op_dtype (LS_F16 / LS_BF16; fp32 accumulation),
 * then the pairs (i, i + head_dim/2) of every q and k head of row t rotated
 * by pos[t].  All pointers are device memory; qkv is written in op_dtype.
 * The rotation runs in the GEMM's epilogue on its fp32 accumulators when
 * head_dim == 128 and the problem fills the chip with 256x256 tiles; otherwise
 * the GEMM stores 16-bit values and lsk_rope rotates those in place (one more
 * rounding; both are within the 16-bit tolerance).  LS_EINVAL on null
 * pointers or d != n_heads * head_dim.
 */
ls_status lsk_gemm_qkv_rope(int op_dtype, int T, int d, const void* H, const void* Wqkv,
                            void* qkv, int n_heads, int head_dim, const int32_t* pos,
                            const float* table, void* stream);

/*
 * Backward through the LLaMA block's FFN-down projection and its SwiGLU
 * activation in one call (training backward of y = x1 + (SiLU(gate) * up) Wd^T):
 *   da[T, F] = dY[T, d] Wd[d, F]            (the projection's input gradient)
 *   dgate = da * up * s * (1 + gate * (1 - s)),  dup = da * gate * s,  s = sigmoid(gate)
 * pre [dev] [T, 2F] holds the saved pre-activations (gate columns, then up
 * columns), grad [dev] [T, 2F] receives (dgate | dup), both op_dtype (LS_F16 /
 * LS_BF16); da is rounded to op_dtype before the activation's derivative is
 * applied.  With enough 256 x 256 tiles the derivative runs in the product's
 * epilogue and da never leaves the chip; otherwise the product is written to
 * da_scratch [dev] [T, F] and lsk_swiglu_bwd follows - the same values either
 * way.  F % 8 == 0; LS_EINVAL on null pointers or other operand types.
 */
ls_status lsk_gemm_swiglu_bwd(int op_dtype, int T, int F, int d, const void* dY, const void* Wd,
                              const void* pre, void* grad, void* da_scratch, void* stream);

/*
 * Serving attention over the paged pool.  Row t of qkv[T, 3d] belongs to
 * request req[t] and sits at absolute position pos[t]; its K and V are first
 * written to the request's page, then its query attends to keys 0..pos[t].
 * k_pool/v_pool point at this layer's [n_pages][n_heads][page][head_dim] slab.
 */
ls_status lsk_kv_write(const void* qkv, int dtype, int T, int n_heads, int head_dim,
                       const int32_t* pos, const int32_t* req, void* k_pool, void* v_pool,
                       const int32_t* block_table, int max_pages_per_req, int page_size,
                       void* stream);
/*
 * lsk_kv_write with the rotary embedding in the same pass (serving path of the blocks of Table 2's
 * LLaMA family): when table is non-null, q and k of qkv (device, [T, 3d], modified in place) are rotated
 * by pos[t] exactly as lsk_rope does with sign +1, and the rotated k rows and the v rows go to the page
 * slots; with a null table only the page write happens.  head_dim even.  16-bit data with head_dim a
 * multiple of 8 and 8-byte-aligned buffers take a vectorised kernel.  LS_EINVAL on null arguments.
 */
ls_status lsk_rope_kv_write(void* qkv, int dtype, int T, int n_heads, int head_dim, const int32_t* pos,
                            const int32_t* req, const float* table, void* k_pool, void* v_pool,
                            const int32_t* block_table, int max_pages_per_req, int page_size, void* stream);
ls_status lsk_attn_paged(int impl, const void* qkv, int dtype, int T, int n_heads, int head_dim,
                         const int32_t* pos, const int32_t* req, const void* k_pool,
                         const void* v_pool, const int32_t* block_table, int max_pages_per_req,
                         int page_size, int max_ctx, void* o, float* scratch, void* stream);
/* impl 0: plain kernel.  impl 1 (16-bit pools): the bandwidth-bound kernel that
 * reads whole pages with 16-byte-per-lane loads and may split a long context
 * over several workgroups; `scratch` then holds the per-split partial results
 * (this many floats; null = never split). */
size_t lsk_attn_paged_scratch_floats(int T, int n_heads, int head_dim, int max_ctx, int page_size);

/*
 * lsk_attn_paged (impl 1: 16-bit pools, head_dim 64 or 128, page_size * head_dim a multiple of 512) for callers
 * that cannot allocate device memory: code under HIP graph capture, tight serving loops, harnesses that
 * forbid it.  Same arguments without `scratch`, same kernels, same result bit for bit; the per-split partial
 * results go to a static array inside the library (8 MiB per GPU, held until the process ends) and the call
 * allocates nothing, on the device or through any library.  LS_EINVAL when the launch would need more than the
 * array holds - lsk_attn_paged_scratch_floats(...) above 2 097 152 floats: batches of 2048 or more (row, head)
 * pairs whose longest context takes many 512-token chunks, e.g. 128 rows x 40 heads with 4096-token contexts;
 * every smaller launch fits - or on the argument errors of lsk_attn_paged.  Every call on one GPU shares that GPU's array: calls that overlap in time
 * on the same GPU (two streams, two threads) race on it and must be serialised by the caller.  Nothing in the
 * array needs clearing between calls: every launch writes each partial it later reads.
 */
ls_status lsk_attn_paged_noalloc(const void* qkv, int dtype, int T, int n_heads, int head_dim,
                                 const int32_t* pos, const int32_t* req, const void* k_pool,
                                 const void* v_pool, const int32_t* block_table, int max_pages_per_req,
                                 int page_size, int max_ctx, void* o, void* stream);

/*
 * Backward-pass gradient scaling.  stage_train_bwd runs the whole backward on
 * dY * 2^e so that 16-bit gradient operands stay in the fp16 normal range (the
 * matrix cores flush fp16 subnormal inputs), and multiplies every fp32 result by
 * 2^-e, which is exact.  lsk_grad_scale writes out3 = {2^e, 2^-e, max|x|} with
 * max|x| * 2^e in (8, 16].  The *_scaled variants take a device scalar that
 * multiplies the accumulator / sum / element before it is added or stored
 * (null = 1); the unscaled entry points above are these with null.
 */
ls_status lsk_grad_scale(const void* x, int dtype, size_t n, float* out3, void* stream);
ls_status lsk_gemm_scaled(int op_dtype, int M, int N, int K, const void* A, long lda, int a_kmajor,
                          const void* B, long ldb, int b_kmajor, void* C, long ldc, int c_dtype,
                          const void* bias, int bias_dtype, const float* resid, long ldr,
                          int accumulate, const float* alpha_dev, void* stream);
ls_status lsk_convert_scaled(const void* src, int src_dtype, void* dst, int dst_dtype, size_t n,
                             const float* scale_dev, void* stream);
ls_status lsk_norm_bwd_scaled(int kind, const void* dh, int dh_dtype, const float* x,
                              const float* mean, const float* rstd, const void* gamma, int p_dtype,
                              int T, int d, const float* dres, float* dx, void* dx16,
                              int dx16_dtype, float* dgamma, float* dbeta, int accumulate,
                              float* partial, const float* alpha_dev, void* stream);
ls_status lsk_colsum_scaled(const void* x, int dtype, int T, int N, long ld, float* out,
                            int accumulate, float* partial, const float* alpha_dev, void* stream);

/*
 * Decode batches (Autoregressive Generation: decoding requests extend their
 * prefilled context one token per iteration; at most 128 rows per call).  The
 * projections of such a batch stream the weights once and split the
 * contraction over workgroups; lsk_gemm_partials leaves the split results
 *   partial[s][M][N] (device, fp32), s < *splits (host, written on return),
 *   sum over s = X[M, K] W[N, K]^T,
 * and each lsk_finish_* call sums them in the order s = 0, 1, .. and applies,
 * in the same pass, the step that follows that projection in the block
 * (Model Architecture: attention and feed-forward sub-layers with residual
 * connections and normalisation).  16-bit operands; M <= 128, N >= 64 and a
 * multiple of 4, K a multiple of 64, partial_floats >= M * N (more allows more
 * splits, at most 16).  LS_EINVAL outside these limits.
 */
ls_status lsk_gemm_partials(int op_dtype, int M, int N, int K, const void* X, long ldx, const void* W,
                            long ldw, float* partial, size_t partial_floats, int* splits, void* stream);

/*
 * x_out[T, d] (fp32) = sum of partials + bias + resid, then, unless kind < 0,
 * h[T, d] (hdt) = LayerNorm (kind 0) or RMSNorm (kind 1) of x_out with gamma,
 * beta (pdt; beta may be null), eps inside the square root.  bias (pdt) and
 * resid (fp32) may be null; x_out may be resid.  d a multiple of 4, <= 8192.
 */
ls_status lsk_finish_resid_norm(const float* partial, int splits, int T, int d, const void* bias,
                                const float* resid, float* x_out, int kind, const void* gamma,
                                const void* beta, int pdt, float eps, void* h, int hdt, void* stream);

/*
 * FFN-up: out[T, F] (odt) = GELU(sum of partials[T, F] + bias) for act
 * LS_ACT_GELU_*, or SiLU(gate) * up with [gate | up] = sum of partials[T, 2F]
 * + bias for LS_ACT_SWIGLU.  bias (pdt) may be null.  F a multiple of 4.
 */
ls_status lsk_finish_act(const float* partial, int splits, int T, int F, int act, const void* bias, int pdt,
                         void* out, int odt, void* stream);

/*
 * QKV: [q | k | v][T, 3 h dh] = sum of partials + bias (pdt, may be null); when
 * table is non-null q and k are rotated by pos[t] (half-split pairs, table as
 * in lsk_rope); q, k, v are written to qkv (dt, 16-bit) and the k and v rows
 * into the page slot of request req[t], position pos[t], as lsk_kv_write does.
 */
ls_status lsk_finish_qkv(const float* partial, int splits, int T, int h, int dh, const void* bias, int pdt,
                         const int32_t* pos, const int32_t* req, const float* table, void* qkv, int dt,
                         void* k_pool, void* v_pool, const int32_t* block_table, int max_pages, int page,
                         void* stream);

/*
 * Per-kind launch timing, for measurement inside a running program: between lsk_timing_begin and
 * lsk_timing_end every kernel-level entry point of the kinds below brackets its launches with two HIP events on
 * its stream (a nested entry point counts once, under the outermost kind).  lsk_timing_end waits for the
 * events, writes the summed milliseconds and the number of bracketed entry-point calls per kind
 * ([LSK_TIMED_KINDS] each, host) and switches the recording off.  Process-wide, one recording at a time, at most
 * 65536 brackets (further ones are dropped and counted in *dropped when it is non-null).  The events add a few
 * microseconds between launches, so a program records in a pass of its own, not in the one it reports as
 * throughput.
 */
enum {
  LSK_TIMED_GEMM = 0,        /* lsk_gemm / lsk_gemm_scaled / lsk_gemm_qkv_rope / lsk_gemm_ws with 256 rows or more */
  LSK_TIMED_ATTN_FWD = 1,    /* matrix-core attention forward (training and prompt chunks) */
  LSK_TIMED_ATTN_BWD = 2,    /* matrix-core attention backward (all its kernels) */
  LSK_TIMED_DECODE_ATTN = 3, /* the paged decode-attention kernel and its merge */
  LSK_TIMED_DECODE_GEMM = 4, /* weight-streaming projections of decode batches (lsk_gemm_partials, lsk_gemm_ws below 256 rows) */
  LSK_TIMED_FINISH = 5,      /* lsk_finish_* */
  LSK_TIMED_KINDS = 6
};
ls_status lsk_timing_begin(void);
ls_status lsk_timing_end(double* ms_by_kind, int32_t* calls_by_kind, int32_t* dropped);

#ifdef __cplusplus
}
#endif
#endif
