// Stage-level entry points: a run of decoder blocks executed for inference
// tasks (prefill, KV-cached decode) and training tasks (forward, backward), and
// the two-stream interference probe.  This file only sequences the kernels
// (lsk_*) and lays out the workspace / saved-activation buffers.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <new>
#include <vector>

#include "common.h"

// ------------------------------------------------------------ error string
static thread_local char g_err[512] = "";
void ls_set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}
extern "C" const char* ls_last_error(void) { return g_err; }

// ------------------------------------------------------------ launch timing by kind
#include <mutex>
namespace {
struct TimingRec { int kind; hipEvent_t e0, e1; };
struct TimingState {
  std::mutex mu;
  bool on = false;
  int dropped = 0;
  std::vector<TimingRec> recs;
};
TimingState g_timing;
thread_local int g_timed_depth = 0;
thread_local int g_timed_slot = -1;
constexpr size_t kMaxTimingRecs = 65536;
}  // namespace

LsTimed::LsTimed(int kind, void* st) : armed(false), stream(st) {
  if (g_timed_depth++ > 0 || !g_timing.on) return;
  std::lock_guard<std::mutex> lock(g_timing.mu);
  if (!g_timing.on) return;
  if (g_timing.recs.size() >= kMaxTimingRecs) { ++g_timing.dropped; return; }
  TimingRec r{kind, nullptr, nullptr};
  if (hipEventCreate(&r.e0) != hipSuccess || hipEventCreate(&r.e1) != hipSuccess ||
      hipEventRecord(r.e0, (hipStream_t)st) != hipSuccess) {
    if (r.e0) (void)hipEventDestroy(r.e0);
    if (r.e1) (void)hipEventDestroy(r.e1);
    (void)hipGetLastError();
    ++g_timing.dropped;
    return;
  }
  g_timing.recs.push_back(r);
  g_timed_slot = (int)g_timing.recs.size() - 1;
  armed = true;
}
LsTimed::~LsTimed() {
  --g_timed_depth;
  if (!armed) return;
  std::lock_guard<std::mutex> lock(g_timing.mu);
  if (g_timed_slot >= 0 && g_timed_slot < (int)g_timing.recs.size())
    (void)hipEventRecord(g_timing.recs[g_timed_slot].e1, (hipStream_t)stream);
  g_timed_slot = -1;
}

extern "C" ls_status lsk_timing_begin(void) {
  std::lock_guard<std::mutex> lock(g_timing.mu);
  if (g_timing.on) {
    ls_set_error("timing_begin: a recording is already running");
    return LS_ESTATE;
  }
  g_timing.on = true;
  g_timing.dropped = 0;
  return LS_OK;
}

extern "C" ls_status lsk_timing_end(double* ms_by_kind, int32_t* calls_by_kind, int32_t* dropped) {
  LS_REQUIRE(ms_by_kind && calls_by_kind, "timing_end: null result");
  std::vector<TimingRec> recs;
  {
    std::lock_guard<std::mutex> lock(g_timing.mu);
    if (!g_timing.on) {
      ls_set_error("timing_end: no recording is running");
      return LS_ESTATE;
    }
    g_timing.on = false;
    recs.swap(g_timing.recs);
    if (dropped) *dropped = g_timing.dropped;
  }
  for (int k = 0; k < LSK_TIMED_KINDS; ++k) { ms_by_kind[k] = 0.0; calls_by_kind[k] = 0; }
  ls_status rc = LS_OK;
  for (const TimingRec& r : recs) {
    float ms = 0.f;
    if (hipEventSynchronize(r.e1) != hipSuccess || hipEventElapsedTime(&ms, r.e0, r.e1) != hipSuccess) {
      (void)hipGetLastError();
      rc = LS_EHIP;
    } else if (r.kind >= 0 && r.kind < LSK_TIMED_KINDS) {
      ms_by_kind[r.kind] += ms;
      ++calls_by_kind[r.kind];
    }
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
  }
  if (rc != LS_OK) ls_set_error("timing_end: an event of the recording could not be read");
  return rc;
}

// internal kernel-level entry points that are not part of the public kernel header
extern "C" {
ls_status lsk_attn_fwd_simple(const void*, int, int, int, int, int, void*, float*, void*);
ls_status lsk_attn_bwd_simple(const void*, const void*, const void*, const float*, int, int, int, int, int,
                              void*, float*, void*);
ls_status lsk_gemm_scaled(int, int, int, int, const void*, long, int, const void*, long, int, void*, long, int,
                          const void*, int, const float*, long, int, const float*, void*);
ls_status lsk_convert_scaled(const void*, int, void*, int, size_t, const float*, void*);
ls_status lsk_grad_scale(const void*, int, size_t, float*, void*);
ls_status lsk_norm_bwd_scaled(int, const void*, int, const float*, const float*, const float*, const void*, int,
                              int, int, const float*, float*, void*, int, float*, float*, int, float*,
                              const float*, void*);
ls_status lsk_colsum_scaled(const void*, int, int, int, long, float*, int, float*, const float*, void*);
ls_status lsk_attn_prefill_mfma(const void*, int, int, const int32_t*, int, int, const void*, const void*,
                                const int32_t*, const int32_t*, int, int, void*, void*);
ls_status lsk_gemm_qkv_rope(int, int, int, const void*, const void*, void*, int, int, const int32_t*, const float*,
                            void*);
ls_status lsk_gemm_ws(int, int, int, int, const void*, long, const void*, long, void*, long, int, const void*, int,
                      const float*, long, float*, size_t, void*);
ls_status lsk_gemm_partials(int, int, int, int, const void*, long, const void*, long, float*, size_t, int*, void*);
ls_status lsk_gemm_swiglu_bwd(int, int, int, int, const void*, const void*, const void*, void*, void*, void*);
}
bool gemm_qkv_rope_fuses(int op_dtype, int T, int d, int head_dim);
ls_status gemm_dma_splitk_partials(int, int, int, int, const void*, long, const void*, long, float*, size_t, int*,
                                   hipStream_t);
extern "C" {
ls_status lsk_finish_resid_norm(const float*, int, int, int, const void*, const float*, float*, int, const void*,
                                const void*, int, float, void*, int, void*);
ls_status lsk_finish_act(const float*, int, int, int, int, const void*, int, void*, int, void*);
ls_status lsk_finish_qkv(const float*, int, int, int, int, const void*, int, const int32_t*, const int32_t*,
                         const float*, void*, int, void*, void*, const int32_t*, int, int, void*);
ls_status lsk_optimizer(int, float, float, float, float, float, float, float, int, size_t, const float*, float*, float*,
                        float*, void*, int, void*, int, void*);
ls_status lsk_attn_bwd_rope(int, const void*, const void*, const void*, const float*, int, int, int, int, int,
                            void*, float*, const int32_t*, const float*, void*);
ls_status lsk_rope_kv_write(void*, int, int, int, int, const int32_t*, const int32_t*, const float*, void*, void*,
                            const int32_t*, int, int, void*);
}

namespace {

struct LayerOff {  // element offsets into the parameter vector
  size_t n1_g, n1_b, w_qkv, b_qkv, w_o, b_o, n2_g, n2_b, w_up, b_up, w_dn, b_dn;
};

}  // namespace

struct ls_stage {
  ls_config cfg;
  size_t n_params;
  std::vector<LayerOff> off;
  const void* params;   // caller's vector (cfg.dtype), borrowed
  void* params_op;      // weights in the operand format (owned when it differs from params)
  bool owns_op;
  float* rope_table;    // [max_pos][head_dim/2][2]
  int up_cols;          // F (GPT) or 2F (LLaMA)
};

namespace {

// bump allocator over a caller buffer, 256-byte aligned pieces
struct Bump {
  char* p;
  size_t used;
  explicit Bump(void* base) : p((char*)base), used(0) {}
  void* take(size_t bytes) {
    void* r = p ? p + used : nullptr;
    used += align_up(bytes, 256);
    return r;
  }
};

struct Chunks {  // prefill requests passed by value to the index kernel
  int n;
  int start[33];
};

__global__ void token_index_kernel(Chunks ch, const int32_t* ctx_len, int32_t* pos, int32_t* req) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= ch.start[ch.n]) return;
  int b = 0;
  while (t >= ch.start[b + 1]) ++b;
  pos[t] = ctx_len[b] + (t - ch.start[b]);
  req[t] = b;
}
// hybrid batch: n_dec single-token rows (request t), then the chunk rows of requests n_dec + b
__global__ void hybrid_index_kernel(int n_dec, Chunks ch, const int32_t* ctx_len, int32_t* pos, int32_t* req) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t < n_dec) {
    pos[t] = ctx_len[t];
    req[t] = t;
    return;
  }
  const int u = t - n_dec;
  if (u >= ch.start[ch.n]) return;
  int b = 0;
  while (u >= ch.start[b + 1]) ++b;
  pos[t] = ctx_len[n_dec + b] + (u - ch.start[b]);
  req[t] = n_dec + b;
}
__global__ void decode_index_kernel(int B, const int32_t* ctx_len, int32_t* pos, int32_t* req) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= B) return;
  pos[t] = ctx_len[t];
  req[t] = t;
}
__global__ void train_index_kernel(int T, int L, int32_t* pos) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t < T) pos[t] = t % L;
}

inline const void* pptr(const ls_stage* s, size_t off) {  // gains / biases: caller's dtype
  return (const char*)s->params + off * dtype_size(s->cfg.dtype);
}
inline const void* wptr(const ls_stage* s, size_t off) {  // weights: operand format
  return (const char*)s->params_op + off * dtype_size(s->cfg.mma_dtype);
}
inline size_t osz(const ls_stage* s) { return dtype_size(s->cfg.mma_dtype); }

ls_status check_stage(const ls_stage* s, bool need_params) {
  LS_REQUIRE(s != nullptr, "null stage");
  if (need_params && !s->params) {
    ls_set_error("no parameters bound (call ls_bind_params first)");
    return LS_ESTATE;
  }
  return LS_OK;
}

// per-layer slices of the saved-activation buffer
struct Saved {
  float *x_in, *mean1, *rstd1, *lse, *x1, *mean2, *rstd2;
  void *h1, *qkv, *o, *h2, *up, *act;
};
size_t carve_saved(const ls_stage* s, void* base, int T, std::vector<Saved>* out) {
  const ls_config& c = s->cfg;
  const size_t d = c.d_model, e = osz(s);
  Bump b(base);
  for (int l = 0; l < c.n_layers; ++l) {
    Saved v;
    v.x_in = (float*)b.take(T * d * 4);
    v.mean1 = (float*)b.take((size_t)T * 4);
    v.rstd1 = (float*)b.take((size_t)T * 4);
    v.h1 = b.take(T * d * e);
    v.qkv = b.take(T * 3 * d * e);
    v.o = b.take(T * d * e);
    v.lse = (float*)b.take((size_t)T * c.n_heads * 4);
    v.x1 = (float*)b.take(T * d * 4);
    v.mean2 = (float*)b.take((size_t)T * 4);
    v.rstd2 = (float*)b.take((size_t)T * 4);
    v.h2 = b.take(T * d * e);
    v.up = b.take((size_t)T * s->up_cols * e);
    v.act = b.take((size_t)T * c.d_ff * e);
    if (out) out->push_back(v);
  }
  return b.used;
}

// forward / serving scratch
struct FwdWs {
  int32_t *pos, *req;
  float *xa, *xb, *scratch;
  void *h, *qkv, *o, *up, *act;
};
// fp32 scratch for split decode attention and split-K decode GEMMs (both are
// only used for small row counts, where these bounds hold)
size_t serve_scratch_floats(const ls_stage* s) {
  const ls_config& c = s->cfg;
  const size_t attn = (size_t)4096 * (c.head_dim + 2);
  const size_t widest = (size_t)(3 * c.d_model > s->up_cols ? 3 * c.d_model : s->up_cols);
  const size_t gemm = (size_t)8 * 128 * widest;
  return attn > gemm ? attn : gemm;
}
size_t carve_fwd(const ls_stage* s, void* base, int T, FwdWs* w) {
  const ls_config& c = s->cfg;
  const size_t d = c.d_model, e = osz(s);
  Bump b(base);
  FwdWs v;
  v.pos = (int32_t*)b.take((size_t)T * 4);
  v.req = (int32_t*)b.take((size_t)T * 4);
  v.xa = (float*)b.take(T * d * 4);
  v.xb = (float*)b.take(T * d * 4);
  v.h = b.take(T * d * e);
  v.qkv = b.take(T * 3 * d * e);
  v.o = b.take(T * d * e);
  v.up = b.take((size_t)T * s->up_cols * e);
  v.act = b.take((size_t)T * c.d_ff * e);
  v.scratch = (float*)b.take(serve_scratch_floats(s) * 4);
  if (w) *w = v;
  return b.used;
}

// backward scratch
struct BwdWs {
  int32_t* pos;
  float *g, *g1, *dvec, *partial, *gscale;
  void *g16, *dact, *dup, *dh, *dqkv, *d_o;
};
size_t carve_bwd(const ls_stage* s, void* base, int T, BwdWs* w) {
  const ls_config& c = s->cfg;
  const size_t d = c.d_model, e = osz(s);
  Bump b(base);
  BwdWs v;
  v.pos = (int32_t*)b.take((size_t)T * 4);
  v.gscale = (float*)b.take(4 * 4);
  v.g = (float*)b.take(T * d * 4);
  v.g1 = (float*)b.take(T * d * 4);
  v.g16 = b.take(T * d * e);
  v.dact = b.take((size_t)T * c.d_ff * e);
  v.dup = b.take((size_t)T * s->up_cols * e);
  v.dh = b.take(T * d * e);
  v.dqkv = b.take(T * 3 * d * e);
  v.d_o = b.take(T * d * e);
  v.dvec = (float*)b.take(lsk_attn_bwd_scratch_floats(1, T, c.n_heads) * 4);
  size_t pf = lsk_norm_bwd_partial_floats(T, c.d_model);
  const size_t widest = (size_t)(3 * c.d_model > s->up_cols ? 3 * c.d_model : s->up_cols);
  const size_t cf = lsk_colsum_partial_floats(T, (int)widest);
  if (cf > pf) pf = cf;
  v.partial = (float*)b.take(pf * 4);
  if (w) *w = v;
  return b.used;
}

// one block's forward on the fp32 stream x -> y.  Training keeps everything in
// `sv`; serving passes its scratch and a KV descriptor.
struct FwdBufs {
  const float* x;
  float *x1, *y, *mean1, *rstd1, *mean2, *rstd2, *lse;
  void *h1, *qkv, *o, *h2, *up, *act;
  float* scratch;
};

// forward linear map (the launcher picks weight-streaming tiles for decode-sized batches, split-K for prompt
// chunks, the large-tile kernels otherwise)
ls_status linear(const ls_stage* s, int T, int N, int K, const void* X, const void* W, void* C, int c_dtype,
                 const void* bias, const float* resid, float* scratch, hipStream_t st) {
  const int mt = s->cfg.mma_dtype;
  return lsk_gemm_ws(mt, T, N, K, X, K, W, K, C, N, c_dtype, bias, s->cfg.dtype, resid, N, scratch,
                     scratch ? serve_scratch_floats(s) : 0, st);
}

// attention of a serving call over the pages of layer-local pools kp / vp (the new rows are already in them)
// the caller's scratch for the decode-attention kernel's split partials, when it is large enough for this launch
float* attn_scratch(const ls_stage* s, int rows, int max_ctx, float* scratch) {
  const ls_config& c = s->cfg;
  if (!scratch) return nullptr;
  return lsk_attn_paged_scratch_floats(rows, c.n_heads, c.head_dim, max_ctx, c.page_size) <= serve_scratch_floats(s)
             ? scratch : nullptr;
}

ls_status serve_attention(const ls_stage* s, int T, const FwdBufs& f, const int32_t* pos, const int32_t* req, int B,
                          const ls_kv* kv, void* kp, void* vp, int max_ctx, const int32_t* chunk_start, int n_decode,
                          hipStream_t st) {
  const ls_config& c = s->cfg;
  const int d = c.d_model, mt = c.mma_dtype;
  if (chunk_start && mt != LS_F32 && c.head_dim >= 64) {
    // decode rows of a hybrid batch: the bandwidth-bound kernel, one row per request
    if (n_decode > 0)
      LS_TRY(lsk_attn_paged(1, f.qkv, mt, n_decode, c.n_heads, c.head_dim, pos, req, kp, vp, kv->block_table,
                            kv->max_pages_per_req, c.page_size, max_ctx, f.o,
                            attn_scratch(s, n_decode, max_ctx, f.scratch), st));
    // prompt chunks: matrix-core attention over the pages (queries of a chunk share the K/V tiles)
    const size_t e = osz(s);
    if (B > n_decode)
      LS_TRY(lsk_attn_prefill_mfma((const char*)f.qkv + (size_t)n_decode * 3 * d * e, mt, B - n_decode, chunk_start,
                                   c.n_heads, c.head_dim, kp, vp,
                                   kv->block_table + (size_t)n_decode * kv->max_pages_per_req,
                                   kv->ctx_len + n_decode, kv->max_pages_per_req, c.page_size,
                                   (char*)f.o + (size_t)n_decode * d * e, st));
    return LS_OK;
  }
  return lsk_attn_paged(mt == LS_F32 ? 0 : 1, f.qkv, mt, T, c.n_heads, c.head_dim, pos, req, kp, vp,
                        kv->block_table, kv->max_pages_per_req, c.page_size, max_ctx, f.o,
                        attn_scratch(s, T, max_ctx, f.scratch), st);
}

// n_decode (serving with chunk_start only): the first n_decode rows are single-token decode rows of
// requests 0 .. n_decode - 1; chunk_start then describes requests n_decode .. B - 1 (rows after them)
// h1_ready (serving calls only, else null): on entry, whether the previous block's last kernel has already
// written this block's normalised input to f.h1; on return, whether this block has done so for the next one.
ls_status block_forward(const ls_stage* s, int l, int T, const FwdBufs& f, const int32_t* pos,
                        const int32_t* req, int B, int L, const ls_kv* kv, int max_ctx,
                        const int32_t* chunk_start, int n_decode, hipStream_t st, bool* h1_ready = nullptr) {
  const ls_config& c = s->cfg;
  const LayerOff& o = s->off[l];
  const int d = c.d_model, F = c.d_ff, mt = c.mma_dtype, pt = c.dtype;
  const bool gpt = c.block == LS_BLOCK_GPT_PRELN;
  const int nk = gpt ? 0 : 1;
  if (!(h1_ready && *h1_ready))
    LS_TRY(lsk_norm_fwd(nk, f.x, T, d, pptr(s, o.n1_g), gpt ? pptr(s, o.n1_b) : nullptr, pt, c.norm_eps,
                        f.h1, mt, f.mean1, f.rstd1, st));
  if (h1_ready) *h1_ready = false;
  // training: rotary embedding in the projection's epilogue where the tile shape allows, else by the rotary
  // kernel.  Serving: in the epilogue only where it is fused there; otherwise the kernel that writes K and V
  // to the pages rotates q and k in the same pass (a prompt chunk of 512 rows has too few tiles for the fused
  // epilogue, and a rotary kernel of its own before the page write cost 13 us per block).
  const bool roped = !gpt && mt != LS_F32 && (!kv || gemm_qkv_rope_fuses(mt, T, d, c.head_dim));
  if (roped) {
    LS_TRY(lsk_gemm_qkv_rope(mt, T, d, f.h1, wptr(s, o.w_qkv), f.qkv, c.n_heads, c.head_dim, pos, s->rope_table, st));
  } else {
    LS_TRY(linear(s, T, 3 * d, d, f.h1, wptr(s, o.w_qkv), f.qkv, mt, gpt ? pptr(s, o.b_qkv) : nullptr, nullptr,
                  f.scratch, st));
    if (!gpt && !kv) LS_TRY(lsk_rope(f.qkv, mt, T, c.n_heads, c.head_dim, pos, s->rope_table, 1.0f, st));
  }
  if (kv) {
    const size_t slab = (size_t)kv->n_pages * c.n_heads * c.page_size * c.head_dim * osz(s);
    void* kp = (char*)kv->k_pool + (size_t)l * slab;
    void* vp = (char*)kv->v_pool + (size_t)l * slab;
    LS_TRY(lsk_rope_kv_write(f.qkv, mt, T, c.n_heads, c.head_dim, pos, req, gpt || roped ? nullptr : s->rope_table, kp, vp,
                             kv->block_table, kv->max_pages_per_req, c.page_size, st));
    LS_TRY(serve_attention(s, T, f, pos, req, B, kv, kp, vp, max_ctx, chunk_start, n_decode, st));
  } else {
    LS_TRY(lsk_attn_fwd(mt == LS_F32 ? 0 : 1, f.qkv, mt, B, L, c.n_heads, c.head_dim, f.o, f.lse, st));
  }
  // serving calls whose output projection is split over k (prompt chunks): the kernel that sums the partial
  // products also adds the residual and normalises for the FFN, in place of a reduce kernel and a norm kernel
  int splits = 0;
  // LS_ESTATE from the split-K launcher means "this shape is not split": the plain path runs instead.
  // Any other status is a failure of the launch itself and ends the call.
  bool split_o = false;
  if (kv && mt != LS_F32 && d <= 8192 && d % 4 == 0 && f.scratch) {
    const ls_status r = gemm_dma_splitk_partials(mt, T, d, d, f.o, d, wptr(s, o.w_o), d, f.scratch,
                                                 serve_scratch_floats(s), &splits, st);
    if (r != LS_OK && r != LS_ESTATE) return r;
    split_o = r == LS_OK;
  }
  if (split_o) {
    LS_TRY(lsk_finish_resid_norm(f.scratch, splits, T, d, gpt ? pptr(s, o.b_o) : nullptr, f.x, f.x1, nk, pptr(s, o.n2_g),
                                 gpt ? pptr(s, o.n2_b) : nullptr, pt, c.norm_eps, f.h2, mt, st));
  } else {
    LS_TRY(linear(s, T, d, d, f.o, wptr(s, o.w_o), f.x1, LS_F32, gpt ? pptr(s, o.b_o) : nullptr, f.x, f.scratch, st));
    LS_TRY(lsk_norm_fwd(nk, f.x1, T, d, pptr(s, o.n2_g), gpt ? pptr(s, o.n2_b) : nullptr, pt, c.norm_eps,
                        f.h2, mt, f.mean2, f.rstd2, st));
  }
  LS_TRY(linear(s, T, s->up_cols, d, f.h2, wptr(s, o.w_up), f.up, mt, gpt ? pptr(s, o.b_up) : nullptr, nullptr,
                f.scratch, st));
  if (gpt) LS_TRY(lsk_gelu_fwd(f.up, f.act, mt, (size_t)T * F, c.act, st));
  else LS_TRY(lsk_swiglu_fwd(f.up, f.act, mt, T, F, st));
  // the same for the down projection, whose sum kernel normalises for the next block
  bool split_dn = false;
  if (h1_ready && kv && mt != LS_F32 && d <= 8192 && d % 4 == 0 && f.scratch) {
    const ls_status r = gemm_dma_splitk_partials(mt, T, d, F, f.act, F, wptr(s, o.w_dn), F, f.scratch,
                                                 serve_scratch_floats(s), &splits, st);
    if (r != LS_OK && r != LS_ESTATE) return r;
    split_dn = r == LS_OK;
  }
  if (split_dn) {
    const bool last = l + 1 == c.n_layers;
    const LayerOff& nx = s->off[last ? l : l + 1];
    LS_TRY(lsk_finish_resid_norm(f.scratch, splits, T, d, gpt ? pptr(s, o.b_dn) : nullptr, f.x1, f.y, last ? -1 : nk,
                                 pptr(s, nx.n1_g), gpt ? pptr(s, nx.n1_b) : nullptr, pt, c.norm_eps, f.h1, mt, st));
    *h1_ready = !last;
    return LS_OK;
  }
  LS_TRY(linear(s, T, d, F, f.act, wptr(s, o.w_dn), f.y, LS_F32, gpt ? pptr(s, o.b_dn) : nullptr, f.x1, f.scratch, st));
  return LS_OK;
}

// Serving calls of at most 128 rows with 16-bit operands: every projection leaves split-K partial
// products and one small kernel per projection sums them and applies what follows it in the block
// (rotary embedding + K/V page write, residual + next normalisation, activation).  h1 of block l + 1
// is produced by block l's last kernel; block 0 normalises its input itself.
bool fused_decode_ok(const ls_stage* s, int T) {
  const ls_config& c = s->cfg;
  return T <= 128 && c.mma_dtype != LS_F32 && c.d_model % 64 == 0 && c.d_ff % 64 == 0 &&
         c.d_model <= 8192;
}

ls_status block_forward_fused(const ls_stage* s, int l, int T, const FwdBufs& f, const int32_t* pos, const int32_t* req,
                              int B, const ls_kv* kv, int max_ctx, const int32_t* chunk_start, int n_decode,
                              hipStream_t st) {
  const ls_config& c = s->cfg;
  const LayerOff& o = s->off[l];
  const int d = c.d_model, F = c.d_ff, mt = c.mma_dtype, pt = c.dtype;
  const bool gpt = c.block == LS_BLOCK_GPT_PRELN, last = l + 1 == c.n_layers;
  const int nk = gpt ? 0 : 1;
  const size_t sf = serve_scratch_floats(s);
  int splits = 0;
  if (l == 0)
    LS_TRY(lsk_norm_fwd(nk, f.x, T, d, pptr(s, o.n1_g), gpt ? pptr(s, o.n1_b) : nullptr, pt, c.norm_eps, f.h1, mt,
                        nullptr, nullptr, st));
  const size_t slab = (size_t)kv->n_pages * c.n_heads * c.page_size * c.head_dim * osz(s);
  void* kp = (char*)kv->k_pool + (size_t)l * slab;
  void* vp = (char*)kv->v_pool + (size_t)l * slab;
  LS_TRY(lsk_gemm_partials(mt, T, 3 * d, d, f.h1, d, wptr(s, o.w_qkv), d, f.scratch, sf, &splits, st));
  LS_TRY(lsk_finish_qkv(f.scratch, splits, T, c.n_heads, c.head_dim, gpt ? pptr(s, o.b_qkv) : nullptr, pt, pos, req,
                        gpt ? nullptr : s->rope_table, f.qkv, mt, kp, vp, kv->block_table, kv->max_pages_per_req,
                        c.page_size, st));
  LS_TRY(serve_attention(s, T, f, pos, req, B, kv, kp, vp, max_ctx, chunk_start, n_decode, st));
  LS_TRY(lsk_gemm_partials(mt, T, d, d, f.o, d, wptr(s, o.w_o), d, f.scratch, sf, &splits, st));
  LS_TRY(lsk_finish_resid_norm(f.scratch, splits, T, d, gpt ? pptr(s, o.b_o) : nullptr, f.x, f.x1, nk, pptr(s, o.n2_g),
                               gpt ? pptr(s, o.n2_b) : nullptr, pt, c.norm_eps, f.h2, mt, st));
  LS_TRY(lsk_gemm_partials(mt, T, s->up_cols, d, f.h2, d, wptr(s, o.w_up), d, f.scratch, sf, &splits, st));
  LS_TRY(lsk_finish_act(f.scratch, splits, T, F, c.act, gpt ? pptr(s, o.b_up) : nullptr, pt, f.act, mt, st));
  LS_TRY(lsk_gemm_partials(mt, T, d, F, f.act, F, wptr(s, o.w_dn), F, f.scratch, sf, &splits, st));
  const LayerOff& nx = s->off[last ? l : l + 1];
  return lsk_finish_resid_norm(f.scratch, splits, T, d, gpt ? pptr(s, o.b_dn) : nullptr, f.x1, f.y, last ? -1 : nk,
                               pptr(s, nx.n1_g), gpt ? pptr(s, nx.n1_b) : nullptr, pt, c.norm_eps, f.h1, mt, st);
}

ls_status check_kv(const ls_stage* s, const ls_kv* kv, int B, const int32_t* new_tokens, int* max_ctx) {
  const ls_config& c = s->cfg;
  LS_REQUIRE(kv && kv->k_pool && kv->v_pool && kv->block_table && kv->ctx_len, "kv: null field");
  LS_REQUIRE(kv->n_pages > 0 && kv->max_pages_per_req > 0, "kv: non-positive page counts");
  int mc = 0;
  for (int b = 0; b < B; ++b) {
    const int nt = new_tokens ? new_tokens[b] : 1;
    LS_REQUIRE(nt > 0, "request %d has %d new tokens", b, nt);
    if (kv->ctx_len_host) {
      const long tot = (long)kv->ctx_len_host[b] + nt;
      LS_REQUIRE(kv->ctx_len_host[b] >= 0, "request %d has negative context length", b);
      LS_REQUIRE((tot + c.page_size - 1) / c.page_size <= kv->max_pages_per_req,
                 "request %d needs %ld tokens of KV but the block table holds %d pages of %d", b, tot,
                 kv->max_pages_per_req, c.page_size);
      LS_REQUIRE(c.block != LS_BLOCK_LLAMA || tot <= c.max_pos, "request %d reaches position %ld >= max_pos %d",
                 b, tot, c.max_pos);
      if (tot > mc) mc = (int)tot;
    }
  }
  if (!kv->ctx_len_host) mc = kv->max_pages_per_req * c.page_size;
  *max_ctx = mc;
  return LS_OK;
}

ls_status serve_forward(ls_stage* s, const void* X, int T, int B, const ls_kv* kv, int max_ctx, void* Y,
                        const FwdWs& w, const int32_t* chunk_start, int n_decode, hipStream_t st) {
  const ls_config& c = s->cfg;
  LS_TRY(lsk_convert(X, c.io_dtype, w.xa, LS_F32, (size_t)T * c.d_model, st));
  const bool fused = fused_decode_ok(s, T);
  bool h1_ready = false;
  for (int l = 0; l < c.n_layers; ++l) {
    FwdBufs f{w.xa, w.xb, w.xa, nullptr, nullptr, nullptr, nullptr, nullptr,
              w.h, w.qkv, w.o, w.h, w.up, w.act, w.scratch};
    if (fused) LS_TRY(block_forward_fused(s, l, T, f, w.pos, w.req, B, kv, max_ctx, chunk_start, n_decode, st));
    else LS_TRY(block_forward(s, l, T, f, w.pos, w.req, B, 0, kv, max_ctx, chunk_start, n_decode, st, &h1_ready));
  }
  return lsk_convert(w.xa, LS_F32, Y, c.io_dtype, (size_t)T * c.d_model, st);
}

}  // namespace

extern "C" {

ls_status ls_create(const ls_config* cfg, ls_stage** out) {
  LS_REQUIRE(cfg && out, "ls_create: null argument");
  const ls_config& c = *cfg;
  LS_REQUIRE(c.block == LS_BLOCK_GPT_PRELN || c.block == LS_BLOCK_LLAMA, "unknown block type %d", c.block);
  LS_REQUIRE(c.dtype == LS_F32 || c.dtype == LS_BF16, "dtype must be LS_F32 or LS_BF16");
  LS_REQUIRE(c.io_dtype == LS_F32 || c.io_dtype == LS_BF16, "io_dtype must be LS_F32 or LS_BF16");
  if (c.dtype == LS_F32)
    LS_REQUIRE(c.mma_dtype == LS_F32 && c.io_dtype == LS_F32, "an fp32 stage needs fp32 io and operands");
  else
    LS_REQUIRE(c.mma_dtype == LS_BF16 || c.mma_dtype == LS_F16, "a bf16 stage needs bf16 or fp16 operands");
  LS_REQUIRE(c.n_layers > 0 && c.d_model > 0 && c.n_heads > 0 && c.d_ff > 0, "non-positive size");
  LS_REQUIRE(c.head_dim == 32 || c.head_dim == 64 || c.head_dim == 128, "head_dim must be 32, 64 or 128");
  LS_REQUIRE(c.d_model == c.n_heads * c.head_dim, "d_model %d != n_heads %d * head_dim %d", c.d_model,
             c.n_heads, c.head_dim);
  LS_REQUIRE(c.d_ff % 8 == 0, "d_ff must be a multiple of 8");
  LS_REQUIRE(c.page_size >= 8 && c.page_size <= 64 && (c.page_size & (c.page_size - 1)) == 0,
             "page_size must be a power of two in 8..64");
  if (c.block == LS_BLOCK_GPT_PRELN)
    LS_REQUIRE(c.act == LS_ACT_GELU_TANH || c.act == LS_ACT_GELU_ERF, "GPT blocks use a GELU activation");
  else
    LS_REQUIRE(c.act == LS_ACT_SWIGLU && c.max_pos > 0 && c.rope_theta > 0, "LLaMA blocks use SwiGLU and RoPE");
  LS_REQUIRE(c.norm_eps > 0, "norm_eps must be positive");

  ls_stage* s = new (std::nothrow) ls_stage();
  if (!s) { ls_set_error("host allocation failed"); return LS_ENOMEM; }
  s->cfg = c;
  s->params = nullptr; s->params_op = nullptr; s->owns_op = false; s->rope_table = nullptr;
  const bool gpt = c.block == LS_BLOCK_GPT_PRELN;
  const size_t d = c.d_model, F = c.d_ff;
  s->up_cols = gpt ? (int)F : (int)(2 * F);
  size_t off = 0;
  for (int l = 0; l < c.n_layers; ++l) {
    LayerOff o{};
    if (gpt) {
      o.n1_g = off; off += d; o.n1_b = off; off += d;
      o.w_qkv = off; off += 3 * d * d; o.b_qkv = off; off += 3 * d;
      o.w_o = off; off += d * d; o.b_o = off; off += d;
      o.n2_g = off; off += d; o.n2_b = off; off += d;
      o.w_up = off; off += F * d; o.b_up = off; off += F;
      o.w_dn = off; off += d * F; o.b_dn = off; off += d;
    } else {
      o.n1_g = off; off += d;
      o.w_qkv = off; off += 3 * d * d;
      o.w_o = off; off += d * d;
      o.n2_g = off; off += d;
      o.w_up = off; off += 2 * F * d;
      o.w_dn = off; off += d * F;
    }
    s->off.push_back(o);
  }
  s->n_params = off;
  if (c.mma_dtype != c.dtype) {
    if (hipMalloc(&s->params_op, off * dtype_size(c.mma_dtype)) != hipSuccess) {
      ls_set_error("device allocation of %zu bytes for the operand-format weights failed",
                   off * dtype_size(c.mma_dtype));
      delete s;
      return LS_ENOMEM;
    }
    s->owns_op = true;
  }
  if (!gpt) {
    const int half = c.head_dim / 2;
    std::vector<float> tab((size_t)c.max_pos * half * 2);
    for (int p = 0; p < c.max_pos; ++p)
      for (int i = 0; i < half; ++i) {
        const double ang = (double)p * pow((double)c.rope_theta, -2.0 * i / c.head_dim);
        tab[((size_t)p * half + i) * 2] = (float)cos(ang);
        tab[((size_t)p * half + i) * 2 + 1] = (float)sin(ang);
      }
    if (hipMalloc(&s->rope_table, tab.size() * 4) != hipSuccess ||
        hipMemcpy(s->rope_table, tab.data(), tab.size() * 4, hipMemcpyHostToDevice) != hipSuccess) {
      ls_set_error("device allocation of the RoPE table failed");
      ls_destroy(s);
      return LS_ENOMEM;
    }
  }
  *out = s;
  return LS_OK;
}

void ls_destroy(ls_stage* s) {
  if (!s) return;
  if (s->owns_op && s->params_op) (void)hipFree(s->params_op);
  if (s->rope_table) (void)hipFree(s->rope_table);
  delete s;
}

size_t ls_param_count(const ls_stage* s) { return s ? s->n_params : 0; }

ls_status ls_get_config(const ls_stage* s, ls_config* out) {
  LS_REQUIRE(s && out, "ls_get_config: null argument");
  *out = s->cfg;
  return LS_OK;
}

ls_status ls_bind_params(ls_stage* s, const void* params, void* stream) {
  LS_TRY(check_stage(s, false));
  LS_REQUIRE(params != nullptr, "ls_bind_params: null parameter vector");
  LS_REQUIRE(((uintptr_t)params % 16) == 0, "ls_bind_params: parameter vector must be 16-byte aligned");
  s->params = params;
  if (s->owns_op) return lsk_convert(params, s->cfg.dtype, s->params_op, s->cfg.mma_dtype, s->n_params, stream);
  s->params_op = const_cast<void*>(params);
  return LS_OK;
}

size_t ls_workspace_bytes(const ls_stage* s, int max_tokens) {
  if (!s || max_tokens <= 0) return 0;
  const size_t a = carve_fwd(s, nullptr, max_tokens, nullptr);
  const size_t b = carve_bwd(s, nullptr, max_tokens, nullptr);
  return (a > b ? a : b) + 256;
}

size_t ls_saved_bytes(const ls_stage* s, int B, int L) {
  if (!s || B <= 0 || L <= 0) return 0;
  return carve_saved(s, nullptr, B * L, nullptr) + 256;
}

ls_status stage_prefill(ls_stage* s, const void* X, const int32_t* chunk_len, int B, const ls_kv* kv,
                        void* Y, void* workspace, void* stream) {
  LS_TRY(check_stage(s, true));
  LS_REQUIRE(X && Y && workspace && chunk_len, "stage_prefill: null argument");
  LS_REQUIRE(B > 0 && B <= 32, "stage_prefill: B must be in 1..32, got %d", B);
  int max_ctx = 0;
  LS_TRY(check_kv(s, kv, B, chunk_len, &max_ctx));
  Chunks ch;
  ch.n = B;
  ch.start[0] = 0;
  for (int b = 0; b < B; ++b) ch.start[b + 1] = ch.start[b] + chunk_len[b];
  const int T = ch.start[B];
  hipStream_t st = (hipStream_t)stream;
  FwdWs w;
  carve_fwd(s, workspace, T, &w);
  token_index_kernel<<<(T + 255) / 256, 256, 0, st>>>(ch, kv->ctx_len, w.pos, w.req);
  LS_CHECK_LAUNCH();
  return serve_forward(s, X, T, B, kv, max_ctx, Y, w, ch.start, 0, st);
}

ls_status stage_decode(ls_stage* s, const void* X, int B, const ls_kv* kv, void* Y, void* workspace,
                       void* stream) {
  LS_TRY(check_stage(s, true));
  LS_REQUIRE(X && Y && workspace, "stage_decode: null argument");
  LS_REQUIRE(B > 0, "stage_decode: B must be positive, got %d", B);
  int max_ctx = 0;
  LS_TRY(check_kv(s, kv, B, nullptr, &max_ctx));
  hipStream_t st = (hipStream_t)stream;
  FwdWs w;
  carve_fwd(s, workspace, B, &w);
  decode_index_kernel<<<(B + 255) / 256, 256, 0, st>>>(B, kv->ctx_len, w.pos, w.req);
  LS_CHECK_LAUNCH();
  return serve_forward(s, X, B, B, kv, max_ctx, Y, w, nullptr, 0, st);
}

ls_status stage_step(ls_stage* s, const void* X, int n_decode, const int32_t* chunk_len, int n_prefill,
                     const ls_kv* kv, void* Y, void* workspace, void* stream) {
  LS_TRY(check_stage(s, true));
  LS_REQUIRE(X && Y && workspace, "stage_step: null argument");
  LS_REQUIRE(n_decode >= 0 && n_prefill >= 0 && n_decode + n_prefill > 0, "stage_step: empty batch (%d decode, %d prefill)",
             n_decode, n_prefill);
  LS_REQUIRE(n_prefill <= 32, "stage_step: at most 32 prompt chunks per call, got %d", n_prefill);
  LS_REQUIRE(n_prefill == 0 || chunk_len, "stage_step: null chunk_len");
  const int B = n_decode + n_prefill;
  std::vector<int32_t> new_tokens((size_t)B, 1);
  Chunks ch;
  ch.n = n_prefill;
  ch.start[0] = 0;
  for (int b = 0; b < n_prefill; ++b) {
    new_tokens[(size_t)n_decode + b] = chunk_len[b];
    LS_REQUIRE(chunk_len[b] > 0, "stage_step: chunk %d has %d tokens", b, chunk_len[b]);
    ch.start[b + 1] = ch.start[b] + chunk_len[b];
  }
  int max_ctx = 0;
  LS_TRY(check_kv(s, kv, B, new_tokens.data(), &max_ctx));
  const int T = n_decode + ch.start[n_prefill];
  hipStream_t st = (hipStream_t)stream;
  FwdWs w;
  carve_fwd(s, workspace, T, &w);
  hybrid_index_kernel<<<(T + 255) / 256, 256, 0, st>>>(n_decode, ch, kv->ctx_len, w.pos, w.req);
  LS_CHECK_LAUNCH();
  // without prompt chunks this is a decode step (no chunk table: every row goes to the decode kernel)
  return serve_forward(s, X, T, B, kv, max_ctx, Y, w, n_prefill > 0 ? ch.start : nullptr, n_decode, st);
}

ls_status stage_train_fwd(ls_stage* s, const void* X, int B, int L, void* Y, void* saved, void* workspace,
                          void* stream) {
  LS_TRY(check_stage(s, true));
  LS_REQUIRE(X && Y && saved && workspace, "stage_train_fwd: null argument");
  LS_REQUIRE(B > 0 && L > 0, "stage_train_fwd: B and L must be positive (B=%d L=%d)", B, L);
  const ls_config& c = s->cfg;
  LS_REQUIRE(c.block != LS_BLOCK_LLAMA || L <= c.max_pos, "stage_train_fwd: L %d exceeds max_pos %d", L, c.max_pos);
  const int T = B * L;
  hipStream_t st = (hipStream_t)stream;
  std::vector<Saved> sv;
  carve_saved(s, saved, T, &sv);
  FwdWs w;
  carve_fwd(s, workspace, T, &w);
  train_index_kernel<<<(T + 255) / 256, 256, 0, st>>>(T, L, w.pos);
  LS_CHECK_LAUNCH();
  LS_TRY(lsk_convert(X, c.io_dtype, sv[0].x_in, LS_F32, (size_t)T * c.d_model, st));
  for (int l = 0; l < c.n_layers; ++l) {
    float* y = l + 1 < c.n_layers ? sv[l + 1].x_in : w.xa;
    FwdBufs f{sv[l].x_in, sv[l].x1, y, sv[l].mean1, sv[l].rstd1, sv[l].mean2, sv[l].rstd2, sv[l].lse,
              sv[l].h1, sv[l].qkv, sv[l].o, sv[l].h2, sv[l].up, sv[l].act, w.scratch};
    LS_TRY(block_forward(s, l, T, f, w.pos, nullptr, B, L, nullptr, 0, nullptr, 0, st));
  }
  return lsk_convert(w.xa, LS_F32, Y, c.io_dtype, (size_t)T * c.d_model, st);
}

ls_status stage_train_bwd(ls_stage* s, const void* dY, int B, int L, const void* saved, void* dX,
                          float* dParams, int accumulate, void* workspace, void* stream) {
  LS_TRY(check_stage(s, true));
  LS_REQUIRE(dY && saved && dX && dParams && workspace, "stage_train_bwd: null argument");
  LS_REQUIRE(B > 0 && L > 0, "stage_train_bwd: B and L must be positive (B=%d L=%d)", B, L);
  const ls_config& c = s->cfg;
  const int T = B * L, d = c.d_model, F = c.d_ff, mt = c.mma_dtype, pt = c.dtype, U = s->up_cols;
  const bool gpt = c.block == LS_BLOCK_GPT_PRELN;
  const int nk = gpt ? 0 : 1, acc = accumulate ? 1 : 0;
  hipStream_t st = (hipStream_t)stream;
  std::vector<Saved> sv;
  carve_saved(s, const_cast<void*>(saved), T, &sv);
  BwdWs w;
  carve_bwd(s, workspace, T, &w);
  train_index_kernel<<<(T + 255) / 256, 256, 0, st>>>(T, L, w.pos);
  LS_CHECK_LAUNCH();
  // the whole backward runs on dY * 2^e (gscale[0]); every fp32 result is multiplied by 2^-e (gscale[1])
  LS_TRY(lsk_grad_scale(dY, c.io_dtype, (size_t)T * d, w.gscale, st));
  const float* inv = w.gscale + 1;
  LS_TRY(lsk_convert_scaled(dY, c.io_dtype, w.g, LS_F32, (size_t)T * d, w.gscale, st));
  LS_TRY(lsk_convert_scaled(dY, c.io_dtype, w.g16, mt, (size_t)T * d, w.gscale, st));
  for (int l = c.n_layers - 1; l >= 0; --l) {
    const LayerOff& o = s->off[l];
    const Saved& v = sv[l];
    // y = x1 + act W_dn^T (+ b_dn)
    if (gpt) {
      LS_TRY(lsk_gemm(mt, T, F, d, w.g16, d, 1, wptr(s, o.w_dn), F, 0, w.dact, F, mt, nullptr, 0, nullptr, 0, 0, st));
    } else if (mt == LS_F32) {
      LS_TRY(lsk_gemm(mt, T, F, d, w.g16, d, 1, wptr(s, o.w_dn), F, 0, w.dact, F, mt, nullptr, 0, nullptr, 0, 0, st));
      LS_TRY(lsk_swiglu_bwd(w.dact, v.up, w.dup, mt, T, F, st));
    } else {
      // the activation's backward in the epilogue of the product that feeds it (no dact round trip)
      LS_TRY(lsk_gemm_swiglu_bwd(mt, T, F, d, w.g16, wptr(s, o.w_dn), v.up, w.dup, w.dact, st));
    }
    LS_TRY(lsk_gemm_scaled(mt, d, F, T, w.g16, d, 0, v.act, F, 0, dParams + o.w_dn, F, LS_F32, nullptr, 0, nullptr, 0, acc, inv, st));
    if (gpt) {
      LS_TRY(lsk_colsum_scaled(w.g16, mt, T, d, d, dParams + o.b_dn, acc, w.partial, inv, st));
      LS_TRY(lsk_gelu_bwd(w.dact, v.up, w.dup, mt, (size_t)T * F, c.act, st));
    }
    // up = h2 W_up^T (+ b_up)
    LS_TRY(lsk_gemm(mt, T, d, U, w.dup, U, 1, wptr(s, o.w_up), d, 0, w.dh, d, mt, nullptr, 0, nullptr, 0, 0, st));
    LS_TRY(lsk_gemm_scaled(mt, U, d, T, w.dup, U, 0, v.h2, d, 0, dParams + o.w_up, d, LS_F32, nullptr, 0, nullptr, 0, acc, inv, st));
    if (gpt) LS_TRY(lsk_colsum_scaled(w.dup, mt, T, U, U, dParams + o.b_up, acc, w.partial, inv, st));
    // h2 = norm2(x1);  g1 = g + norm2_bwd(dh)
    LS_TRY(lsk_norm_bwd_scaled(nk, w.dh, mt, v.x1, v.mean2, v.rstd2, pptr(s, o.n2_g), pt, T, d, w.g, w.g1, w.g16, mt,
                        dParams + o.n2_g, gpt ? dParams + o.n2_b : nullptr, acc, w.partial, inv, st));
    // x1 = x + o W_o^T (+ b_o)
    LS_TRY(lsk_gemm(mt, T, d, d, w.g16, d, 1, wptr(s, o.w_o), d, 0, w.d_o, d, mt, nullptr, 0, nullptr, 0, 0, st));
    LS_TRY(lsk_gemm_scaled(mt, d, d, T, w.g16, d, 0, v.o, d, 0, dParams + o.w_o, d, LS_F32, nullptr, 0, nullptr, 0, acc, inv, st));
    if (gpt) LS_TRY(lsk_colsum_scaled(w.g16, mt, T, d, d, dParams + o.b_o, acc, w.partial, inv, st));
    if (gpt)
      LS_TRY(lsk_attn_bwd(mt == LS_F32 ? 0 : 1, v.qkv, v.o, w.d_o, v.lse, mt, B, L, c.n_heads, c.head_dim, w.dqkv,
                          w.dvec, st));
    else
      LS_TRY(lsk_attn_bwd_rope(mt == LS_F32 ? 0 : 1, v.qkv, v.o, w.d_o, v.lse, mt, B, L, c.n_heads, c.head_dim,
                               w.dqkv, w.dvec, w.pos, s->rope_table, st));
    // qkv = h1 W_qkv^T (+ b_qkv)
    LS_TRY(lsk_gemm(mt, T, d, 3 * d, w.dqkv, 3 * d, 1, wptr(s, o.w_qkv), d, 0, w.dh, d, mt, nullptr, 0, nullptr, 0, 0, st));
    LS_TRY(lsk_gemm_scaled(mt, 3 * d, d, T, w.dqkv, 3 * d, 0, v.h1, d, 0, dParams + o.w_qkv, d, LS_F32, nullptr, 0, nullptr, 0, acc, inv, st));
    if (gpt) LS_TRY(lsk_colsum_scaled(w.dqkv, mt, T, 3 * d, 3 * d, dParams + o.b_qkv, acc, w.partial, inv, st));
    // h1 = norm1(x);  g = g1 + norm1_bwd(dh)
    LS_TRY(lsk_norm_bwd_scaled(nk, w.dh, mt, v.x_in, v.mean1, v.rstd1, pptr(s, o.n1_g), pt, T, d, w.g1, w.g, w.g16, mt,
                        dParams + o.n1_g, gpt ? dParams + o.n1_b : nullptr, acc, w.partial, inv, st));
  }
  return lsk_convert_scaled(w.g, LS_F32, dX, c.io_dtype, (size_t)T * d, inv, st);
}

// Model update: one fused pass per parameter tensor (decay on the weight matrices only)
ls_status stage_optimizer_step(ls_stage* s, const ls_optim* opt, void* params, float* master, float* m, float* v,
                               const float* dParams, void* stream) {
  LS_TRY(check_stage(s, true));
  LS_REQUIRE(opt && params && master && m && dParams, "stage_optimizer_step: null argument");
  LS_REQUIRE(params == s->params, "stage_optimizer_step: params must be the vector bound with ls_bind_params");
  LS_REQUIRE(opt->kind == LS_OPT_SGD || opt->kind == LS_OPT_ADAMW, "stage_optimizer_step: unknown optimizer %d", opt->kind);
  LS_REQUIRE(opt->kind == LS_OPT_SGD || v, "stage_optimizer_step: AdamW needs the second-moment vector");
  LS_REQUIRE(opt->step >= 1, "stage_optimizer_step: steps count from 1 (got %d)", opt->step);
  const ls_config& c = s->cfg;
  const size_t d = c.d_model, F = c.d_ff, U = s->up_cols;
  const bool gpt = c.block == LS_BLOCK_GPT_PRELN;
  const size_t psz = dtype_size(c.dtype), osz_ = dtype_size(c.mma_dtype);
  auto one = [&](size_t off, size_t n, bool decay) -> ls_status {
    void* pop = s->owns_op ? (char*)s->params_op + off * osz_ : nullptr;
    return lsk_optimizer(opt->kind, opt->lr, opt->beta1, opt->beta2, opt->eps, decay ? opt->weight_decay : 0.f,
                         opt->momentum, opt->grad_scale, opt->step, n, dParams + off, m + off, v ? v + off : nullptr,
                         master + off, (char*)params + off * psz, c.dtype, pop, c.mma_dtype, stream);
  };
  for (int l = 0; l < c.n_layers; ++l) {
    const LayerOff& o = s->off[l];
    LS_TRY(one(o.n1_g, d, false));
    if (gpt) LS_TRY(one(o.n1_b, d, false));
    LS_TRY(one(o.w_qkv, 3 * d * d, true));
    if (gpt) LS_TRY(one(o.b_qkv, 3 * d, false));
    LS_TRY(one(o.w_o, d * d, true));
    if (gpt) LS_TRY(one(o.b_o, d, false));
    LS_TRY(one(o.n2_g, d, false));
    if (gpt) LS_TRY(one(o.n2_b, d, false));
    LS_TRY(one(o.w_up, U * d, true));
    if (gpt) LS_TRY(one(o.b_up, U, false));
    LS_TRY(one(o.w_dn, d * F, true));
    if (gpt) LS_TRY(one(o.b_dn, d, false));
  }
  return LS_OK;
}

ls_status stage_probe_interference(ls_stage* s, const void* dec_X, int dec_B, const ls_kv* kv, void* dec_Y,
                                   void* ws_a, const void* trn_X, int trn_B, int trn_L, void* trn_Y,
                                   void* trn_saved, const void* trn_dY, void* trn_dX, float* trn_dParams,
                                   void* ws_b, void* stream_a, void* stream_b, int iters, float* out_ms) {
  LS_TRY(check_stage(s, true));
  LS_REQUIRE(out_ms && iters > 0, "probe: bad iters or null out_ms");
  LS_REQUIRE(stream_a != stream_b, "probe: the two streams must differ");
  LS_REQUIRE(ws_a && ws_b && ws_a != ws_b, "probe: the two calls need separate, non-null workspaces");
  LS_REQUIRE(dec_X && dec_Y && kv, "probe: null decode argument");
  LS_REQUIRE(trn_X && trn_Y && trn_saved && trn_dY && trn_dX && trn_dParams, "probe: null training argument");
  LS_REQUIRE(dec_B > 0 && trn_B > 0 && trn_L > 0, "probe: non-positive batch (decode %d, train %d x %d)", dec_B, trn_B,
             trn_L);
  hipStream_t sa = (hipStream_t)stream_a, sb = (hipStream_t)stream_b;
  // the four events are destroyed on every way out of the call
  struct Events {
    hipEvent_t e[4] = {nullptr, nullptr, nullptr, nullptr};
    ~Events() {
      for (hipEvent_t v : e)
        if (v) (void)hipEventDestroy(v);
    }
  } ev;
  for (hipEvent_t& v : ev.e) LS_CHECK_HIP(hipEventCreate(&v));
  hipEvent_t ea0 = ev.e[0], ea1 = ev.e[1], eb0 = ev.e[2], eb1 = ev.e[3];
  ls_status rc = LS_OK;
  auto run_a = [&]() { return stage_decode(s, dec_X, dec_B, kv, dec_Y, ws_a, sa); };
  auto run_b = [&]() {
    ls_status r = stage_train_fwd(s, trn_X, trn_B, trn_L, trn_Y, trn_saved, ws_b, sb);
    if (r != LS_OK) return r;
    return stage_train_bwd(s, trn_dY, trn_B, trn_L, trn_saved, trn_dX, trn_dParams, 0, ws_b, sb);
  };
  float ms = 0.f;
  memset(out_ms, 0, 6 * sizeof(float));
  do {
    // warm-up of both paths
    if ((rc = run_a()) != LS_OK) break;
    if ((rc = run_b()) != LS_OK) break;
    if (hipStreamSynchronize(sa) != hipSuccess || hipStreamSynchronize(sb) != hipSuccess) { rc = LS_EHIP; break; }
    // A alone
    (void)hipEventRecord(ea0, sa);
    for (int i = 0; i < iters && rc == LS_OK; ++i) rc = run_a();
    (void)hipEventRecord(ea1, sa);
    if (rc != LS_OK) break;
    if (hipEventSynchronize(ea1) != hipSuccess) { rc = LS_EHIP; break; }
    (void)hipEventElapsedTime(&ms, ea0, ea1);
    out_ms[0] = ms / iters;
    // B alone
    (void)hipEventRecord(eb0, sb);
    for (int i = 0; i < iters && rc == LS_OK; ++i) rc = run_b();
    (void)hipEventRecord(eb1, sb);
    if (rc != LS_OK) break;
    if (hipEventSynchronize(eb1) != hipSuccess) { rc = LS_EHIP; break; }
    (void)hipEventElapsedTime(&ms, eb0, eb1);
    out_ms[1] = ms / iters;
    // together: the training stream is enqueued first (it is the long one),
    // the decode stream keeps issuing steps until it has done `iters` of them
    (void)hipEventRecord(eb0, sb);
    (void)hipEventRecord(ea0, sa);
    for (int i = 0; i < iters && rc == LS_OK; ++i) {
      rc = run_b();
      if (rc == LS_OK) rc = run_a();
    }
    (void)hipEventRecord(ea1, sa);
    (void)hipEventRecord(eb1, sb);
    if (rc != LS_OK) break;
    if (hipEventSynchronize(ea1) != hipSuccess || hipEventSynchronize(eb1) != hipSuccess) { rc = LS_EHIP; break; }
    (void)hipEventElapsedTime(&ms, ea0, ea1);
    out_ms[2] = ms / iters;
    (void)hipEventElapsedTime(&ms, eb0, eb1);
    out_ms[3] = ms / iters;
    float w0 = 0.f;
    (void)hipEventElapsedTime(&w0, eb0, ea1);
    out_ms[4] = (ms > w0 ? ms : w0) / iters;
  } while (0);
  if (rc == LS_EHIP) ls_set_error("probe: a HIP synchronisation failed");
  (void)hipStreamSynchronize(sa);
  (void)hipStreamSynchronize(sb);
  return rc;
}

}  // extern "C"
