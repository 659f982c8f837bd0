// Public attention entry points: choose between the plain kernels and the
// matrix-core kernels.
#include "common.h"

extern "C" {
ls_status lsk_attn_fwd_simple(const void*, int, int, int, int, int, void*, float*, void*);
ls_status lsk_attn_bwd_simple(const void*, const void*, const void*, const float*, int, int, int, int, int,
                              void*, float*, void*);
ls_status lsk_attn_paged_simple(const void*, int, int, int, int, const int32_t*, const int32_t*,
                                const void*, const void*, const int32_t*, int, int, int, void*, void*);

ls_status lsk_attn_fwd_mfma(const void*, int, int, int, int, int, void*, float*, void*);
ls_status lsk_attn_bwd_mfma(const void*, const void*, const void*, const float*, int, int, int, int, int,
                            void*, float*, const float*, void*);

static bool mfma_ok(int impl, int dtype, int head_dim) {
  return impl == 1 && (dtype == LS_BF16 || dtype == LS_F16) && (head_dim == 64 || head_dim == 128);
}

ls_status lsk_attn_fwd(int impl, const void* qkv, int dtype, int B, int L, int n_heads, int head_dim,
                       void* o, float* lse, void* stream) {
  if (mfma_ok(impl, dtype, head_dim)) return lsk_attn_fwd_mfma(qkv, dtype, B, L, n_heads, head_dim, o, lse, stream);
  return lsk_attn_fwd_simple(qkv, dtype, B, L, n_heads, head_dim, o, lse, stream);
}

ls_status lsk_attn_bwd(int impl, const void* qkv, const void* o, const void* dO, const float* lse,
                       int dtype, int B, int L, int n_heads, int head_dim, void* dqkv, float* dvec,
                       void* stream) {
  if (mfma_ok(impl, dtype, head_dim))
    return lsk_attn_bwd_mfma(qkv, o, dO, lse, dtype, B, L, n_heads, head_dim, dqkv, dvec, nullptr, stream);
  return lsk_attn_bwd_simple(qkv, o, dO, lse, dtype, B, L, n_heads, head_dim, dqkv, dvec, stream);
}

// Attention backward followed by the backward of the rotary embedding on dq and dk
// (rotation by -pos[t]); pos[t] must be t mod L.  Fused into the matrix-core kernels' stores
// when they apply, otherwise the in-place rotary kernel runs afterwards.
ls_status lsk_attn_bwd_rope(int impl, const void* qkv, const void* o, const void* dO, const float* lse,
                            int dtype, int B, int L, int n_heads, int head_dim, void* dqkv, float* dvec,
                            const int32_t* pos, const float* table, void* stream) {
  LS_REQUIRE(pos && table, "attn_bwd_rope: null rotary arguments");
  if (mfma_ok(impl, dtype, head_dim))
    return lsk_attn_bwd_mfma(qkv, o, dO, lse, dtype, B, L, n_heads, head_dim, dqkv, dvec, table, stream);
  LS_TRY(lsk_attn_bwd_simple(qkv, o, dO, lse, dtype, B, L, n_heads, head_dim, dqkv, dvec, stream));
  return lsk_rope(dqkv, dtype, B * L, n_heads, head_dim, pos, table, -1.0f, stream);
}

size_t lsk_attn_bwd_scratch_floats(int B, int L, int n_heads) {
  const size_t items = (size_t)B * L * n_heads;
  return 2 * items + (items + 3) / 4 + 1;   // D, per-workgroup maxima of |dO|, their maximum, log-sum-exp in base 2
}

size_t lsk_attn_decode_scratch_floats(int, int, int, int, int);
ls_status lsk_attn_decode(const void*, int, int, int, int, const int32_t*, const int32_t*, const void*,
                          const void*, const int32_t*, int, int, int, void*, float*, void*);

size_t lsk_attn_paged_scratch_floats(int T, int n_heads, int head_dim, int max_ctx, int page_size) {
  return lsk_attn_decode_scratch_floats(T, n_heads, head_dim, max_ctx, page_size);
}

ls_status lsk_attn_paged(int impl, const void* qkv, int dtype, int T, int n_heads, int head_dim,
                         const int32_t* pos, const int32_t* req, const void* k_pool, const void* v_pool,
                         const int32_t* block_table, int max_pages_per_req, int page_size, int max_ctx,
                         void* o, float* scratch, void* stream) {
  if (mfma_ok(impl, dtype, head_dim) && (page_size * head_dim) % 512 == 0)
    return lsk_attn_decode(qkv, dtype, T, n_heads, head_dim, pos, req, k_pool, v_pool, block_table,
                           max_pages_per_req, page_size, max_ctx, o, scratch, stream);
  return lsk_attn_paged_simple(qkv, dtype, T, n_heads, head_dim, pos, req, k_pool, v_pool, block_table,
                               max_pages_per_req, page_size, max_ctx, o, stream);
}
}
