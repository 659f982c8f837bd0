// Decode batches (at most 128 rows): the split-K projections leave fp32 partial
// products; the kernels here sum them in a fixed order and apply, in the same
// pass, the step that follows the projection in the block:
//   QKV projection   -> bias, rotary embedding of q and k, K/V page write
//   output / FFN-down -> bias, residual add, and the normalisation that comes next
//   FFN-up           -> bias, GELU or SwiGLU
// so that a decode step launches one small kernel per projection instead of a
// reduce kernel plus the elementwise kernel after it.
#include "common.h"

ls_status gemm_dma_skinny_partials(int, int, int, int, const void*, long, const void*, long, float*, size_t, int*,
                                   hipStream_t);

namespace {

__device__ __forceinline__ f32x4 sum_partials(const float* partial, int splits, long stride, long i) {
  f32x4 v = *(const f32x4*)(partial + i);
#pragma unroll 4
  for (int s = 1; s < splits; ++s) v += *(const f32x4*)(partial + s * stride + i);
  return v;
}

template <class TH> __device__ __forceinline__ void store4(TH* p, f32x4 v) {
  typedef TH V4 __attribute__((ext_vector_type(4)));
  V4 o;
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = from_f<TH>(v[e]);
  *(V4*)p = o;
}
template <> __device__ __forceinline__ void store4<float>(float* p, f32x4 v) { *(f32x4*)p = v; }

// one workgroup of up to 1024 threads per row (a decode batch has few rows, so the parallelism has to
// come from the columns): x_out = sum of partials + bias + resid; h = norm(x_out) (kind 0 LayerNorm,
// 1 RMSNorm, < 0 none).  d % 4 == 0, d <= 8192 = 1024 threads x FN_MAX float4.
constexpr int FN_MAX = 2;
template <class TH>
__global__ __launch_bounds__(1024) void finish_resid_norm_kernel(const float* partial, int splits, int T, int d,
                                                                const void* bias, const float* resid, float* x_out,
                                                                int kind, const void* gamma, const void* beta,
                                                                int pdt, float eps, TH* h) {
  __shared__ float red[16];
  const long row = blockIdx.x, stride = (long)T * d;
  f32x4 v[FN_MAX];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < FN_MAX; ++i) {
    const int c = (threadIdx.x + i * (int)blockDim.x) * 4;
    v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (c < d) {
      v[i] = sum_partials(partial, splits, stride, row * d + c);
      if (bias)
#pragma unroll
        for (int e = 0; e < 4; ++e) v[i][e] += load_as_f(bias, c + e, pdt);
      if (resid) v[i] += *(const f32x4*)(resid + row * d + c);
      *(f32x4*)(x_out + row * d + c) = v[i];
      s += (v[i][0] + v[i][1]) + (v[i][2] + v[i][3]);
    }
  }
  if (kind < 0) return;
  const float mu = kind == 0 ? block_sum(s, red) / d : 0.f;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < FN_MAX; ++i)
    if ((threadIdx.x + i * (int)blockDim.x) * 4 < d)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float t = v[i][e] - mu;
        q += t * t;
      }
  const float r = 1.0f / sqrtf(block_sum(q, red) / d + eps);
#pragma unroll
  for (int i = 0; i < FN_MAX; ++i) {
    const int c = (threadIdx.x + i * (int)blockDim.x) * 4;
    if (c < d) {
      f32x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        o[e] = (v[i][e] - mu) * r * load_as_f(gamma, c + e, pdt);
        if (kind == 0 && beta) o[e] += load_as_f(beta, c + e, pdt);
      }
      store4<TH>(h + row * d + c, o);
    }
  }
}

// four hidden units per thread.  act LS_ACT_SWIGLU: the projection has 2F columns (gate, then up).
template <class TH>
__global__ void finish_act_kernel(const float* partial, int splits, int T, int F, int act, const void* bias, int pdt,
                                  TH* out) {
  const int cols = act == LS_ACT_SWIGLU ? 2 * F : F;
  const long stride = (long)T * cols, n4 = (long)T * (F / 4);
  for (long idx = blockIdx.x * (long)blockDim.x + threadIdx.x; idx < n4; idx += (long)gridDim.x * blockDim.x) {
    const long t = idx / (F / 4);
    const int f = (int)(idx % (F / 4)) * 4;
    f32x4 a = sum_partials(partial, splits, stride, t * cols + f), o;
    if (bias)
#pragma unroll
      for (int e = 0; e < 4; ++e) a[e] += load_as_f(bias, f + e, pdt);
    if (act == LS_ACT_SWIGLU) {
      f32x4 u = sum_partials(partial, splits, stride, t * cols + F + f);
      if (bias)
#pragma unroll
        for (int e = 0; e < 4; ++e) u[e] += load_as_f(bias, F + f + e, pdt);
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = a[e] / (1.f + __expf(-a[e])) * u[e];
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = gelu_f(a[e], act);
    }
    store4<TH>(out + t * F + f, o);
  }
}

// one thread per (row, q / k / v, head, four pairs i .. i + 3 < dh / 2); rotation of q and k by
// pos[row] when a table is given; the values go to the qkv buffer and those of k and v also to
// the request's page slot.  dh % 8 == 0.
template <class TH>
__global__ void finish_qkv_kernel(const float* partial, int splits, int T, int h, int dh, const void* bias, int pdt,
                                  const int32_t* pos, const int32_t* req, const float* table, TH* qkv, TH* k_pool,
                                  TH* v_pool, const int32_t* block_table, int max_pages, int page) {
  const int half = dh / 2, d = h * dh, q4 = half / 4;
  const long stride = (long)T * 3 * d, n = (long)T * 3 * h * q4;
  for (long idx = blockIdx.x * (long)blockDim.x + threadIdx.x; idx < n; idx += (long)gridDim.x * blockDim.x) {
    const int i = (int)(idx % q4) * 4, hp = (int)((idx / q4) % (3 * h));   // hp = part * h + head
    const int part = hp / h, head = hp % h;
    const long t = idx / ((long)q4 * 3 * h);
    const long qi = t * 3 * d + (long)hp * dh + i;
    f32x4 xa = sum_partials(partial, splits, stride, qi), xb = sum_partials(partial, splits, stride, qi + half);
    if (bias)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        xa[e] += load_as_f(bias, (long)hp * dh + i + e, pdt);
        xb[e] += load_as_f(bias, (long)hp * dh + i + half + e, pdt);
      }
    const int p = pos[t];
    if (table && part < 2) {
      const float* tb = table + ((long)p * half + i) * 2;   // (cos, sin) pairs
      const f32x4 cs0 = *(const f32x4*)tb, cs1 = *(const f32x4*)(tb + 4);
      const f32x4 c = {cs0[0], cs0[2], cs1[0], cs1[2]}, sn = {cs0[1], cs0[3], cs1[1], cs1[3]};
      const f32x4 ra = xa * c - xb * sn, rb = xb * c + xa * sn;
      xa = ra; xb = rb;
    }
    typedef TH V4 __attribute__((ext_vector_type(4)));
    V4 oa, ob;
#pragma unroll
    for (int e = 0; e < 4; ++e) { oa[e] = from_f<TH>(xa[e]); ob[e] = from_f<TH>(xb[e]); }
    *(V4*)(qkv + qi) = oa;
    *(V4*)(qkv + qi + half) = ob;
    if (part > 0) {
      TH* pool = part == 1 ? k_pool : v_pool;
      const int pg = block_table[(long)req[t] * max_pages + p / page];
      const long dst = (((long)pg * h + head) * page + p % page) * dh + i;
      *(V4*)(pool + dst) = oa;
      *(V4*)(pool + dst + half) = ob;
    }
  }
}

inline unsigned grid_of(long n, unsigned cap = 8192) {
  long g = (n + 255) / 256;
  return (unsigned)(g < 1 ? 1 : (g > cap ? cap : g));
}
inline bool half_type(int dt) { return dt == LS_BF16 || dt == LS_F16; }

}  // namespace

extern "C" {

ls_status lsk_gemm_partials(int op_dtype, int M, int N, int K, const void* X, long ldx, const void* W, long ldw,
                            float* partial, size_t partial_floats, int* splits, void* stream) {
  LsTimed timed(LSK_TIMED_DECODE_GEMM, stream);
  LS_REQUIRE(X && W && partial && splits, "gemm_partials: null argument");
  LS_REQUIRE(half_type(op_dtype), "gemm_partials: 16-bit operands only");
  LS_REQUIRE(M >= 1 && M <= 128 && N >= 64 && N % 4 == 0 && K >= 64 && K % 64 == 0,
             "gemm_partials: need 1 <= M <= 128, N >= 64 and a multiple of 4, K a multiple of 64 (M=%d N=%d K=%d)", M, N, K);
  LS_REQUIRE(ldx % 8 == 0 && ldw % 8 == 0 && (uintptr_t)X % 16 == 0 && (uintptr_t)W % 16 == 0 &&
                 (uintptr_t)partial % 16 == 0,
             "gemm_partials: operands must be 16-byte aligned with leading dimensions that are multiples of 8");
  LS_REQUIRE(partial_floats >= (size_t)M * N, "gemm_partials: the partial buffer holds %zu floats, one M x N result needs %zu",
             partial_floats, (size_t)M * N);
  const ls_status r = gemm_dma_skinny_partials(op_dtype, M, N, K, X, ldx, W, ldw, partial, partial_floats, splits,
                                               (hipStream_t)stream);
  LS_REQUIRE(r != LS_ESTATE, "gemm_partials: shape not covered (M=%d N=%d K=%d)", M, N, K);
  return r;
}

ls_status lsk_finish_resid_norm(const float* partial, int splits, int T, int d, const void* bias, const float* resid,
                                float* x_out, int kind, const void* gamma, const void* beta, int pdt, float eps,
                                void* h, int hdt, void* stream) {
  LsTimed timed(LSK_TIMED_FINISH, stream);
  LS_REQUIRE(partial && x_out && splits >= 1 && T > 0 && d > 0, "finish_resid_norm: bad argument");
  LS_REQUIRE(d % 4 == 0 && d <= 4096 * FN_MAX, "finish_resid_norm: d_model %d must be a multiple of 4, at most %d", d,
             4096 * FN_MAX);
  LS_REQUIRE(kind < 0 || (kind <= 1 && gamma && h), "finish_resid_norm: the normalisation needs gamma and an output");
  LS_REQUIRE((uintptr_t)partial % 16 == 0 && (uintptr_t)x_out % 16 == 0 && (!resid || (uintptr_t)resid % 16 == 0) &&
                 (!h || (uintptr_t)h % 16 == 0),
             "finish_resid_norm: buffers must be 16-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  int nt = (d / 4 + 63) / 64 * 64;   // one float4 per thread up to 4096 columns, two beyond
  if (nt > 1024) nt = 1024;
  if (hdt == LS_F32)
    finish_resid_norm_kernel<float><<<T, nt, 0, st>>>(partial, splits, T, d, bias, resid, x_out, kind, gamma, beta, pdt, eps, (float*)h);
  else if (hdt == LS_BF16)
    finish_resid_norm_kernel<bf16_t><<<T, nt, 0, st>>>(partial, splits, T, d, bias, resid, x_out, kind, gamma, beta, pdt, eps, (bf16_t*)h);
  else
    finish_resid_norm_kernel<f16_t><<<T, nt, 0, st>>>(partial, splits, T, d, bias, resid, x_out, kind, gamma, beta, pdt, eps, (f16_t*)h);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

ls_status lsk_finish_act(const float* partial, int splits, int T, int F, int act, const void* bias, int pdt, void* out,
                         int odt, void* stream) {
  LsTimed timed(LSK_TIMED_FINISH, stream);
  LS_REQUIRE(partial && out && splits >= 1 && T > 0 && F > 0, "finish_act: bad argument");
  LS_REQUIRE(F % 4 == 0, "finish_act: d_ff must be a multiple of 4");
  LS_REQUIRE(act == LS_ACT_GELU_TANH || act == LS_ACT_GELU_ERF || act == LS_ACT_SWIGLU, "finish_act: unknown activation %d", act);
  LS_REQUIRE((uintptr_t)partial % 16 == 0 && (uintptr_t)out % 16 == 0, "finish_act: buffers must be 16-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  const unsigned g = grid_of((long)T * (F / 4));
  if (odt == LS_F32) finish_act_kernel<float><<<g, 256, 0, st>>>(partial, splits, T, F, act, bias, pdt, (float*)out);
  else if (odt == LS_BF16) finish_act_kernel<bf16_t><<<g, 256, 0, st>>>(partial, splits, T, F, act, bias, pdt, (bf16_t*)out);
  else finish_act_kernel<f16_t><<<g, 256, 0, st>>>(partial, splits, T, F, act, bias, pdt, (f16_t*)out);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

ls_status lsk_finish_qkv(const float* partial, int splits, int T, int h, int dh, const void* bias, int pdt,
                         const int32_t* pos, const int32_t* req, const float* table, void* qkv, int dt, void* k_pool,
                         void* v_pool, const int32_t* block_table, int max_pages, int page, void* stream) {
  LsTimed timed(LSK_TIMED_FINISH, stream);
  LS_REQUIRE(partial && pos && req && qkv && k_pool && v_pool && block_table, "finish_qkv: null argument");
  LS_REQUIRE(splits >= 1 && T > 0 && h > 0 && dh > 0 && dh % 8 == 0 && max_pages > 0 && page > 0,
             "finish_qkv: bad size (head_dim must be a multiple of 8)");
  LS_REQUIRE((uintptr_t)partial % 16 == 0 && (uintptr_t)qkv % 8 == 0 && (uintptr_t)k_pool % 8 == 0 &&
                 (uintptr_t)v_pool % 8 == 0 && (!table || (uintptr_t)table % 16 == 0),
             "finish_qkv: buffers must be aligned to their vector accesses");
  LS_REQUIRE(half_type(dt), "finish_qkv: 16-bit q, k, v only");
  hipStream_t st = (hipStream_t)stream;
  const unsigned g = grid_of((long)T * 3 * h * (dh / 8));
  if (dt == LS_BF16)
    finish_qkv_kernel<bf16_t><<<g, 256, 0, st>>>(partial, splits, T, h, dh, bias, pdt, pos, req, table, (bf16_t*)qkv,
                                                (bf16_t*)k_pool, (bf16_t*)v_pool, block_table, max_pages, page);
  else
    finish_qkv_kernel<f16_t><<<g, 256, 0, st>>>(partial, splits, T, h, dh, bias, pdt, pos, req, table, (f16_t*)qkv,
                                               (f16_t*)k_pool, (f16_t*)v_pool, block_table, max_pages, page);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

}  // extern "C"
