// Plain (no matrix core) attention kernels: forward over contiguous sequences
// or over the paged pool, and the training backward.  One wavefront owns one
// (query row, head) pair - or one (key row, head) pair in the dK/dV kernel -
// and works in two passes: lanes over keys for the scores (kept in LDS), then
// lanes over head dimensions for the weighted sums.  Deterministic: no atomics.
// These kernels serve the fp32 stage mode and any shape the MFMA kernels do
// not cover.
#include "common.h"

namespace {

struct KvView {
  // contiguous: keys of the row's sequence live in qkv rows seq0 .. seq0+pos
  // paged: keys live in the pool, found through the request's block table
  const void* qkv;
  const void* k_pool;
  const void* v_pool;
  const int32_t* block_table;
  int paged, dt, h, dh, d, max_pages, page;
};

__device__ __forceinline__ size_t k_index(const KvView& kv, int seq0, int req, int j, int head) {
  if (!kv.paged) return (size_t)(seq0 + j) * 3 * kv.d + kv.d + (size_t)head * kv.dh;
  const int pg = kv.block_table[(size_t)req * kv.max_pages + j / kv.page];
  return (((size_t)pg * kv.h + head) * kv.page + j % kv.page) * kv.dh;
}
__device__ __forceinline__ size_t v_index(const KvView& kv, int seq0, int req, int j, int head) {
  if (!kv.paged) return (size_t)(seq0 + j) * 3 * kv.d + 2 * kv.d + (size_t)head * kv.dh;
  return k_index(kv, seq0, req, j, head);
}

// grid: (ceil(T*h / 4)), block 256 (4 wavefronts), dynamic LDS: 4 * (max_ctx + dh) floats
__global__ __launch_bounds__(256) void attn_fwd_simple_kernel(KvView kv, int T, int L,
                                                              const int32_t* pos_arr,
                                                              const int32_t* req_arr, int max_ctx,
                                                              void* o, float* lse) {
  extern __shared__ float smem[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long item = (long)blockIdx.x * 4 + wave;
  if (item >= (long)T * kv.h) return;
  const int t = item / kv.h, head = item % kv.h;
  float* sc = smem + (size_t)wave * (max_ctx + kv.dh);
  float* qs = sc + max_ctx;
  int pos, req = 0, seq0 = 0;
  if (kv.paged) { pos = pos_arr[t]; req = req_arr[t]; }
  else { pos = t % L; seq0 = t - pos; }
  const int nkeys = pos + 1;
  const float scale = 1.0f / sqrtf((float)kv.dh);
  const void* kbase = kv.paged ? kv.k_pool : kv.qkv;
  const void* vbase = kv.paged ? kv.v_pool : kv.qkv;
  for (int c = lane; c < kv.dh; c += 64)
    qs[c] = load_as_f(kv.qkv, (size_t)t * 3 * kv.d + (size_t)head * kv.dh + c, kv.dt);
  __builtin_amdgcn_wave_barrier();
  float m = -INFINITY;
  for (int j = lane; j < nkeys; j += 64) {
    const size_t ki = k_index(kv, seq0, req, j, head);
    float s = 0.f;
    for (int c = 0; c < kv.dh; ++c) s = fmaf(qs[c], load_as_f(kbase, ki + c, kv.dt), s);
    s *= scale;
    sc[j] = s;
    m = fmaxf(m, s);
  }
  m = wave_max(m);
  float l = 0.f;
  for (int j = lane; j < nkeys; j += 64) {
    const float p = expf(sc[j] - m);
    sc[j] = p;
    l += p;
  }
  l = wave_sum(l);
  __builtin_amdgcn_wave_barrier();
  const float inv = 1.0f / l;
  for (int c = lane; c < kv.dh; c += 64) {
    float acc = 0.f;
    for (int j = 0; j < nkeys; ++j)
      acc = fmaf(sc[j], load_as_f(vbase, v_index(kv, seq0, req, j, head) + c, kv.dt), acc);
    store_from_f(o, (size_t)t * kv.d + (size_t)head * kv.dh + c, kv.dt, acc * inv);
  }
  if (lse && lane == 0) lse[(size_t)t * kv.h + head] = m + logf(l);
}

// D[t, head] = sum_c dO * O
__global__ void attn_dvec_kernel(const void* o, const void* dO, int dt, long n_items, int dh, float* dvec) {
  const long item = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (item >= n_items) return;
  float s = 0.f;
  for (int c = lane; c < dh; c += 64)
    s += load_as_f(o, item * dh + c, dt) * load_as_f(dO, item * dh + c, dt);
  s = wave_sum(s);
  if (lane == 0) dvec[item] = s;
}

// dQ: one wavefront per (query row, head)
__global__ __launch_bounds__(256) void attn_bwd_dq_simple_kernel(const void* qkv, const void* dO,
                                                                 const float* lse, const float* dvec,
                                                                 int dt, int T, int L, int h, int dh,
                                                                 void* dqkv) {
  extern __shared__ float smem[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long item = (long)blockIdx.x * 4 + wave;
  if (item >= (long)T * h) return;
  const int t = item / h, head = item % h, d = h * dh;
  float* ds = smem + (size_t)wave * (L + 2 * dh);
  float* qs = ds + L;
  float* gs = qs + dh;
  const int pos = t % L, seq0 = t - pos;
  const float scale = 1.0f / sqrtf((float)dh);
  for (int c = lane; c < dh; c += 64) {
    qs[c] = load_as_f(qkv, (size_t)t * 3 * d + (size_t)head * dh + c, dt);
    gs[c] = load_as_f(dO, (size_t)t * d + (size_t)head * dh + c, dt);
  }
  __builtin_amdgcn_wave_barrier();
  const float ls = lse[item], dv = dvec[item];
  for (int j = lane; j <= pos; j += 64) {
    const size_t ki = (size_t)(seq0 + j) * 3 * d + d + (size_t)head * dh;
    float s = 0.f, dp = 0.f;
    for (int c = 0; c < dh; ++c) {
      s = fmaf(qs[c], load_as_f(qkv, ki + c, dt), s);
      dp = fmaf(gs[c], load_as_f(qkv, ki + d + c, dt), dp);
    }
    ds[j] = expf(s * scale - ls) * (dp - dv);
  }
  __builtin_amdgcn_wave_barrier();
  for (int c = lane; c < dh; c += 64) {
    float acc = 0.f;
    for (int j = 0; j <= pos; ++j)
      acc = fmaf(ds[j], load_as_f(qkv, (size_t)(seq0 + j) * 3 * d + d + (size_t)head * dh + c, dt), acc);
    store_from_f(dqkv, (size_t)t * 3 * d + (size_t)head * dh + c, dt, acc * scale);
  }
}

// dK, dV: one wavefront per (key row, head); queries i >= j of the same sequence
__global__ __launch_bounds__(256) void attn_bwd_dkv_simple_kernel(const void* qkv, const void* dO,
                                                                  const float* lse, const float* dvec,
                                                                  int dt, int T, int L, int h, int dh,
                                                                  void* dqkv) {
  extern __shared__ float smem[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long item = (long)blockIdx.x * 4 + wave;
  if (item >= (long)T * h) return;
  const int t = item / h, head = item % h, d = h * dh;
  float* ps = smem + (size_t)wave * (2 * L + 2 * dh);
  float* ds = ps + L;
  float* ks = ds + L;
  float* vs = ks + dh;
  const int pos = t % L, seq0 = t - pos;
  const float scale = 1.0f / sqrtf((float)dh);
  for (int c = lane; c < dh; c += 64) {
    ks[c] = load_as_f(qkv, (size_t)t * 3 * d + d + (size_t)head * dh + c, dt);
    vs[c] = load_as_f(qkv, (size_t)t * 3 * d + 2 * d + (size_t)head * dh + c, dt);
  }
  __builtin_amdgcn_wave_barrier();
  for (int i = pos + lane; i < L; i += 64) {
    const size_t qi = (size_t)(seq0 + i) * 3 * d + (size_t)head * dh;
    const size_t gi = (size_t)(seq0 + i) * d + (size_t)head * dh;
    float s = 0.f, dp = 0.f;
    for (int c = 0; c < dh; ++c) {
      s = fmaf(ks[c], load_as_f(qkv, qi + c, dt), s);
      dp = fmaf(vs[c], load_as_f(dO, gi + c, dt), dp);
    }
    const long it = (long)(seq0 + i) * h + head;
    const float p = expf(s * scale - lse[it]);
    ps[i] = p;
    ds[i] = p * (dp - dvec[it]);
  }
  __builtin_amdgcn_wave_barrier();
  for (int c = lane; c < dh; c += 64) {
    float ak = 0.f, av = 0.f;
    for (int i = pos; i < L; ++i) {
      ak = fmaf(ds[i], load_as_f(qkv, (size_t)(seq0 + i) * 3 * d + (size_t)head * dh + c, dt), ak);
      av = fmaf(ps[i], load_as_f(dO, (size_t)(seq0 + i) * d + (size_t)head * dh + c, dt), av);
    }
    store_from_f(dqkv, (size_t)t * 3 * d + d + (size_t)head * dh + c, dt, ak * scale);
    store_from_f(dqkv, (size_t)t * 3 * d + 2 * d + (size_t)head * dh + c, dt, av);
  }
}

// scatter the new K/V rows into their pages: one thread per (row, head, 8-lane of dh)
__global__ void kv_write_kernel(const void* qkv, int dt, int T, int h, int dh, const int32_t* pos,
                                const int32_t* req, void* k_pool, void* v_pool,
                                const int32_t* block_table, int max_pages, int page) {
  const size_t n = (size_t)T * h * dh;
  const int d = h * dh;
  for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < n;
       idx += (size_t)gridDim.x * blockDim.x) {
    const int c = idx % dh, head = (idx / dh) % h;
    const size_t t = idx / ((size_t)dh * h);
    const int p = pos[t];
    const int pg = block_table[(size_t)req[t] * max_pages + p / page];
    const size_t dst = (((size_t)pg * h + head) * page + p % page) * dh + c;
    const size_t src = t * 3 * d + d + (size_t)head * dh + c;
    if (dt == LS_F32) {
      ((float*)k_pool)[dst] = ((const float*)qkv)[src];
      ((float*)v_pool)[dst] = ((const float*)qkv)[src + d];
    } else {
      ((uint16_t*)k_pool)[dst] = ((const uint16_t*)qkv)[src];
      ((uint16_t*)v_pool)[dst] = ((const uint16_t*)qkv)[src + d];
    }
  }
}

// serving: rotary embedding of q and k (optional) fused with the K/V page write;
// one thread per (row, head, pair i < dh/2)
__global__ void rope_kv_kernel(void* qkv, int dt, int T, int h, int dh, const int32_t* pos,
                               const int32_t* req, const float* table, void* k_pool, void* v_pool,
                               const int32_t* block_table, int max_pages, int page) {
  const int half = dh / 2, d = h * dh;
  const size_t n = (size_t)T * h * half;
  for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < n;
       idx += (size_t)gridDim.x * blockDim.x) {
    const int i = idx % half, head = (idx / half) % h;
    const size_t t = idx / ((size_t)half * h);
    const int p = pos[t];
    const size_t qi = t * 3 * d + (size_t)head * dh + i;
    float ka = load_as_f(qkv, qi + d, dt), kb = load_as_f(qkv, qi + d + half, dt);
    if (table) {
      const float c = table[((size_t)p * half + i) * 2], s = table[((size_t)p * half + i) * 2 + 1];
      const float qa = load_as_f(qkv, qi, dt), qb = load_as_f(qkv, qi + half, dt);
      store_from_f(qkv, qi, dt, qa * c - qb * s);
      store_from_f(qkv, qi + half, dt, qb * c + qa * s);
      const float ra = ka * c - kb * s, rb = kb * c + ka * s;
      ka = ra; kb = rb;
      store_from_f(qkv, qi + d, dt, ka);
      store_from_f(qkv, qi + d + half, dt, kb);
    }
    const int pg = block_table[(size_t)req[t] * max_pages + p / page];
    const size_t dst = (((size_t)pg * h + head) * page + p % page) * dh + i;
    store_from_f(k_pool, dst, dt, ka);
    store_from_f(k_pool, dst + half, dt, kb);
    if (dt == LS_F32) {
      ((float*)v_pool)[dst] = ((const float*)qkv)[qi + 2 * d];
      ((float*)v_pool)[dst + half] = ((const float*)qkv)[qi + 2 * d + half];
    } else {
      ((uint16_t*)v_pool)[dst] = ((const uint16_t*)qkv)[qi + 2 * d];
      ((uint16_t*)v_pool)[dst + half] = ((const uint16_t*)qkv)[qi + 2 * d + half];
    }
  }
}

// The same for 16-bit data, head_dim % 8 == 0: one thread per (row, q / k / v, head, four pairs
// i .. i + 3 < dh / 2), 8-byte accesses.  v and (without a table) q are not rewritten in place.
template <class TH>
__global__ void rope_kv_vec_kernel(TH* qkv, int T, int h, int dh, const int32_t* pos, const int32_t* req,
                                   const float* table, TH* k_pool, TH* v_pool, const int32_t* block_table,
                                   int max_pages, int page) {
  typedef TH V4 __attribute__((ext_vector_type(4)));
  const int half = dh / 2, d = h * dh, q4 = half / 4;
  const size_t n = (size_t)T * 3 * h * q4;
  for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < n; idx += (size_t)gridDim.x * blockDim.x) {
    const int i = (int)(idx % q4) * 4, hp = (int)((idx / q4) % (3 * h));   // hp = part * h + head
    const int part = hp / h, head = hp % h;
    const size_t t = idx / ((size_t)q4 * 3 * h);
    if (part == 0 && !table) continue;
    const size_t qi = t * 3 * d + (size_t)hp * dh + i;
    V4 a = *(const V4*)(qkv + qi), b = *(const V4*)(qkv + qi + half);
    const int p = pos[t];
    if (table && part < 2) {
      const float* tb = table + ((size_t)p * half + i) * 2;   // (cos, sin) pairs
      const f32x4 cs0 = *(const f32x4*)tb, cs1 = *(const f32x4*)(tb + 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float c = e < 2 ? cs0[2 * e] : cs1[2 * (e - 2)], sn = e < 2 ? cs0[2 * e + 1] : cs1[2 * (e - 2) + 1];
        const float xa = to_f(a[e]), xb = to_f(b[e]);
        a[e] = from_f<TH>(xa * c - xb * sn);
        b[e] = from_f<TH>(xb * c + xa * sn);
      }
      *(V4*)(qkv + qi) = a;
      *(V4*)(qkv + qi + half) = b;
    }
    if (part > 0) {
      TH* pool = part == 1 ? k_pool : v_pool;
      const int pg = block_table[(size_t)req[t] * max_pages + p / page];
      const size_t dst = (((size_t)pg * h + head) * page + p % page) * dh + i;
      *(V4*)(pool + dst) = a;
      *(V4*)(pool + dst + half) = b;
    }
  }
}

ls_status set_lds(const void* fn, size_t bytes) {
  LS_REQUIRE(bytes <= 160 * 1024, "attention: context too long for the plain kernel (%zu bytes of LDS)", bytes);
  if (bytes > 48 * 1024)
    LS_CHECK_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  return LS_OK;
}

}  // namespace

extern "C" {

ls_status lsk_attn_fwd_simple(const void* qkv, int dt, int B, int L, int h, int dh, void* o,
                              float* lse, void* stream) {
  LS_REQUIRE(qkv && o && B > 0 && L > 0 && h > 0 && dh > 0, "attn_fwd: bad argument");
  KvView kv{qkv, nullptr, nullptr, nullptr, 0, dt, h, dh, h * dh, 0, 1};
  const int T = B * L;
  const size_t lds = 4 * (size_t)(L + dh) * sizeof(float);
  LS_TRY(set_lds((const void*)attn_fwd_simple_kernel, lds));
  const long items = (long)T * h;
  attn_fwd_simple_kernel<<<(unsigned)((items + 3) / 4), 256, lds, (hipStream_t)stream>>>(
      kv, T, L, nullptr, nullptr, L, o, lse);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

ls_status lsk_attn_bwd_simple(const void* qkv, const void* o, const void* dO, const float* lse,
                              int dt, int B, int L, int h, int dh, void* dqkv, float* dvec,
                              void* stream) {
  LS_REQUIRE(qkv && o && dO && lse && dqkv && dvec && B > 0 && L > 0, "attn_bwd: bad argument");
  const int T = B * L;
  const long items = (long)T * h;
  hipStream_t st = (hipStream_t)stream;
  attn_dvec_kernel<<<(unsigned)((items + 3) / 4), 256, 0, st>>>(o, dO, dt, items, dh, dvec);
  LS_CHECK_LAUNCH();
  size_t lds = 4 * (size_t)(L + 2 * dh) * sizeof(float);
  LS_TRY(set_lds((const void*)attn_bwd_dq_simple_kernel, lds));
  attn_bwd_dq_simple_kernel<<<(unsigned)((items + 3) / 4), 256, lds, st>>>(qkv, dO, lse, dvec, dt, T, L, h,
                                                                          dh, dqkv);
  LS_CHECK_LAUNCH();
  lds = 4 * (size_t)(2 * L + 2 * dh) * sizeof(float);
  LS_TRY(set_lds((const void*)attn_bwd_dkv_simple_kernel, lds));
  attn_bwd_dkv_simple_kernel<<<(unsigned)((items + 3) / 4), 256, lds, st>>>(qkv, dO, lse, dvec, dt, T, L, h,
                                                                           dh, dqkv);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

ls_status lsk_kv_write(const void* qkv, int dt, int T, int h, int dh, const int32_t* pos,
                       const int32_t* req, void* k_pool, void* v_pool, const int32_t* block_table,
                       int max_pages, int page, void* stream) {
  LS_REQUIRE(qkv && pos && req && k_pool && v_pool && block_table && T > 0, "kv_write: bad argument");
  const size_t n = (size_t)T * h * dh;
  size_t g = (n + 255) / 256;
  if (g > 8192) g = 8192;
  kv_write_kernel<<<(unsigned)g, 256, 0, (hipStream_t)stream>>>(qkv, dt, T, h, dh, pos, req, k_pool, v_pool,
                                                                block_table, max_pages, page);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

ls_status lsk_rope_kv_write(void* qkv, int dt, int T, int h, int dh, const int32_t* pos, const int32_t* req,
                            const float* table, void* k_pool, void* v_pool, const int32_t* block_table,
                            int max_pages, int page, void* stream) {
  LS_REQUIRE(qkv && pos && req && k_pool && v_pool && block_table && T > 0 && dh % 2 == 0,
             "rope_kv_write: bad argument");
  if (dt != LS_F32 && dh % 8 == 0 && ((uintptr_t)qkv | (uintptr_t)k_pool | (uintptr_t)v_pool) % 8 == 0 &&
      (!table || (uintptr_t)table % 16 == 0)) {
    const size_t nv = (size_t)T * 3 * h * (dh / 8);
    size_t gv = (nv + 255) / 256;
    if (gv > 8192) gv = 8192;
    if (dt == LS_BF16)
      rope_kv_vec_kernel<bf16_t><<<(unsigned)gv, 256, 0, (hipStream_t)stream>>>(
          (bf16_t*)qkv, T, h, dh, pos, req, table, (bf16_t*)k_pool, (bf16_t*)v_pool, block_table, max_pages, page);
    else
      rope_kv_vec_kernel<f16_t><<<(unsigned)gv, 256, 0, (hipStream_t)stream>>>(
          (f16_t*)qkv, T, h, dh, pos, req, table, (f16_t*)k_pool, (f16_t*)v_pool, block_table, max_pages, page);
    LS_CHECK_LAUNCH();
    return LS_OK;
  }
  const size_t n = (size_t)T * h * (dh / 2);
  size_t g = (n + 255) / 256;
  if (g > 8192) g = 8192;
  rope_kv_kernel<<<(unsigned)g, 256, 0, (hipStream_t)stream>>>(qkv, dt, T, h, dh, pos, req, table, k_pool,
                                                               v_pool, block_table, max_pages, page);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

ls_status lsk_attn_paged_simple(const void* qkv, int dt, int T, int h, int dh, const int32_t* pos,
                                const int32_t* req, const void* k_pool, const void* v_pool,
                                const int32_t* block_table, int max_pages, int page, int max_ctx,
                                void* o, void* stream) {
  LS_REQUIRE(qkv && pos && req && k_pool && v_pool && block_table && o && T > 0 && max_ctx > 0,
             "attn_paged: bad argument");
  KvView kv{qkv, k_pool, v_pool, block_table, 1, dt, h, dh, h * dh, max_pages, page};
  const size_t lds = 4 * (size_t)(max_ctx + dh) * sizeof(float);
  LS_TRY(set_lds((const void*)attn_fwd_simple_kernel, lds));
  const long items = (long)T * h;
  attn_fwd_simple_kernel<<<(unsigned)((items + 3) / 4), 256, lds, (hipStream_t)stream>>>(
      kv, T, 0, pos, req, max_ctx, o, nullptr);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

}  // extern "C"
