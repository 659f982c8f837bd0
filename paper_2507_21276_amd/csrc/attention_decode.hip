// Ragged paged decode attention: one query row per request, keys gathered page
// by page from the pool.  Bandwidth-bound: every K and V byte is read once, in
// 16-byte-per-lane loads that cover whole pages contiguously (a page of one
// head is page_size * head_dim 16-bit elements, 4 KB for 16 x 128).
//
// Work split: a workgroup of 4 wavefronts owns one (row, head, split); the
// split's pages are dealt round-robin to the wavefronts.  A lane holds 8
// consecutive head-dimension elements of one token; the q.k dot product is
// finished with a butterfly over the head_dim/8 lanes that share a token.
// Softmax is online per wavefront; the four partial (max, sum, output) triples
// are merged in LDS, and when the context was split across workgroups a second
// kernel merges the per-split partials (deterministic, no atomics).
#include <mutex>

#include "common.h"

namespace {

// Scratch of the entry point that allocates nothing (lsk_attn_paged_noalloc): the per-split partial results
// (output, maximum, sum; head_dim + 2 floats) of contexts split over workgroups.  8 MiB hold 16 131 (row, head,
// split) items at head_dim 128: every launch below 2048 (row, head) pairs (fewer than 4096 items), and e.g. 64
// rows x 32 heads with contexts up to 3584 tokens.  One copy per GPU, held until the process ends; every call
// on a GPU shares it.
constexpr size_t kStaticScratchFloats = (size_t)2 << 20;   // 8 MiB
static __device__ __align__(256) float scratch[kStaticScratchFloats];

template <class T, int DH>
__global__ __launch_bounds__(256) void decode_attn_kernel(
    const T* __restrict__ qkv, const int32_t* __restrict__ pos_arr, const int32_t* __restrict__ req_arr,
    const T* __restrict__ k_pool, const T* __restrict__ v_pool, const int32_t* __restrict__ block_table,
    int max_pages, int page, int h, int nsplit, int chunk_pages, float scale_log2, T* __restrict__ o,
    float* __restrict__ partial) {
  constexpr int LPT = DH / 8;        // lanes per token
  constexpr int TPL = 64 / LPT;      // tokens per wave-wide load (1 KB)
  typedef typename vec8<T>::type V8;
  __shared__ float s_m[4], s_l[4];
  __shared__ float s_o[4][DH];

  const int t = blockIdx.x / h, head = blockIdx.x % h, split = blockIdx.y;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int sub = lane % LPT;        // which 8-element chunk of the head dimension
  const int tok_in = lane / LPT;     // token within a load
  const int d = h * DH;
  const int nkeys = pos_arr[t] + 1;
  const int req = req_arr[t];
  const int npages = (nkeys + page - 1) / page;
  // chunk_pages > 0: every split covers that many pages whatever the request's length (splits past its end
  // are empty), so that the work items of a ragged batch are all about the same size; otherwise the
  // request's own pages are divided evenly over the splits
  const int per = chunk_pages > 0 ? chunk_pages : (npages + nsplit - 1) / nsplit;
  const int p_lo = split * per, p_hi = min(npages, p_lo + per);
  if (p_lo >= p_hi && nsplit > 1) {   // an empty split: only its marker is read by the merge
    if (threadIdx.x == 0) {
      float* pp = partial + (((long)t * h + head) * nsplit + split) * (DH + 2);
      pp[DH] = -INFINITY;
      pp[DH + 1] = 0.f;
    }
    return;
  }
  const int loads_per_page = page / TPL;   // page * DH * 2 bytes / 1 KB
  const int32_t* bt = block_table + (long)req * max_pages;

  float q[8];
  {
    const V8 qv = *(const V8*)(qkv + (long)t * 3 * d + (long)head * DH + sub * 8);
#pragma unroll
    for (int i = 0; i < 8; ++i) q[i] = to_f(qv[i]) * scale_log2;
  }
  float m = -INFINITY, l = 0.f, acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;

  for (int p = p_lo + wave; p < p_hi; p += 4) {
    const long base = ((long)bt[p] * h + head) * page * DH;
    const int tok0 = p * page;
    // up to 4 loads per page (page 16, DH 128); generic in page size via the loop
    for (int i0 = 0; i0 < loads_per_page; i0 += 4) {
      V8 kv[4], vv[4];
      float s[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (i0 + i < loads_per_page) {
          kv[i] = __builtin_nontemporal_load((const V8*)(k_pool + base + (long)(i0 + i) * 512 + lane * 8));
          vv[i] = __builtin_nontemporal_load((const V8*)(v_pool + base + (long)(i0 + i) * 512 + lane * 8));
        }
      float mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        s[i] = -INFINITY;
        if (i0 + i < loads_per_page) {
          float a = 0.f;
#pragma unroll
          for (int c = 0; c < 8; ++c) a = fmaf(q[c], to_f(kv[i][c]), a);
#pragma unroll
          for (int off = 1; off < LPT; off <<= 1) a += __shfl_xor(a, off, 64);
          const int tok = tok0 + (i0 + i) * TPL + tok_in;
          s[i] = tok < nkeys ? a : -INFINITY;
          mx = fmaxf(mx, s[i]);
        }
      }
#pragma unroll
      for (int off = LPT; off < 64; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
      const float m_new = fmaxf(m, mx);   // finite: token tok0 of a visited page is always < nkeys
      const float alpha = __builtin_amdgcn_exp2f(m - m_new);
      l *= alpha;
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[c] *= alpha;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (i0 + i < loads_per_page) {
          const float pr = __builtin_amdgcn_exp2f(s[i] - m_new);
          l += pr;
          // slots of the last page beyond the context were never written: whatever bit patterns they hold
          // (NaN, infinity) must not reach the sum through 0 * x
          if (s[i] == -INFINITY) vv[i] = V8{};
#pragma unroll
          for (int c = 0; c < 8; ++c) acc[c] = fmaf(pr, to_f(vv[i][c]), acc[c]);
        }
      m = m_new;
    }
  }
  // sum over the token groups of the wavefront (lanes with equal `sub`)
#pragma unroll
  for (int off = LPT; off < 64; off <<= 1) {
    l += __shfl_xor(l, off, 64);
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] += __shfl_xor(acc[c], off, 64);
  }
  if (lane < LPT) {
#pragma unroll
    for (int c = 0; c < 8; ++c) s_o[wave][lane * 8 + c] = acc[c];
  }
  if (lane == 0) { s_m[wave] = m; s_l[wave] = l; }
  __syncthreads();
  if (threadIdx.x < DH) {
    const float mm = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));
    float ll = 0.f, oo = 0.f;
    if (mm != -INFINITY) {
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float f = __builtin_amdgcn_exp2f(s_m[w] - mm);   // 0 for a wavefront that saw no page
        ll += s_l[w] * f;
        oo += s_o[w][threadIdx.x] * f;
      }
    }
    if (nsplit == 1) {
      o[(long)t * d + (long)head * DH + threadIdx.x] = from_f<T>(oo / ll);
    } else {
      float* pp = partial + (((long)t * h + head) * nsplit + split) * (DH + 2);
      pp[threadIdx.x] = oo;
      if (threadIdx.x == 0) { pp[DH] = mm; pp[DH + 1] = ll; }
    }
  }
}

template <class T, int DH>
__global__ void decode_merge_kernel(const float* __restrict__ partial, int nsplit, int h, T* __restrict__ o) {
  const long item = blockIdx.x;   // t * h + head
  const float* pp = partial + item * nsplit * (DH + 2);
  float mm = -INFINITY;
  for (int s = 0; s < nsplit; ++s) mm = fmaxf(mm, pp[s * (DH + 2) + DH]);
  float ll = 0.f, oo = 0.f;
  for (int s = 0; s < nsplit; ++s) {
    const float ms = pp[s * (DH + 2) + DH];
    if (ms == -INFINITY) continue;   // an empty split
    const float f = __builtin_amdgcn_exp2f(ms - mm);
    ll += pp[s * (DH + 2) + DH + 1] * f;
    oo += pp[s * (DH + 2) + threadIdx.x] * f;
  }
  const long t = item / h, head = item % h;
  o[t * (long)h * DH + head * DH + threadIdx.x] = from_f<T>(oo / ll);
}

// Pages per split when the batch alone fills the chip (2048 or more (row, head) pairs): contexts of a ragged
// batch differ by an order of magnitude, and with one workgroup per pair the compute units that drew the
// long ones are still streaming when the others have finished.  Chunks of 512 tokens make every work item
// about the same size; the partial results cost (dh + 2) floats per chunk against 512 * dh * 4 bytes read.
constexpr int kChunkTokens = 512;

int pick_nsplit(long items, int max_ctx, int page, int* chunk_pages) {
  // enough workgroups to fill 256 compute units a few times over, but never
  // fewer than 8 pages per split
  const int max_pages = (max_ctx + page - 1) / page;
  *chunk_pages = 0;
  if (items >= 2048) {
    const int cp = kChunkTokens / page > 0 ? kChunkTokens / page : 1;
    if (max_pages <= cp + cp / 2) return 1;
    const int ns = (max_pages + cp - 1) / cp;
    if (ns > 32) return 1;
    *chunk_pages = cp;
    return ns;
  }
  int ns = (int)((2048 + items - 1) / items);
  const int cap = max_pages / 8 > 1 ? max_pages / 8 : 1;
  if (ns > cap) ns = cap;
  if (ns > 32) ns = 32;
  return ns < 1 ? 1 : ns;
}

template <class T, int DH>
ls_status launch(const void* qkv, int T_, int h, const int32_t* pos, const int32_t* req, const void* kp,
                 const void* vp, const int32_t* bt, int max_pages, int page, int max_ctx, void* o,
                 float* scratch, hipStream_t st) {
  const long items = (long)T_ * h;
  int chunk_pages = 0;
  const int ns = scratch ? pick_nsplit(items, max_ctx, page, &chunk_pages) : 1;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)DH);
  decode_attn_kernel<T, DH><<<dim3((unsigned)items, ns), 256, 0, st>>>(
      (const T*)qkv, pos, req, (const T*)kp, (const T*)vp, bt, max_pages, page, h, ns, chunk_pages, scale_log2,
      (T*)o, scratch);
  LS_CHECK_LAUNCH();
  if (ns > 1) {
    decode_merge_kernel<T, DH><<<(unsigned)items, DH, 0, st>>>(scratch, ns, h, (T*)o);
    LS_CHECK_LAUNCH();
  }
  return LS_OK;
}

// Device address of `scratch` on the current GPU.  The array's name is a host-side stand-in, not a device
// address: the address comes from hipGetSymbolAddress, once per device with that device current (each GPU has
// its own copy at its own address), and only that pointer is handed to kernels.
ls_status static_scratch(float** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static float* ptrs[kMaxDevices] = {};
  int dev = -1;
  LS_CHECK_HIP(hipGetDevice(&dev));
  LS_REQUIRE(dev >= 0 && dev < kMaxDevices, "attn_paged_noalloc: device index %d outside 0..%d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(mu);
  if (!ptrs[dev]) {
    float* p = nullptr;
    LS_CHECK_HIP(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
    LS_REQUIRE(p != nullptr, "attn_paged_noalloc: the scratch array has no device address");
    ptrs[dev] = p;
  }
  *out = ptrs[dev];
  return LS_OK;
}

}  // namespace

extern "C" {

size_t lsk_attn_decode_scratch_floats(int T, int h, int dh, int max_ctx, int page) {
  int chunk_pages = 0;
  const int ns = pick_nsplit((long)T * h, max_ctx, page, &chunk_pages);
  return ns > 1 ? (size_t)T * h * ns * (dh + 2) : 0;
}

ls_status lsk_attn_decode(const void* qkv, int dt, int T, int h, int dh, const int32_t* pos,
                          const int32_t* req, const void* k_pool, const void* v_pool,
                          const int32_t* block_table, int max_pages, int page, int max_ctx, void* o,
                          float* scratch, void* stream) {
  LsTimed timed(LSK_TIMED_DECODE_ATTN, stream);
  LS_REQUIRE(qkv && pos && req && k_pool && v_pool && block_table && o && T > 0 && max_ctx > 0,
             "attn_decode: bad argument");
  LS_REQUIRE(dt == LS_BF16 || dt == LS_F16, "attn_decode: 16-bit pools only");
  LS_REQUIRE(dh == 64 || dh == 128, "attn_decode: head_dim must be 64 or 128");
  LS_REQUIRE(page * dh % 512 == 0, "attn_decode: a page of one head must be a multiple of 1 KB");
  LS_REQUIRE((long)T * h <= 0x7fffffffL, "attn_decode: too many (row, head) pairs");
  hipStream_t st = (hipStream_t)stream;
  if (dt == LS_BF16)
    return dh == 64 ? launch<bf16_t, 64>(qkv, T, h, pos, req, k_pool, v_pool, block_table, max_pages, page, max_ctx, o, scratch, st)
                    : launch<bf16_t, 128>(qkv, T, h, pos, req, k_pool, v_pool, block_table, max_pages, page, max_ctx, o, scratch, st);
  return dh == 64 ? launch<f16_t, 64>(qkv, T, h, pos, req, k_pool, v_pool, block_table, max_pages, page, max_ctx, o, scratch, st)
                  : launch<f16_t, 128>(qkv, T, h, pos, req, k_pool, v_pool, block_table, max_pages, page, max_ctx, o, scratch, st);
}

// lsk_attn_paged with impl 1 for callers that cannot allocate: the split partials go to the library's static
// per-GPU scratch instead of a caller buffer.  No allocation of any kind happens in this call.
ls_status lsk_attn_paged_noalloc(const void* qkv, int dt, int T, int h, int dh, const int32_t* pos, const int32_t* req,
                                 const void* k_pool, const void* v_pool, const int32_t* block_table, int max_pages,
                                 int page, int max_ctx, void* o, void* stream) {
  LS_REQUIRE(T > 0 && h > 0 && max_ctx > 0 && page > 0, "attn_paged_noalloc: non-positive size");
  LS_REQUIRE(dh == 64 || dh == 128, "attn_paged_noalloc: head_dim must be 64 or 128");
  const size_t need = lsk_attn_decode_scratch_floats(T, h, dh, max_ctx, page);
  LS_REQUIRE(need <= kStaticScratchFloats,
             "attn_paged_noalloc: this launch needs %zu scratch floats, the static scratch holds %zu", need,
             kStaticScratchFloats);
  float* sp = nullptr;
  LS_TRY(static_scratch(&sp));
  return lsk_attn_decode(qkv, dt, T, h, dh, pos, req, k_pool, v_pool, block_table, max_pages, page, max_ctx, o, sp,
                         stream);
}

}  // extern "C"
