// Bandwidth-bound steps of the block: dtype conversion, LayerNorm / RMSNorm
// forward and backward (fused with the residual-gradient add), rotary
// embedding, GELU / SwiGLU forward and backward, column sums for bias
// gradients.  All statistics and transcendental math are fp32.
#include "common.h"

namespace {

// ------------------------------------------------------------------ convert
__global__ void convert_kernel(const void* src, int sdt, void* dst, int ddt, size_t n, const float* scale) {
  const float sc = scale ? *scale : 1.f;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x)
    store_from_f(dst, i, ddt, load_as_f(src, i, sdt) * sc);
}

// ------------------------------------------------------------ gradient scale
// out[0] = 2^e with max|x| * 2^e in (8, 16], out[1] = 2^-e.  Multiplying the
// upstream gradient by out[0] keeps every 16-bit gradient operand of the
// backward pass well inside the fp16 normal range (the matrix cores flush
// fp16 subnormal inputs); results are multiplied by out[1], which is exact.
// A workgroup's maximum (256 threads) into the global one: one atomic per workgroup - with one per wavefront
// the eight thousand atomics on one address took 90 of the kernel's 100 us at 4096 x 4096 elements.  Values
// that are not finite are left out (the scale then comes from the finite ones).
__device__ __forceinline__ void block_amax(float m, unsigned* amax_bits) {
  __shared__ float wave_m[4];
  m = wave_max(m);
  if ((threadIdx.x & 63) == 0) wave_m[threadIdx.x >> 6] = m <= 3.0e38f ? m : 0.f;
  __syncthreads();
  if (threadIdx.x == 0) {
    m = fmaxf(fmaxf(wave_m[0], wave_m[1]), fmaxf(wave_m[2], wave_m[3]));
    if (__float_as_uint(m) > __hip_atomic_load(amax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
      atomicMax(amax_bits, __float_as_uint(m));
  }
}
__global__ void amax_kernel(const void* x, int dt, size_t n, unsigned* amax_bits) {
  float m = 0.f;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x)
    m = fmaxf(m, fabsf(load_as_f(x, i, dt)));
  block_amax(m, amax_bits);
}
__global__ void scale_reset_kernel(float* out) { out[2] = 0.f; }
__global__ void scale_finish_kernel(float* out) {
  const float a = out[2];
  float e = 0.f;
  if (a > 0.f && a <= 3.0e38f) e = fminf(fmaxf(floorf(log2f(16.f / a)), -24.f), 40.f);
  out[0] = exp2f(e);
  out[1] = exp2f(-e);
}

// ---------------------------------------------------------------- norm fwd
// one 256-thread workgroup per row; the row is read once and held in registers
constexpr int NF_MAXCOL = 32;  // d <= 256 * 32
__global__ __launch_bounds__(256) void norm_fwd_kernel(int kind, const float* x, int d,
                                                       const void* gamma, const void* beta,
                                                       int pdt, float eps, void* h, int hdt,
                                                       float* mean, float* rstd) {
  __shared__ float red[16];
  const size_t row = blockIdx.x;
  const float* xr = x + row * d;
  float v[NF_MAXCOL];
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < NF_MAXCOL; ++c) {
    const int i = threadIdx.x + c * 256;
    v[c] = i < d ? xr[i] : 0.f;
    s += v[c];
  }
  float mu = 0.f;
  if (kind == 0) mu = block_sum(s, red) / d;
  float q = 0.f;
#pragma unroll
  for (int c = 0; c < NF_MAXCOL; ++c) {
    const int i = threadIdx.x + c * 256;
    const float t = i < d ? v[c] - mu : 0.f;
    q += t * t;
  }
  const float var = block_sum(q, red) / d;
  const float r = 1.0f / sqrtf(var + eps);
#pragma unroll
  for (int c = 0; c < NF_MAXCOL; ++c) {
    const int i = threadIdx.x + c * 256;
    if (i < d) {
      float o = (v[c] - mu) * r * load_as_f(gamma, i, pdt);
      if (kind == 0 && beta) o += load_as_f(beta, i, pdt);
      store_from_f(h, row * d + i, hdt, o);
    }
  }
  if (threadIdx.x == 0) {
    if (mean && kind == 0) mean[row] = mu;
    if (rstd) rstd[row] = r;
  }
}

// ---------------------------------------------------------------- norm bwd
// Two kernels.  (1) per-row statistics m1 = mean(dh*gamma), m2 = mean(dh*gamma*xhat),
// one wavefront per row.  (2) dx and the column partial sums: a thread owns 8
// consecutive columns (16-byte loads) and walks NB_ROWS rows, so a workgroup
// covers a 2048-column x NB_ROWS-row patch; its dgamma/dbeta partials go to
// partial[row chunk][2][d] and a last kernel sums them in a fixed order.
constexpr int NB_ROWS = 16;

template <class TD> struct Ld8 {
  static __device__ __forceinline__ void load(const TD* p, float (&v)[8]) {
    typedef typename vec8<TD>::type V8;
    const V8 t = *(const V8*)p;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = to_f(t[i]);
  }
  static __device__ __forceinline__ void store(TD* p, const float (&v)[8]) {
    typedef typename vec8<TD>::type V8;
    V8 t;
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = from_f<TD>(v[i]);
    *(V8*)p = t;
  }
};
template <> struct Ld8<float> {
  static __device__ __forceinline__ void load(const float* p, float (&v)[8]) {
    const f32x4 a = *(const f32x4*)p, b = *(const f32x4*)(p + 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[i] = a[i]; v[4 + i] = b[i]; }
  }
  static __device__ __forceinline__ void store(float* p, const float (&v)[8]) {
    *(f32x4*)p = f32x4{v[0], v[1], v[2], v[3]};
    *(f32x4*)(p + 4) = f32x4{v[4], v[5], v[6], v[7]};
  }
};

// conversion of eight consecutive elements per thread (16-byte accesses on the 16-bit side)
template <class TS, class TD>
__global__ void convert8_kernel(const TS* src, TD* dst, size_t n8, const float* scale) {
  const float sc = scale ? *scale : 1.f;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n8; i += (size_t)gridDim.x * blockDim.x) {
    float v[8];
    Ld8<TS>::load(src + i * 8, v);
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] *= sc;
    Ld8<TD>::store(dst + i * 8, v);
  }
}

// maximum of |x| over eight consecutive elements per thread
template <class TS>
__global__ void amax8_kernel(const TS* x, size_t n8, unsigned* amax_bits) {
  float m = 0.f;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n8; i += (size_t)gridDim.x * blockDim.x) {
    float v[8];
    Ld8<TS>::load(x + i * 8, v);
#pragma unroll
    for (int k = 0; k < 8; ++k) m = fmaxf(m, fabsf(v[k]));
  }
  block_amax(m, amax_bits);
}

// eight consecutive values of a parameter vector whose type is known only at run time
__device__ __forceinline__ void load8_param(const void* p, int c, int dt, float (&v)[8]) {
  if (dt == LS_F32) Ld8<float>::load((const float*)p + c, v);
  else if (dt == LS_BF16) Ld8<bf16_t>::load((const bf16_t*)p + c, v);
  else Ld8<f16_t>::load((const f16_t*)p + c, v);
}

// eight values kept in the form they were loaded in (four registers for a 16-bit type)
template <class TD> struct Raw8 {
  typename vec8<TD>::type t;
  __device__ __forceinline__ void load(const TD* p) { t = *(const typename vec8<TD>::type*)p; }
  __device__ __forceinline__ float get(int i) const { return to_f(t[i]); }
};
template <> struct Raw8<float> {
  f32x4 a, b;
  __device__ __forceinline__ void load(const float* p) { a = *(const f32x4*)p; b = *(const f32x4*)(p + 4); }
  __device__ __forceinline__ float get(int i) const { return i < 4 ? a[i] : b[i - 4]; }
};

// Forward, one wavefront per row (four rows per workgroup): a lane owns eight
// consecutive columns out of every 512, the row stays in registers between the
// statistics and the output, and no LDS or barrier is involved.  Needs
// d % 8 == 0, d <= 512 * NIT and 16-byte aligned rows and parameters.
template <class TH, int NIT>
__global__ __launch_bounds__(256) void norm_fwd_rows_kernel(int kind, const float* x, int T, int d,
                                                            const void* gamma, const void* beta, int pdt,
                                                            float eps, TH* h, float* mean, float* rstd) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= T) return;
  const size_t off = (size_t)row * d;
  float v[NIT][8];
  float s = 0.f;
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int c = lane * 8 + it * 512;
    if (c < d) Ld8<float>::load(x + off + c, v[it]);
    else
#pragma unroll
      for (int i = 0; i < 8; ++i) v[it][i] = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += v[it][i];
  }
  const float mu = kind == 0 ? wave_sum(s) / d : 0.f;
  float q = 0.f;
#pragma unroll
  for (int it = 0; it < NIT; ++it)
    if (lane * 8 + it * 512 < d)
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float t = v[it][i] - mu;
        q += t * t;
      }
  const float r = 1.0f / sqrtf(wave_sum(q) / d + eps);
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int c = lane * 8 + it * 512;
    if (c < d) {
      float gam[8], o[8];
      load8_param(gamma, c, pdt, gam);
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = (v[it][i] - mu) * r * gam[i];
      if (kind == 0 && beta) {
        load8_param(beta, c, pdt, gam);
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] += gam[i];
      }
      Ld8<TH>::store(h + off + c, o);
    }
  }
  if (lane == 0) {
    if (mean && kind == 0) mean[row] = mu;
    if (rstd) rstd[row] = r;
  }
}

// Backward in one pass over the data, one wavefront per row and NB_ROWS rows per
// 512-thread workgroup: the row's dh and xhat stay in registers between the two
// row means and dx, each wave keeps its dgamma / dbeta column sums in registers
// and the eight waves' sums are combined in a fixed order through LDS into
// partial[workgroup][2][d] (RMSNorm leaves the dbeta half unwritten).  Needs d % 8 == 0, d <= 512 * NIT, 16-byte alignment.
template <class TD, int KIND, int NIT>
__global__ __launch_bounds__(512) void norm_bwd_rows_kernel(const TD* dh, const float* x, const float* mean,
                                                            const float* rstd, const void* gamma, int pdt,
                                                            int T, int d, const float* dres, float* dx,
                                                            TD* dx16, float* partial) {
  extern __shared__ float sred[];  // [8][d]
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r0 = blockIdx.x * NB_ROWS, r1 = min(T, r0 + NB_ROWS);
  constexpr int NB = KIND == 0 ? NIT : 1;
  float dg[NIT][8], db[NB][8];
#pragma unroll
  for (int it = 0; it < NIT; ++it)
#pragma unroll
    for (int i = 0; i < 8; ++i) dg[it][i] = 0.f;
#pragma unroll
  for (int it = 0; it < NB; ++it)
#pragma unroll
    for (int i = 0; i < 8; ++i) db[it][i] = 0.f;
  for (int row = r0 + w; row < r1; row += 8) {
    const size_t off = (size_t)row * d;
    const float mu = KIND == 0 ? mean[row] : 0.f, r = rstd[row];
    Raw8<TD> g[NIT];
    float xh[NIT][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = lane * 8 + it * 512;
      if (c < d) {
        float gam[8];
        g[it].load(dh + off + c);
        Ld8<float>::load(x + off + c, xh[it]);
        load8_param(gamma, c, pdt, gam);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float dxh = g[it].get(i) * gam[i];
          xh[it][i] = (xh[it][i] - mu) * r;
          s1 += dxh;
          s2 += dxh * xh[it][i];
        }
      }
    }
    const float m1 = KIND == 0 ? wave_sum(s1) / d : 0.f;
    const float m2 = wave_sum(s2) / d;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = lane * 8 + it * 512;
      if (c < d) {
        float gam[8], o[8];
        load8_param(gamma, c, pdt, gam);
        if (dres) Ld8<float>::load(dres + off + c, o);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float gi = g[it].get(i);
          const float val = r * (gi * gam[i] - m1 - xh[it][i] * m2);
          o[i] = dres ? o[i] + val : val;
          dg[it][i] += gi * xh[it][i];
          if (KIND == 0) db[it][i] += gi;
        }
        Ld8<float>::store(dx + off + c, o);
        if (dx16) Ld8<TD>::store(dx16 + off + c, o);
      }
    }
  }
  float* p = partial + (size_t)blockIdx.x * 2 * d;
#pragma unroll
  for (int pass = 0; pass < (KIND == 0 ? 2 : 1); ++pass) {
    if (pass) __syncthreads();
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = lane * 8 + it * 512;
      if (c < d) Ld8<float>::store(sred + (size_t)w * d + c, pass == 0 ? dg[it] : db[KIND == 0 ? it : 0]);
    }
    __syncthreads();
    for (int c = threadIdx.x * 4; c < d; c += 2048) {
      f32x4 a = *(const f32x4*)(sred + c);
#pragma unroll
      for (int k = 1; k < 8; ++k) a += *(const f32x4*)(sred + (size_t)k * d + c);
      *(f32x4*)(p + pass * d + c) = a;
    }
  }
}

template <class TD>
__global__ __launch_bounds__(256) void norm_bwd_stats_kernel(int kind, const TD* dh, const float* x,
                                                             const float* mean, const float* rstd,
                                                             const void* gamma, int pdt, int T, int d,
                                                             float* stats) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= T) return;
  const size_t off = (size_t)row * d;
  const float mu = kind == 0 ? mean[row] : 0.f, r = rstd[row];
  float s1 = 0.f, s2 = 0.f;
  for (int c = lane * 8; c < d; c += 512) {
    float g[8], xv[8];
    Ld8<TD>::load(dh + off + c, g);
    Ld8<float>::load(x + off + c, xv);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float dxh = g[i] * load_as_f(gamma, c + i, pdt);
      s1 += dxh;
      s2 += dxh * (xv[i] - mu) * r;
    }
  }
  s1 = wave_sum(s1);
  s2 = wave_sum(s2);
  if (lane == 0) {
    stats[2 * row] = s1 / d;
    stats[2 * row + 1] = s2 / d;
  }
}

template <class TD>
__global__ __launch_bounds__(256) void norm_bwd_apply_kernel(int kind, const TD* dh, const float* x,
                                                             const float* mean, const float* rstd,
                                                             const void* gamma, int pdt, int T, int d,
                                                             const float* stats, const float* dres,
                                                             float* dx, TD* dx16, float* partial) {
  const int c = (blockIdx.x * 256 + threadIdx.x) * 8;
  if (c >= d) return;
  float gam[8], dg[8], db[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    gam[i] = load_as_f(gamma, c + i, pdt);
    dg[i] = db[i] = 0.f;
  }
  const int r0 = blockIdx.y * NB_ROWS, r1 = min(T, r0 + NB_ROWS);
  for (int row = r0; row < r1; ++row) {
    const size_t off = (size_t)row * d + c;
    const float mu = kind == 0 ? mean[row] : 0.f, r = rstd[row];
    const float m1 = kind == 0 ? stats[2 * row] : 0.f, m2 = stats[2 * row + 1];
    float g[8], xv[8], o[8];
    Ld8<TD>::load(dh + off, g);
    Ld8<float>::load(x + off, xv);
    if (dres) Ld8<float>::load(dres + off, o);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float xh = (xv[i] - mu) * r;
      const float v = r * (g[i] * gam[i] - m1 - xh * m2);
      o[i] = dres ? o[i] + v : v;
      dg[i] += g[i] * xh;
      db[i] += g[i];
    }
    Ld8<float>::store(dx + off, o);
    if (dx16) Ld8<TD>::store(dx16 + off, o);
  }
  float* p = partial + (size_t)blockIdx.y * 2 * d + c;
  Ld8<float>::store(p, dg);
  Ld8<float>::store(p + d, db);
}

// 32 columns (eight float4 lanes) x 32 row groups per workgroup; the 32 partial sums of a
// column are combined in a fixed order through LDS.  d % 4 == 0.
__global__ __launch_bounds__(256) void norm_bwd_finish_kernel(const float* partial, int nwg, int d, float* dgamma,
                                                              float* dbeta, int accumulate, const float* alpha) {
  __shared__ float sg[32][32], sb[32][32];
  const int cg = threadIdx.x & 7, rg = threadIdx.x >> 3;
  const int i = blockIdx.x * 32 + cg * 4;
  f32x4 g = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
  if (i < d)
    for (int w = rg; w < nwg; w += 32) {
      g += *(const f32x4*)(partial + (size_t)w * 2 * d + i);
      if (dbeta) b += *(const f32x4*)(partial + (size_t)w * 2 * d + d + i);
    }
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    sg[rg][cg * 4 + k] = g[k];
    sb[rg][cg * 4 + k] = b[k];
  }
  __syncthreads();
  const int col = blockIdx.x * 32 + threadIdx.x;
  if (threadIdx.x >= 32 || col >= d) return;
  float tg = 0.f, tb = 0.f;
#pragma unroll
  for (int k = 0; k < 32; ++k) {
    tg += sg[k][threadIdx.x];
    tb += sb[k][threadIdx.x];
  }
  if (alpha) { tg *= *alpha; tb *= *alpha; }
  if (dgamma) dgamma[col] = accumulate ? dgamma[col] + tg : tg;
  if (dbeta) dbeta[col] = accumulate ? dbeta[col] + tb : tb;
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

template <class TD, int KIND, int NIT>
ls_status launch_norm_bwd_rows(const void* dh, const float* x, const float* mean, const float* rstd,
                               const void* gamma, int pdt, int T, int d, const float* dres, float* dx,
                               void* dx16, float* partial, hipStream_t st) {
  static bool attr_set = false;
  const size_t lds = (size_t)8 * d * sizeof(float);
  auto* kern = norm_bwd_rows_kernel<TD, KIND, NIT>;
  if (!attr_set) {
    LS_CHECK_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 8 * 512 * NIT * 4));
    attr_set = true;
  }
  kern<<<(T + NB_ROWS - 1) / NB_ROWS, 512, lds, st>>>((const TD*)dh, x, mean, rstd, gamma, pdt, T, d, dres, dx,
                                                      (TD*)dx16, partial);
  return LS_OK;
}

template <class TD>
ls_status launch_norm_bwd(int kind, const void* dh, const float* x, const float* mean, const float* rstd,
                          const void* gamma, int pdt, int T, int d, const float* dres, float* dx, void* dx16,
                          float* partial, hipStream_t st) {
  // LayerNorm's second set of column sums does not fit the register file beyond 2048 columns
  const bool rows_ok = d <= (kind == 0 ? 2048 : 4096) && aligned16(dh) && aligned16(x) && aligned16(gamma) && aligned16(dx) &&
                       aligned16(partial) && (!dres || aligned16(dres)) && (!dx16 || aligned16(dx16));
  if (rows_ok) {
#define LS_NB(K, N) launch_norm_bwd_rows<TD, K, N>(dh, x, mean, rstd, gamma, pdt, T, d, dres, dx, dx16, partial, st)
    if (kind == 0) return LS_NB(0, 4);
    return d <= 2048 ? LS_NB(1, 4) : LS_NB(1, 8);
#undef LS_NB
  }
  const int nchunk = (T + NB_ROWS - 1) / NB_ROWS;
  float* stats = partial + (size_t)nchunk * 2 * d;
  norm_bwd_stats_kernel<TD><<<(T + 3) / 4, 256, 0, st>>>(kind, (const TD*)dh, x, mean, rstd, gamma, pdt, T, d, stats);
  norm_bwd_apply_kernel<TD><<<dim3((d + 2047) / 2048, nchunk), 256, 0, st>>>(
      kind, (const TD*)dh, x, mean, rstd, gamma, pdt, T, d, stats, dres, dx, (TD*)dx16, partial);
  return LS_OK;
}

template <class TH>
void launch_norm_fwd_rows(int kind, const float* x, int T, int d, const void* gamma, const void* beta, int pdt,
                          float eps, void* h, float* mean, float* rstd, hipStream_t st) {
  const int grid = (T + 3) / 4;
  if (d <= 2048)
    norm_fwd_rows_kernel<TH, 4><<<grid, 256, 0, st>>>(kind, x, T, d, gamma, beta, pdt, eps, (TH*)h, mean, rstd);
  else if (d <= 4096)
    norm_fwd_rows_kernel<TH, 8><<<grid, 256, 0, st>>>(kind, x, T, d, gamma, beta, pdt, eps, (TH*)h, mean, rstd);
  else
    norm_fwd_rows_kernel<TH, 16><<<grid, 256, 0, st>>>(kind, x, T, d, gamma, beta, pdt, eps, (TH*)h, mean, rstd);
}

// -------------------------------------------------------------------- rope
// one thread per (row, head, pair)
__global__ void rope_kernel(void* qkv, int dt, int T, int h, int dh, const int32_t* pos,
                            const float* table, float sign) {
  const int half = dh / 2;
  const size_t n = (size_t)T * 2 * h * half;
  const int d = h * dh;
  for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < n;
       idx += (size_t)gridDim.x * blockDim.x) {
    const int i = idx % half;
    const int hh = (idx / half) % (2 * h);  // q heads then k heads
    const size_t t = idx / ((size_t)half * 2 * h);
    const size_t base = t * 3 * d + (size_t)hh * dh + i;
    const float c = table[((size_t)pos[t] * half + i) * 2];
    const float s = table[((size_t)pos[t] * half + i) * 2 + 1] * sign;
    const float a = load_as_f(qkv, base, dt), b = load_as_f(qkv, base + half, dt);
    store_from_f(qkv, base, dt, a * c - b * s);
    store_from_f(qkv, base + half, dt, b * c + a * s);
  }
}

// ------------------------------------------------------------- activations
__device__ __forceinline__ float gelu_grad_f(float u, int kind) {
  if (kind == LS_ACT_GELU_TANH) {
    const float t = tanhf(kGeluC * (u + 0.044715f * u * u * u));
    return 0.5f * (1.f + t) + 0.5f * u * (1.f - t * t) * kGeluC * (1.f + 3.f * 0.044715f * u * u);
  }
  const float Phi = 0.5f * (1.f + erff(u * 0.70710678118654752f));
  const float phi = 0.3989422804014327f * expf(-0.5f * u * u);
  return Phi + u * phi;
}

__global__ void gelu_fwd_kernel(const void* u, void* g, int dt, size_t n, int kind) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x)
    store_from_f(g, i, dt, gelu_f(load_as_f(u, i, dt), kind));
}
__global__ void gelu_bwd_kernel(const void* dg, const void* u, void* du, int dt, size_t n, int kind) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x)
    store_from_f(du, i, dt, load_as_f(dg, i, dt) * gelu_grad_f(load_as_f(u, i, dt), kind));
}
// SwiGLU: a thread owns 8 consecutive hidden units (16-byte loads of gate, up)
template <class TD>
__global__ void swiglu_fwd_kernel(const TD* gu, TD* a, size_t T, int F) {
  const size_t n8 = T * (size_t)(F / 8);
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n8;
       i += (size_t)gridDim.x * blockDim.x) {
    const size_t t = i / (F / 8), f = (i % (F / 8)) * 8;
    float gt[8], up[8], o[8];
    Ld8<TD>::load(gu + t * 2 * F + f, gt);
    Ld8<TD>::load(gu + t * 2 * F + F + f, up);
#pragma unroll
    for (int k = 0; k < 8; ++k) o[k] = gt[k] / (1.f + __expf(-gt[k])) * up[k];
    Ld8<TD>::store(a + t * F + f, o);
  }
}
template <class TD>
__global__ void swiglu_bwd_kernel(const TD* da, const TD* gu, TD* dgu, size_t T, int F) {
  const size_t n8 = T * (size_t)(F / 8);
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n8;
       i += (size_t)gridDim.x * blockDim.x) {
    const size_t t = i / (F / 8), f = (i % (F / 8)) * 8;
    float gt[8], up[8], g[8], og[8], ou[8];
    Ld8<TD>::load(gu + t * 2 * F + f, gt);
    Ld8<TD>::load(gu + t * 2 * F + F + f, up);
    Ld8<TD>::load(da + t * F + f, g);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const float sg = 1.f / (1.f + __expf(-gt[k]));
      og[k] = g[k] * up[k] * sg * (1.f + gt[k] * (1.f - sg));
      ou[k] = g[k] * gt[k] * sg;
    }
    Ld8<TD>::store(dgu + t * 2 * F + f, og);
    Ld8<TD>::store(dgu + t * 2 * F + F + f, ou);
  }
}

// ------------------------------------------------------------------ colsum
constexpr int CS_ROWS = 128;
__global__ __launch_bounds__(256) void colsum_kernel(const void* x, int dt, int T, int N, long ld,
                                                     float* partial) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  const int r0 = blockIdx.y * CS_ROWS;
  if (n >= N) return;
  float s = 0.f;
  const int r1 = min(T, r0 + CS_ROWS);
  for (int r = r0; r < r1; ++r) s += load_as_f(x, (size_t)r * ld + n, dt);
  partial[(size_t)blockIdx.y * N + n] = s;
}
__global__ void colsum_finish_kernel(const float* partial, int nchunk, int N, float* out, int accumulate,
                                     const float* alpha) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N) return;
  float s = 0.f;
  for (int c = 0; c < nchunk; ++c) s += partial[(size_t)c * N + n];
  if (alpha) s *= *alpha;
  out[n] = accumulate ? out[n] + s : s;
}

inline int grid_for(size_t n, int block = 256, int cap = 256 * 32) {
  size_t g = (n + block - 1) / block;
  return (int)(g < 1 ? 1 : (g > (size_t)cap ? cap : g));
}
bool ok_dtype(int dt) { return dt == LS_F32 || dt == LS_BF16 || dt == LS_F16; }

}  // namespace

extern "C" {

ls_status lsk_convert_scaled(const void* src, int sdt, void* dst, int ddt, size_t n, const float* scale_dev,
                             void* stream) {
  LS_REQUIRE(src && dst && ok_dtype(sdt) && ok_dtype(ddt), "convert: bad argument");
  if (n == 0) return LS_OK;
  hipStream_t st = (hipStream_t)stream;
  if (n % 8 == 0 && ((uintptr_t)src & 15) == 0 && ((uintptr_t)dst & 15) == 0) {
    const size_t n8 = n / 8;
    const int g = grid_for(n8);
#define LS_CV(TS, TD) convert8_kernel<TS, TD><<<g, 256, 0, st>>>((const TS*)src, (TD*)dst, n8, scale_dev)
    if (sdt == LS_F32) { if (ddt == LS_F32) LS_CV(float, float); else if (ddt == LS_BF16) LS_CV(float, bf16_t); else LS_CV(float, f16_t); }
    else if (sdt == LS_BF16) { if (ddt == LS_F32) LS_CV(bf16_t, float); else if (ddt == LS_BF16) LS_CV(bf16_t, bf16_t); else LS_CV(bf16_t, f16_t); }
    else { if (ddt == LS_F32) LS_CV(f16_t, float); else if (ddt == LS_BF16) LS_CV(f16_t, bf16_t); else LS_CV(f16_t, f16_t); }
#undef LS_CV
  } else {
    convert_kernel<<<grid_for(n), 256, 0, st>>>(src, sdt, dst, ddt, n, scale_dev);
  }
  LS_CHECK_LAUNCH();
  return LS_OK;
}
ls_status lsk_convert(const void* src, int sdt, void* dst, int ddt, size_t n, void* stream) {
  return lsk_convert_scaled(src, sdt, dst, ddt, n, nullptr, stream);
}

ls_status lsk_grad_scale(const void* x, int dt, size_t n, float* out3, void* stream) {
  LS_REQUIRE(x && out3 && ok_dtype(dt) && n > 0, "grad_scale: bad argument");
  hipStream_t st = (hipStream_t)stream;
  scale_reset_kernel<<<1, 1, 0, st>>>(out3);
  if (n % 8 == 0 && ((uintptr_t)x & 15) == 0) {
    const int g = grid_for(n / 8, 256, 2048);
    if (dt == LS_F32) amax8_kernel<float><<<g, 256, 0, st>>>((const float*)x, n / 8, (unsigned*)(out3 + 2));
    else if (dt == LS_BF16) amax8_kernel<bf16_t><<<g, 256, 0, st>>>((const bf16_t*)x, n / 8, (unsigned*)(out3 + 2));
    else amax8_kernel<f16_t><<<g, 256, 0, st>>>((const f16_t*)x, n / 8, (unsigned*)(out3 + 2));
  } else {
    amax_kernel<<<grid_for(n, 256, 2048), 256, 0, st>>>(x, dt, n, (unsigned*)(out3 + 2));
  }
  scale_finish_kernel<<<1, 1, 0, st>>>(out3);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

ls_status lsk_norm_fwd(int kind, const float* x, int T, int d, const void* gamma, const void* beta,
                       int pdt, float eps, void* h, int hdt, float* mean, float* rstd, void* stream) {
  LS_REQUIRE(x && gamma && h && T > 0 && d > 0, "norm_fwd: bad argument");
  LS_REQUIRE(kind == 0 || kind == 1, "norm_fwd: kind must be 0 (LayerNorm) or 1 (RMSNorm)");
  LS_REQUIRE(d <= 256 * NF_MAXCOL, "norm_fwd: d_model %d exceeds %d", d, 256 * NF_MAXCOL);
  hipStream_t st = (hipStream_t)stream;
  if (d % 8 == 0 && aligned16(x) && aligned16(h) && aligned16(gamma) && (!beta || aligned16(beta))) {
    if (hdt == LS_F32) launch_norm_fwd_rows<float>(kind, x, T, d, gamma, beta, pdt, eps, h, mean, rstd, st);
    else if (hdt == LS_BF16) launch_norm_fwd_rows<bf16_t>(kind, x, T, d, gamma, beta, pdt, eps, h, mean, rstd, st);
    else launch_norm_fwd_rows<f16_t>(kind, x, T, d, gamma, beta, pdt, eps, h, mean, rstd, st);
  } else {
    norm_fwd_kernel<<<T, 256, 0, st>>>(kind, x, d, gamma, beta, pdt, eps, h, hdt, mean, rstd);
  }
  LS_CHECK_LAUNCH();
  return LS_OK;
}

size_t lsk_norm_bwd_partial_floats(int T, int d) {
  return (size_t)((T + NB_ROWS - 1) / NB_ROWS) * 2 * d + 2 * (size_t)T;
}

ls_status lsk_norm_bwd_scaled(int kind, const void* dh, int dhdt, const float* x, const float* mean,
                              const float* rstd, const void* gamma, int pdt, int T, int d,
                              const float* dres, float* dx, void* dx16, int dx16dt, float* dgamma,
                              float* dbeta, int accumulate, float* partial, const float* alpha_dev,
                              void* stream) {
  LS_REQUIRE(dh && x && rstd && gamma && dx && partial && T > 0 && d > 0, "norm_bwd: bad argument");
  LS_REQUIRE(kind == 1 || mean, "norm_bwd: LayerNorm needs the saved mean");
  LS_REQUIRE(d % 8 == 0, "norm_bwd: d_model must be a multiple of 8");
  LS_REQUIRE(!dx16 || dx16dt == dhdt, "norm_bwd: the 16-bit copy of dx must have the type of dh");
  hipStream_t st = (hipStream_t)stream;
  if (dhdt == LS_F32) LS_TRY(launch_norm_bwd<float>(kind, dh, x, mean, rstd, gamma, pdt, T, d, dres, dx, dx16, partial, st));
  else if (dhdt == LS_BF16) LS_TRY(launch_norm_bwd<bf16_t>(kind, dh, x, mean, rstd, gamma, pdt, T, d, dres, dx, dx16, partial, st));
  else LS_TRY(launch_norm_bwd<f16_t>(kind, dh, x, mean, rstd, gamma, pdt, T, d, dres, dx, dx16, partial, st));
  LS_CHECK_LAUNCH();
  if (dgamma || dbeta) {
    const int nchunk = (T + NB_ROWS - 1) / NB_ROWS;
    norm_bwd_finish_kernel<<<(d + 31) / 32, 256, 0, st>>>(partial, nchunk, d, dgamma,
                                                            kind == 0 ? dbeta : nullptr, accumulate, alpha_dev);
    LS_CHECK_LAUNCH();
  }
  return LS_OK;
}
ls_status lsk_norm_bwd(int kind, const void* dh, int dhdt, const float* x, const float* mean,
                       const float* rstd, const void* gamma, int pdt, int T, int d,
                       const float* dres, float* dx, void* dx16, int dx16dt, float* dgamma,
                       float* dbeta, int accumulate, float* partial, void* stream) {
  return lsk_norm_bwd_scaled(kind, dh, dhdt, x, mean, rstd, gamma, pdt, T, d, dres, dx, dx16, dx16dt, dgamma,
                             dbeta, accumulate, partial, nullptr, stream);
}

ls_status lsk_rope(void* qkv, int dt, int T, int h, int dh, const int32_t* pos, const float* table,
                   float sign, void* stream) {
  LS_REQUIRE(qkv && pos && table && T > 0 && h > 0 && dh > 0 && dh % 2 == 0, "rope: bad argument");
  const size_t n = (size_t)T * 2 * h * (dh / 2);
  rope_kernel<<<grid_for(n), 256, 0, (hipStream_t)stream>>>(qkv, dt, T, h, dh, pos, table, sign);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

ls_status lsk_gelu_fwd(const void* u, void* g, int dt, size_t n, int kind, void* stream) {
  LS_REQUIRE(u && g && n > 0, "gelu_fwd: bad argument");
  gelu_fwd_kernel<<<grid_for(n), 256, 0, (hipStream_t)stream>>>(u, g, dt, n, kind);
  LS_CHECK_LAUNCH();
  return LS_OK;
}
ls_status lsk_gelu_bwd(const void* dg, const void* u, void* du, int dt, size_t n, int kind, void* stream) {
  LS_REQUIRE(dg && u && du && n > 0, "gelu_bwd: bad argument");
  gelu_bwd_kernel<<<grid_for(n), 256, 0, (hipStream_t)stream>>>(dg, u, du, dt, n, kind);
  LS_CHECK_LAUNCH();
  return LS_OK;
}
ls_status lsk_swiglu_fwd(const void* gu, void* a, int dt, int T, int F, void* stream) {
  LS_REQUIRE(gu && a && T > 0 && F > 0, "swiglu_fwd: bad argument");
  LS_REQUIRE(F % 8 == 0, "swiglu_fwd: d_ff must be a multiple of 8");
  const int gr = grid_for((size_t)T * F / 8);
  hipStream_t st = (hipStream_t)stream;
  if (dt == LS_F32) swiglu_fwd_kernel<float><<<gr, 256, 0, st>>>((const float*)gu, (float*)a, T, F);
  else if (dt == LS_BF16) swiglu_fwd_kernel<bf16_t><<<gr, 256, 0, st>>>((const bf16_t*)gu, (bf16_t*)a, T, F);
  else swiglu_fwd_kernel<f16_t><<<gr, 256, 0, st>>>((const f16_t*)gu, (f16_t*)a, T, F);
  LS_CHECK_LAUNCH();
  return LS_OK;
}
ls_status lsk_swiglu_bwd(const void* da, const void* gu, void* dgu, int dt, int T, int F, void* stream) {
  LS_REQUIRE(da && gu && dgu && T > 0 && F > 0, "swiglu_bwd: bad argument");
  LS_REQUIRE(F % 8 == 0, "swiglu_bwd: d_ff must be a multiple of 8");
  const int gr = grid_for((size_t)T * F / 8);
  hipStream_t st = (hipStream_t)stream;
  if (dt == LS_F32) swiglu_bwd_kernel<float><<<gr, 256, 0, st>>>((const float*)da, (const float*)gu, (float*)dgu, T, F);
  else if (dt == LS_BF16) swiglu_bwd_kernel<bf16_t><<<gr, 256, 0, st>>>((const bf16_t*)da, (const bf16_t*)gu, (bf16_t*)dgu, T, F);
  else swiglu_bwd_kernel<f16_t><<<gr, 256, 0, st>>>((const f16_t*)da, (const f16_t*)gu, (f16_t*)dgu, T, F);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

size_t lsk_colsum_partial_floats(int T, int N) { return (size_t)((T + CS_ROWS - 1) / CS_ROWS) * N; }

ls_status lsk_colsum_scaled(const void* x, int dt, int T, int N, long ld, float* out, int accumulate,
                            float* partial, const float* alpha_dev, void* stream) {
  LS_REQUIRE(x && out && partial && T > 0 && N > 0, "colsum: bad argument");
  const int nchunk = (T + CS_ROWS - 1) / CS_ROWS;
  colsum_kernel<<<dim3((N + 255) / 256, nchunk), 256, 0, (hipStream_t)stream>>>(x, dt, T, N, ld, partial);
  LS_CHECK_LAUNCH();
  colsum_finish_kernel<<<(N + 255) / 256, 256, 0, (hipStream_t)stream>>>(partial, nchunk, N, out, accumulate,
                                                                         alpha_dev);
  LS_CHECK_LAUNCH();
  return LS_OK;
}
ls_status lsk_colsum(const void* x, int dt, int T, int N, long ld, float* out, int accumulate,
                     float* partial, void* stream) {
  return lsk_colsum_scaled(x, dt, T, N, ld, out, accumulate, partial, nullptr, stream);
}

}  // extern "C"
