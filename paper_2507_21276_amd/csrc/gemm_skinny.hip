// Weight-streaming GEMM for decode batches: Y[M,N] = X[M,K] W[N,K]^T (+ bias)
// (+ residual) with M <= 128 rows.  The weights are read exactly once, straight
// from HBM into MFMA operand registers (no LDS: nothing in W is reused inside a
// workgroup); the few activation rows come through the caches.
//
// The activation slab a workgroup needs is staged in LDS in double-buffered chunks.
// 16x16x32 MFMA with W as the A operand: a lane holds 8 consecutive k of one
// weight row, four lanes share a row, so one wave-wide load covers 16 rows x
// 64 contiguous bytes and two successive k steps consume whole 128-byte lines.
// A workgroup = 4 wavefronts x 16 weight rows; the grid is (N/64) x ksplit,
// ksplit slabs of K chosen so that a few hundred workgroups are in flight even
// for the square projections.  Split results go to an fp32 scratch and are
// summed in a fixed order by a second kernel that also applies the epilogue.
#include "common.h"

namespace {

template <class T> struct Mfma16;
template <> struct Mfma16<bf16_t> {
  static __device__ __forceinline__ f32x4 run(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
};
template <> struct Mfma16<f16_t> {
  static __device__ __forceinline__ f32x4 run(f16x8 a, f16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
  }
};

struct SkinnyArgs {
  int M, N, K, kslab, ksplit;
  const void* X; long ldx;
  const void* W; long ldw;
  void* C; long ldc; int c_dtype;
  const void* bias; int bias_dtype;
  const float* resid; long ldr;
  float* partial;   // [ksplit][M][N] when ksplit > 1
};

template <class T>
__device__ __forceinline__ void epilogue_store(const SkinnyArgs& g, int m, int n, float v) {
  if (g.bias) v += load_as_f(g.bias, n, g.bias_dtype);
  if (g.resid) v += g.resid[(long)m * g.ldr + n];
  if (g.c_dtype == LS_F32) ((float*)g.C)[(long)m * g.ldc + n] = v;
  else ((T*)g.C)[(long)m * g.ldc + n] = from_f<T>(v);
}

// KC = k extent of one activation chunk staged in LDS (two buffers of
// [MT*16][KC + 8] elements).  The weight stream is a rolling prefetch: as soon as
// the MFMAs of k step u have consumed their weight fragment, the same registers
// receive the load for step u of the next chunk, so every wavefront keeps KC/32
// 16-byte weight loads per lane in flight at all times.
template <class T, int MT, int KC>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(SkinnyArgs g) {
  typedef typename vec8<T>::type V8;
  constexpr int MP = MT * 16, XSTR = KC + 8;
  constexpr int NSTEP = KC / 32;                 // MFMA k steps per chunk
  constexpr int XLD = MP * (KC / 8) / 256;       // 16-byte activation loads per thread per chunk
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* xs = (T*)smem_raw;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r16 = lane & 15, kc = (lane >> 4) * 8;
  const int n = blockIdx.x * 64 + wave * 16 + r16;
  const int k_lo = blockIdx.y * g.kslab, k_hi = min(g.K, k_lo + g.kslab);
  const T* W = (const T*)g.W;
  const T* X = (const T*)g.X;
  const bool n_ok = n < g.N;
  const T* wrow = W + (long)(n_ok ? n : 0) * g.ldw;
  f32x4 acc[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  const u32x4 zero = {0u, 0u, 0u, 0u};

  auto load_w = [&](int k0, int u) -> V8 {
    const int k = k0 + u * 32 + kc;
    u32x4 w = zero;
    if (n_ok && k < k_hi) w = __builtin_nontemporal_load((const u32x4*)(wrow + k));
    return __builtin_bit_cast(V8, w);
  };
  u32x4 xr[XLD];
  auto load_x = [&](int k0) {
#pragma unroll
    for (int i = 0; i < XLD; ++i) {
      const int c = threadIdx.x + i * 256;
      const int m = c / (KC / 8), k = k0 + (c % (KC / 8)) * 8;
      u32x4 x = zero;
      if (m < g.M && k < k_hi) x = *(const u32x4*)(X + (long)m * g.ldx + k);
      xr[i] = x;
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int i = 0; i < XLD; ++i) {
      const int c = threadIdx.x + i * 256;
      const int m = c / (KC / 8), kk = (c % (KC / 8)) * 8;
      *(u32x4*)(xs + buf * (MP * XSTR) + m * XSTR + kk) = xr[i];
    }
  };

  // weight fragments of two chunks are always in flight (rolling prefetch, distance 2 chunks)
  V8 wf[2][NSTEP];
#pragma unroll
  for (int u = 0; u < NSTEP; ++u) wf[0][u] = load_w(k_lo, u);
#pragma unroll
  for (int u = 0; u < NSTEP; ++u) wf[1][u] = load_w(k_lo + KC, u);
  load_x(k_lo);
  store_x(0);
  __syncthreads();
  int buf = 0;
  for (int k0 = k_lo; k0 < k_hi; k0 += 2 * KC) {
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int kc0 = k0 + half * KC;
      if (kc0 < k_hi) {     // uniform across the workgroup
        const bool more = kc0 + KC < k_hi;
        if (more) load_x(kc0 + KC);
        const T* xb = xs + buf * (MP * XSTR);
#pragma unroll
        for (int u = 0; u < NSTEP; ++u) {
          const V8 w = wf[half][u];
          wf[half][u] = load_w(kc0 + 2 * KC, u);   // zero-filled past the slab
#pragma unroll
          for (int t = 0; t < MT; ++t) {
            const V8 xf = *(const V8*)(xb + (t * 16 + r16) * XSTR + u * 32 + kc);
            acc[t] = Mfma16<T>::run(w, xf, acc[t]);
          }
        }
        if (more) store_x(buf ^ 1);   // the other buffer was last read one chunk ago
        __syncthreads();
        buf ^= 1;
      }
    }
  }
  // accumulator: column (lane % 16) = batch row m, rows 4 * (lane / 16) + e = weight row
  const int nb = blockIdx.x * 64 + wave * 16 + (lane >> 4) * 4;
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    const int m = t * 16 + r16;
    if (m >= g.M) continue;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int nn = nb + e;
      if (nn >= g.N) continue;
      if (g.ksplit == 1) epilogue_store<T>(g, m, nn, acc[t][e]);
      else g.partial[((long)blockIdx.y * g.M + m) * g.N + nn] = acc[t][e];
    }
  }
}

template <class T>
__global__ void skinny_reduce_kernel(SkinnyArgs g) {
  const long total = (long)g.M * g.N;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    float v = 0.f;
    for (int s = 0; s < g.ksplit; ++s) v += g.partial[(long)s * total + i];
    epilogue_store<T>(g, (int)(i / g.N), (int)(i % g.N), v);
  }
}

void plan(int N, int K, int* ksplit, int* kslab) {
  const int bn = (N + 63) / 64;
  int ks = (640 + bn - 1) / bn;
  if (ks > 8) ks = 8;
  while (ks > 1 && K / ks < 512) --ks;
  if (ks < 1) ks = 1;
  int slab = ((K + ks - 1) / ks + 511) / 512 * 512;   // whole LDS chunks
  *ksplit = (K + slab - 1) / slab;
  *kslab = slab;
}

template <class T, int MT, int KC>
ls_status launch_one(const SkinnyArgs& g, dim3 grid, hipStream_t st) {
  const size_t lds = 2 * (size_t)MT * 16 * (KC + 8) * sizeof(T);
  static bool attr_set = false;   // per instantiation; the attribute is idempotent
  if (lds > 48 * 1024 && !attr_set) {
    LS_CHECK_HIP(hipFuncSetAttribute((const void*)gemm_skinny_kernel<T, MT, KC>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set = true;
  }
  gemm_skinny_kernel<T, MT, KC><<<grid, 256, lds, st>>>(g);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

template <class T>
ls_status run(SkinnyArgs g, hipStream_t st) {
  dim3 grid((g.N + 63) / 64, g.ksplit);
  const int mt = (g.M + 15) / 16;
  if (mt <= 1) LS_TRY((launch_one<T, 1, 512>(g, grid, st)));
  else if (mt <= 2) LS_TRY((launch_one<T, 2, 512>(g, grid, st)));
  else if (mt <= 4) LS_TRY((launch_one<T, 4, 256>(g, grid, st)));
  else LS_TRY((launch_one<T, 8, 128>(g, grid, st)));
  if (g.ksplit > 1) {
    const long total = (long)g.M * g.N;
    skinny_reduce_kernel<T><<<(unsigned)((total + 255) / 256), 256, 0, st>>>(g);
    LS_CHECK_LAUNCH();
  }
  return LS_OK;
}

}  // namespace

extern "C" {

size_t lsk_gemm_skinny_scratch_floats(int M, int N, int K) {
  int ks, slab;
  plan(N, K, &ks, &slab);
  return ks > 1 ? (size_t)ks * M * N : 0;
}

ls_status lsk_gemm_skinny(int op_dtype, int M, int N, int K, const void* X, long ldx, const void* W,
                          long ldw, void* C, long ldc, int c_dtype, const void* bias, int bias_dtype,
                          const float* resid, long ldr, float* scratch, void* stream) {
  LS_REQUIRE(M > 0 && M <= 128 && N > 0 && K > 0, "gemm_skinny: need 0 < M <= 128 (M=%d N=%d K=%d)", M, N, K);
  LS_REQUIRE(X && W && C, "gemm_skinny: null operand");
  LS_REQUIRE(op_dtype == LS_BF16 || op_dtype == LS_F16, "gemm_skinny: 16-bit operands only");
  LS_REQUIRE(K % 8 == 0 && ldx % 8 == 0 && ldw % 8 == 0, "gemm_skinny: K and leading dimensions must be multiples of 8");
  LS_REQUIRE(((uintptr_t)X % 16) == 0 && ((uintptr_t)W % 16) == 0, "gemm_skinny: operands must be 16-byte aligned");
  LS_REQUIRE(c_dtype == LS_F32 || c_dtype == op_dtype, "gemm_skinny: output type must be fp32 or the operand type");
  SkinnyArgs g{M, N, K, K, 1, X, ldx, W, ldw, C, ldc, c_dtype, bias, bias_dtype, resid, ldr, scratch};
  if (scratch) plan(N, K, &g.ksplit, &g.kslab);
  else g.kslab = (K + 511) / 512 * 512;
  hipStream_t st = (hipStream_t)stream;
  return op_dtype == LS_BF16 ? run<bf16_t>(g, st) : run<f16_t>(g, st);
}

}  // extern "C"
