// Weight-streaming GEMM for decode batches: Y[M,N] = X[M,K] W[N,K]^T (+ bias)
// (+ residual) with M <= 128 rows.  The weights are read exactly once, straight
// from HBM into MFMA operand registers (no LDS: nothing in W is reused inside a
// workgroup); the few activation rows come through the caches.
//
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

template <class T, int MT>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(SkinnyArgs g) {
  typedef typename vec8<T>::type V8;
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

  constexpr int UN = 4;
  for (int k0 = k_lo; k0 < k_hi; k0 += 32 * UN) {
    V8 wf[UN], xf[UN][MT];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int k = k0 + u * 32 + kc;
      u32x4 w = zero;
      if (n_ok && k < k_hi) w = __builtin_nontemporal_load((const u32x4*)(wrow + k));
      wf[u] = __builtin_bit_cast(V8, w);
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        const int m = t * 16 + r16;
        u32x4 x = zero;
        if (m < g.M && k < k_hi) x = *(const u32x4*)(X + (long)m * g.ldx + k);
        xf[u][t] = __builtin_bit_cast(V8, x);
      }
    }
#pragma unroll
    for (int u = 0; u < UN; ++u)
#pragma unroll
      for (int t = 0; t < MT; ++t) acc[t] = Mfma16<T>::run(wf[u], xf[u][t], acc[t]);
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
  int slab = ((K + ks - 1) / ks + 31) / 32 * 32;
  *ksplit = (K + slab - 1) / slab;
  *kslab = slab;
}

template <class T>
ls_status run(SkinnyArgs g, hipStream_t st) {
  dim3 grid((g.N + 63) / 64, g.ksplit);
  const int mt = (g.M + 15) / 16;
  if (mt <= 1) gemm_skinny_kernel<T, 1><<<grid, 256, 0, st>>>(g);
  else if (mt <= 2) gemm_skinny_kernel<T, 2><<<grid, 256, 0, st>>>(g);
  else if (mt <= 4) gemm_skinny_kernel<T, 4><<<grid, 256, 0, st>>>(g);
  else gemm_skinny_kernel<T, 8><<<grid, 256, 0, st>>>(g);
  LS_CHECK_LAUNCH();
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
  else g.kslab = (K + 31) / 32 * 32;
  hipStream_t st = (hipStream_t)stream;
  return op_dtype == LS_BF16 ? run<bf16_t>(g, st) : run<f16_t>(g, st);
}

}  // extern "C"
