// Dense contractions of the stage:  C[M,N] (+)= A * B^T (+ bias) (+ residual)
//
//   A(m,k), B(n,k) are 16-bit (bf16 or fp16) matrix-core operands, or fp32 for
//   the plain-FMA path.  Each operand is either "k-major" (element (r,k) at
//   r*ld + k: activations X[T,K], weights W[N,K]) or "k-strided" (element
//   (r,k) at k*ld + r).  The three uses in a decoder block:
//     forward     Y  = X  W^T   A k-major,   B k-major
//     input grad  dX = dY W     A k-major,   B k-strided (W[k][n])
//     weight grad dW = dY^T X   A k-strided, B k-strided (contraction over tokens)
//
// MFMA kernel: BM x BN block tile, BK = 64, 256 threads = 4 wavefronts in a
// 2 x 2 grid, each owning a (BM/2) x (BN/2) tile built from 32x32x16 MFMAs.
// Operand tiles are staged in LDS as [row][k] with k contiguous (row stride
// padded by 16 bytes so that the 16-byte fragment reads of 16 consecutive rows
// fall in distinct banks); k-strided operands are transposed in registers on
// the way in (8x8 blocks per thread), so the MFMA loop is the same for all
// three layouts.  Global loads for tile k+1 are in flight while tile k is
// multiplied; two LDS buffers, one barrier per k step.
#include <stdlib.h>
#include <string.h>

#include "common.h"

namespace {

template <class T> struct Mfma;
template <> struct Mfma<bf16_t> {
  static __device__ __forceinline__ f32x16 run(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
};
template <> struct Mfma<f16_t> {
  static __device__ __forceinline__ f32x16 run(f16x8 a, f16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
};

struct GemmArgs {
  int M, N, K;
  const void* A; long lda; int a_kmajor;
  const void* B; long ldb; int b_kmajor;
  void* C; long ldc; int c_dtype;
  const void* bias; int bias_dtype;
  const float* resid; long ldr;
  int accumulate;
  const float* alpha;   // device scalar multiplying the accumulator (null = 1)
};

constexpr int BK = 64;
constexpr int LDS_STRIDE = BK + 8;  // elements; 144 bytes per row

// ---- global -> register staging -------------------------------------------------
// k-major operand tile [ROWS][BK]: ROWS*8 chunks of 16 bytes, ROWS*8/256 per thread.
template <class T, int ROWS>
struct StageK {
  static constexpr int N = ROWS * 8 / 256;
  u32x4 v[N];
  __device__ __forceinline__ void load(const T* base, long ld, int row0, int nrows, int k0, int K) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = threadIdx.x + i * 256;
      const int r = c >> 3, kc = (c & 7) * 8;
      const int gr = row0 + r, gk = k0 + kc;
      u32x4 z = {0u, 0u, 0u, 0u};
      if (gr < nrows && gk < K) z = *(const u32x4*)(base + (long)gr * ld + gk);
      v[i] = z;
    }
  }
  __device__ __forceinline__ void store(T* lds) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = threadIdx.x + i * 256;
      const int r = c >> 3, kc = (c & 7) * 8;
      *(u32x4*)(lds + r * LDS_STRIDE + kc) = v[i];
    }
  }
};

// k-strided operand tile: element (r,k) at k*ld + r.  Each thread owns 8 rows x 8 k
// blocks: eight 16-byte loads (8 rows at one k), transposed in registers, eight
// 16-byte LDS stores (8 k at one row).  ROWS/8 row groups x 8 k groups.
template <class T, int ROWS>
struct StageS {
  static constexpr int NB = ROWS;                // (ROWS/8 row groups) x (8 k groups)
  static constexpr int N = (NB + 255) / 256;     // blocks per thread
  u32x4 v[N][8];
  __device__ __forceinline__ void load(const T* base, long ld, int row0, int nrows, int k0, int K) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int b = threadIdx.x + i * 256;
      const int rg = b % (ROWS / 8), kg = b / (ROWS / 8);
      const int gr = row0 + rg * 8;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int gk = k0 + kg * 8 + j;
        u32x4 z = {0u, 0u, 0u, 0u};
        if (b < NB && gr < nrows && gk < K) z = *(const u32x4*)(base + (long)gk * ld + gr);
        v[i][j] = z;
      }
    }
  }
  __device__ __forceinline__ void store(T* lds) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int b = threadIdx.x + i * 256;
      if (b >= NB) continue;
      const int rg = b % (ROWS / 8), kg = b / (ROWS / 8);
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        // row r of the block: element r of each of the eight k vectors
        u32x4 o;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const uint32_t lo = v[i][2 * p][r >> 1], hi = v[i][2 * p + 1][r >> 1];
          o[p] = (r & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u)
                         : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
        }
        *(u32x4*)(lds + (rg * 8 + r) * LDS_STRIDE + kg * 8) = o;
      }
    }
  }
};

template <class T, int ROWS, bool KMAJOR> struct StageSel { typedef StageK<T, ROWS> type; };
template <class T, int ROWS> struct StageSel<T, ROWS, false> { typedef StageS<T, ROWS> type; };

template <class T, int BM, int BN, bool AK, bool BKM>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmArgs g) {
  constexpr int WM = BM / 2, WN = BN / 2;  // wavefront tile
  constexpr int TM = WM / 32, TN = WN / 32;
  typedef typename vec8<T>::type V8;
  __shared__ __attribute__((aligned(16))) T lds[2][(BM + BN) * LDS_STRIDE];

  // tile order: consecutive workgroups walk down M inside a band of N so that
  // the workgroups resident at one time share few B tiles (L2 reuse)
  const int tiles_m = (g.M + BM - 1) / BM;
  const int tm = blockIdx.x % tiles_m, tn = blockIdx.x / tiles_m;
  const int m0 = tm * BM, n0 = tn * BN;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = (wave >> 1) * WM, wn = (wave & 1) * WN;

  typename StageSel<T, BM, AK>::type sa;
  typename StageSel<T, BN, BKM>::type sb;
  const T* A = (const T*)g.A;
  const T* B = (const T*)g.B;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int nk = (g.K + BK - 1) / BK;
  sa.load(A, g.lda, m0, g.M, 0, g.K);
  sb.load(B, g.ldb, n0, g.N, 0, g.K);
  sa.store(&lds[0][0]);
  sb.store(&lds[0][BM * LDS_STRIDE]);
  __syncthreads();

  const int frow = lane & 31, fk = (lane >> 5) * 8;
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) {
      sa.load(A, g.lda, m0, g.M, (kt + 1) * BK, g.K);
      sb.load(B, g.ldb, n0, g.N, (kt + 1) * BK, g.K);
    }
    const T* la = &lds[cur][0];
    const T* lb = &lds[cur][BM * LDS_STRIDE];
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      V8 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[i] = *(const V8*)(la + (wm + i * 32 + frow) * LDS_STRIDE + ks * 16 + fk);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        fb[j] = *(const V8*)(lb + (wn + j * 32 + frow) * LDS_STRIDE + ks * 16 + fk);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = Mfma<T>::run(fa[i], fb[j], acc[i][j]);
    }
    if (kt + 1 < nk) {
      sa.store(&lds[cur ^ 1][0]);
      sb.store(&lds[cur ^ 1][BM * LDS_STRIDE]);
    }
    __syncthreads();
  }

  // epilogue: 32x32 accumulator tile: column = lane % 32,
  // row = 8 * (e / 4) + 4 * (lane / 32) + e % 4
  const int col_in = lane & 31, row_in = (lane >> 5) * 4;
  const float alpha = g.alpha ? *g.alpha : 1.f;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = n0 + wn + j * 32 + col_in;
    if (n >= g.N) continue;
    const float bv = g.bias ? load_as_f(g.bias, n, g.bias_dtype) : 0.f;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = m0 + wm + i * 32 + 8 * (e >> 2) + row_in + (e & 3);
        if (m >= g.M) continue;
        float v = acc[i][j][e] * alpha + bv;
        if (g.resid) v += g.resid[(long)m * g.ldr + n];
        const long ci = (long)m * g.ldc + n;
        if (g.c_dtype == LS_F32) {
          float* c = (float*)g.C;
          c[ci] = g.accumulate ? c[ci] + v : v;
        } else {
          ((T*)g.C)[ci] = from_f<T>(v);
        }
      }
    }
  }
}

// ---- plain fp32 FMA path (fp32 stage mode; any strides, any sizes) ---------------
// 64x64 tile, 256 threads, 4x4 outputs per thread, BK = 16.
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs g) {
  __shared__ float sa[16][64 + 1], sb[16][64 + 1];
  const float* A = (const float*)g.A;
  const float* B = (const float*)g.B;
  const int tiles_m = (g.M + 63) / 64;
  const int m0 = (blockIdx.x % tiles_m) * 64, n0 = (blockIdx.x / tiles_m) * 64;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const long a_rs = g.a_kmajor ? g.lda : 1, a_ks = g.a_kmajor ? 1 : g.lda;
  const long b_rs = g.b_kmajor ? g.ldb : 1, b_ks = g.b_kmajor ? 1 : g.ldb;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < g.K; k0 += 16) {
    for (int i = threadIdx.x; i < 64 * 16; i += 256) {
      int r, k;
      if (g.a_kmajor) { r = i >> 4; k = i & 15; } else { r = i & 63; k = i >> 6; }
      sa[k][r] = (m0 + r < g.M && k0 + k < g.K) ? A[(long)(m0 + r) * a_rs + (long)(k0 + k) * a_ks] : 0.f;
      if (g.b_kmajor) { r = i >> 4; k = i & 15; } else { r = i & 63; k = i >> 6; }
      sb[k][r] = (n0 + r < g.N && k0 + k < g.K) ? B[(long)(n0 + r) * b_rs + (long)(k0 + k) * b_ks] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { av[i] = sa[k][ty * 4 + i]; bv[i] = sb[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
    __syncthreads();
  }
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m >= g.M || n >= g.N) continue;
      float v = acc[i][j] * (g.alpha ? *g.alpha : 1.f);
      if (g.bias) v += load_as_f(g.bias, n, g.bias_dtype);
      if (g.resid) v += g.resid[(long)m * g.ldr + n];
      float* c = (float*)g.C;
      const long ci = (long)m * g.ldc + n;
      c[ci] = g.accumulate ? c[ci] + v : v;
    }
}

template <class T, int BM, int BN>
ls_status launch_mfma(const GemmArgs& g, hipStream_t st) {
  const int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  dim3 grid(tiles), block(256);
  if (g.a_kmajor && g.b_kmajor) gemm_mfma_kernel<T, BM, BN, true, true><<<grid, block, 0, st>>>(g);
  else if (g.a_kmajor && !g.b_kmajor) gemm_mfma_kernel<T, BM, BN, true, false><<<grid, block, 0, st>>>(g);
  else if (!g.a_kmajor && !g.b_kmajor) gemm_mfma_kernel<T, BM, BN, false, false><<<grid, block, 0, st>>>(g);
  else gemm_mfma_kernel<T, BM, BN, false, true><<<grid, block, 0, st>>>(g);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

template <class T>
ls_status dispatch_mfma(const GemmArgs& g, hipStream_t st) {
  // 256x256 tiles when they still give every compute unit work, else 128x128
  const long big = (long)((g.M + 255) / 256) * ((g.N + 255) / 256);
  if (big >= 200) return launch_mfma<T, 256, 256>(g, st);
  return launch_mfma<T, 128, 128>(g, st);
}

}  // namespace

ls_status gemm_dma_try(int, int, int, int, const void*, long, int, const void*, long, int, void*, long, int,
                       const void*, int, const float*, long, int, const float*, const int32_t*, const float*, int,
                       hipStream_t);

ls_status gemm_dma_splitk_try(int, int, int, int, const void*, long, const void*, long, void*, long, int, const void*,
                              int, const float*, long, float*, size_t, hipStream_t);
ls_status gemm_dma_skinny_try(int, int, int, int, const void*, long, const void*, long, void*, long, int, const void*,
                              int, const float*, long, float*, size_t, hipStream_t);

extern "C" ls_status lsk_gemm_scaled(int op_dtype, int M, int N, int K, const void* A, long lda,
                                     int a_kmajor, const void* B, long ldb, int b_kmajor, void* C,
                                     long ldc, int c_dtype, const void* bias, int bias_dtype,
                                     const float* resid, long ldr, int accumulate,
                                     const float* alpha_dev, void* stream) {
  LS_REQUIRE(M > 0 && N > 0 && K > 0, "gemm: non-positive size M=%d N=%d K=%d", M, N, K);
  LS_REQUIRE(A && B && C, "gemm: null operand");
  LS_REQUIRE(!accumulate || c_dtype == LS_F32, "gemm: accumulate needs an fp32 output");
  LsTimed timed(M >= 256 ? LSK_TIMED_GEMM : LSK_TIMED_DECODE_GEMM, stream);
  GemmArgs g{M, N, K, A, lda, a_kmajor, B, ldb, b_kmajor, C, ldc, c_dtype,
             bias, bias_dtype, resid, ldr, accumulate, alpha_dev};
  hipStream_t st = (hipStream_t)stream;
  if (op_dtype == LS_F32) {
    LS_REQUIRE(c_dtype == LS_F32, "gemm: fp32 operands need an fp32 output");
    const int tiles = ((M + 63) / 64) * ((N + 63) / 64);
    gemm_f32_kernel<<<dim3(tiles), dim3(256), 0, st>>>(g);
    LS_CHECK_LAUNCH();
    return LS_OK;
  }
  // 16-byte vector loads: the contiguous dimension of each operand must be a
  // multiple of 8 elements, as must the leading dimensions and base addresses
  LS_REQUIRE(lda % 8 == 0 && ldb % 8 == 0, "gemm: leading dimensions must be multiples of 8");
  LS_REQUIRE(((uintptr_t)A % 16) == 0 && ((uintptr_t)B % 16) == 0, "gemm: operands must be 16-byte aligned");
  LS_REQUIRE(a_kmajor ? (K % 8 == 0) : (M % 8 == 0), "gemm: A contiguous extent must be a multiple of 8");
  LS_REQUIRE(b_kmajor ? (K % 8 == 0) : (N % 8 == 0), "gemm: B contiguous extent must be a multiple of 8");
  LS_REQUIRE(c_dtype == LS_F32 || c_dtype == op_dtype, "gemm: output type must be fp32 or the operand type");
  if (M >= 256) {
    const ls_status r = gemm_dma_try(op_dtype, M, N, K, A, lda, a_kmajor, B, ldb, b_kmajor, C, ldc, c_dtype, bias,
                                     bias_dtype, resid, ldr, accumulate, alpha_dev, nullptr, nullptr, 0, st);
    if (r != LS_ESTATE) return r;
  }
  if (op_dtype == LS_BF16) return dispatch_mfma<bf16_t>(g, st);
  if (op_dtype == LS_F16) return dispatch_mfma<f16_t>(g, st);
  ls_set_error("gemm: unknown operand dtype %d", op_dtype);
  return LS_EINVAL;
}

extern "C" ls_status lsk_gemm(int op_dtype, int M, int N, int K, const void* A, long lda, int a_kmajor,
                              const void* B, long ldb, int b_kmajor, void* C, long ldc, int c_dtype,
                              const void* bias, int bias_dtype, const float* resid, long ldr,
                              int accumulate, void* stream) {
  return lsk_gemm_scaled(op_dtype, M, N, K, A, lda, a_kmajor, B, ldb, b_kmajor, C, ldc, c_dtype, bias,
                         bias_dtype, resid, ldr, accumulate, nullptr, stream);
}

// Forward-layout product C[M, N] = X[M, K] W[N, K]^T (+ bias, + residual) with a caller workspace:
// shapes that give the chip too few output tiles are computed split along K through `scratch`
// (deterministic: partial sums are added in a fixed order); everything else goes to lsk_gemm.
extern "C" ls_status lsk_gemm_ws(int op_dtype, int M, int N, int K, const void* X, long ldx, const void* W,
                                 long ldw, void* C, long ldc, int c_dtype, const void* bias, int bias_dtype,
                                 const float* resid, long ldr, float* scratch, size_t scratch_floats,
                                 void* stream) {
  LS_REQUIRE(M > 0 && N > 0 && K > 0, "gemm_ws: non-positive size M=%d N=%d K=%d", M, N, K);
  LS_REQUIRE(X && W && C, "gemm_ws: null operand");
  LsTimed timed(M >= 256 ? LSK_TIMED_GEMM : LSK_TIMED_DECODE_GEMM, stream);
  // decode batches (M <= 128): weights stream through LDS in 64 x 128 or 128 x 128 tiles
  if (scratch && (op_dtype == LS_BF16 || op_dtype == LS_F16) && M <= 128 && K % 8 == 0 &&
      ldx % 8 == 0 && ldw % 8 == 0 && (uintptr_t)X % 16 == 0 && (uintptr_t)W % 16 == 0 &&
      (c_dtype == LS_F32 || c_dtype == op_dtype)) {
    const ls_status r = gemm_dma_skinny_try(op_dtype, M, N, K, X, ldx, W, ldw, C, ldc, c_dtype, bias, bias_dtype, resid,
                                            ldr, scratch, scratch_floats, (hipStream_t)stream);
    if (r != LS_ESTATE) return r;
  }
  if (scratch && (op_dtype == LS_BF16 || op_dtype == LS_F16) && M >= 256 && K % 8 == 0 &&
      ldx % 8 == 0 && ldw % 8 == 0 && (uintptr_t)X % 16 == 0 && (uintptr_t)W % 16 == 0 &&
      (c_dtype == LS_F32 || c_dtype == op_dtype)) {
    const ls_status r = gemm_dma_splitk_try(op_dtype, M, N, K, X, ldx, W, ldw, C, ldc, c_dtype, bias, bias_dtype, resid,
                                            ldr, scratch, scratch_floats, (hipStream_t)stream);
    if (r != LS_ESTATE) return r;
  }
  return lsk_gemm(op_dtype, M, N, K, X, ldx, 1, W, ldw, 1, C, ldc, c_dtype, bias, bias_dtype, resid, ldr, 0, stream);
}

ls_status gemm_dma16_swiglu_bwd_try(int, int, int, int, const void*, long, const void*, long, const void*, void*,
                                    hipStream_t);

// Backward through the FFN-down projection and the SwiGLU activation in one step: da = dY W_d (W_d stored
// [d, F]: the input-gradient layout), then d(gate | up) from the saved pre-activations.  With enough
// 256 x 256 tiles the activation's backward runs in the product's epilogue and da is never stored;
// otherwise the product goes to `da_scratch` [T, F] and the element-wise kernel follows.  Same result
// either way, bit for bit.
extern "C" ls_status lsk_gemm_swiglu_bwd(int op_dtype, int T, int F, int d, const void* dY, const void* Wd,
                                         const void* pre, void* grad, void* da_scratch, void* stream) {
  LS_REQUIRE(dY && Wd && pre && grad && da_scratch && T > 0 && F > 0 && d > 0, "gemm_swiglu_bwd: bad argument");
  LS_REQUIRE(op_dtype == LS_BF16 || op_dtype == LS_F16, "gemm_swiglu_bwd: 16-bit operands only");
  LS_REQUIRE(F % 8 == 0, "gemm_swiglu_bwd: d_ff must be a multiple of 8");
  {
    LsTimed timed(T >= 256 ? LSK_TIMED_GEMM : LSK_TIMED_DECODE_GEMM, stream);
    const ls_status r = gemm_dma16_swiglu_bwd_try(op_dtype, T, F, d, dY, d, Wd, F, pre, grad, (hipStream_t)stream);
    if (r != LS_ESTATE) return r;
  }
  LS_TRY(lsk_gemm(op_dtype, T, F, d, dY, d, 1, Wd, F, 0, da_scratch, F, op_dtype, nullptr, 0, nullptr, 0, 0, stream));
  return lsk_swiglu_bwd(da_scratch, pre, grad, op_dtype, T, F, stream);
}

// QKV projection with the rotary embedding of q and k fused into the epilogue
// (head_dim 128, no bias): qkv[T, 3d] = h1 Wqkv^T, then the pairs (i, i + 64) of
// every q and k head of row t rotated by pos[t] * theta^(-2i/128).  Falls back to
// the plain GEMM followed by the in-place rotary kernel for shapes the fused
// epilogue does not cover.
// whether lsk_gemm_qkv_rope applies the rotary embedding in the projection's epilogue at this shape (the
// 256 x 256 tile kernel, which needs enough tiles to fill the chip); otherwise it runs the projection and
// the rotary kernel one after the other
bool gemm_qkv_rope_fuses(int op_dtype, int T, int d, int head_dim) {
  return head_dim == 128 && T >= 256 && (long)((T + 255) / 256) * ((3 * d + 255) / 256) >= 160 &&
         (op_dtype == LS_BF16 || op_dtype == LS_F16);
}

extern "C" ls_status lsk_gemm_qkv_rope(int op_dtype, int T, int d, const void* H, const void* Wqkv, void* qkv,
                                       int n_heads, int head_dim, const int32_t* pos, const float* table,
                                       void* stream) {
  LS_REQUIRE(H && Wqkv && qkv && pos && table && T > 0 && d == n_heads * head_dim, "gemm_qkv_rope: bad argument");
  LsTimed timed(T >= 256 ? LSK_TIMED_GEMM : LSK_TIMED_DECODE_GEMM, stream);
  hipStream_t st = (hipStream_t)stream;
  if (gemm_qkv_rope_fuses(op_dtype, T, d, head_dim)) {
    const ls_status r = gemm_dma_try(op_dtype, T, 3 * d, d, H, d, 1, Wqkv, d, 1, qkv, 3 * d, op_dtype, nullptr, 0,
                                     nullptr, 0, 0, nullptr, pos, table, 2 * d, st);
    if (r != LS_ESTATE) return r;
  }
  LS_TRY(lsk_gemm(op_dtype, T, 3 * d, d, H, d, 1, Wqkv, d, 1, qkv, 3 * d, op_dtype, nullptr, 0, nullptr, 0, 0, stream));
  return lsk_rope(qkv, op_dtype, T, n_heads, head_dim, pos, table, 1.0f, stream);
}
