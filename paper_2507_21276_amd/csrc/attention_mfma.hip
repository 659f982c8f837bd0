// Matrix-core causal attention for training (contiguous sequences), 16-bit
// operands, fp32 softmax statistics and accumulation.
//
// Forward.  A workgroup (4 wavefronts) owns BQ = 4*QT*32 consecutive query rows
// of one (sequence, head); each wavefront owns QT 32-row query tiles.  K/V are
// walked in tiles of 64 keys staged in LDS (K as [key][dh], V transposed to
// [dh][key] on the way in).  Both products are computed *transposed* so that a
// lane always holds data of one query (its column):
//     S^T = K Q^T   (A = K rows, B = Q)      lane: query = lane%32, 16 keys/tile
//     O^T = V^T P^T (A = V^T rows, B = P^T)  lane: query = lane%32, dh rows
// The online-softmax maximum, sum and rescale factor are therefore per-lane
// scalars (one exchange with lane^32 for the maximum), and the exponentials of
// S^T feed the second product straight from registers.  K rows are fetched in
// the order pi(r) = r with bits 2 and 3 swapped, which makes the 8 values a lane
// holds per 16-key step consecutive keys, i.e. exactly the B-operand layout.
//
// Backward (dQ, dK, dV) follows the same scheme; see flash_bwd_kernel.
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <queue>
#include <type_traits>

#include "common.h"

namespace {

template <class T> struct Mma;
template <> struct Mma<bf16_t> {
  typedef bf16x8 V8;
  typedef bf16x4 V4;
  static __device__ __forceinline__ f32x16 run(V8 a, V8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
};
template <> struct Mma<f16_t> {
  typedef f16x8 V8;
  typedef f16x4 V4;
  static __device__ __forceinline__ f32x16 run(V8 a, V8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
};

constexpr int KT = 64;  // keys per tile

__device__ __forceinline__ int pi_row(int r) {  // swap bits 2 and 3
  return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1);
}

// 8x8 transpose of 16-bit elements held as eight 16-byte rows
__device__ __forceinline__ void transpose8x8(const u32x4 (&in)[8], u32x4 (&out)[8]) {
#pragma unroll
  for (int r = 0; r < 8; ++r) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const uint32_t lo = in[2 * p][r >> 1], hi = in[2 * p + 1][r >> 1];
      out[r][p] = (r & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
    }
  }
}

// Where the keys of one (sequence, head) live: rows of the training qkv buffer,
// or pages of the serving pool found through the request's block table.
template <class T>
struct KvContig {
  const T* k; const T* v; long ld;
  __device__ __forceinline__ const T* krow(int key) const { return k + (long)key * ld; }
  __device__ __forceinline__ const T* vrow(int key) const { return v + (long)key * ld; }
};
template <class T>
struct KvPaged {
  const T* k; const T* v; const int32_t* bt; int page, h, head, dh;
  __device__ __forceinline__ long off(int key) const {
    return (((long)bt[key / page] * h + head) * page + key % page) * dh;
  }
  __device__ __forceinline__ const T* krow(int key) const { return k + off(key); }
  __device__ __forceinline__ const T* vrow(int key) const { return v + off(key); }
};

// K tile [KT][DH] (row stride DH+8) and V^T tile [DH][KT] (row stride KT+8)
template <class T, int DH>
struct KvStage {
  static constexpr int KCH = KT * DH / 8 / 256;  // 16-byte chunks of K per thread
  static constexpr int VBLK = 8 * (DH / 8);      // 8x8 blocks of V (one per thread below VBLK)
  u32x4 k[KCH];
  u32x4 v[8];
  template <class SRC>
  __device__ __forceinline__ void load(const SRC& src, int key0, int nkeys) {
#pragma unroll
    for (int i = 0; i < KCH; ++i) {
      const int c = threadIdx.x + i * 256;
      const int r = c / (DH / 8), col = (c % (DH / 8)) * 8;
      u32x4 z = {0u, 0u, 0u, 0u};
      if (key0 + r < nkeys) z = *(const u32x4*)(src.krow(key0 + r) + col);
      k[i] = z;
    }
    if (threadIdx.x < VBLK) {
      const int kg = threadIdx.x & 7, dg = threadIdx.x >> 3;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int key = key0 + kg * 8 + j;
        u32x4 z = {0u, 0u, 0u, 0u};
        if (key < nkeys) z = *(const u32x4*)(src.vrow(key) + dg * 8);
        v[j] = z;
      }
    }
  }
  __device__ __forceinline__ void store(T* ks, T* vt) const {
#pragma unroll
    for (int i = 0; i < KCH; ++i) {
      const int c = threadIdx.x + i * 256;
      const int r = c / (DH / 8), col = (c % (DH / 8)) * 8;
      *(u32x4*)(ks + r * (DH + 8) + col) = k[i];
    }
    if (threadIdx.x < VBLK) {
      const int kg = threadIdx.x & 7, dg = threadIdx.x >> 3;
      u32x4 t[8];
      transpose8x8(v, t);
#pragma unroll
      for (int r = 0; r < 8; ++r) *(u32x4*)(vt + (dg * 8 + r) * (KT + 8) + kg * 8) = t[r];
    }
  }
};

// Serving geometry: request r owns rows start[r] .. start[r+1]-1 of qkv / o, its queries sit at
// absolute positions ctx_len[r] + i and its keys 0 .. ctx_len[r] + chunk - 1 are in the pool.
struct PagedGeom {
  const void* k_pool; const void* v_pool; const int32_t* block_table; const int32_t* ctx_len;
  int max_pages, page, n_req;
  int start[33];
};

template <class T, int DH, int QT, bool PAGED>
__global__ __launch_bounds__(256) void flash_fwd_kernel(const T* __restrict__ qkv, T* __restrict__ o,
                                                        float* __restrict__ lse, int L, int h,
                                                        float scale_log2, PagedGeom pg) {
  typedef typename Mma<T>::V8 V8;
  typedef typename Mma<T>::V4 V4;
  constexpr int BQ = 4 * QT * 32;
  constexpr int KS = DH / 16;   // k steps over the head dimension
  constexpr int DT = DH / 32;   // 32-row tiles of O^T
  constexpr int KSTR = DH + 8, VSTR = KT + 8;
  __shared__ __attribute__((aligned(16))) T ks_lds[2][KT * KSTR];
  __shared__ __attribute__((aligned(16))) T vt_lds[2][DH * VSTR];

  // query tiles in grid.y (dispatched slowest): the long workgroups of all heads start first
  const int b = blockIdx.x / h, head = blockIdx.x % h;
  const int d = h * DH;
  const long ld = 3L * d;
  // rows of this sequence / request chunk, number of cached tokens before it
  const long row0 = PAGED ? pg.start[b] : (long)b * L;
  const int Lq = PAGED ? pg.start[b + 1] - pg.start[b] : L;
  const int past = PAGED ? pg.ctx_len[b] : 0;
  const int n_qt = (Lq + BQ - 1) / BQ;
  if ((int)blockIdx.y >= n_qt) return;
  const int qtile = n_qt - 1 - blockIdx.y;  // heaviest tiles first
  const T* qb = qkv + row0 * ld + (long)head * DH;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int col = lane & 31, hf = lane >> 5;
  const int wq0 = qtile * BQ + wave * QT * 32;  // first query row of this wavefront
  const int nkeys = past + Lq;
  const KvContig<T> src_c{qb + d, qb + 2 * d, ld};
  const KvPaged<T> src_p{(const T*)pg.k_pool, (const T*)pg.v_pool,
                         pg.block_table + (PAGED ? (long)b * pg.max_pages : 0), pg.page, h, head, DH};

  // Q fragments (B operand): column = query, k = head dimension
  V8 qf[QT][KS];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const int q = wq0 + t * 32 + col;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      u32x4 z = {0u, 0u, 0u, 0u};
      if (q < Lq) z = *(const u32x4*)(qb + (long)q * ld + s * 16 + hf * 8);
      qf[t][s] = __builtin_bit_cast(V8, z);
    }
  }

  f32x16 oacc[QT][DT];
  float m_run[QT], l_run[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    m_run[t] = -INFINITY;
    l_run[t] = 0.f;
#pragma unroll
    for (int j = 0; j < DT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[t][j][e] = 0.f;
  }

  const int q_hi = min(Lq, qtile * BQ + BQ) - 1;  // last query row of the workgroup
  const int n_kt = (past + q_hi) / KT + 1;
  KvStage<T, DH> stg;
  auto load_tile = [&](int key0) {
    if (PAGED) stg.load(src_p, key0, nkeys);
    else stg.load(src_c, key0, nkeys);
  };
  load_tile(0);
  stg.store(ks_lds[0], vt_lds[0]);
  __syncthreads();

  for (int kt = 0; kt < n_kt; ++kt) {
    const int cur = kt & 1;
    const int key0 = kt * KT;
    if (kt + 1 < n_kt) load_tile(key0 + KT);
    // this wavefront's rows end at wq0 + QT*32 - 1: skip tiles entirely above its diagonal
    if (key0 <= past + wq0 + QT * 32 - 1) {
      const T* ks = ks_lds[cur];
      const T* vt = vt_lds[cur];
      f32x16 sacc[QT][2];
#pragma unroll
      for (int t = 0; t < QT; ++t)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
          for (int e = 0; e < 16; ++e) sacc[t][c][e] = 0.f;
      // S^T = K Q^T
#pragma unroll
      for (int s = 0; s < KS; ++s) {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const V8 kf = *(const V8*)(ks + (c * 32 + pi_row(col)) * KSTR + s * 16 + hf * 8);
#pragma unroll
          for (int t = 0; t < QT; ++t) sacc[t][c] = Mma<T>::run(kf, qf[t][s], sacc[t][c]);
        }
      }
      // online softmax per query (lane), keys of element e: key0 + c*32 + 16*(e/8) + 8*hf + e%8
      V8 pf[QT][4];
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        const int q = past + wq0 + t * 32 + col;           // absolute position of this lane's query
        const bool diag = key0 + KT - 1 > past + wq0 + t * 32;  // tile reaches past the first row's diagonal
        float mx = -INFINITY;
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            float v = sacc[t][c][e] * scale_log2;
            if (diag) {
              const int key = key0 + c * 32 + 16 * (e >> 3) + 8 * hf + (e & 7);
              if (key > q) v = -INFINITY;
            }
            sacc[t][c][e] = v;
            mx = fmaxf(mx, v);
          }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run[t], mx);
        // a row with no visible key yet keeps m = -inf; use 0 as the reference then
        const float m_ref = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run[t] - m_ref);
        float rs = 0.f;
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
          for (int g = 0; g < 2; ++g) {
            V8 pv;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
              const float p = __builtin_amdgcn_exp2f(sacc[t][c][g * 8 + i] - m_ref);
              rs += p;
              pv[i] = from_f<T>(p);
            }
            pf[t][c * 2 + g] = pv;
          }
        l_run[t] = l_run[t] * alpha + rs;
        m_run[t] = m_new;
#pragma unroll
        for (int j = 0; j < DT; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) oacc[t][j][e] *= alpha;
      }
      // O^T += V^T P^T
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
        for (int j = 0; j < DT; ++j) {
          const V8 vf = *(const V8*)(vt + (j * 32 + col) * VSTR + kk * 16 + hf * 8);
#pragma unroll
          for (int t = 0; t < QT; ++t) oacc[t][j] = Mma<T>::run(vf, pf[t][kk], oacc[t][j]);
        }
      }
    }
    if (kt + 1 < n_kt) stg.store(ks_lds[cur ^ 1], vt_lds[cur ^ 1]);
    __syncthreads();
  }

  // normalise and write O[q][dh]; lane holds dh rows j*32 + 8*(e/4) + 4*hf + e%4 of its query
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const int q = wq0 + t * 32 + col;
    const float l = l_run[t] + __shfl_xor(l_run[t], 32, 64);
    if (q >= Lq) continue;
    const float inv = 1.0f / l;
    T* orow = o + (row0 + q) * d + (long)head * DH;
#pragma unroll
    for (int j = 0; j < DT; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        V4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = from_f<T>(oacc[t][j][g * 4 + i] * inv);
        *(V4*)(orow + j * 32 + 8 * g + 4 * hf) = v;
      }
    if (lse && hf == 0)
      lse[(row0 + q) * h + head] = (m_run[t] + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
  }
}

// ---------------------------------------------------------------------------------
// Backward.  Two kernels, no atomics (deterministic):
//   flash_bwd_dq_kernel : a workgroup owns 128 query rows, walks key tiles j <= i
//   flash_bwd_dkv_kernel: a workgroup owns 128 keys, walks query tiles i >= j
// Both recompute P from the saved log-sum-exp.  An MFMA result has its row index
// in registers and its column index in lanes, which is the B-operand layout of a
// following product that contracts over the rows; so each kernel forms its first
// products with the contraction index of the second products as rows:
//   dq : S^T, dP^T [key, q]  ->  dQ^T[dh, q]   = K^T[dh, key] dS^T[key, q]
//   dkv: S,   dP   [q, key]  ->  dV^T[dh, key] = dO^T[dh, q] P[q, key]
//                                dK^T[dh, key] = Q^T[dh, q]  dS[q, key]
// The transposed A operands (K^T, Q^T, dO^T) are made in registers on the way
// into LDS.  D = rowsum(dO * O) comes from a separate bandwidth-bound kernel.
// ---------------------------------------------------------------------------------

// multiply the eight 16-bit elements of a raw 16-byte chunk by a power of two (exact)
template <class T>
__device__ __forceinline__ u32x4 scale_chunk(u32x4 raw, float sc) {
  typedef typename Mma<T>::V8 V8;
  V8 v = __builtin_bit_cast(V8, raw);
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = from_f<T>(to_f(v[i]) * sc);
  return __builtin_bit_cast(u32x4, v);
}

// Power-of-two factor that brings the largest |dO| element into (16, 32].  dS = P (dP - D)
// is linear in dO and carries the softmax probabilities (~1/context), so without it
// dS sits in the fp16 subnormal range for small upstream gradients.  dP <= 32 * sum|v|
// stays far below the fp16 maximum.
__device__ __forceinline__ float do_scale(const float* amax_ptr) {
  const float a = *amax_ptr;
  if (!(a > 0.f) || a > 3.0e38f) return 1.f;
  float e = floorf(__builtin_amdgcn_logf(32.f / a));   // log2
  e = fminf(fmaxf(e, -14.f), 24.f);
  return __builtin_amdgcn_exp2f(e);
}

// natural tile [ROWS][DH] -> LDS row stride DH+8
template <class T, int ROWS, int DH>
struct NatStage {
  static constexpr int N = (ROWS * DH / 8 + 255) / 256;
  u32x4 v[N];
  __device__ __forceinline__ void load(const T* base, long ld, int row0, int nrows) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = threadIdx.x + i * 256;
      const int r = c / (DH / 8), col = (c % (DH / 8)) * 8;
      u32x4 z = {0u, 0u, 0u, 0u};
      if (c < ROWS * DH / 8 && row0 + r < nrows) z = *(const u32x4*)(base + (long)(row0 + r) * ld + col);
      v[i] = z;
    }
  }
  __device__ __forceinline__ void scale(float sc) {
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = scale_chunk<T>(v[i], sc);
  }
  __device__ __forceinline__ void store(T* lds) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = threadIdx.x + i * 256;
      const int r = c / (DH / 8), col = (c % (DH / 8)) * 8;
      if (c < ROWS * DH / 8) *(u32x4*)(lds + r * (DH + 8) + col) = v[i];
    }
  }
};

// transposed tile: global [ROWS][DH] -> LDS [DH][ROWS+8]; one 8x8 block per thread
// for threads tid0 .. tid0 + (ROWS/8)*(DH/8) - 1
template <class T, int ROWS, int DH>
struct TrStage {
  static constexpr int NBLK = (ROWS / 8) * (DH / 8);
  u32x4 v[8];
  __device__ __forceinline__ void load(const T* base, long ld, int row0, int nrows, int tid0) {
    const int t = (int)threadIdx.x - tid0;
    if (t >= 0 && t < NBLK) {
      const int rg = t % (ROWS / 8), dg = t / (ROWS / 8);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int r = row0 + rg * 8 + j;
        u32x4 z = {0u, 0u, 0u, 0u};
        if (r < nrows) z = *(const u32x4*)(base + (long)r * ld + dg * 8);
        v[j] = z;
      }
    }
  }
  __device__ __forceinline__ void scale(float sc) {
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = scale_chunk<T>(v[j], sc);
  }
  __device__ __forceinline__ void store(T* lds, int tid0) const {
    const int t = (int)threadIdx.x - tid0;
    if (t >= 0 && t < NBLK) {
      const int rg = t % (ROWS / 8), dg = t / (ROWS / 8);
      u32x4 o[8];
      transpose8x8(v, o);
#pragma unroll
      for (int r = 0; r < 8; ++r) *(u32x4*)(lds + (dg * 8 + r) * (ROWS + 8) + rg * 8) = o[r];
    }
  }
};

// Store one gradient row held as O^T-style accumulators (lane = row, registers = head
// dimension j*32 + 8g + 4hf + i), multiplied by `mul`.  With a rotary table the row is first
// rotated back by its position (the transpose of the forward rotation): the pair
// (i, i + DH/2) lives in tiles j and j + DT/2 of the same lane.
template <class T, int DH>
__device__ __forceinline__ void store_grad_row(T* row, const f32x16 (&acc)[DH / 32], float mul, int hf,
                                               const float* tab) {
  typedef typename Mma<T>::V4 V4;
  constexpr int DT = DH / 32;
  if (tab == nullptr) {
#pragma unroll
    for (int j = 0; j < DT; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        V4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = from_f<T>(acc[j][g * 4 + i] * mul);
        *(V4*)(row + j * 32 + 8 * g + 4 * hf) = v;
      }
    return;
  }
#pragma unroll
  for (int j = 0; j < DT / 2; ++j)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int i0 = j * 32 + 8 * g + 4 * hf;
      const f32x4 cs0 = *(const f32x4*)(tab + i0 * 2), cs1 = *(const f32x4*)(tab + i0 * 2 + 4);
      V4 lo, hi;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float c = i < 2 ? cs0[2 * i] : cs1[2 * (i - 2)], sn = i < 2 ? cs0[2 * i + 1] : cs1[2 * (i - 2) + 1];
        const float a = acc[j][g * 4 + i] * mul, b = acc[j + DT / 2][g * 4 + i] * mul;
        lo[i] = from_f<T>(a * c + b * sn);
        hi[i] = from_f<T>(b * c - a * sn);
      }
      *(V4*)(row + i0) = lo;
      *(V4*)(row + i0 + DH / 2) = hi;
    }
}

// ---- tiles brought in by direct-to-LDS loads ------------------------------------------------
// A tile is ROWS rows of DH 16-bit elements, row-major in LDS, the 16-byte chunks of a row
// XOR-permuted by the row number so that both kinds of fragment read are conflict-free:
//   - 16-byte reads of 8 consecutive head-dimension elements (operand rows = tile rows), and
//   - transposing reads (operand rows = head dimension, contraction over the tile rows).
// A wave load writes 1 KB (lane i -> bytes 16 i), i.e. 1024 / (2 DH) whole rows.
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));

// Chunk permutation of a tile row.  16 consecutive rows (one phase of a 16-byte fragment read)
// must get 16 different bank groups, and 4 consecutive rows (one phase of a transposing read,
// which takes a pair of adjacent chunks from each) 4 different chunk pairs.
template <int DH> __device__ __forceinline__ int tile_swz(int row) {
  return DH == 128 ? (((row & 7) << 1) | ((row >> 3) & 1)) : ((((row >> 1) & 3) << 1) | ((row >> 3) & 1));
}

// wave load `l` of a tile whose first row is global row `row0` (rows past `nrows` re-read the last row)
template <class T, int DH>
__device__ __forceinline__ void dma_rows(const T* base, long ld, int row0, int nrows, char* lds_tile, int l,
                                         int lane) {
  constexpr int CPR = DH / 8, RPL = 64 / CPR;
  const int row = l * RPL + lane / CPR;
  const int gch = (lane % CPR) ^ tile_swz<DH>(row);
  const int gr = min(row0 + row, nrows - 1);
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(base + (long)gr * ld + gch * 8),
                                   (__attribute__((address_space(3))) void*)(lds_tile + l * 1024), 16, 0, 0);
}

// 64 floats, one per lane: element i of a strided vector (stride in floats) -> LDS float i
__device__ __forceinline__ void dma_floats(const float* base, long stride, int i0, int n, char* lds, int lane) {
  const int i = min(i0 + lane, n - 1);
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(base + (long)i * stride),
                                   (__attribute__((address_space(3))) void*)lds, 4, 0, 0);
}

// fragment for operand rows = tile rows: row (of the tile) and the 8 head-dimension elements 8 c .. 8 c + 7
template <class T, int DH>
__device__ __forceinline__ typename Mma<T>::V8 frag_rows(const char* tile, int row, int c) {
  return *(const typename Mma<T>::V8*)(tile + row * (DH * 2) + ((c ^ tile_swz<DH>(row)) * 16));
}

// Fragment for operand rows = head dimension d0 .. d0 + 31, contraction over tile rows
// k0 + 8 (lane >> 5) .. + 7: two transposing LDS reads.  They are issued from inline assembly
// (the builtin form makes the compiler wait for all direct-to-LDS loads in flight), so the
// registers are only valid after tr_wait() has been applied to them.
struct TrFrag { s16x4_t lo, hi; };
template <int DH>
__device__ __forceinline__ void tr_read(TrFrag& f, const char* tile, int d0, int k0, int lane) {
  const int i16 = lane & 15, a = i16 >> 2, j4 = i16 & 3;
  const int nb = d0 + 16 * ((lane >> 4) & 1) + 4 * j4;   // first of the 4 head-dimension elements of this lane
  const int k = k0 + 8 * (lane >> 5) + a;
  const char* p0 = tile + k * (DH * 2) + (((nb >> 3) ^ tile_swz<DH>(k)) * 16) + ((nb >> 2) & 1) * 8;
  const char* p1 = tile + (k + 4) * (DH * 2) + (((nb >> 3) ^ tile_swz<DH>(k + 4)) * 16) + ((nb >> 2) & 1) * 8;
  const uint32_t a0 = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)p0;
  const uint32_t a1 = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)p1;
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(f.lo) : "v"(a0) : "memory");
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(f.hi) : "v"(a1) : "memory");
}
__device__ __forceinline__ void tr_wait(TrFrag (&f)[4]) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi), "+v"(f[2].lo), "+v"(f[2].hi),
                 "+v"(f[3].lo), "+v"(f[3].hi));
}
__device__ __forceinline__ void tr_wait(TrFrag (&f)[2]) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi));
}
template <class T>
__device__ __forceinline__ typename Mma<T>::V8 tr_value(const TrFrag& f) {
  const s16x8_t w = __builtin_shufflevector(f.lo, f.hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(typename Mma<T>::V8, w);
}

// Forward through the tile ring.  A workgroup owns 4 * QT * 32 queries (QT tiles of 32 per
// wavefront, Q fragments in registers) and walks the 64-key tiles below its diagonal; K and V
// tiles arrive by direct-to-LDS loads through a ring of NS stages (three tiles in flight), so no
// wavefront waits on a global load inside the loop.  S^T = K Q^T puts the softmax state of a
// query in one lane; V^T for O^T += V^T P^T is read from the V tile with the transposing LDS
// load, and P goes from the first product's accumulators straight into the second product's
// B operand.  PAGED: the tiles are gathered from the request's pages (block-table row copied
// to LDS once), queries sit at positions past .. past + Lq - 1.
template <class T, int DH>
__device__ __forceinline__ void dma_rows_paged(const T* kpool, const T* vpool, const int* page_of, int shift, int h,
                                               int head, int key0, int nkeys, char* k_tile, char* v_tile, int l,
                                               int lane) {
  constexpr int CPR = DH / 8, RPL = 64 / CPR;
  const int row = l * RPL + lane / CPR;
  const int gch = (lane % CPR) ^ tile_swz<DH>(row);
  const int key = min(key0 + row, nkeys - 1);
  const long off = ((((long)page_of[key >> shift] * h + head) << shift) + (key & ((1 << shift) - 1))) * DH + gch * 8;
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(kpool + off),
                                   (__attribute__((address_space(3))) void*)(k_tile + l * 1024), 16, 0, 0);
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(vpool + off),
                                   (__attribute__((address_space(3))) void*)(v_tile + l * 1024), 16, 0, 0);
}

template <class T, int DH, int QT, bool PAGED, int NS, int OCC>
__global__ __launch_bounds__(256, OCC) void flash_fwd_ring_kernel(const T* __restrict__ qkv, T* __restrict__ o,
                                                             float* __restrict__ lse, int L, int h,
                                                             float scale_log2, PagedGeom pg) {
  typedef typename Mma<T>::V8 V8;
  typedef typename Mma<T>::V4 V4;
  constexpr int BQ = 4 * QT * 32, KS = DH / 16, DT = DH / 32;
  constexpr int TILE_B = KT * DH * 2;            // bytes of a K or V tile
  constexpr int STAGE_B = 2 * TILE_B;
  constexpr int NLT = TILE_B / 1024 / 4;         // wave loads per wavefront and tile
  constexpr int NLD = 2 * NLT;                   // loads per wavefront and stage
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  int* page_of = (int*)(smem + NS * STAGE_B);

  const int b = blockIdx.x / h, head = blockIdx.x % h;
  const int d = h * DH;
  const long ld = 3L * d;
  const long row0 = PAGED ? pg.start[b] : (long)b * L;
  const int Lq = PAGED ? pg.start[b + 1] - pg.start[b] : L;
  const int past = PAGED ? pg.ctx_len[b] : 0;
  const int n_qt = (Lq + BQ - 1) / BQ;
  if ((int)blockIdx.y >= n_qt) return;
  const int qtile = n_qt - 1 - blockIdx.y;   // heaviest tiles of all heads first
  const T* qb = qkv + row0 * ld + (long)head * DH;
  const T* kb = qb + d;
  const T* vb = qb + 2 * d;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int col = lane & 31, hf = lane >> 5;
  const int wq0 = qtile * BQ + wave * QT * 32;
  const int nkeys = past + Lq;
  const int shift = PAGED ? 31 - __builtin_clz(pg.page) : 0;
  if (PAGED) {
    const int np = (nkeys + pg.page - 1) >> shift;
    for (int i = threadIdx.x; i < np; i += 256) page_of[i] = pg.block_table[(long)b * pg.max_pages + i];
  }

  V8 qf[QT][KS];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const int q = wq0 + t * 32 + col;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      u32x4 z = {0u, 0u, 0u, 0u};
      if (q < Lq) z = *(const u32x4*)(qb + (long)q * ld + s * 16 + hf * 8);
      qf[t][s] = __builtin_bit_cast(V8, z);
    }
  }
  f32x16 oacc[QT][DT];
  float m_run[QT], l_run[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    m_run[t] = -INFINITY;
    l_run[t] = 0.f;
#pragma unroll
    for (int j = 0; j < DT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[t][j][e] = 0.f;
  }
  // the wait counts below assume that only direct-to-LDS loads are in flight
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  if (PAGED) __syncthreads();

  const int q_hi = min(Lq, qtile * BQ + BQ) - 1;
  const int nt = (past + q_hi) / KT + 1;
  // tile t -> stage t % NS; tiles past the end re-fetch the last one (never used), so that
  // every wavefront always has the same number of loads in flight
  auto issue = [&](int t) {
    const int key0 = min(t, nt - 1) * KT;
    char* st = smem + (t % NS) * STAGE_B;
#pragma unroll
    for (int j = 0; j < NLT; ++j) {
      if (PAGED) {
        dma_rows_paged<T, DH>((const T*)pg.k_pool, (const T*)pg.v_pool, page_of, shift, h, head, key0, nkeys, st,
                              st + TILE_B, wave * NLT + j, lane);
      } else {
        dma_rows<T, DH>(kb, ld, key0, nkeys, st, wave * NLT + j, lane);
        dma_rows<T, DH>(vb, ld, key0, nkeys, st + TILE_B, wave * NLT + j, lane);
      }
    }
  };
#pragma unroll
  for (int t = 0; t < NS; ++t) issue(t);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 1) * NLD) : "memory");
  __syncthreads();

  // One tile for this wavefront.  MASKED: the tile reaches the diagonal of some query of the wavefront.
  auto tile_body = [&](auto masked_tag, int t) {
    constexpr bool MASKED = decltype(masked_tag)::value;
    const int key0 = t * KT;
    const char* ks = smem + (t % NS) * STAGE_B;
    const char* vs = ks + TILE_B;
    f32x16 sacc[QT][2];
#pragma unroll
    for (int tq = 0; tq < QT; ++tq)
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) sacc[tq][c][e] = 0.f;
    // S^T = K Q^T; MFMA row r is key pi(r): a lane's 8 values per 16-key step are consecutive keys
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const V8 kf = frag_rows<T, DH>(ks, c * 32 + pi_row(col), 2 * s + hf);
#pragma unroll
        for (int tq = 0; tq < QT; ++tq) sacc[tq][c] = Mma<T>::run(kf, qf[tq][s], sacc[tq][c]);
      }
    TrFrag fr[2][DT];
#pragma unroll
    for (int j = 0; j < DT; ++j) tr_read<DH>(fr[0][j], vs, j * 32, 0, lane);
    // online softmax per query (lane); element e of block c <-> key key0 + 32 c + 16 (e / 8) + 8 hf + e % 8.
    // m_run is the reference the exponentials are taken against.  It follows the running maximum
    // lazily: only when some query of the wavefront exceeds it by more than 2^8 are the sums and
    // the accumulators rescaled (exact either way; until then p <= 256, far inside every format
    // involved), which removes the rescaling from all but the first tiles of a row.
    V8 pf[QT][4];
#pragma unroll
    for (int tq = 0; tq < QT; ++tq) {
      const int q = past + wq0 + tq * 32 + col;
      float mx = -INFINITY;
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          if (MASKED) {
            const int key = key0 + c * 32 + 16 * (e >> 3) + 8 * hf + (e & 7);
            if (key > q) sacc[tq][c][e] = -INFINITY;
          }
          mx = fmaxf(mx, sacc[tq][c][e]);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * scale_log2;
      if (__builtin_amdgcn_ballot_w64(mx > m_run[tq] + 8.f) != 0) {
        const float m_new = fmaxf(m_run[tq], mx);
        const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m_run[tq] - m_new);
        l_run[tq] *= alpha;
        m_run[tq] = m_new;
#pragma unroll
        for (int j = 0; j < DT; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) oacc[tq][j][e] *= alpha;
      }
      const float m_ref = m_run[tq] == -INFINITY ? 0.f : m_run[tq];   // a row with no visible key yet
      float rs = 0.f;
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int g = 0; g < 2; ++g) {
          V8 pv;
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[tq][c][g * 8 + i], scale_log2, -m_ref));
            rs += pr;
            pv[i] = from_f<T>(pr);
          }
          pf[tq][c * 2 + g] = pv;
        }
      l_run[tq] += rs;
    }
    // O^T += V^T P^T in four steps of 16 keys
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      tr_wait(fr[kk & 1]);
      if (kk < 3) {
#pragma unroll
        for (int j = 0; j < DT; ++j) tr_read<DH>(fr[(kk + 1) & 1][j], vs, j * 32, (kk + 1) * 16, lane);
      }
#pragma unroll
      for (int j = 0; j < DT; ++j) {
        const V8 vf = tr_value<T>(fr[kk & 1][j]);
#pragma unroll
        for (int tq = 0; tq < QT; ++tq) oacc[tq][j] = Mma<T>::run(vf, pf[tq][kk], oacc[tq][j]);
      }
    }
  };
  // tile t + 1 has landed when only the loads of tiles t + 2 .. t + NS - 1 are outstanding; after the
  // barrier nobody reads tile t any more and its stage is refilled
  auto ring_step = [&](int t) {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((NS - 2) * NLD) : "memory");
    __syncthreads();
    issue(t + NS);
  };
  // This wavefront's rows are past + wq0 .. + QT * 32 - 1.  Tiles entirely below the first row's diagonal
  // need no mask (first loop), the rest are masked, and tiles entirely above the last row's diagonal add
  // nothing.  The two loops together make nt trips in every wavefront, so the barriers match.
  const int t_plain = min(nt, max(0, (past + wq0 + 1) / KT));
  int t = 0;
  for (; t < t_plain; ++t) {
    tile_body(std::false_type{}, t);
    ring_step(t);
  }
  for (; t < nt; ++t) {
    if (t * KT <= past + wq0 + QT * 32 - 1) tile_body(std::true_type{}, t);
    ring_step(t);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no direct-to-LDS write may outlive the workgroup

  // normalise and write O[q][dh]; a lane holds dh rows j * 32 + 8 (e / 4) + 4 hf + e % 4 of its query
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const int q = wq0 + t * 32 + col;
    const float l = l_run[t] + __shfl_xor(l_run[t], 32, 64);
    if (q >= Lq) continue;
    const float inv = 1.0f / l;
    T* orow = o + (row0 + q) * d + (long)head * DH;
#pragma unroll
    for (int j = 0; j < DT; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        V4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = from_f<T>(oacc[t][j][g * 4 + i] * inv);
        *(V4*)(orow + j * 32 + 8 * g + 4 * hf) = v;
      }
    if (lse && hf == 0)
      lse[(row0 + q) * h + head] = (m_run[t] + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
  }
}

#include "attention_sched.h"

// Four stages.  With head_dim 64 (64 KB of ring, under 256 registers) two workgroups share a compute
// unit and cover each other's waits; with head_dim 128 one does (two stages and two workgroups were
// measured slower: 227 against 164 us at 2 x 2048 x 32 heads, the registers no longer fit).
template <int DH> struct RingCfg { static constexpr int NS = 4, OCC = DH == 128 ? 1 : 2; };

template <class T, int DH, int QT, bool PAGED>
ls_status launch_ring(const void* qkv, void* o, float* lse, int L, int h, float scale_log2, const PagedGeom& pg,
                      dim3 grid, int extra_lds, hipStream_t st) {
  constexpr int NS = RingCfg<DH>::NS;
  const int lds = NS * 2 * KT * DH * 2 + extra_lds;
  static bool attr_set = false;
  if (!attr_set) {
    LS_CHECK_HIP(hipFuncSetAttribute((const void*)flash_fwd_ring_kernel<T, DH, QT, PAGED, NS, RingCfg<DH>::OCC>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    attr_set = true;
  }
  flash_fwd_ring_kernel<T, DH, QT, PAGED, NS, RingCfg<DH>::OCC><<<grid, 256, lds, st>>>((const T*)qkv, (T*)o, lse, L, h, scale_log2, pg);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

// How many 128-row tiles of a (sequence, head) one workgroup of a hand-scheduled kernel takes in a row (it keeps
// its ring of key tiles running from one to the next, which saves most of a workgroup's start-up per tile): the
// count that makes the launch shortest under a simple model, if that is a tenth shorter than with one tile per
// workgroup (the model is rough where the launch does not fill the chip).  A workgroup costs 3 units, a query
// tile its key tiles (tile i has i + 1) plus 6 units (measured: a key tile takes about 1 us, a workgroup's first
// query tile 8.8 us more than its key tiles, a further one 5.9); the workgroups start in launch order (all heads'
// workgroup 0, then all heads' workgroup 1, ...), each on the compute unit that is free first.
inline int tiles_per_workgroup(int bh, int n_tiles) {
  static std::mutex mu;
  static std::map<std::pair<int, int>, int> known;
  std::lock_guard<std::mutex> lock(mu);
  const auto hit = known.find({bh, n_tiles});
  if (hit != known.end()) return hit->second;
  constexpr int CUS = 256;
  int best = 1;
  double best_cost = 0;
  for (int ipw = 1; ipw <= 16 && ipw <= n_tiles; ++ipw) {
    const int G = (n_tiles + ipw - 1) / ipw;
    std::priority_queue<double, std::vector<double>, std::greater<double>> free_at;
    for (int i = 0; i < CUS; ++i) free_at.push(0.0);
    double cost = 0;
    for (int y = 0; y < G; ++y) {
      double w = 3;
      for (int k = 0; k < ipw; ++k) {
        const int tile = snake_tile(k, y, G, n_tiles);
        if (tile >= 0) w += tile + 1 + 6;
      }
      for (int i = 0; i < bh; ++i) {
        const double end = free_at.top() + w;
        free_at.pop();
        free_at.push(end);
        cost = end > cost ? end : cost;
      }
    }
    if (ipw == 1) best_cost = 0.9 * cost;
    else if (cost < best_cost) best = ipw, best_cost = cost;
  }
  known[{bh, n_tiles}] = best;
  return best;
}

template <class T, int DH>
ls_status launch_fwd(const void* qkv, int B, int L, int h, void* o, float* lse, hipStream_t st) {
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)DH);
  PagedGeom pg{};
  if constexpr (DH == 128) {
    // the hand-scheduled kernel
    constexpr int lds = FWD128_LDS;
    static bool attr_set = false;
    if (!attr_set) {
      LS_CHECK_HIP(hipFuncSetAttribute((const void*)flash_fwd128_kernel<T>, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
      attr_set = true;
    }
    const int n_qt = (L + 127) / 128;
    const int ipw = tiles_per_workgroup(B * h, n_qt);
    flash_fwd128_kernel<T><<<dim3(B * h, (n_qt + ipw - 1) / ipw), 256, lds, st>>>((const T*)qkv, (T*)o, lse, L, h, scale_log2, ipw);
    LS_CHECK_LAUNCH();
    return LS_OK;
  } else if constexpr (DH >= 64) {
    // the tile-ring kernel.  128 queries per workgroup: with 256 the two code paths of a tile (masked /
    // unmasked, rescaling or not) no longer fit the register file for head_dim 128
    return launch_ring<T, DH, 1, false>(qkv, o, lse, L, h, scale_log2, pg, dim3(B * h, (L + 127) / 128), 0, st);
  } else {
    // head_dim 32: the register-staged kernel
    if (L > 512) {
      constexpr int QT = 2;
      dim3 grid(B * h, (L + 4 * QT * 32 - 1) / (4 * QT * 32));
      flash_fwd_kernel<T, DH, QT, false><<<grid, 256, 0, st>>>((const T*)qkv, (T*)o, lse, L, h, scale_log2, pg);
    } else {
      constexpr int QT = 1;
      dim3 grid(B * h, (L + 4 * QT * 32 - 1) / (4 * QT * 32));
      flash_fwd_kernel<T, DH, QT, false><<<grid, 256, 0, st>>>((const T*)qkv, (T*)o, lse, L, h, scale_log2, pg);
    }
    LS_CHECK_LAUNCH();
    return LS_OK;
  }
}

template <class T, int DH>
ls_status launch_prefill(const void* qkv, int h, void* o, const PagedGeom& pg, int max_chunk, hipStream_t st) {
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)DH);
  constexpr int QT = 1;
  dim3 grid(pg.n_req * h, (max_chunk + 4 * QT * 32 - 1) / (4 * QT * 32));
  if (pg.max_pages <= 4096 && pg.page >= 8 && (pg.page & (pg.page - 1)) == 0)
    return launch_ring<T, DH, 1, true>(qkv, o, nullptr, 0, h, scale_log2, pg, grid, pg.max_pages * 4, st);
  flash_fwd_kernel<T, DH, QT, true><<<grid, 256, 0, st>>>((const T*)qkv, (T*)o, nullptr, 0, h, scale_log2, pg);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

// dQ.  A workgroup owns 128 queries (32 per wavefront, Q and dO fragments in registers) and
// walks the key tiles of 64 keys below its diagonal.  K and V tiles arrive by direct-to-LDS
// loads through a ring of NS stages; K^T for the second product is read from the K tile with
// the transposing LDS load.  Both first products are formed transposed (S^T, dP^T: rows =
// keys, lane column = query), so the softmax statistics are per-lane scalars.
template <class T, int DH>
__global__ __launch_bounds__(256) void flash_bwd_dq_kernel(const T* __restrict__ qkv,
                                                           const T* __restrict__ dO,
                                                           const float* __restrict__ lse,
                                                           const float* __restrict__ dvec,
                                                           T* __restrict__ dqkv, int L, int h,
                                                           float scale, const float* __restrict__ rope) {
  typedef typename Mma<T>::V8 V8;
  constexpr int BQ = 128, NS = 4, KS = DH / 16, DT = DH / 32;
  constexpr int TILE_B = KT * DH * 2;            // bytes of a K or V tile
  constexpr int STAGE_B = 2 * TILE_B;
  constexpr int NLT = TILE_B / 1024 / 4;         // wave loads per wavefront and tile
  constexpr int NLD = 2 * NLT;                   // loads per wavefront and stage
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  const int n_qt = (L + BQ - 1) / BQ;
  const int qtile = n_qt - 1 - blockIdx.y;   // heaviest tiles of all heads first
  const int b = blockIdx.x / h, head = blockIdx.x % h;
  const int d = h * DH;
  const long ld = 3L * d;
  const T* qb = qkv + (long)b * L * ld + (long)head * DH;
  const T* kb = qb + d;
  const T* vb = qb + 2 * d;
  const T* dob = dO + (long)b * L * d + (long)head * DH;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int col = lane & 31, hf = lane >> 5;
  const int wq0 = qtile * BQ + wave * 32;
  const int q = wq0 + col;
  const float scale_log2 = scale * 1.4426950408889634f;
  const float gsc = do_scale(dvec + (long)gridDim.x * L + ((long)gridDim.x * L + 3) / 4);   // after D and the per-workgroup maxima

  V8 qf[KS], dof[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    u32x4 z0 = {0u, 0u, 0u, 0u}, z1 = {0u, 0u, 0u, 0u};
    if (q < L) {
      z0 = *(const u32x4*)(qb + (long)q * ld + s * 16 + hf * 8);
      z1 = *(const u32x4*)(dob + (long)q * d + s * 16 + hf * 8);
    }
    qf[s] = __builtin_bit_cast(V8, z0);
    dof[s] = __builtin_bit_cast(V8, z1);
  }
  float lse2 = INFINITY, dq_ = 0.f;
  if (q < L) {
    lse2 = lse[((long)b * L + q) * h + head] * 1.4426950408889634f;
    dq_ = dvec[((long)b * L + q) * h + head];
  }
  f32x16 acc[DT];
#pragma unroll
  for (int j = 0; j < DT; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
  // the wait counts below assume that only direct-to-LDS loads are in flight
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  const int q_hi = min(L, qtile * BQ + BQ) - 1;
  const int nt = q_hi / KT + 1;
  // tile t -> stage t % NS; tiles past the end re-fetch the last one (never used), so that
  // every wavefront always has the same number of loads in flight
  auto issue = [&](int t) {
    const int key0 = min(t, nt - 1) * KT;
    char* st = smem + (t % NS) * STAGE_B;
#pragma unroll
    for (int j = 0; j < NLT; ++j) {
      dma_rows<T, DH>(kb, ld, key0, L, st, wave * NLT + j, lane);
      dma_rows<T, DH>(vb, ld, key0, L, st + TILE_B, wave * NLT + j, lane);
    }
  };
#pragma unroll
  for (int t = 0; t < NS; ++t) issue(t);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 1) * NLD) : "memory");
  __syncthreads();

  for (int t = 0; t < nt; ++t) {
    const int key0 = t * KT;
    const char* ks = smem + (t % NS) * STAGE_B;
    const char* vs = ks + TILE_B;
    // the tile's 64 keys in two blocks of 32
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      f32x16 sacc, pacc;
#pragma unroll
      for (int e = 0; e < 16; ++e) sacc[e] = pacc[e] = 0.f;
      const int row = c * 32 + pi_row(col);   // MFMA row r is key pi(r): a lane's 8 values per 16-key step are consecutive keys
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        sacc = Mma<T>::run(frag_rows<T, DH>(ks, row, 2 * s + hf), qf[s], sacc);
        pacc = Mma<T>::run(frag_rows<T, DH>(vs, row, 2 * s + hf), dof[s], pacc);
      }
      TrFrag fr[2][DT];
#pragma unroll
      for (int j = 0; j < DT; ++j) tr_read<DH>(fr[0][j], ks, j * 32, c * 32, lane);
      // element e <-> key key0 + 32 c + 16 (e / 8) + 8 hf + e % 8, lane column <-> query
      V8 dsf[2];
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        const int kbase = key0 + 32 * c + 16 * g + 8 * hf;
        V8 td;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int e = g * 8 + i;
          float p = __builtin_amdgcn_exp2f(sacc[e] * scale_log2 - lse2);
          if (kbase + i > q) p = 0.f;
          td[i] = from_f<T>(p * (pacc[e] - dq_) * gsc);
        }
        dsf[g] = td;
      }
      // dQ^T += K^T dS^T over these 32 keys in 2 steps of 16
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        tr_wait(fr[g]);
        if (g == 0) {
#pragma unroll
          for (int j = 0; j < DT; ++j) tr_read<DH>(fr[1][j], ks, j * 32, c * 32 + 16, lane);
        }
#pragma unroll
        for (int j = 0; j < DT; ++j) acc[j] = Mma<T>::run(tr_value<T>(fr[g][j]), dsf[g], acc[j]);
      }
    }
    // tile t + 1 has landed when only the loads of tiles t + 2 .. t + NS - 1 are outstanding;
    // after the barrier nobody reads tile t any more and its stage is refilled
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((NS - 2) * NLD) : "memory");
    __syncthreads();
    issue(t + NS);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no direct-to-LDS write may outlive the workgroup
  if (q < L) {
    T* row = dqkv + ((long)b * L + q) * ld + (long)head * DH;
    store_grad_row<T, DH>(row, acc, scale / gsc, hf, rope ? rope + (long)q * DH : nullptr);
  }
}

// dK, dV.  A workgroup owns 128 keys (32 per wavefront, K and V fragments in registers) and walks
// the query tiles of 64 rows that can see them.  Q, dO, the log-sum-exp and D of a tile arrive by
// direct-to-LDS loads through a ring of NS stages (three tiles in flight); the transposed
// operands dO^T and Q^T of the second pair of products are read from the same tiles with the
// transposing LDS load.  dS is scaled by a power of two before it is rounded to 16 bits.
template <class T, int DH>
__global__ __launch_bounds__(256) void flash_bwd_dkv_kernel(const T* __restrict__ qkv,
                                                            const T* __restrict__ dO,
                                                            const float* __restrict__ lse,
                                                            const float* __restrict__ dvec,
                                                            T* __restrict__ dqkv, int L, int h,
                                                            float scale, const float* __restrict__ rope) {
  typedef typename Mma<T>::V8 V8;
  constexpr int BKEY = 128, QR = 64, NS = 4, KS = DH / 16, DT = DH / 32;
  constexpr int TILE_B = QR * DH * 2;            // bytes of a Q or dO tile
  constexpr int STAGE_B = 2 * TILE_B + 512;      // Q, dO, 64 log-sum-exp, 64 D
  constexpr int NLT = TILE_B / 1024 / 4;         // wave loads per wavefront and tile
  constexpr int NLD = 2 * NLT + 2;               // loads per wavefront and stage
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  // key tiles in grid.y (dispatched slowest): the long workgroups of all heads start first
  const int ktile = blockIdx.y;
  const int b = blockIdx.x / h, head = blockIdx.x % h;
  const int d = h * DH;
  const long ld = 3L * d;
  const T* qb = qkv + (long)b * L * ld + (long)head * DH;
  const T* kb = qb + d;
  const T* vb = qb + 2 * d;
  const T* dob = dO + (long)b * L * d + (long)head * DH;
  const float* lseb = lse + (long)b * L * h + head;
  const float* dvb = dvec + (long)b * L * h + head;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int col = lane & 31, hf = lane >> 5;
  const int wk0 = ktile * BKEY + wave * 32;
  const int key = wk0 + col;
  const float scale_log2 = scale * 1.4426950408889634f;
  const float gsc = do_scale(dvec + (long)gridDim.x * L + ((long)gridDim.x * L + 3) / 4);

  V8 kf[KS], vf[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    u32x4 z0 = {0u, 0u, 0u, 0u}, z1 = {0u, 0u, 0u, 0u};
    if (key < L) {
      z0 = *(const u32x4*)(kb + (long)key * ld + s * 16 + hf * 8);
      z1 = *(const u32x4*)(vb + (long)key * ld + s * 16 + hf * 8);
    }
    kf[s] = __builtin_bit_cast(V8, z0);
    vf[s] = __builtin_bit_cast(V8, z1);
  }
  f32x16 dk[DT], dv[DT];
#pragma unroll
  for (int j = 0; j < DT; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) dk[j][e] = dv[j][e] = 0.f;
  const unsigned vis = (unsigned)max(L - key, 0);   // queries key .. L - 1 see this lane's key

  // the wait counts below assume that only direct-to-LDS loads are in flight
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  const int qt_first = (ktile * BKEY) / QR;   // first query tile that can see these keys
  const int nt = (L + QR - 1) / QR - qt_first;
  // tile t of this workgroup -> stage t % NS; tiles past the end re-fetch the last one (never
  // used), so that every wavefront always has the same number of loads in flight
  auto issue = [&](int t) {
    const int q0 = (qt_first + min(t, nt - 1)) * QR;
    char* st = smem + (t % NS) * STAGE_B;
#pragma unroll
    for (int j = 0; j < NLT; ++j) {
      dma_rows<T, DH>(qb, ld, q0, L, st, wave * NLT + j, lane);
      dma_rows<T, DH>(dob, d, q0, L, st + TILE_B, wave * NLT + j, lane);
    }
    dma_floats(lseb, h, q0, L, st + 2 * TILE_B, lane);          // every wavefront writes the same values
    dma_floats(dvb, h, q0, L, st + 2 * TILE_B + 256, lane);
  };
#pragma unroll
  for (int t = 0; t < NS; ++t) issue(t);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 1) * NLD) : "memory");
  __syncthreads();

  for (int t = 0; t < nt; ++t) {
    const int q0 = (qt_first + t) * QR;
    const char* qs = smem + (t % NS) * STAGE_B;
    const char* dos = qs + TILE_B;
    const float* lses = (const float*)(qs + 2 * TILE_B);
    const float* ds_ = lses + 64;
    {
      // the tile's 64 queries in two blocks of 32 (keeps the live registers within one wavefront's share)
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        // S = Q K^T and dP = dO V^T for 32 queries x 32 keys; MFMA row r is query pi(r), which
        // makes a lane's 8 values per 16-query step consecutive queries
        f32x16 sacc, pacc;
#pragma unroll
        for (int e = 0; e < 16; ++e) sacc[e] = pacc[e] = 0.f;
        const int row = c * 32 + pi_row(col);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          sacc = Mma<T>::run(frag_rows<T, DH>(qs, row, 2 * s + hf), kf[s], sacc);
          pacc = Mma<T>::run(frag_rows<T, DH>(dos, row, 2 * s + hf), vf[s], pacc);
        }
        // first transposed fragments of this block: their latency hides behind the exponentials
        TrFrag fr[2][DT];
#pragma unroll
        for (int j = 0; j < DT; ++j) tr_read<DH>(fr[0][j], dos, j * 32, c * 32, lane);
        // element e <-> query q0 + 32 c + 16 (e / 8) + 8 hf + e % 8, lane column <-> key
        V8 pf[2], dsf[2];
#pragma unroll
        for (int g = 0; g < 2; ++g) {
          const int r0 = 32 * c + 16 * g + 8 * hf;
          const f32x4 l0 = *(const f32x4*)&lses[r0], l1 = *(const f32x4*)&lses[r0 + 4];
          const f32x4 d0 = *(const f32x4*)&ds_[r0], d1 = *(const f32x4*)&ds_[r0 + 4];
          V8 tp, td;
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const int e = g * 8 + i;
            const float lq = (i < 4 ? l0[i & 3] : l1[i & 3]) * 1.4426950408889634f;
            const float dq = i < 4 ? d0[i & 3] : d1[i & 3];
            float p = __builtin_amdgcn_exp2f(sacc[e] * scale_log2 - lq);
            if ((unsigned)(q0 + r0 - key + i) >= vis) p = 0.f;   // key <= query < L, as one unsigned compare
            tp[i] = from_f<T>(p);
            td[i] = from_f<T>(p * (pacc[e] - dq) * gsc);
          }
          pf[g] = tp;
          dsf[g] = td;
        }
        // dV^T += dO^T P and dK^T += Q^T dS over these 32 queries: 4 steps (dO^T, Q^T) x (16, 16)
#pragma unroll
        for (int st4 = 0; st4 < 4; ++st4) {
          const int g = st4 >> 1, which = st4 & 1;   // which: 0 = dO^T P, 1 = Q^T dS
          tr_wait(fr[st4 & 1]);
          if (st4 + 1 < 4) {
            const int g1 = (st4 + 1) >> 1;
            const char* src = ((st4 + 1) & 1) ? qs : dos;
#pragma unroll
            for (int j = 0; j < DT; ++j) tr_read<DH>(fr[(st4 + 1) & 1][j], src, j * 32, c * 32 + g1 * 16, lane);
          }
#pragma unroll
          for (int j = 0; j < DT; ++j) {
            if (which == 0) dv[j] = Mma<T>::run(tr_value<T>(fr[st4 & 1][j]), pf[g], dv[j]);
            else dk[j] = Mma<T>::run(tr_value<T>(fr[st4 & 1][j]), dsf[g], dk[j]);
          }
        }
      }
    }
    // tile t + 1 has landed when only the loads of tiles t + 2 .. t + NS - 1 are outstanding;
    // after the barrier nobody reads tile t any more and its stage is refilled
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((NS - 2) * NLD) : "memory");
    __syncthreads();
    issue(t + NS);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no direct-to-LDS write may outlive the workgroup
  if (key < L) {
    T* rk = dqkv + ((long)b * L + key) * ld + d + (long)head * DH;
    store_grad_row<T, DH>(rk, dk, scale / gsc, hf, rope ? rope + (long)key * DH : nullptr);
    store_grad_row<T, DH>(rk + d, dv, 1.0f, hf, nullptr);
  }
}

// also records max|dO| per workgroup in dvec[n_items + blockIdx.x]; amax_finish_kernel
// folds those into dvec[n_items + gridDim.x] (no atomics: deterministic and contention-free)
// lse2 (nullable): receives the log-sum-exp in base 2, lse * log2(e), which the head_dim-128 dK/dV kernel reads
template <class T, int DH>
__global__ __launch_bounds__(256) void dvec_kernel(const T* o, const T* dO, long n_items, float* dvec,
                                                   const float* lse, float* lse2) {
  typedef typename Mma<T>::V8 V8;
  constexpr int LPI = DH / 8, IPW = 64 / LPI;   // lanes per (row, head) item (16 bytes each), items per wavefront
  __shared__ float wmax[4];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long item = ((long)blockIdx.x * 4 + wave) * IPW + lane / LPI;
  float s = 0.f, m = 0.f;
  if (item < n_items) {
    const V8 a = *(const V8*)(o + item * DH + (lane % LPI) * 8), g = *(const V8*)(dO + item * DH + (lane % LPI) * 8);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float gi = to_f(g[i]);
      s += to_f(a[i]) * gi;
      m = fmaxf(m, fabsf(gi));
    }
  }
#pragma unroll
  for (int off = 1; off < LPI; off <<= 1) s += __shfl_xor(s, off, 64);
  m = wave_max(m);
  if (item < n_items && lane % LPI == 0) {
    dvec[item] = s;
    if (lse2) lse2[item] = lse[item] * 1.4426950408889634f;
  }
  if (lane == 0) wmax[wave] = m;
  __syncthreads();
  if (threadIdx.x == 0) dvec[n_items + blockIdx.x] = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
}
// maximum of blockmax[0 .. nb - 1] -> blockmax[out]
__global__ __launch_bounds__(1024) void amax_finish_kernel(float* blockmax, long nb, long out) {
  __shared__ float red[16];
  // independent partial maxima per thread: the loads of one thread do not wait for each other
  float m0 = 0.f, m1 = 0.f, m2 = 0.f, m3 = 0.f;
  long i = threadIdx.x;
  for (; i + 3 * 1024 < nb; i += 4 * 1024) {
    m0 = fmaxf(m0, blockmax[i]);
    m1 = fmaxf(m1, blockmax[i + 1024]);
    m2 = fmaxf(m2, blockmax[i + 2 * 1024]);
    m3 = fmaxf(m3, blockmax[i + 3 * 1024]);
  }
  for (; i < nb; i += 1024) m0 = fmaxf(m0, blockmax[i]);
  float m = wave_max(fmaxf(fmaxf(m0, m1), fmaxf(m2, m3)));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x < 64) {
    m = wave_max(threadIdx.x < 16 ? red[threadIdx.x] : 0.f);
    if (threadIdx.x == 0) blockmax[out] = m;
  }
}

template <class T, int DH>
ls_status launch_bwd(const void* qkv, const void* o, const void* dO, const float* lse, int B, int L, int h,
                     void* dqkv, float* dvec, const float* rope, hipStream_t st) {
  const float scale = 1.0f / sqrtf((float)DH);
  const long items = (long)B * L * h;
  const long nb = (items + 3) / 4;
  // the scratch keeps room for one maximum per four items; the kernel fills one per 4 * (512 / head_dim)
  const long nwg = (items + 4 * (512 / DH) - 1) / (4 * (512 / DH));
  float* lse2 = DH == 128 ? dvec + items + nb + 1 : nullptr;   // after D, the per-workgroup maxima and their maximum
  dvec_kernel<T, DH><<<(unsigned)nwg, 256, 0, st>>>((const T*)o, (const T*)dO, items, dvec, lse, lse2);
  amax_finish_kernel<<<1, 1024, 0, st>>>(dvec + items, nwg, nb);
  LS_CHECK_LAUNCH();
  dim3 gq(B * h, (L + 127) / 128), gk(B * h, (L + 127) / 128);
  constexpr int dq_lds = 4 * (2 * KT * DH * 2);
  static bool dq_attr = false;
  if constexpr (DH == 128) {
    if (!dq_attr) {
      LS_CHECK_HIP(hipFuncSetAttribute((const void*)flash_bwd_dq128_kernel<T>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, dq_lds));
      dq_attr = true;
    }
    flash_bwd_dq128_kernel<T><<<gq, 256, dq_lds, st>>>((const T*)qkv, (const T*)dO, lse2, dvec, (T*)dqkv, L, h, scale, rope);
  } else {
    if (!dq_attr) {
      LS_CHECK_HIP(hipFuncSetAttribute((const void*)flash_bwd_dq_kernel<T, DH>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, dq_lds));
      dq_attr = true;
    }
    flash_bwd_dq_kernel<T, DH><<<gq, 256, dq_lds, st>>>((const T*)qkv, (const T*)dO, lse, dvec, (T*)dqkv, L, h, scale, rope);
  }
  LS_CHECK_LAUNCH();
  constexpr int dkv_lds = 4 * (2 * 64 * DH * 2 + 512);
  static bool dkv_attr = false;
  if constexpr (DH == 128) {
    if (!dkv_attr) {
      LS_CHECK_HIP(hipFuncSetAttribute((const void*)flash_bwd_dkv128_kernel<T>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, dkv_lds));
      dkv_attr = true;
    }
    flash_bwd_dkv128_kernel<T><<<gk, 256, dkv_lds, st>>>((const T*)qkv, (const T*)dO, lse2, dvec, (T*)dqkv, L, h, scale, rope);
    LS_CHECK_LAUNCH();
    return LS_OK;
  }
  if (!dkv_attr) {
    LS_CHECK_HIP(hipFuncSetAttribute((const void*)flash_bwd_dkv_kernel<T, DH>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, dkv_lds));
    dkv_attr = true;
  }
  flash_bwd_dkv_kernel<T, DH><<<gk, 256, dkv_lds, st>>>((const T*)qkv, (const T*)dO, lse, dvec, (T*)dqkv, L, h, scale, rope);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

}  // namespace

extern "C" ls_status lsk_attn_fwd_mfma(const void* qkv, int dt, int B, int L, int h, int dh, void* o,
                                       float* lse, void* stream) {
  LsTimed timed(LSK_TIMED_ATTN_FWD, stream);
  LS_REQUIRE(qkv && o && B > 0 && L > 0 && h > 0, "attn_fwd: bad argument");
  LS_REQUIRE(dt == LS_BF16 || dt == LS_F16, "attn_fwd: the matrix-core kernel needs 16-bit operands");
  LS_REQUIRE(dh == 64 || dh == 128, "attn_fwd: the matrix-core kernel needs head_dim 64 or 128");
  LS_REQUIRE((long)B * h <= 65535, "attn_fwd: B * n_heads exceeds the grid limit");
  hipStream_t st = (hipStream_t)stream;
  if (dt == LS_BF16) return dh == 64 ? launch_fwd<bf16_t, 64>(qkv, B, L, h, o, lse, st)
                                     : launch_fwd<bf16_t, 128>(qkv, B, L, h, o, lse, st);
  return dh == 64 ? launch_fwd<f16_t, 64>(qkv, B, L, h, o, lse, st)
                  : launch_fwd<f16_t, 128>(qkv, B, L, h, o, lse, st);
}

// Prefill attention over the paged pool: request r owns rows start[r] .. start[r+1]-1 of qkv
// (start on the host, n_req + 1 entries, n_req <= 32); its K/V rows are already in the pool.
extern "C" ls_status lsk_attn_prefill_mfma(const void* qkv, int dt, int n_req, const int32_t* start_host, int h,
                                           int dh, const void* k_pool, const void* v_pool,
                                           const int32_t* block_table, const int32_t* ctx_len, int max_pages,
                                           int page, void* o, void* stream) {
  LsTimed timed(LSK_TIMED_ATTN_FWD, stream);
  LS_REQUIRE(qkv && o && start_host && k_pool && v_pool && block_table && ctx_len, "attn_prefill: null argument");
  LS_REQUIRE(n_req > 0 && n_req <= 32, "attn_prefill: 1..32 requests per call");
  LS_REQUIRE(dt == LS_BF16 || dt == LS_F16, "attn_prefill: 16-bit operands only");
  LS_REQUIRE(dh == 64 || dh == 128, "attn_prefill: head_dim must be 64 or 128");
  PagedGeom pg{k_pool, v_pool, block_table, ctx_len, max_pages, page, n_req, {0}};
  int max_chunk = 0;
  for (int r = 0; r <= n_req; ++r) pg.start[r] = start_host[r];
  for (int r = 0; r < n_req; ++r) max_chunk = max_chunk > pg.start[r + 1] - pg.start[r] ? max_chunk : pg.start[r + 1] - pg.start[r];
  LS_REQUIRE(max_chunk > 0, "attn_prefill: empty chunks");
  hipStream_t st = (hipStream_t)stream;
  if (dt == LS_BF16) return dh == 64 ? launch_prefill<bf16_t, 64>(qkv, h, o, pg, max_chunk, st)
                                     : launch_prefill<bf16_t, 128>(qkv, h, o, pg, max_chunk, st);
  return dh == 64 ? launch_prefill<f16_t, 64>(qkv, h, o, pg, max_chunk, st)
                  : launch_prefill<f16_t, 128>(qkv, h, o, pg, max_chunk, st);
}

// rope_table (nullable): [position][head_dim/2][cos, sin]; when given, dq and dk are rotated back
// by their positions before they are stored (the backward of the rotary embedding, fused)
extern "C" ls_status lsk_attn_bwd_mfma(const void* qkv, const void* o, const void* dO, const float* lse,
                                       int dt, int B, int L, int h, int dh, void* dqkv, float* dvec,
                                       const float* rope_table, void* stream) {
  LsTimed timed(LSK_TIMED_ATTN_BWD, stream);
  LS_REQUIRE(qkv && o && dO && lse && dqkv && dvec && B > 0 && L > 0 && h > 0, "attn_bwd: bad argument");
  LS_REQUIRE(dt == LS_BF16 || dt == LS_F16, "attn_bwd: the matrix-core kernel needs 16-bit operands");
  LS_REQUIRE(dh == 64 || dh == 128, "attn_bwd: the matrix-core kernel needs head_dim 64 or 128");
  LS_REQUIRE((long)B * h <= 65535, "attn_bwd: B * n_heads exceeds the grid limit");
  hipStream_t st = (hipStream_t)stream;
  if (dt == LS_BF16) return dh == 64 ? launch_bwd<bf16_t, 64>(qkv, o, dO, lse, B, L, h, dqkv, dvec, rope_table, st)
                                     : launch_bwd<bf16_t, 128>(qkv, o, dO, lse, B, L, h, dqkv, dvec, rope_table, st);
  return dh == 64 ? launch_bwd<f16_t, 64>(qkv, o, dO, lse, B, L, h, dqkv, dvec, rope_table, st)
                  : launch_bwd<f16_t, 128>(qkv, o, dO, lse, B, L, h, dqkv, dvec, rope_table, st);
}
