// Large-tile MFMA GEMM whose operand tiles go from global memory straight into
// LDS (16-byte direct-to-LDS loads, no register staging, no LDS store
// instructions).  256 x 256 x 64 tiles (4 wavefronts of 128 x 128) or 128 x 128 x 64
// tiles (4 wavefronts of 64 x 64) for problems with few tiles, 32x32x16 MFMA, two
// LDS buffers.  Used when the contraction length is a multiple of 64; the
// register-staged kernel in gemm.hip covers everything else.
//
// LDS layouts (a direct-to-LDS wave load writes 1 KB: lane i -> bytes 16 i):
//   k-major operand  (element (r,k) at r*ld + k): [256 rows][64 k], 128 B per
//     row, the eight 16-byte chunks of a row XOR-permuted with (row >> 1) & 7,
//     so that the 16-byte fragment reads of 16 consecutive rows hit 16
//     different bank groups.  Fragments: one 16-byte LDS read per 8 k.
//   k-strided operand (element (r,k) at k*ld + r): [64 k][256 rows], 512 B per
//     k, chunk index XOR-permuted with 4 * (k & 3).  Fragments are read with the
//     transposing LDS load (4 k x 16 rows per 16 lanes), two per 8 k.
// The permutations are applied by choosing which global chunk each lane fetches.
//
// With one wavefront per SIMD nothing hides a stalled wavefront, so the k loop is
// software-pipelined by hand: the next tile's loads are issued a few at a time
// between the MFMAs of the first half of a tile (a burst of 16 loads blocks the
// wavefront on the address path for about as long as the tile's MFMAs take), the
// LDS reads of the next fragments run under the current MFMAs, and the single
// workgroup barrier per tile sits before the last quarter of the MFMAs.
#include "gemm_dma_common.h"

namespace {

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

template <class T> struct Mf;
template <> struct Mf<bf16_t> {
  typedef bf16x8 V8;
  typedef bf16x4 V4;
  static __device__ __forceinline__ f32x16 run(V8 a, V8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ V4 tr(const void* p) {
    return __builtin_bit_cast(V4, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p));
  }
};
template <> struct Mf<f16_t> {
  typedef f16x8 V8;
  typedef f16x4 V4;
  static __device__ __forceinline__ f32x16 run(V8 a, V8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ V4 tr(const void* p) {
    return __builtin_bit_cast(V4, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p));
  }
};

// One operand fragment: 8 k for 32 rows of an operand tile.
//  - k-major tiles: one ordinary 16-byte LDS load, tracked by the compiler.
//  - k-strided tiles: two transposing LDS loads.  These are issued from inline assembly: before
//    the builtin form the compiler waits for every direct-to-LDS load in flight (it cannot tell
//    that the tile being filled is another one), which serialises loads and arithmetic.  The
//    assembly form is invisible to the compiler's wait-count bookkeeping, so wait_frags() must
//    run between the reads and the first use; it redefines the registers, which pins the order.
template <class T, bool KMAJOR> struct Frag { typename Mf<T>::V8 v; };
template <class T> struct Frag<T, false> { s16x4 lo, hi; };

template <class T, bool KMAJOR, int ROWS>
__device__ __forceinline__ void read_frag(Frag<T, KMAJOR>& f, const char* lds_tile, int r0, int ks, int lane) {
  typedef typename Mf<T>::V8 V8;
  const int hf = lane >> 5;
  if constexpr (KMAJOR) {
    const int r = r0 + (lane & 31);
    const int kc = (ks * 2 + hf) ^ ((r >> 1) & 7);
    f.v = *(const V8*)(lds_tile + r * 128 + kc * 16);
  } else {
    constexpr int KROW = ROWS * 2;  // bytes per k row
    const int i16 = lane & 15, a = i16 >> 2, j4 = i16 & 3;
    const int nb = r0 + 16 * ((lane >> 4) & 1) + 4 * j4;  // first of the 4 rows this lane addresses
    const int kb = ks * 16 + 8 * hf;
    const int phys = (nb >> 3) ^ (4 * a);
    const char* p0 = lds_tile + (kb + a) * KROW + phys * 16 + ((nb >> 2) & 1) * 8;
    const uint32_t addr = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)p0;
    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(f.lo) : "v"(addr) : "memory");
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.hi) : "v"(addr), "n"(4 * KROW) : "memory");
  }
}

template <class T, bool KMAJOR, int N>
__device__ __forceinline__ void wait_frags(Frag<T, KMAJOR> (&f)[N]) {
  static_assert(KMAJOR || N == 2 || N == 4, "fragment count");
  if constexpr (!KMAJOR) {
    if constexpr (N == 4)
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi), "+v"(f[2].lo), "+v"(f[2].hi),
                     "+v"(f[3].lo), "+v"(f[3].hi));
    else
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi));
  }
}

template <class T, bool KMAJOR>
__device__ __forceinline__ typename Mf<T>::V8 frag_value(const Frag<T, KMAJOR>& f) {
  if constexpr (KMAJOR) {
    return f.v;
  } else {
    const s16x8 w = __builtin_shufflevector(f.lo, f.hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(typename Mf<T>::V8, w);
  }
}

// MODE 0: C (16-bit) = acc + bias;  1: C (fp32) = resid + acc + bias;  2: C (fp32) = acc;  4: C (fp32) += acc;
// MODE 3: as 0 without bias, and the half-split rotary embedding (head_dim 128) applied to the
//         columns below rope_cols: a wavefront's 128 columns are one head, so the pair
//         (c, c + 64) sits in accumulator tiles j and j + 2 of the same lane
template <class T, int BM, int BN, bool AK, bool BK, int MODE>
__global__ __launch_bounds__(256) void gemm_dma_kernel(DmaArgs g) {
  typedef typename Mf<T>::V8 V8;
  constexpr int TM = BM, TN = BN;
  constexpr int WM = BM / 2, WN = BN / 2;       // wavefront tile
  constexpr int TI = WM / 32, TJ = WN / 32;     // 32x32 MFMA tiles per wavefront
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, BUF_BYTES = A_BYTES + B_BYTES;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  // buffer b: A tile at smem + b BUF_BYTES, B tile A_BYTES after it

  // workgroups that run at the same time share operand tiles through L2:
  // walk M fastest inside bands of 8 N tiles
  // (consecutive workgroup ids are dealt round-robin to the 8 XCDs, each with its
  // own L2: give every XCD a contiguous run of the tile order instead)
  const int total = g.tiles_m * g.tiles_n, per_xcd = total / 8;
  int bid = blockIdx.x;
  if (bid < per_xcd * 8) bid = (bid % 8) * per_xcd + bid / 8;
  const int band = 8;
  const int per_band = band * g.tiles_m;
  const int b0 = (bid / per_band) * band;
  const int bw = min(band, g.tiles_n - b0);
  const int rem = bid % per_band;
  const int tn = b0 + rem % bw, tm = rem / bw;
  const int m0 = tm * TM, n0 = tn * TN;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wm = (wave >> 1) * WM, wn = (wave & 1) * WN;
  // uniform tile bases (bytes) and their advance per k step
  const char* a_base = (const char*)g.A + (AK ? (long)m0 * g.lda : (long)m0) * 2;
  const char* b_base = (const char*)g.B + (BK ? (long)n0 * g.ldb : (long)n0) * 2;
  const long a_step = (AK ? (long)TK : (long)TK * g.lda) * 2;
  const long b_step = (BK ? (long)TK : (long)TK * g.ldb) * 2;
  uint32_t a_off[BM / 32], b_off[BN / 32];
  tile_offsets<AK, BM>(a_off, g.lda, m0, g.M, wave, lane);
  tile_offsets<BK, BN>(b_off, g.ldb, n0, g.N, wave, lane);

  f32x16 acc[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // gridDim.y > 1: split-K, this workgroup contracts over its share of the k tiles
  const int nk_all = g.K / TK;
  const int kt0 = (int)((long)blockIdx.y * nk_all / gridDim.y);
  const int nk = (int)((long)(blockIdx.y + 1) * nk_all / gridDim.y) - kt0;
  a_base += kt0 * a_step;
  b_base += kt0 * b_step;
  issue_tile<BM>(a_base, a_off, smem, wave);
  issue_tile<BN>(b_base, b_off, smem + A_BYTES, wave);

  // Software pipeline of one k tile (4 sub-steps of 16 k): while the MFMAs of a sub-step run, the
  // fragments of the next one are read from LDS, and during LDKS sub-steps direct-to-LDS loads are
  // issued, at most one memory instruction between two MFMAs (a burst would stall the wavefront,
  // and with it the matrix pipe, on the address path).  The workgroup barrier sits
  // before the last sub-step: by then every wavefront holds its last fragments of the current
  // tile in registers, so the fragments read during the last sub-step come from the next tile.
  // Every MFMA and what follows it are fenced with scheduling barriers: the source order below is the issue order.
  constexpr int NM = TI * TJ;            // MFMAs per k sub-step
  constexpr int NF = TI + TJ;            // fragments per k sub-step
  constexpr int NLD = (BM + BN) / 32;    // direct-to-LDS loads per tile and wavefront
  constexpr int LDKS = 2;                // k sub-steps over which they are issued
  constexpr int LD_FIRST = 3;            // the first of them: sub-step 3 is the first after the barrier that frees a buffer
  constexpr int LPK = NLD / LDKS;        // loads per sub-step
  static_assert(NLD % LDKS == 0, "loads per sub-step");
  constexpr GapPlan<NM, NF, LPK> plan{};
  if (LD_FIRST > 0) {
    // what sub-steps LD_FIRST .. 3 of the tile before the first would have issued
    const int t1 = nk > 1 ? 1 : 0;
#pragma unroll
    for (int l = 0; l < (4 - LD_FIRST) * NLD / LDKS; ++l)
      issue_one<BM, BN>(l, a_base + t1 * a_step, a_off, b_base + t1 * b_step, b_off, smem + BUF_BYTES,
                        smem + BUF_BYTES + A_BYTES, wave);
  }
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  Frag<T, AK> fa[2][TI];
  Frag<T, BK> fb[2][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i) read_frag<T, AK, BM>(fa[0][i], smem, wm + i * 32, 0, lane);
#pragma unroll
  for (int j = 0; j < TJ; ++j) read_frag<T, BK, BN>(fb[0][j], smem + A_BYTES, wn + j * 32, 0, lane);

  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    const char* la = smem + cur * BUF_BYTES;
    const char* lb = la + A_BYTES;
    char* na = smem + (cur ^ 1) * BUF_BYTES;
    char* nb = na + A_BYTES;
    // tiles after the last are the last again: fetched, never multiplied
    const int t1 = min(kt + 1, nk - 1), t2 = min(kt + 2, nk - 1);
    const char* ga1 = a_base + t1 * a_step;
    const char* gb1 = b_base + t1 * b_step;
    const char* ga2 = a_base + t2 * a_step;
    const char* gb2 = b_base + t2 * b_step;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int c = ks & 1;
      wait_frags<T, AK, TI>(fa[c]);
      wait_frags<T, BK, TJ>(fb[c]);
      if (ks == 3) {
        __builtin_amdgcn_s_waitcnt(0);   // this wavefront's share of the next tile has landed
        __syncthreads();
      }
      V8 va[TI], vb[TJ];
#pragma unroll
      for (int i = 0; i < TI; ++i) va[i] = frag_value<T, AK>(fa[c][i]);
#pragma unroll
      for (int j = 0; j < TJ; ++j) vb[j] = frag_value<T, BK>(fb[c][j]);
      const char* ra = ks < 3 ? la : na;
      const char* rb = ks < 3 ? lb : nb;
      const int kn = (ks + 1) & 3;
      __builtin_amdgcn_sched_barrier(0);
      // sub-steps LD_FIRST .. 3 come after this tile's barrier: the buffer being vacated takes the tile
      // after the next; sub-steps before LD_FIRST complete the next tile in the other buffer
      const int ph = (ks - LD_FIRST) & 3;
      const bool ahead = LD_FIRST > 0 && ks >= LD_FIRST;
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        // the wavefront's 32 x 32 tiles in boustrophedon order: consecutive MFMAs share an operand (0.4 %)
        const int ti = m / TJ, tj = (ti & 1) ? TJ - 1 - m % TJ : m % TJ;
        acc[ti][tj] = Mf<T>::run(vb[tj], va[ti], acc[ti][tj]);
        __builtin_amdgcn_sched_barrier(0);   // the MFMA first: what follows issues in its shadow
#pragma unroll
        for (int r = 0; r < NF; ++r) {
          if (plan.read_gap[r] != m) continue;
          if (r < TI) read_frag<T, AK, BM>(fa[c ^ 1][r], ra, wm + r * 32, kn, lane);
          else read_frag<T, BK, BN>(fb[c ^ 1][r - TI], rb, wn + (r - TI) * 32, kn, lane);
        }
        if (ph < LDKS) {
#pragma unroll
          for (int l = 0; l < LPK; ++l) {
            if (plan.load_gap[l] != m) continue;
            issue_one<BM, BN>(ph * LPK + l, ahead ? ga2 : ga1, a_off, ahead ? gb2 : gb1, b_off, ahead ? (char*)la : na,
                              ahead ? (char*)lb : nb, wave);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  // The last iteration read the fragments of a tile that does not exist.  Their registers must
  // stay allocated until the reads have returned: the compiler does not know that the
  // transposing reads issued from assembly are still in flight and would hand the registers to
  // the epilogue, where the late LDS data would overwrite live values.
  wait_frags<T, AK, TI>(fa[0]);
  wait_frags<T, BK, TJ>(fb[0]);
  __builtin_amdgcn_s_waitcnt(0);

  // Epilogue.  The MFMAs ran with the operands swapped, so the accumulators hold C^T tiles:
  // lane -> row m (lane & 31), register 4 q + e -> column 8 q + 4 (lane >> 5) + e.  Storing
  // from that layout touches 32 rows per instruction, 16 bytes in each, which the memory
  // pipeline takes far longer over than over the same bytes as whole cache lines.  So each
  // wavefront stages its tile in its quarter of the (now idle) LDS, row-major with the 16-byte
  // chunks of a row XOR-permuted by the row number, and writes it out as full rows; residual
  // and accumulation operands are read with the same coalesced pattern.
  typedef typename Mf<T>::V4 V4;
  constexpr int ESZ = (MODE == 0 || MODE == 3) ? 2 : 4;
  constexpr int REGION = (BM + BN) * 128 * 2 / 4;   // bytes of LDS per wavefront
  constexpr int ROWB = WN * ESZ;                    // bytes of a staged row
  constexpr int CPR = ROWB / 16;                    // 16-byte chunks per row
  constexpr int NPASS = (WM * ROWB + REGION - 1) / REGION;
  constexpr int TIP = TI / NPASS;                   // 32-row MFMA tiles per pass
  constexpr int ROWS_P = TIP * 32;
  const int row_in = lane & 31, hf = lane >> 5;
  const float alpha = g.alpha ? *g.alpha : 1.f;
  __syncthreads();   // every wavefront is done with the operand tiles
  char* stg = smem + wave * REGION;
  // A lane's columns are the same for all of its rows: its bias values are fetched once, outside the
  // staging loops (a fetch with a type switch inside them, once per element, made the epilogue some
  // thousands of instructions long and cost 3 - 6 us per launch even without a bias).
  float bv[TJ][4][4];
#pragma unroll
  for (int j = 0; j < TJ; ++j)
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int e = 0; e < 4; ++e) bv[j][q][e] = 0.f;
  if ((MODE == 0 || MODE == 1) && g.bias) {
    const int nb = n0 + wn + 4 * hf;
    auto fetch = [&](auto* b) {
#pragma unroll
      for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int n = nb + j * 32 + 8 * q + e;
            bv[j][q][e] = (float)b[n < g.N ? n : g.N - 1];
          }
    };
    if (g.bias_dtype == LS_F32) fetch((const float*)g.bias);
    else if (g.bias_dtype == LS_BF16) fetch((const bf16_t*)g.bias);
    else fetch((const f16_t*)g.bias);
  }
#pragma unroll
  for (int pass = 0; pass < NPASS; ++pass) {
    // results added to a buffer (the residual stream, or the output itself): what the pass adds to is fetched
    // first, all of it at once, and arrives while the accumulators are staged (a load per store, each behind its
    // own branch and wait, made an accumulating launch a sixth longer)
    constexpr int NOUT = ROWS_P * CPR / 64;
    constexpr bool ADDS = MODE == 1 || MODE == 4;
    f32x4 c_old[ADDS ? NOUT : 1];
    if constexpr (ADDS) {
      const float* src = MODE == 1 ? g.resid : (const float*)g.C + blockIdx.y * g.split_stride;
      const long ld_src = MODE == 1 ? g.ldr : g.ldc;
#pragma unroll
      for (int it = 0; it < NOUT; ++it) {
        const int idx = it * 64 + lane;
        const int m = m0 + wm + pass * ROWS_P + idx / CPR;
        const int n = n0 + wn + (idx % CPR) * (16 / ESZ);
        c_old[it] = m < g.M && n < g.N ? *(const f32x4*)(src + (long)m * ld_src + n) : f32x4{0.f, 0.f, 0.f, 0.f};
      }
    }
#pragma unroll
    for (int ii = 0; ii < TIP; ++ii) {
      const int i = pass * TIP + ii;
      const int r = ii * 32 + row_in;
      char* srow = stg + r * ROWB;
      const int sw = r & (CPR - 1);
      if constexpr (MODE == 3) {
        if constexpr (TJ == 4) {
          const int m = min(m0 + wm + i * 32 + row_in, g.M - 1);   // rows past the edge are staged, never stored
          const bool rot = n0 + wn < g.rope_cols;   // q or k section: uniform over the wavefront
          const float* tab = g.rope_table + (long)g.rope_pos[m] * 128 + 8 * hf;   // 64 (cos, sin) pairs
#pragma unroll
          for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              V4 lo, hi;
              if (rot) {
                const f32x4 cs0 = *(const f32x4*)(tab + (j * 32 + 8 * q) * 2);
                const f32x4 cs1 = *(const f32x4*)(tab + (j * 32 + 8 * q) * 2 + 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  const float c = e < 2 ? cs0[2 * e] : cs1[2 * (e - 2)];
                  const float sn = e < 2 ? cs0[2 * e + 1] : cs1[2 * (e - 2) + 1];
                  const float a = acc[i][j][4 * q + e], bb = acc[i][j + 2][4 * q + e];
                  lo[e] = from_f<T>(a * c - bb * sn);
                  hi[e] = from_f<T>(bb * c + a * sn);
                }
              } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  lo[e] = from_f<T>(acc[i][j][4 * q + e]);
                  hi[e] = from_f<T>(acc[i][j + 2][4 * q + e]);
                }
              }
              *(u32x2_a*)(srow + (((j * 4 + q) ^ sw) * 16) + hf * 8) = __builtin_bit_cast(u32x2_t, lo);
              *(u32x2_a*)(srow + (((j * 4 + q + 8) ^ sw) * 16) + hf * 8) = __builtin_bit_cast(u32x2_t, hi);
            }
        }
      } else {
#pragma unroll
        for (int j = 0; j < TJ; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            f32x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * q + e] * alpha;
            if constexpr (MODE == 0 || MODE == 1) {
#pragma unroll
              for (int e = 0; e < 4; ++e) v[e] += bv[j][q][e];
            }
            if constexpr (ESZ == 2) {
              V4 o;
#pragma unroll
              for (int e = 0; e < 4; ++e) o[e] = from_f<T>(v[e]);
              *(u32x2_a*)(srow + (((j * 4 + q) ^ sw) * 16) + hf * 8) = __builtin_bit_cast(u32x2_t, o);
            } else {
              *(f32x4_a*)(srow + (((j * 8 + 2 * q + hf) ^ sw) * 16)) = v;
            }
          }
      }
    }
    // full rows out: 64 / CPR rows per instruction, 16 bytes per lane
    constexpr int NIT = ROWS_P * CPR / 64, GRP = NIT % 8 == 0 ? 8 : NIT;
    auto put = [&](int it, int m, int n, const f32x4& v) {
      if constexpr (ESZ == 2) {
        *(f32x4_a*)((T*)g.C + (long)m * g.ldc + n) = v;
      } else if constexpr (MODE == 1) {
        *(f32x4*)((float*)g.C + (long)m * g.ldc + n) = v + c_old[it];
      } else {
        *(f32x4*)((float*)g.C + blockIdx.y * g.split_stride + (long)m * g.ldc + n) = MODE == 4 ? c_old[it] + v : v;
      }
    };
    if (m0 + wm + pass * ROWS_P + ROWS_P <= g.M && n0 + wn + WN <= g.N) {
      // uniform: every row and column of the pass exists, so nothing depends on the lane and a group of staged
      // pieces is read before it is stored (under the per-lane bounds check below the compiler moves each read to
      // its store and waits for it there: one LDS round trip after the other)
#pragma unroll
      for (int it0 = 0; it0 < NIT; it0 += GRP) {
        f32x4 v[GRP];
#pragma unroll
        for (int u = 0; u < GRP; ++u) {
          const int idx = (it0 + u) * 64 + lane;
          const int r = idx / CPR, c = idx % CPR;
          v[u] = *(const f32x4_a*)(stg + r * ROWB + ((c ^ (r & (CPR - 1))) * 16));
        }
#pragma unroll
        for (int u = 0; u < GRP; ++u) {
          const int idx = (it0 + u) * 64 + lane;
          put(it0 + u, m0 + wm + pass * ROWS_P + idx / CPR, n0 + wn + (idx % CPR) * (16 / ESZ), v[u]);
        }
      }
    } else {
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int idx = it * 64 + lane;
        const int r = idx / CPR, c = idx % CPR;
        const int m = m0 + wm + pass * ROWS_P + r;
        const int n = n0 + wn + c * (16 / ESZ);
        if (m >= g.M || n >= g.N) continue;
        put(it, m, n, *(const f32x4_a*)(stg + r * ROWB + ((c ^ (r & (CPR - 1))) * 16)));
      }
    }
  }
}

template <class T, int BM, int BN, bool AK, bool BK, int MODE>
ls_status launch(DmaArgs g, hipStream_t st, int splits = 1) {
  static bool attr_set = false;
  const int lds = 2 * (BM + BN) * 128;
  if (!attr_set) {
    LS_CHECK_HIP(hipFuncSetAttribute((const void*)gemm_dma_kernel<T, BM, BN, AK, BK, MODE>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    attr_set = true;
  }
  g.tiles_m = (g.M + BM - 1) / BM;
  g.tiles_n = (g.N + BN - 1) / BN;
  gemm_dma_kernel<T, BM, BN, AK, BK, MODE><<<dim3(g.tiles_m * g.tiles_n, splits), 256, lds, st>>>(g);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

// the combinations a decoder block uses: forward (k-major x k-major, 16-bit or
// residual output), input gradient (k-major x k-strided, 16-bit output), weight
// gradient (k-strided x k-strided, fp32 output)
template <class T, int BM, int BN>
ls_status dispatch_layout(const DmaArgs& g, hipStream_t st) {
  if (g.rope_table) {
    if (BM == 256 && g.a_kmajor && g.b_kmajor && g.c_dtype != LS_F32 && !g.bias)
      return launch<T, 256, 256, true, true, 3>(g, st);
    return LS_ESTATE;
  }
  const int mode = g.c_dtype != LS_F32 ? 0 : (g.resid ? 1 : (g.accumulate ? 4 : 2));
  if (mode >= 2 && g.bias) return LS_ESTATE;
  if (mode == 1 && g.accumulate) return LS_ESTATE;
  if (g.a_kmajor && g.b_kmajor && mode == 0) return launch<T, BM, BN, true, true, 0>(g, st);
  if (g.a_kmajor && g.b_kmajor && mode == 1) return launch<T, BM, BN, true, true, 1>(g, st);
  if (g.a_kmajor && g.b_kmajor && mode == 2) return launch<T, BM, BN, true, true, 2>(g, st);
  if (g.a_kmajor && g.b_kmajor && mode == 4) return launch<T, BM, BN, true, true, 4>(g, st);
  if (g.a_kmajor && !g.b_kmajor && mode == 0) return launch<T, BM, BN, true, false, 0>(g, st);
  if (g.a_kmajor && !g.b_kmajor && mode == 2) return launch<T, BM, BN, true, false, 2>(g, st);
  if (g.a_kmajor && !g.b_kmajor && mode == 4) return launch<T, BM, BN, true, false, 4>(g, st);
  if (!g.a_kmajor && !g.b_kmajor && mode == 2) return launch<T, BM, BN, false, false, 2>(g, st);
  if (!g.a_kmajor && !g.b_kmajor && mode == 4) return launch<T, BM, BN, false, false, 4>(g, st);
  return LS_ESTATE;
}

// 256 x 256 tiles when they still give most compute units a workgroup, else 128 x 128
template <class T>
ls_status dispatch(const DmaArgs& g, hipStream_t st) {
  const long big = (long)((g.M + 255) / 256) * ((g.N + 255) / 256);
  if (big >= 160) return dispatch_layout<T, 256, 256>(g, st);
  return dispatch_layout<T, 128, 128>(g, st);
}

}  // namespace

namespace {

// C = sum over the splits (in order) of the fp32 partial results, + bias + residual
template <class T>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* partial, int splits, long MN, int N,
                                                            void* C, long ldc, int c_dtype, const void* bias,
                                                            int bias_dtype, const float* resid, long ldr) {
  const long i4 = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i4 >= MN) return;
  f32x4 v = *(const f32x4*)(partial + i4);
  for (int s = 1; s < splits; ++s) v += *(const f32x4*)(partial + s * MN + i4);
  const long m = i4 / N;
  const int n = (int)(i4 % N);
  if (bias) {
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] += load_as_f(bias, n + e, bias_dtype);
  }
  if (resid) v += *(const f32x4*)(resid + m * ldr + n);
  if (c_dtype == LS_F32) {
    *(f32x4*)((float*)C + m * ldc + n) = v;
  } else {
    typename Mf<T>::V4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = from_f<T>(v[e]);
    *(typename Mf<T>::V4*)((T*)C + m * ldc + n) = o;
  }
}

template <class T, int BM = 128>
ls_status run_splitk(DmaArgs g, int splits, float* scratch, void* C, long ldc, int c_dtype, const void* bias,
                     int bias_dtype, const float* resid, long ldr, hipStream_t st) {
  const long MN = (long)g.M * g.N;
  g.C = scratch; g.ldc = g.N; g.c_dtype = LS_F32; g.bias = nullptr; g.resid = nullptr; g.accumulate = 0;
  g.split_stride = MN;
  LS_TRY((launch<T, BM, 128, true, true, 2>(g, st, splits)));
  splitk_reduce_kernel<T><<<(unsigned)((MN / 4 + 255) / 256), 256, 0, st>>>(scratch, splits, MN, g.N, C, ldc, c_dtype,
                                                                          bias, bias_dtype, resid, ldr);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

}  // namespace

// Forward-layout GEMM (both operands k-major) for problems with too few output tiles to fill
// the chip: the contraction is split over `splits` workgroups per tile, partial results go to
// `scratch` (fp32, splits * M * N) and are summed in a fixed order (deterministic).  Returns
// LS_ESTATE when the shape does not call for it or the scratch is too small.
ls_status gemm_dma_splitk_try(int op_dtype, int M, int N, int K, const void* A, long lda, const void* B, long ldb,
                              void* C, long ldc, int c_dtype, const void* bias, int bias_dtype,
                              const float* resid, long ldr, float* scratch, size_t scratch_floats,
                              hipStream_t st) {
  if (!scratch || K % TK != 0 || M < 64 || N < 64 || N % 4 != 0) return LS_ESTATE;
  const int per16 = c_dtype == LS_F32 ? 4 : 8;
  if (ldc % per16 != 0 || (uintptr_t)C % 16 != 0 || (uintptr_t)scratch % 16 != 0) return LS_ESTATE;
  if (resid && (ldr % 4 != 0 || (uintptr_t)resid % 16 != 0)) return LS_ESTATE;
  const long tiles = (long)((M + 127) / 128) * ((N + 127) / 128);
  const int nk = K / TK;
  if (tiles >= 200 || nk < 32) return LS_ESTATE;
  int splits = (int)(512 / tiles);
  if (splits > 8) splits = 8;
  while (splits > 1 && nk / splits < 8) --splits;
  while (splits > 1 && (size_t)splits * M * N > scratch_floats) --splits;
  if (splits < 2) return LS_ESTATE;
  DmaArgs g{M, N, K, A, lda, 1, B, ldb, 1, nullptr, 0, LS_F32, nullptr, 0, nullptr, 0, 0, nullptr, 0, 0, 0, nullptr,
            nullptr, 0};
  if (op_dtype == LS_BF16)
    return run_splitk<bf16_t>(g, splits, scratch, C, ldc, c_dtype, bias, bias_dtype, resid, ldr, st);
  if (op_dtype == LS_F16)
    return run_splitk<f16_t>(g, splits, scratch, C, ldc, c_dtype, bias, bias_dtype, resid, ldr, st);
  return LS_ESTATE;
}

// The first half of gemm_dma_splitk_try: the partial products stay in `scratch` as [splits][M][N] for a
// caller that sums them together with its next step.  LS_ESTATE when the shape does not call for a split.
ls_status gemm_dma_splitk_partials(int op_dtype, int M, int N, int K, const void* A, long lda, const void* B, long ldb,
                                   float* scratch, size_t scratch_floats, int* splits_out, hipStream_t st) {
  if (!scratch || K % TK != 0 || M < 256 || N < 64 || N % 4 != 0 || (uintptr_t)scratch % 16 != 0) return LS_ESTATE;
  if (lda % 8 != 0 || ldb % 8 != 0 || (uintptr_t)A % 16 != 0 || (uintptr_t)B % 16 != 0) return LS_ESTATE;
  const long tiles = (long)((M + 127) / 128) * ((N + 127) / 128);
  const int nk = K / TK;
  if (tiles >= 200 || nk < 32) return LS_ESTATE;
  int splits = (int)(512 / tiles);
  if (splits > 8) splits = 8;
  while (splits > 1 && nk / splits < 8) --splits;
  while (splits > 1 && (size_t)splits * M * N > scratch_floats) --splits;
  if (splits < 2) return LS_ESTATE;
  DmaArgs g{M, N, K, A, lda, 1, B, ldb, 1, scratch, N, LS_F32, nullptr, 0, nullptr, 0, 0, nullptr, 0, 0, 0, nullptr,
            nullptr, 0};
  g.split_stride = (long)M * N;
  if (op_dtype == LS_BF16) LS_TRY((launch<bf16_t, 128, 128, true, true, 2>(g, st, splits)));
  else if (op_dtype == LS_F16) LS_TRY((launch<f16_t, 128, 128, true, true, 2>(g, st, splits)));
  else return LS_ESTATE;
  *splits_out = splits;
  return LS_OK;
}

// Weight-streaming product for a few rows (decode batches, M <= 128): tiles of 64 x 128 so that
// three workgroups share a compute unit (128 x 128 and two workgroups above 64 rows), the weights stream through LDS as whole cache lines,
// and the contraction is split until the chip has about three workgroups per compute unit.
ls_status gemm_dma_skinny_partials(int op_dtype, int M, int N, int K, const void* A, long lda, const void* B,
                                   long ldb, float* scratch, size_t scratch_floats, int* splits_out, hipStream_t st) {
  if (!scratch || K % TK != 0 || M < 1 || M > 128 || N < 64 || N % 4 != 0) return LS_ESTATE;
  if ((uintptr_t)scratch % 16 != 0) return LS_ESTATE;
  // up to 64 rows: 64 x 128 tiles, three 48 KB workgroups per compute unit; up to 128 rows: 128 x 128
  // tiles, two 64 KB workgroups
  const bool tall = M > 64;
  const long tiles = (N + 127) / 128;
  const int nk = K / TK;
  int splits = (int)((tall ? 512 : 768) / tiles);   // one round of workgroups
  if (splits < 1) splits = 1;
  if (splits > 16) splits = 16;
  while (splits > 1 && nk / splits < 6) --splits;
  while (splits > 1 && (size_t)splits * M * N > scratch_floats) --splits;
  if ((size_t)splits * M * N > scratch_floats) return LS_ESTATE;
  DmaArgs g{M, N, K, A, lda, 1, B, ldb, 1, scratch, N, LS_F32, nullptr, 0, nullptr, 0, 0, nullptr, 0, 0, 0, nullptr,
            nullptr, 0};
  g.split_stride = (long)M * N;
  if (op_dtype == LS_BF16) {
    if (tall) LS_TRY((launch<bf16_t, 128, 128, true, true, 2>(g, st, splits)));
    else LS_TRY((launch<bf16_t, 64, 128, true, true, 2>(g, st, splits)));
  } else if (op_dtype == LS_F16) {
    if (tall) LS_TRY((launch<f16_t, 128, 128, true, true, 2>(g, st, splits)));
    else LS_TRY((launch<f16_t, 64, 128, true, true, 2>(g, st, splits)));
  } else {
    return LS_ESTATE;
  }
  *splits_out = splits;
  return LS_OK;
}

ls_status gemm_dma_skinny_try(int op_dtype, int M, int N, int K, const void* A, long lda, const void* B, long ldb,
                              void* C, long ldc, int c_dtype, const void* bias, int bias_dtype,
                              const float* resid, long ldr, float* scratch, size_t scratch_floats,
                              hipStream_t st) {
  const int per16 = c_dtype == LS_F32 ? 4 : 8;
  if (ldc % per16 != 0 || (uintptr_t)C % 16 != 0) return LS_ESTATE;
  if (resid && (ldr % 4 != 0 || (uintptr_t)resid % 16 != 0)) return LS_ESTATE;
  int splits = 0;
  const ls_status r = gemm_dma_skinny_partials(op_dtype, M, N, K, A, lda, B, ldb, scratch, scratch_floats, &splits, st);
  if (r != LS_OK) return r;
  const long MN = (long)M * N;
  const unsigned grid = (unsigned)((MN / 4 + 255) / 256);
  if (op_dtype == LS_BF16)
    splitk_reduce_kernel<bf16_t><<<grid, 256, 0, st>>>(scratch, splits, MN, N, C, ldc, c_dtype, bias, bias_dtype, resid, ldr);
  else
    splitk_reduce_kernel<f16_t><<<grid, 256, 0, st>>>(scratch, splits, MN, N, C, ldc, c_dtype, bias, bias_dtype, resid, ldr);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

ls_status gemm_dma16_try(int, int, int, int, const void*, long, int, const void*, long, int, void*, long, int,
                         const void*, int, const float*, long, int, const float*, const int32_t*, const float*, int,
                         hipStream_t);

// Returns LS_OK after launching, or LS_ESTATE (without touching the error text)
// when the shape is outside what this kernel covers.
ls_status gemm_dma_try(int op_dtype, int M, int N, int K, const void* A, long lda, int a_kmajor,
                       const void* B, long ldb, int b_kmajor, void* C, long ldc, int c_dtype,
                       const void* bias, int bias_dtype, const float* resid, long ldr, int accumulate,
                       const float* alpha, const int32_t* rope_pos, const float* rope_table, int rope_cols,
                       hipStream_t st) {
  if (K % TK != 0 || M < 64 || N < 64) return LS_ESTATE;
  // the epilogue stores 16-byte pieces of rows
  const int per16 = c_dtype == LS_F32 ? 4 : 8;
  if (N % per16 != 0 || ldc % per16 != 0 || (uintptr_t)C % 16 != 0) return LS_ESTATE;
  if (resid && (ldr % 4 != 0 || (uintptr_t)resid % 16 != 0)) return LS_ESTATE;
  // problems with enough 256 x 256 tiles run the 16x16x32 kernel
  const ls_status r16 = gemm_dma16_try(op_dtype, M, N, K, A, lda, a_kmajor, B, ldb, b_kmajor, C, ldc, c_dtype, bias,
                                       bias_dtype, resid, ldr, accumulate, alpha, rope_pos, rope_table, rope_cols, st);
  if (r16 != LS_ESTATE) return r16;
  DmaArgs g{M, N, K, A, lda, a_kmajor, B, ldb, b_kmajor, C, ldc, c_dtype, bias, bias_dtype, resid, ldr,
            accumulate, alpha, 0, 0, 0, rope_pos, rope_table, rope_cols};
  if (op_dtype == LS_BF16) return dispatch<bf16_t>(g, st);
  if (op_dtype == LS_F16) return dispatch<f16_t>(g, st);
  return LS_ESTATE;
}
