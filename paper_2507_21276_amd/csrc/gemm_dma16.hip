// The 256 x 256 x 64 direct-to-LDS GEMM with the 16x16x32 MFMA.
//
// Same tiles, LDS layouts, loads, barrier and epilogue staging as gemm_dma_kernel (gemm_dma.hip);
// what differs is the matrix instruction.  On real (Gaussian) operands the chip holds its power limit
// by clocking down, and a register-only loop of 16x16x32 MFMAs sustains 15 % more than one of
// 32x32x16 MFMAs there (1730 - 1870 against 1500 - 1610 TFLOP/s; on all-zero operands both reach the
// same 2230 - 2330): per FLOP the 16x16x32 form moves half the accumulator data.
//
// A wavefront owns 128 x 128 of the tile: 8 x 8 blocks of 16 x 16, 64 accumulators of 4 registers.
// Fragments: 16 rows x 32 k, lane -> row lane & 15, k 8 (lane >> 4) .. + 7: one 16-byte LDS read from
// a k-major tile, two transposing reads (4 k x 16 rows per 16 lanes) from a k-strided one.
// The k tile is walked in four quarters: (k 0..31, rows 0..63), (k 0..31, rows 64..127), then the
// same for k 32..63; a quarter is 32 MFMAs and needs 4 A fragments and the 8 B fragments of its k half.
// The quarters take the place of the four k sub-steps of gemm_dma_kernel: fragments of the next quarter
// are read under the MFMAs of the present one, the workgroup barrier sits before the last quarter, and
// the loads of the tile after the next are issued during the last quarter and the first of the next tile.
#include "gemm_dma_common.h"
#include <cstdlib>
#include <cstring>

namespace {

template <class T> struct Mf16;
template <> struct Mf16<bf16_t> {
  typedef bf16x8 V8;
  typedef bf16x4 V4;
  static __device__ __forceinline__ f32x4 run(V8 a, V8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
};
template <> struct Mf16<f16_t> {
  typedef f16x8 V8;
  typedef f16x4 V4;
  static __device__ __forceinline__ f32x4 run(V8 a, V8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
  }
};

// k-major fragments are ordinary LDS loads (tracked by the compiler); k-strided ones are issued from
// assembly and waited for by wait_frags16, which redefines their registers (see gemm_dma.hip)
template <class T, bool KMAJOR> struct Frag16 { typename Mf16<T>::V8 v; };
template <class T> struct Frag16<T, false> { s16x4 lo, hi; };

// fragment of rows r0 .. r0 + 15, k 32 kh .. 32 kh + 31 of an operand tile
template <class T, bool KMAJOR, int ROWS>
__device__ __forceinline__ void read_frag16(Frag16<T, KMAJOR>& f, const char* lds_tile, int r0, int kh, int lane) {
  typedef typename Mf16<T>::V8 V8;
  const int kg = lane >> 4;
  if constexpr (KMAJOR) {
    const int r = r0 + (lane & 15);
    const int kc = (kh * 4 + kg) ^ ((r >> 1) & 7);
    f.v = *(const V8*)(lds_tile + r * 128 + kc * 16);
  } else {
    constexpr int KROW = ROWS * 2;  // bytes per k row
    const int i16 = lane & 15, a = i16 >> 2, j4 = i16 & 3;
    const int nb = r0 + 4 * j4;     // first of the 4 rows this lane addresses
    const int kb = kh * 32 + 8 * kg;
    // chunk permutation of the tile: 4 (k & 3) as in the 32x32x16 kernel, and 2 ((k >> 3) & 1) = 2 (kg & 1),
    // which keeps the two 16-lane groups of a 32-lane access (k and k + 8) on different banks
    const int phys = (nb >> 3) ^ (4 * a) ^ (2 * (kg & 1));
    const char* p0 = lds_tile + (kb + a) * KROW + phys * 16 + ((nb >> 2) & 1) * 8;
    const uint32_t addr = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)p0;
    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(f.lo) : "v"(addr) : "memory");
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.hi) : "v"(addr), "n"(4 * KROW) : "memory");
  }
}

template <class T, bool KMAJOR, int N>
__device__ __forceinline__ void wait_frags16(Frag16<T, KMAJOR> (&f)[N]) {
  static_assert(KMAJOR || N == 4 || N == 8, "fragment count");
  if constexpr (!KMAJOR) {
    if constexpr (N == 8)
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi), "+v"(f[2].lo), "+v"(f[2].hi),
                     "+v"(f[3].lo), "+v"(f[3].hi), "+v"(f[4].lo), "+v"(f[4].hi), "+v"(f[5].lo), "+v"(f[5].hi),
                     "+v"(f[6].lo), "+v"(f[6].hi), "+v"(f[7].lo), "+v"(f[7].hi));
    else
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi), "+v"(f[2].lo), "+v"(f[2].hi),
                     "+v"(f[3].lo), "+v"(f[3].hi));
  }
}

template <class T, bool KMAJOR>
__device__ __forceinline__ typename Mf16<T>::V8 frag_value16(const Frag16<T, KMAJOR>& f) {
  if constexpr (KMAJOR) {
    return f.v;
  } else {
    const s16x8 w = __builtin_shufflevector(f.lo, f.hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(typename Mf16<T>::V8, w);
  }
}

// Gaps (after MFMA m of a quarter of NM) for the NF fragment reads and the LPK loads of a quarter.  A
// 16x16x32 MFMA is half as long as a 32x32x16 one, and the compute unit's load path takes a wave load
// per 16 cycles: the loads are spread evenly over the quarter (one per NM / LPK MFMAs, from the first gap
// on), stepping aside where a read sits; the reads are spread over the first three quarters (this
// placement measured 0.3 - 0.5 % better than reads over seven eighths and loads from the third gap on).
template <int NM, int NF, int LPK>
struct SpreadPlan {
  int read_at[NM];   // fragment read in the gap after MFMA m, or -1
  int load_at[NM];   // load issued in that gap, or -1
  constexpr SpreadPlan() : read_at{}, load_at{} {
    for (int m = 0; m < NM; ++m) read_at[m] = load_at[m] = -1;
    for (int r = 0; r < NF; ++r) read_at[r * (NM * 3 / 4) / NF] = r;
    for (int l = 0; l < LPK; ++l) {
      int g = l * NM / LPK;
      while (read_at[g] >= 0 || load_at[g] >= 0) g = (g + 1) % NM;
      load_at[g] = l;
    }
  }
};
static_assert(32 * 3 / 4 >= 12, "one read per gap");

// MODE 0: C (16-bit) = acc + bias;  1: C (fp32) = resid + acc + bias;  2: C (fp32) = acc;  4: C (fp32) += acc;
// MODE 5: the product da[M, N] is not stored: it is the gradient of a = SiLU(gate) * up, and the rows written are
//         those of the gradient of (gate | up) [M, 2 N], from the saved pre-activations:
//         dgate = da up s (1 + gate (1 - s)), dup = da gate s, s = sigmoid(gate); da is rounded to the operand
//         type first, as the staged 16-bit tile of MODE 0 is, so the result is that of MODE 0 followed by the
//         element-wise kernel
// MODE 3: as 0 without bias, and the half-split rotary embedding (head_dim 128) applied to the
//         columns below rope_cols: a wavefront's 128 columns are one head, so the pair
//         (c, c + 64) sits in accumulator blocks j and j + 4 of the same lane
template <class T, bool AK, bool BK, int MODE>
__global__ __launch_bounds__(256) void gemm_dma16_kernel(DmaArgs g) {
  typedef typename Mf16<T>::V8 V8;
  typedef typename Mf16<T>::V4 V4;
  constexpr int BM = 256, BN = 256;
  constexpr int WM = BM / 2, WN = BN / 2;       // wavefront tile
  constexpr int TI = WM / 16, TJ = WN / 16;     // 16 x 16 blocks per wavefront
  constexpr int HI = TI / 2;                    // row blocks per quarter
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, BUF_BYTES = A_BYTES + B_BYTES;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  // buffer b: A tile at smem + b BUF_BYTES, B tile A_BYTES after it

  // the tile order of gemm_dma_kernel: every XCD a contiguous run, M fastest inside bands of 8 N tiles
  const int total = g.tiles_m * g.tiles_n, per_xcd = total / 8;
  int bid = blockIdx.x;
  if (bid < per_xcd * 8) bid = (bid % 8) * per_xcd + bid / 8;
  const int band = 8;
  const int per_band = band * g.tiles_m;
  const int b0 = (bid / per_band) * band;
  const int bw = min(band, g.tiles_n - b0);
  const int rem = bid % per_band;
  const int tn = b0 + rem % bw, tm = rem / bw;
  const int m0 = tm * BM, n0 = tn * BN;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wm = (wave >> 1) * WM, wn = (wave & 1) * WN;
  const char* a_base = (const char*)g.A + (AK ? (long)m0 * g.lda : (long)m0) * 2;
  const char* b_base = (const char*)g.B + (BK ? (long)n0 * g.ldb : (long)n0) * 2;
  const long a_step = (AK ? (long)TK : (long)TK * g.lda) * 2;
  const long b_step = (BK ? (long)TK : (long)TK * g.ldb) * 2;
  uint32_t a_off[BM / 32], b_off[BN / 32];
  tile_offsets<AK, BM, true>(a_off, g.lda, m0, g.M, wave, lane);
  tile_offsets<BK, BN, true>(b_off, g.ldb, n0, g.N, wave, lane);

  f32x4 acc[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

  const int nk = g.K / TK;
  issue_tile<BM>(a_base, a_off, smem, wave);
  issue_tile<BN>(b_base, b_off, smem + A_BYTES, wave);

  constexpr int NM = HI * TJ;            // MFMAs per quarter
  constexpr int NLD = (BM + BN) / 32;    // direct-to-LDS loads per tile and wavefront
  constexpr int LPK = NLD / 2;           // issued over two quarters
  constexpr SpreadPlan<NM, HI, LPK> plan_a{};        // quarters that read the other row half's A fragments only
  constexpr SpreadPlan<NM, HI + TJ, LPK> plan_ab{};  // quarters that also read the next k half's B fragments
  {
    // what the last quarter of the tile before the first would have issued
    const int t1 = nk > 1 ? 1 : 0;
#pragma unroll
    for (int l = 0; l < LPK; ++l)
      issue_one<BM, BN>(l, a_base + t1 * a_step, a_off, b_base + t1 * b_step, b_off, smem + BUF_BYTES,
                        smem + BUF_BYTES + A_BYTES, wave);
  }
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  Frag16<T, AK> fa[2][HI];     // by quarter parity
  Frag16<T, BK> fb[2][TJ];     // by k half
#pragma unroll
  for (int i = 0; i < HI; ++i) read_frag16<T, AK, BM>(fa[0][i], smem, wm + i * 16, 0, lane);
#pragma unroll
  for (int j = 0; j < TJ; ++j) read_frag16<T, BK, BN>(fb[0][j], smem + A_BYTES, wn + j * 16, 0, lane);

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
    for (int q = 0; q < 4; ++q) {
      const int kh = q >> 1, half = q & 1;
      wait_frags16<T, AK, HI>(fa[q & 1]);
      if (half == 0) wait_frags16<T, BK, TJ>(fb[kh]);
      if (q == 3) {
        __builtin_amdgcn_s_waitcnt(0);   // this wavefront's share of the next tile has landed
        __syncthreads();
      }
      V8 va[HI], vb[TJ];
#pragma unroll
      for (int i = 0; i < HI; ++i) va[i] = frag_value16<T, AK>(fa[q & 1][i]);
#pragma unroll
      for (int j = 0; j < TJ; ++j) vb[j] = frag_value16<T, BK>(fb[kh][j]);
      // the next quarter: the other row half of this k half, or the first row half of the next k half
      // (of the next tile after the last quarter)
      const int nq = (q + 1) & 3, nkh = nq >> 1, nhalf = nq & 1;
      const char* ra = q < 3 ? la : na;
      const char* rb = q < 3 ? lb : nb;
      // the last quarter and the first come after the barrier that frees a buffer: the last quarter starts
      // the tile after the next in the buffer being vacated, the first completes it in the next trip
      const bool loads = q == 3 || q == 0;
      const bool ahead = q == 3;
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        // the quarter's blocks in boustrophedon order: consecutive MFMAs share an operand
        const int ii = m / TJ, tj = (ii & 1) ? TJ - 1 - m % TJ : m % TJ;
        const int ti = half * HI + ii;
        acc[ti][tj] = Mf16<T>::run(vb[tj], va[ii], acc[ti][tj]);
        __builtin_amdgcn_sched_barrier(0);   // the MFMA first: what follows issues in its shadow
        if (nhalf == 1) {
          const int r = plan_a.read_at[m];
          if (r >= 0) read_frag16<T, AK, BM>(fa[nq & 1][r], ra, wm + (HI + r) * 16, nkh, lane);
        } else {
          const int r = plan_ab.read_at[m];
          if (r >= 0 && r < HI) read_frag16<T, AK, BM>(fa[nq & 1][r], ra, wm + r * 16, nkh, lane);
          if (r >= HI) read_frag16<T, BK, BN>(fb[nkh][r - HI], rb, wn + (r - HI) * 16, nkh, lane);
        }
        if (loads) {
          const int l = nhalf == 1 ? plan_a.load_at[m] : plan_ab.load_at[m];
          if (l >= 0)
            issue_one<BM, BN>((ahead ? 0 : LPK) + l, ahead ? ga2 : ga1, a_off, ahead ? gb2 : gb1, b_off,
                              ahead ? (char*)la : na, ahead ? (char*)lb : nb, wave);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  // The last quarter read the fragments of a tile that does not exist.  Their registers must stay
  // allocated until the reads have returned (see gemm_dma.hip).
  wait_frags16<T, AK, HI>(fa[0]);
  wait_frags16<T, BK, TJ>(fb[0]);
  __builtin_amdgcn_s_waitcnt(0);

  // Epilogue.  The MFMAs ran with the operands swapped, so the accumulators hold C^T blocks:
  // lane -> row m (lane & 15), register e -> column 4 (lane >> 4) + e of the block.  Each wavefront
  // stages its tile in its quarter of the (now idle) LDS, row-major with the 16-byte chunks of a row
  // XOR-permuted by the row number, and writes it out as full rows; residual and accumulation operands
  // are read with the same coalesced pattern.
  constexpr int ESZ = (MODE == 0 || MODE == 3 || MODE == 5) ? 2 : 4;
  constexpr int REGION = (BM + BN) * 128 * 2 / 4;   // bytes of LDS per wavefront
  constexpr int ROWB = WN * ESZ;                    // bytes of a staged row
  constexpr int CPR = ROWB / 16;                    // 16-byte chunks per row
  constexpr int NPASS = (WM * ROWB + REGION - 1) / REGION;
  constexpr int TIP = TI / NPASS;                   // 16-row blocks per pass
  constexpr int ROWS_P = TIP * 16;
  const int row_in = lane & 15, cg = lane >> 4;
  const float alpha = g.alpha ? *g.alpha : 1.f;
  __syncthreads();   // every wavefront is done with the operand tiles
  char* stg = smem + wave * REGION;
  // a lane's columns are the same for all of its rows: its bias values are fetched once
  float bv[TJ][4];
#pragma unroll
  for (int j = 0; j < TJ; ++j)
#pragma unroll
    for (int e = 0; e < 4; ++e) bv[j][e] = 0.f;
  if ((MODE == 0 || MODE == 1) && g.bias) {
    const int nbase = n0 + wn + 4 * cg;
    auto fetch = [&](auto* b) {
#pragma unroll
      for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int n = nbase + j * 16 + e;
          bv[j][e] = (float)b[n < g.N ? n : g.N - 1];
        }
    };
    if (g.bias_dtype == LS_F32) fetch((const float*)g.bias);
    else if (g.bias_dtype == LS_BF16) fetch((const bf16_t*)g.bias);
    else fetch((const f16_t*)g.bias);
  }
  // MODE 3: q or k section (uniform over the wavefront), and the table rows of this lane's row blocks
  const bool rot = MODE == 3 && n0 + wn < g.rope_cols;
  f32x4 cs_cur[TJ / 2][2], cs_nxt[TJ / 2][2];
#pragma unroll
  for (int j = 0; j < TJ / 2; ++j) cs_cur[j][0] = cs_cur[j][1] = cs_nxt[j][0] = cs_nxt[j][1] = f32x4{1.f, 0.f, 1.f, 0.f};
  auto rope_fetch = [&](int i, f32x4 (&cs)[TJ / 2][2]) {
    const int m = min(m0 + wm + i * 16 + row_in, g.M - 1);   // rows past the edge are staged, never stored
    const float* tab = g.rope_table + (long)g.rope_pos[m] * 128 + 8 * cg;   // 64 (cos, sin) pairs per position
#pragma unroll
    for (int j = 0; j < TJ / 2; ++j) {
      cs[j][0] = *(const f32x4*)(tab + j * 32);       // pairs 16 j + 4 cg + 0, 1
      cs[j][1] = *(const f32x4*)(tab + j * 32 + 4);   // pairs 16 j + 4 cg + 2, 3
    }
  };
#pragma unroll
  for (int pass = 0; pass < NPASS; ++pass) {
    // results added to a buffer (the residual stream, or the output itself): what the pass adds to is fetched
    // first, all of it at once, and arrives while the accumulators are staged (a load per store, each behind its
    // own branch and wait, made an accumulating launch a sixth longer)
    constexpr int NOUT = ROWS_P * CPR / 64;
    constexpr bool ADDS = MODE == 1 || MODE == 4;
    f32x4 c_old[ADDS ? NOUT : 1];
    if constexpr (ADDS) {
      const float* src = MODE == 1 ? g.resid : (const float*)g.C;
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
      const int r = ii * 16 + row_in;
      char* srow = stg + r * ROWB;
      const int sw = r & (CPR - 1);
      if constexpr (MODE == 3) {
        // (cos, sin) of this lane's four column pairs in each of the TJ / 2 block pairs; the values for the
        // next row block are fetched while this one is rotated (a fetch per block pair, each behind its own
        // branch and wait, cost 50 us per tile)
        if (rot) {
          if (ii == 0) rope_fetch(i, cs_cur);
          if (ii + 1 < TIP) rope_fetch(i + 1, cs_nxt);
        }
#pragma unroll
        for (int j = 0; j < TJ / 2; ++j) {
          V4 lo, hi;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float c = e < 2 ? cs_cur[j][0][2 * e] : cs_cur[j][1][2 * (e - 2)];
            const float sn = e < 2 ? cs_cur[j][0][2 * e + 1] : cs_cur[j][1][2 * (e - 2) + 1];
            const float a = acc[i][j][e], bb = acc[i][j + TJ / 2][e];
            lo[e] = from_f<T>(rot ? a * c - bb * sn : a);
            hi[e] = from_f<T>(rot ? bb * c + a * sn : bb);
          }
          // columns 16 j + 4 cg .. + 3: chunk 2 j + (cg >> 1), half cg & 1
          *(u32x2_a*)(srow + (((2 * j + (cg >> 1)) ^ sw) * 16) + (cg & 1) * 8) = __builtin_bit_cast(u32x2_t, lo);
          *(u32x2_a*)(srow + (((2 * (j + TJ / 2) + (cg >> 1)) ^ sw) * 16) + (cg & 1) * 8) = __builtin_bit_cast(u32x2_t, hi);
        }
#pragma unroll
        for (int j = 0; j < TJ / 2; ++j) {
          cs_cur[j][0] = cs_nxt[j][0];
          cs_cur[j][1] = cs_nxt[j][1];
        }
      } else {
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = acc[i][j][e] * alpha;
          if constexpr (MODE == 0 || MODE == 1) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] += bv[j][e];
          }
          if constexpr (ESZ == 2) {
            V4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = from_f<T>(v[e]);
            *(u32x2_a*)(srow + (((2 * j + (cg >> 1)) ^ sw) * 16) + (cg & 1) * 8) = __builtin_bit_cast(u32x2_t, o);
          } else {
            *(f32x4_a*)(srow + (((4 * j + cg) ^ sw) * 16)) = v;
          }
        }
      }
    }
    // full rows out: 64 / CPR rows per instruction, 16 bytes per lane
    if constexpr (MODE == 5) {
      // the saved pre-activations of a group of rows are fetched together, before any of the group's results is
      // stored (the buffers may alias as far as the compiler knows, so a load per store would wait for each in turn)
      typedef typename Mf16<T>::V8 V8;
      constexpr int NIT = ROWS_P * CPR / 64, GRP = 8;
      static_assert(NIT % GRP == 0, "row groups of the activation epilogue");
      const T* pre = (const T*)g.glu_pre;
      T* grad = (T*)g.glu_grad;
#pragma unroll 1
      for (int it0 = 0; it0 < NIT; it0 += GRP) {
        V8 gt[GRP], up[GRP], da[GRP];
        long at[GRP];
#pragma unroll
        for (int u = 0; u < GRP; ++u) {
          const int idx = (it0 + u) * 64 + lane;
          const int r = idx / CPR, c = idx % CPR;
          const int m = m0 + wm + pass * ROWS_P + r, n = n0 + wn + c * 8;
          at[u] = m < g.M && n < g.N ? (long)m * 2 * g.N + n : -1;
          const long a = at[u] < 0 ? 0 : at[u];
          gt[u] = *(const V8*)(pre + a);
          up[u] = *(const V8*)(pre + a + g.N);
          da[u] = __builtin_bit_cast(V8, *(const f32x4_a*)(stg + r * ROWB + ((c ^ (r & (CPR - 1))) * 16)));
        }
#pragma unroll
        for (int u = 0; u < GRP; ++u) {
          V8 og, ou;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float a = to_f(da[u][e]), gf = to_f(gt[u][e]), uf = to_f(up[u][e]);
            const float sg = 1.f / (1.f + __expf(-gf));
            og[e] = from_f<T>(a * uf * sg * (1.f + gf * (1.f - sg)));
            ou[e] = from_f<T>(a * gf * sg);
          }
          if (at[u] >= 0) {
            *(V8*)(grad + at[u]) = og;
            *(V8*)(grad + at[u] + g.N) = ou;
          }
        }
      }
    } else {
      constexpr int NIT = ROWS_P * CPR / 64, GRP = 8;
      static_assert(NIT % GRP == 0, "row groups of the store loop");
      auto put = [&](int it, int m, int n, const f32x4& v) {
        if constexpr (ESZ == 2) {
          *(f32x4_a*)((T*)g.C + (long)m * g.ldc + n) = v;
        } else if constexpr (MODE == 1) {
          *(f32x4*)((float*)g.C + (long)m * g.ldc + n) = v + c_old[it];
        } else {
          *(f32x4*)((float*)g.C + (long)m * g.ldc + n) = MODE == 4 ? c_old[it] + v : v;
        }
      };
      if (m0 + wm + pass * ROWS_P + ROWS_P <= g.M && n0 + wn + WN <= g.N) {
        // uniform: every row and column of the pass exists, so nothing depends on the lane and eight staged
        // pieces are read before eight are stored (under the per-lane bounds check below the compiler moves each
        // read to its store and waits for it there: 32 or 64 LDS round trips in a row per tile)
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
}

template <class T, bool AK, bool BK, int MODE>
ls_status launch16(DmaArgs g, hipStream_t st) {
  static bool attr_set = false;
  const int lds = 2 * (256 + 256) * 128;
  if (!attr_set) {
    LS_CHECK_HIP(hipFuncSetAttribute((const void*)gemm_dma16_kernel<T, AK, BK, MODE>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    attr_set = true;
  }
  g.tiles_m = (g.M + 255) / 256;
  g.tiles_n = (g.N + 255) / 256;
  gemm_dma16_kernel<T, AK, BK, MODE><<<dim3(g.tiles_m * g.tiles_n), 256, lds, st>>>(g);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

template <class T>
ls_status dispatch16(const DmaArgs& g, hipStream_t st) {
  if (g.rope_table) {
    if (g.a_kmajor && g.b_kmajor && g.c_dtype != LS_F32 && !g.bias) return launch16<T, true, true, 3>(g, st);
    return LS_ESTATE;
  }
  if (g.glu_pre) {
    if (g.a_kmajor && !g.b_kmajor && g.c_dtype != LS_F32 && !g.bias && !g.alpha && g.N % 8 == 0)
      return launch16<T, true, false, 5>(g, st);
    return LS_ESTATE;
  }
  const int mode = g.c_dtype != LS_F32 ? 0 : (g.resid ? 1 : (g.accumulate ? 4 : 2));
  if (mode >= 2 && g.bias) return LS_ESTATE;
  if (mode == 1 && g.accumulate) return LS_ESTATE;
  if (g.a_kmajor && g.b_kmajor && mode == 0) return launch16<T, true, true, 0>(g, st);
  if (g.a_kmajor && g.b_kmajor && mode == 1) return launch16<T, true, true, 1>(g, st);
  if (g.a_kmajor && g.b_kmajor && mode == 2) return launch16<T, true, true, 2>(g, st);
  if (g.a_kmajor && g.b_kmajor && mode == 4) return launch16<T, true, true, 4>(g, st);
  if (g.a_kmajor && !g.b_kmajor && mode == 0) return launch16<T, true, false, 0>(g, st);
  if (g.a_kmajor && !g.b_kmajor && mode == 2) return launch16<T, true, false, 2>(g, st);
  if (g.a_kmajor && !g.b_kmajor && mode == 4) return launch16<T, true, false, 4>(g, st);
  // Both operands k-strided (weight gradients): left to the 32x32x16 kernel.  Every fragment is two
  // transposing reads there, 24 in a quarter of 32 short MFMAs, and this kernel measured 8 - 10 % slower on
  // those shapes (faster by 5 - 12 % on the other two layouts), also with the LDS reads free of bank conflicts.
  return LS_ESTATE;
}

}  // namespace

// The large-tile GEMM for problems with enough 256 x 256 tiles; LS_ESTATE (error text untouched) when the
// shape or the combination of layouts is outside what this kernel covers.  Arguments as gemm_dma_try, whose
// checks of alignment and sizes have run before this is called.
ls_status gemm_dma16_try(int op_dtype, int M, int N, int K, const void* A, long lda, int a_kmajor, const void* B,
                         long ldb, int b_kmajor, void* C, long ldc, int c_dtype, const void* bias, int bias_dtype,
                         const float* resid, long ldr, int accumulate, const float* alpha, const int32_t* rope_pos,
                         const float* rope_table, int rope_cols, hipStream_t st) {
  if (K % TK != 0 || M < 64 || N < 64) return LS_ESTATE;
  const long big = (long)((M + 255) / 256) * ((N + 255) / 256);
  if (big < 160) return LS_ESTATE;
  DmaArgs g{M, N, K, A, lda, a_kmajor, B, ldb, b_kmajor, C, ldc, c_dtype, bias, bias_dtype, resid, ldr,
            accumulate, alpha, 0, 0, 0, rope_pos, rope_table, rope_cols};
  if (op_dtype == LS_BF16) return dispatch16<bf16_t>(g, st);
  if (op_dtype == LS_F16) return dispatch16<f16_t>(g, st);
  return LS_ESTATE;
}

// da[M, N] = dY[M, K] W[K, N] (W k-strided: the input-gradient layout of a linear map whose weight is stored
// [K, N]) with the backward of SwiGLU in the epilogue: `pre` holds the saved (gate | up) pre-activations
// [M, 2 N], `grad` receives their gradients [M, 2 N]; da itself is not stored.  LS_ESTATE when the shape is
// outside what the large-tile kernel covers (the caller then runs the product and the element-wise kernel).
ls_status gemm_dma16_swiglu_bwd_try(int op_dtype, int M, int N, int K, const void* dY, long ldy, const void* W, long ldw,
                                    const void* pre, void* grad, hipStream_t st) {
  if (K % TK != 0 || M < 64 || N < 64 || N % 8 != 0) return LS_ESTATE;
  if (ldy % 8 != 0 || ldw % 8 != 0 || (uintptr_t)dY % 16 != 0 || (uintptr_t)W % 16 != 0 || (uintptr_t)pre % 16 != 0 ||
      (uintptr_t)grad % 16 != 0)
    return LS_ESTATE;
  const long big = (long)((M + 255) / 256) * ((N + 255) / 256);
  if (big < 160) return LS_ESTATE;
  DmaArgs g{M, N, K, dY, ldy, 1, W, ldw, 0, grad, 2L * N, op_dtype, nullptr, 0, nullptr, 0, 0, nullptr, 0, 0, 0,
            nullptr, nullptr, 0};
  g.glu_pre = pre;
  g.glu_grad = grad;
  if (op_dtype == LS_BF16) return dispatch16<bf16_t>(g, st);
  if (op_dtype == LS_F16) return dispatch16<f16_t>(g, st);
  return LS_ESTATE;
}
