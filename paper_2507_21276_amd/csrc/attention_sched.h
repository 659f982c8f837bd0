// Hand-scheduled attention kernels for head_dim 128: dK/dV, dQ and the training forward (included by
// attention_mfma.hip, inside its anonymous namespace).  Same tiles, layouts and arithmetic as the
// compiler-scheduled kernels of that file (flash_bwd_dkv_kernel, flash_bwd_dq_kernel, flash_fwd_ring_kernel,
// which stay for head_dim 64 and for prompt chunks over pages); what differs is who places the instructions:
//   * every MFMA, LDS read and wait of the tile loop is issued from assembly, in source order, with
//     scheduling barriers between the steps, so that the matrix pipe, the vector unit and the LDS
//     work at the same time inside the one wavefront a SIMD holds;
//   * S and dP accumulate in ordinary vector registers (the vector unit reads them directly), the
//     dK / dV accumulators and the K / V operands of the workgroup live in the accumulator file;
//   * LDS addresses are a per-lane register plus an immediate: one vector add per table entry and
//     tile instead of address arithmetic per read;
//   * fragments are fetched a fixed number of MFMAs ahead and waited for by count.
//
// A tile (64 queries in two blocks of 32, against the wavefront's 32 keys) is 64 MFMAs; "gap g" is the slot
// after MFMA g, and everything else of the tile is placed into the gaps so that no gap holds much more than
// the 32 cycles its MFMA runs:
//   MFMA  0.. 7  S of block 0        8..15  dP of block 0      16..23  S of block 1     24..31  dP of block 1
//        32..47  dV, dK of block 0  48..63  dV, dK of block 1
//   exponentials of block 0 in gaps 8..23 (one element each), its dS in 24..31 (two each); exponentials of
//   block 1 in 32..47, its dS in 48..59; fragment reads 8 MFMAs ahead (transposed ones 4 ahead), the
//   log-sum-exp / D vectors a few gaps before their first use; the ten direct-to-LDS loads that refill the
//   stage of the previous tile in every second gap of 5..15 and 25..31 (bunched after the barrier, the four
//   wavefronts queue up at the compute unit's one load path: 450 ns per tile); the ring step after gap 59.
//
// The compiler does not know what the assembly statements do, so the hazards it normally covers
// are handled here: an MFMA result is read by vector instructions only after bwd_mfma_settle(),
// and every LDS read is retired by a counted wait before its register is used (tests/isa_lint.py
// checks the compiled code for that).
#pragma once

template <int I> using IC = std::integral_constant<int, I>;
template <int B, int E, class F> __device__ __forceinline__ void static_for(F&& f) {
  if constexpr (B < E) {
    f(IC<B>{});
    static_for<B + 1, E>(f);
  }
}

// The MFMAs of this file.  An MFMA may read a register that a vector instruction wrote only two wait states
// after it.  The compiler keeps that distance for its own MFMAs; here it cannot know that a statement is one (and
// it does move the conversions that complete an operand down to the statement that first uses it), so operands
// made by vector instructions go through operand_ready() at least one MFMA before they are used.
template <class V> __device__ __forceinline__ void operand_ready(V& a) { asm volatile("" : "+v"(a)); }
// D (vector registers) = A (vector registers) x B (accumulator file) [+ D]
template <class T, bool FIRST>
__device__ __forceinline__ void mma_to_vgpr(f32x16& d, const typename Mma<T>::V8& a, const typename Mma<T>::V8& b) {
  if constexpr (std::is_same<T, f16_t>::value) {
    if constexpr (FIRST) asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "a"(b));
    else asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "a"(b));
  } else {
    if constexpr (FIRST) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "a"(b));
    else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "a"(b));
  }
}
// D (accumulator file) += A (vector registers) x B (vector registers)
template <class T>
__device__ __forceinline__ void mma_to_agpr(f32x16& d, const typename Mma<T>::V8& a, const typename Mma<T>::V8& b) {
  if constexpr (std::is_same<T, f16_t>::value)
    asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(d) : "v"(a), "v"(b));
  else
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(d) : "v"(a), "v"(b));
}
// Wait states between the last MFMA that wrote these registers and a vector instruction that reads them: 11
// for this MFMA (its 8 passes + 3; the MFMA issued in between runs meanwhile).
__device__ __forceinline__ void bwd_mfma_settle(f32x16& a) { asm volatile("s_nop 10" : "+v"(a)); }
// The same, generously, for the eight accumulator blocks of a kernel at the end of every tile: whatever the
// compiler places after the tile's last MFMA (copies of an accumulator at a loop edge, the epilogue's reads)
// comes after it.
__device__ __forceinline__ void bwd_mfma_settle_acc(f32x16 (&a)[4], f32x16 (&b)[4]) {
  asm volatile("s_nop 15\n\ts_nop 7"
               : "+a"(a[0]), "+a"(a[1]), "+a"(a[2]), "+a"(a[3]), "+a"(b[0]), "+a"(b[1]), "+a"(b[2]), "+a"(b[3]));
}

// From here on the value lives in the accumulator file (it is only ever an operand of the MFMAs above).
template <class V> __device__ __forceinline__ void pin_agpr(V& v) { asm volatile("" : "+a"(v)); }

template <int IMM, class V> __device__ __forceinline__ void lds_read16(V& d, uint32_t addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(d) : "v"(addr), "n"(IMM) : "memory");
}
template <int IMM> __device__ __forceinline__ void lds_read_tr(s16x4_t& d, uint32_t addr) {
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(d) : "v"(addr), "n"(IMM) : "memory");
}
template <int N> __device__ __forceinline__ void lgkm_wait() {
  static_assert(N >= 0 && N <= 15, "lgkmcnt holds 0 .. 15");
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
}

// One direct-to-LDS wave load, 16 or 4 bytes per lane: address = uniform 64-bit base + per-lane 32-bit offset,
// LDS destination = `lds` + 16 (or 4) x lane.  Issued from assembly, so the compiler neither counts these loads
// nor forms a 64-bit address per lane; every wait for them in this file is an explicit s_waitcnt.
__device__ __forceinline__ void dma16(const void* base, uint32_t off, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds), "v"(off), "s"(base) : "memory", "m0");
}
__device__ __forceinline__ void dma4(const void* base, uint32_t off, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" : : "s"(lds), "v"(off), "s"(base) : "memory", "m0");
}

// Store a wavefront's 32 gradient rows (O^T-style accumulators: lane = row, registers = head dimension
// j * 32 + 8 g + 4 hf + i, as store_grad_row takes them) through LDS: each lane puts its 8-byte pieces into a
// [32][128] tile of 16-bit values (rows padded to 272 bytes: two-way bank conflicts at most), then the tile is
// written out as whole rows, 16 bytes per lane, four rows per store instruction - instead of 64 instructions
// that each touch 32 rows with 8 bytes.  `tile` is this wavefront's own 8704 bytes of LDS; row r of the tile goes
// to out + r * ld if r < rows.  With a rotary table (this lane's row of it) the row is rotated back first.
template <class T>
__device__ __forceinline__ void store_grad_rows_staged(T* out, long ld, int rows, const f32x16 (&acc)[4], float mul,
                                                       int lane, const float* tab, char* tile) {
  typedef typename Mma<T>::V4 V4;
  constexpr int DH = 128, DT = 4, RS = DH * 2 + 16;
  const int col = lane & 31, hf = lane >> 5;
  char* my = tile + col * RS;
  if (tab == nullptr) {
#pragma unroll
    for (int j = 0; j < DT; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        V4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = from_f<T>(acc[j][g * 4 + i] * mul);
        *(V4*)(my + (j * 32 + 8 * g + 4 * hf) * 2) = v;
      }
  } else {
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
        *(V4*)(my + i0 * 2) = lo;
        *(V4*)(my + (i0 + DH / 2) * 2) = hi;
      }
  }
  // the LDS executes one wavefront's operations in order: the reads below see the writes above
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int r = it * 4 + (lane >> 4);
    const u32x4 v = *(const u32x4*)(tile + r * RS + (lane & 15) * 16);
    if (r < rows) *(u32x4*)(out + (long)r * ld + (lane & 15) * 8) = v;
  }
}

// ---- the LDS read schedule of a dK/dV tile, as a table the wait counts are derived from ----------
// A cycle starts at the ring step (after gap 59), which leaves no read outstanding; position tau counts the
// gaps from there: gaps 60..63 are tau 0..3, gaps 0..59 are tau 4..63.
struct DkvPlan {
  static constexpr int tau(int gap) { return gap >= 60 ? gap - 60 : gap + 4; }
  static constexpr int reads_at(int t) {
    const int gap = t < 4 ? 60 + t : t - 4;
    if (gap >= 60) return 2;        // two fragments of the next tile
    if (gap < 4) return 2;          // fragment, log-sum-exp of block 0
    if (gap < 16) return 1;         // fragment
    if (gap < 24) return 2;         // fragment, D of block 0 (16..19) or log-sum-exp of block 1 (20..23)
    if (gap < 32) return 1;         // half a transposed fragment
    if (gap < 40) return 2;         // transposed fragment
    if (gap < 44) return 3;         // transposed fragment, D of block 1
    return 2;                       // transposed fragment
  }
  static constexpr int issued_through(int t) {   // reads issued at positions 0 .. t
    int n = 0;
    for (int i = 0; i <= t; ++i) n += reads_at(i);
    return n;
  }
  // reads issued after read number `pos` of position tr and before the MFMA that precedes gap `gap`
  static constexpr int newer(int gap, int tr, int pos) { return issued_through(tau(gap) - 1) - issued_through(tr - 1) - pos - 1; }
  // position of the (last) read that MFMA g waits for
  static constexpr int need_tau(int g) {
    if (g < 8) return g / 2;
    if (g < 32) return g - 4;                       // issued in gap g - 8
    const int M = g - 32;
    return M < 4 ? 29 + 2 * M : 32 + M;             // second half: gap 25 + 2 M, or gap 28 + M
  }
  static constexpr int need_pos(int g) { return g < 8 ? g % 2 : g < 32 ? 0 : (g - 32 < 4 ? 0 : 1); }
  // One wait serves two MFMAs: before MFMA g (even) the operands of g and g + 1 must have landed.
  static constexpr int wait(int g) { return newer(g, need_tau(g + 1), need_pos(g + 1)); }
};

// dK, dV for head_dim 128.  Grid, LDS layout and arguments of flash_bwd_dkv_kernel, except that lse2 is the
// log-sum-exp in base 2 (natural value times log2 e; dvec_kernel writes it beside D).
template <class T>
__global__ __launch_bounds__(256) void flash_bwd_dkv128_kernel(const T* __restrict__ qkv, const T* __restrict__ dO,
                                                               const float* __restrict__ lse2,
                                                               const float* __restrict__ dvec, T* __restrict__ dqkv,
                                                               int L, int h, float scale,
                                                               const float* __restrict__ rope) {
  typedef typename Mma<T>::V8 V8;
  constexpr int DH = 128, BKEY = 128, QR = 64, NS = 4, KS = DH / 16, DT = DH / 32;
  constexpr int TILE_B = QR * DH * 2;            // bytes of a Q or dO tile
  constexpr int STAGE_B = 2 * TILE_B + 512;      // Q, dO, 64 log-sum-exp, 64 D
  constexpr int NLT = TILE_B / 1024 / 4;         // wave loads per wavefront and tile
  constexpr int NLD = 2 * NLT + 2;               // loads per wavefront and stage
  static_assert(NLD == 10, "the refill of a stage is spread as two loads over each of the last five gaps");
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  const int ktile = blockIdx.y;
  const int b = blockIdx.x / h, head = blockIdx.x % h;
  const int d = h * DH;
  const long ld = 3L * d;
  const T* qb = qkv + (long)b * L * ld + (long)head * DH;
  const T* kb = qb + d;
  const T* vb = qb + 2 * d;
  const T* dob = dO + (long)b * L * d + (long)head * DH;
  const float* lseb = lse2 + (long)b * L * h + head;
  const float* dvb = dvec + (long)b * L * h + head;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int col = lane & 31, hf = lane >> 5;
  const int wk0 = ktile * BKEY + wave * 32;
  const int key = wk0 + col;
  const float scale_log2 = scale * 1.4426950408889634f;
  const float gsc = do_scale(dvec + (long)gridDim.x * L + ((long)gridDim.x * L + 3) / 4);

  // per-lane byte offsets inside a stage (see frag_rows / tr_read for the layouts)
  const uint32_t lds0 = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)smem;
  uint32_t nat[KS], tr0[DT], tr1[DT], lsv;
  {
    const int row = pi_row(col);
#pragma unroll
    for (int s = 0; s < KS; ++s) nat[s] = lds0 + row * (DH * 2) + (((2 * s + hf) ^ tile_swz<DH>(row)) * 16);
    const int i16 = lane & 15, a = i16 >> 2, j4 = i16 & 3;
    const int k = 8 * (lane >> 5) + a;
#pragma unroll
    for (int j = 0; j < DT; ++j) {
      const int nb = j * 32 + 16 * ((lane >> 4) & 1) + 4 * j4;
      tr0[j] = lds0 + k * (DH * 2) + (((nb >> 3) ^ tile_swz<DH>(k)) * 16) + ((nb >> 2) & 1) * 8;
      tr1[j] = lds0 + (k + 4) * (DH * 2) + (((nb >> 3) ^ tile_swz<DH>(k + 4)) * 16) + ((nb >> 2) & 1) * 8;
    }
    lsv = lds0 + 2 * TILE_B + 32 * hf;
  }

  const int qt_first = (ktile * BKEY) / QR;   // first query tile that can see these keys
  const int nt = (L + QR - 1) / QR - qt_first;
  // Direct-to-LDS loads of a stage: load i = 0 .. NLD - 1 of this wavefront (Q rows, dO rows, then the 64
  // log-sum-exp and the 64 D values, which every wavefront writes alike).  The per-lane offsets from the tile's
  // first row are the same for every full tile (registers, set once); a tile cut off by the end of the sequence
  // re-reads row L - 1 for the rows past it.  Tile t -> stage t % NS; tiles past the end re-fetch the last one (never used), so
  // that every wavefront always has the same number of loads in flight.
  constexpr int CPR = DH / 8, RPL = 64 / CPR;
  uint32_t qoff[NLT], ooff[NLT], foff;
  // offsets for a tile of `rows` valid rows (64 for all but a cut-off last tile)
  auto set_offsets = [&](int rows) {
#pragma unroll
    for (int j = 0; j < NLT; ++j) {
      const int row = (wave * NLT + j) * RPL + lane / CPR;
      const int gch = (lane % CPR) ^ tile_swz<DH>(row);
      const int r = min(row, rows - 1);
      qoff[j] = (uint32_t)((r * ld + gch * 8) * 2);
      ooff[j] = (uint32_t)(((long)r * d + gch * 8) * 2);
    }
    foff = (uint32_t)(min(lane, rows - 1) * h * 4);
  };
  set_offsets(QR);
  const int last_rows = L - (qt_first + nt - 1) * QR;   // rows of the last tile, <= 64
  // Called once per tile before its loads, in tile order: the last tile (which all fetches past the end repeat)
  // switches the offsets to its row count, and nothing switches them back.
  auto prepare_tile = [&](int t) {
    if (t >= nt - 1 && last_rows < QR) set_offsets(last_rows);
  };
  auto issue_one = [&](int t, auto i_) {
    constexpr int i = decltype(i_)::value;
    const int q0 = (qt_first + min(t, nt - 1)) * QR;
    const uint32_t st = lds0 + (t % NS) * STAGE_B;
    if constexpr (i < 2 * NLT) {
      constexpr int j = i % NLT;
      if constexpr (i < NLT) dma16(qb + (long)q0 * ld, qoff[j], st + (wave * NLT + j) * 1024);
      else dma16(dob + (long)q0 * d, ooff[j], st + TILE_B + (wave * NLT + j) * 1024);
    } else {
      dma4((i == 2 * NLT ? lseb : dvb) + (long)q0 * h, foff, st + 2 * TILE_B + (i == 2 * NLT ? 0 : 256));
    }
  };
#pragma unroll
  for (int t = 0; t < NS - 1; ++t) {   // the tile loop refills a stage one tile after it was used: tile 0 fetches tile NS - 1
    prepare_tile(t);
    static_for<0, NLD>([&](auto i_) { issue_one(t, i_); });
  }

  // this wavefront's 32 keys: K and V fragments, all requested before the first is used
  V8 kf[KS], vf[KS];
  {
    // every lane loads (rows past the end read the last row and are cleared afterwards): loads under a per-lane
    // condition compile to one branch and one full wait each, sixteen round trips in a row
    u32x4 z0[KS], z1[KS];
    const long row_off = (long)min(key, L - 1) * ld + hf * 8;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      z0[s] = *(const u32x4*)(kb + row_off + s * 16);
      z1[s] = *(const u32x4*)(vb + row_off + s * 16);
    }
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      z0[s] = key < L ? z0[s] : u32x4{0u, 0u, 0u, 0u};
      z1[s] = key < L ? z1[s] : u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      kf[s] = __builtin_bit_cast(V8, z0[s]);
      vf[s] = __builtin_bit_cast(V8, z1[s]);
      pin_agpr(kf[s]);
      pin_agpr(vf[s]);
    }
  }
  f32x16 dk[DT], dv[DT];
#pragma unroll
  for (int j = 0; j < DT; ++j) {
#pragma unroll
    for (int e = 0; e < 16; ++e) dk[j][e] = dv[j][e] = 0.f;
    pin_agpr(dk[j]);
    pin_agpr(dv[j]);
  }
  const unsigned vis = (unsigned)max(L - key, 0);   // queries key .. L - 1 see this lane's key
  // the K / V fragments were requested after the four stages: when they are here, so are the stages
  asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");

  // fragment n = 0 .. 31 of a tile's first products, in MFMA order: block n / 16, Q (S) or dO (dP) by (n % 16) / 8,
  // k step n % 8
  V8 nf[8];
  auto read_frag = [&](auto n_) {
    constexpr int n = decltype(n_)::value;
    lds_read16<(n / 16) * 32 * (DH * 2) + ((n % 16) / 8) * TILE_B>(nf[n % 8], nat[n % 8]);
  };
  static_for<0, 8>([&](auto i_) { read_frag(i_); });

  TrFrag tf[8];
  f32x16 sacc0, pacc0, sacc1, pacc1;
  f32x4 ls[2][4], dd[2][4];      // per block: log-sum-exp and D of the lane's queries, [16-query step][first / second four]
  u32x4 pw[2][2], dw[2][2];      // P and dS of a block, 16 bits each: per 16-query step the B operand of the second products

  // transposed fragment for MFMA 32 + M of the second products, M = 16 c + m: step st4 = m / 4 (dO^T P, Q^T dS for
  // the first 16 queries of the block, then for the second 16), head-dimension block j = m % 4
  auto read_tr = [&](auto M_, auto half_) {
    constexpr int M = decltype(M_)::value, half = decltype(half_)::value;
    constexpr int c = M / 16, m = M % 16, st4 = m / 4, j = m % 4, g = st4 >> 1, which = st4 & 1;
    constexpr int imm = (c * 32 + g * 16) * (DH * 2) + (which ? 0 : TILE_B);
    if constexpr (half == 0) lds_read_tr<imm>(tf[M % 8].lo, tr0[j]);
    else lds_read_tr<imm>(tf[M % 8].hi, tr1[j]);
  };
  // vector r = 0 .. 3 of a block's log-sum-exp (is_d = 0) or D (is_d = 1) values: 16-query step r / 2, half r % 2
  auto read_lv = [&](auto c_, auto is_d_, auto r_) {
    constexpr int c = decltype(c_)::value, is_d = decltype(is_d_)::value, r = decltype(r_)::value;
    constexpr int imm = 128 * c + 64 * (r / 2) + (r % 2) * 16 + is_d * 256;
    if constexpr (is_d) lds_read16<imm>(dd[c][r], lsv);
    else lds_read16<imm>(ls[c][r], lsv);
  };

  auto tile = [&](auto masked_tag, int t) {
    constexpr bool MASKED = decltype(masked_tag)::value;
    const int q0 = (qt_first + t) * QR;
    // element e of block c is query q0 + 32 c + 16 (e / 8) + 8 hf + e % 8.  First half of its arithmetic: the
    // probability, which replaces the score in the accumulator register and goes into the P operand.
    auto exp_part = [&](auto c_, auto e_, f32x16& sacc) {
      constexpr int c = decltype(c_)::value, e = decltype(e_)::value, g = e >> 3, i = e & 7;
      float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[e], scale_log2, -ls[c][g * 2 + (i >> 2)][i & 3]));
      if constexpr (MASKED) {
        const int r0 = 32 * c + 16 * g + 8 * hf;
        if ((unsigned)(q0 + r0 - key + i) >= vis) p = 0.f;   // key <= query < L, as one unsigned compare
      }
      sacc[e] = p;
      if constexpr (e & 1) {
        typedef T T2 __attribute__((ext_vector_type(2)));
        T2 a;
        a[0] = from_f<T>(sacc[e - 1]);
        a[1] = from_f<T>(p);
        pw[c][g][i >> 1] = __builtin_bit_cast(uint32_t, a);
        if constexpr (i == 7) operand_ready(pw[c][g]);
      }
    };
    // second half: dS = P (dP - D), times the power of two that keeps it in the 16-bit format's range
    auto ds_part = [&](auto c_, auto e_, f32x16& sacc, const f32x16& pacc) {
      constexpr int c = decltype(c_)::value, e = decltype(e_)::value, g = e >> 3, i = e & 7;
      sacc[e] = sacc[e] * (pacc[e] - dd[c][g * 2 + (i >> 2)][i & 3]) * gsc;
      if constexpr (e & 1) {
        typedef T T2 __attribute__((ext_vector_type(2)));
        T2 a;
        a[0] = from_f<T>(sacc[e - 1]);
        a[1] = from_f<T>(sacc[e]);
        dw[c][g][i >> 1] = __builtin_bit_cast(uint32_t, a);
        if constexpr (i == 7) operand_ready(dw[c][g]);
      }
    };
    auto operand = [&](const u32x4& w) { return __builtin_bit_cast(V8, w); };

    static_for<0, 64>([&](auto g_) {
      constexpr int g = decltype(g_)::value;
      // ---- the MFMA
      if constexpr (g < 60 && g % 2 == 0) lgkm_wait<DkvPlan::wait(g)>();
      if constexpr (g < 32) {
        constexpr int s = g % 8;
        if constexpr (g < 8) mma_to_vgpr<T, s == 0>(sacc0, nf[g % 8], kf[s]);
        else if constexpr (g < 16) mma_to_vgpr<T, s == 0>(pacc0, nf[g % 8], vf[s]);
        else if constexpr (g < 24) mma_to_vgpr<T, s == 0>(sacc1, nf[g % 8], kf[s]);
        else mma_to_vgpr<T, s == 0>(pacc1, nf[g % 8], vf[s]);
      } else {
        constexpr int M = g - 32, c = M / 16, m = M % 16, st4 = m / 4, j = m % 4, gq = st4 >> 1;
        if constexpr ((st4 & 1) == 0) mma_to_agpr<T>(dv[j], tr_value<T>(tf[M % 8]), operand(pw[c][gq]));
        else mma_to_agpr<T>(dk[j], tr_value<T>(tf[M % 8]), operand(dw[c][gq]));
      }
      // ---- LDS reads of this gap
      if constexpr (g < 24) read_frag(IC<g + 8>{});
      if constexpr (g < 4) read_lv(IC<0>{}, IC<0>{}, g_);
      if constexpr (g >= 16 && g < 20) read_lv(IC<0>{}, IC<1>{}, IC<g - 16>{});
      if constexpr (g >= 20 && g < 24) read_lv(IC<1>{}, IC<0>{}, IC<g - 20>{});
      if constexpr (g >= 24 && g < 32) read_tr(IC<(g - 24) / 2>{}, IC<(g - 24) % 2>{});
      if constexpr (g >= 32 && g < 60) {
        read_tr(IC<g - 32 + 4>{}, IC<0>{});
        read_tr(IC<g - 32 + 4>{}, IC<1>{});
      }
      if constexpr (g >= 40 && g < 44) read_lv(IC<1>{}, IC<1>{}, IC<g - 40>{});
      // ---- direct-to-LDS loads of tile t + NS - 1 into the stage that tile t - 1 left
      if constexpr (g == 4) prepare_tile(t + NS - 1);
      if constexpr (g >= 5 && g < 16 && g % 2 == 1) issue_one(t + NS - 1, IC<(g - 5) / 2>{});
      if constexpr (g >= 25 && g < 32 && g % 2 == 1) issue_one(t + NS - 1, IC<6 + (g - 25) / 2>{});
      // ---- vector work of this gap
      if constexpr (g == 8) bwd_mfma_settle(sacc0);
      if constexpr (g >= 8 && g < 24) exp_part(IC<0>{}, IC<g - 8>{}, sacc0);
      if constexpr (g >= 24 && g < 32) {
        ds_part(IC<0>{}, IC<2 * (g - 24)>{}, sacc0, pacc0);
        ds_part(IC<0>{}, IC<2 * (g - 24) + 1>{}, sacc0, pacc0);
      }
      if constexpr (g >= 32 && g < 48) exp_part(IC<1>{}, IC<g - 32>{}, sacc1);
      if constexpr (g >= 48 && g < 52) {
        ds_part(IC<1>{}, IC<2 * (g - 48)>{}, sacc1, pacc1);
        ds_part(IC<1>{}, IC<2 * (g - 48) + 1>{}, sacc1, pacc1);
      }
      if constexpr (g >= 52 && g < 60) ds_part(IC<1>{}, IC<g - 44>{}, sacc1, pacc1);
      // ---- ring step and the first fragments of the next tile
      if constexpr (g == 59) {
        // every read of this tile has been issued: when they have landed, and tile t + 1 too (only the loads
        // of tiles t + 2 and t + 3 outstanding), the stage is handed back.  (The barrier is issued from
        // assembly: before its own the compiler waits for every load in flight.)
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"((NS - 2) * NLD) : "memory");
        const int step = ((t + 1) % NS == 0) ? -(NS - 1) * STAGE_B : STAGE_B;
#pragma unroll
        for (int s = 0; s < KS; ++s) nat[s] += step;
#pragma unroll
        for (int jj = 0; jj < DT; ++jj) {
          tr0[jj] += step;
          tr1[jj] += step;
        }
        lsv += step;
      }
      if constexpr (g >= 60) {
        read_frag(IC<2 * (g - 60)>{});
        read_frag(IC<2 * (g - 60) + 1>{});
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    bwd_mfma_settle_acc(dk, dv);
  };

  // Tiles on the diagonal (the first two: 128 keys against 64-query tiles) and, when L is not a multiple of
  // 64, the last one need the mask; with such an L every tile takes the masked path.
  const int n_masked = (L % QR) ? nt : min(nt, BKEY / QR);
  int t = 0;
  for (; t < n_masked; ++t) tile(std::true_type{}, t);
  for (; t < nt; ++t) tile(std::false_type{}, t);
  // The fragments read ahead for a tile that does not exist are dropped; when every wavefront's loads have landed
  // (no direct-to-LDS write may outlive the workgroup, or hit the tiles staged below) the ring is free.
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
  {
    char* stage_k = smem + wave * (2 * 8704);
    T* rk = dqkv + ((long)b * L + wk0) * ld + d + (long)head * DH;
    store_grad_rows_staged<T>(rk, ld, L - wk0, dk, scale / gsc, lane, (rope && key < L) ? rope + (long)key * DH : nullptr,
                              stage_k);
    store_grad_rows_staged<T>(rk + d, ld, L - wk0, dv, 1.0f, lane, nullptr, stage_k + 8704);
  }
}

// ---- dQ ------------------------------------------------------------------------------------------
// The same treatment for flash_bwd_dq_kernel at head_dim 128.  A workgroup owns 128 queries (32 per
// wavefront, Q and dO fragments in the accumulator file) and walks the key tiles of 64 keys below its diagonal.
// Both first products are formed transposed (S^T, dP^T: rows = keys, lane = query), so the softmax statistics are
// per-lane scalars.  A tile is 48 MFMAs: 0..15 S^T and dP^T of keys 0..31 (alternating), 16..31 of keys
// 32..63, 32..39 dQ^T += K^T dS^T of the first block, 40..47 of the second; the exponentials and dS of the first
// block in gaps 16..31, of the second in 32..43; the eight direct-to-LDS loads in the odd gaps 1..15; the ring
// step after gap 43.
struct DqPlan {
  static constexpr int tau(int gap) { return gap >= 44 ? gap - 44 : gap + 4; }
  static constexpr int reads_at(int t) {
    const int gap = t < 4 ? 44 + t : t - 4;
    if (gap >= 44) return 2;        // two fragments of the next tile
    if (gap < 24) return 1;         // fragment
    if (gap < 32) return 1;         // half a transposed fragment
    return 2;                       // transposed fragment (gaps 32..43)
  }
  static constexpr int issued_through(int t) {
    int n = 0;
    for (int i = 0; i <= t; ++i) n += reads_at(i);
    return n;
  }
  static constexpr int newer(int gap, int tr, int pos) { return issued_through(tau(gap) - 1) - issued_through(tr - 1) - pos - 1; }
  static constexpr int need_tau(int g) {
    if (g < 8) return g / 2;
    if (g < 32) return g - 4;                       // issued in gap g - 8
    const int M = g - 32;
    return M < 4 ? 29 + 2 * M : 32 + M;             // second half: gap 25 + 2 M, or gap 28 + M
  }
  static constexpr int need_pos(int g) { return g < 8 ? g % 2 : g < 32 ? 0 : (g - 32 < 4 ? 0 : 1); }
  static constexpr int wait(int g) { return newer(g, need_tau(g + 1), need_pos(g + 1)); }
};

template <class T>
__global__ __launch_bounds__(256) void flash_bwd_dq128_kernel(const T* __restrict__ qkv, const T* __restrict__ dO,
                                                              const float* __restrict__ lse2v,
                                                              const float* __restrict__ dvec, T* __restrict__ dqkv,
                                                              int L, int h, float scale,
                                                              const float* __restrict__ rope) {
  typedef typename Mma<T>::V8 V8;
  constexpr int DH = 128, BQ = 128, NS = 4, KS = DH / 16, DT = DH / 32;
  constexpr int TILE_B = KT * DH * 2;            // bytes of a K or V tile
  constexpr int STAGE_B = 2 * TILE_B;
  constexpr int NLT = TILE_B / 1024 / 4;         // wave loads per wavefront and tile
  constexpr int NLD = 2 * NLT;                   // loads per wavefront and stage
  static_assert(NLD == 8, "the refill of a stage takes the eight odd gaps 1 .. 15");
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

  const uint32_t lds0 = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)smem;
  uint32_t nat[KS], tr0[DT], tr1[DT];
  {
    const int row = pi_row(col);   // MFMA row r is key pi(r): a lane's 8 values per 16-key step are consecutive keys
#pragma unroll
    for (int s = 0; s < KS; ++s) nat[s] = lds0 + row * (DH * 2) + (((2 * s + hf) ^ tile_swz<DH>(row)) * 16);
    const int i16 = lane & 15, a = i16 >> 2, j4 = i16 & 3;
    const int k = 8 * (lane >> 5) + a;
#pragma unroll
    for (int j = 0; j < DT; ++j) {
      const int nb = j * 32 + 16 * ((lane >> 4) & 1) + 4 * j4;
      tr0[j] = lds0 + k * (DH * 2) + (((nb >> 3) ^ tile_swz<DH>(k)) * 16) + ((nb >> 2) & 1) * 8;
      tr1[j] = lds0 + (k + 4) * (DH * 2) + (((nb >> 3) ^ tile_swz<DH>(k + 4)) * 16) + ((nb >> 2) & 1) * 8;
    }
  }

  const int q_hi = min(L, qtile * BQ + BQ) - 1;
  const int nt = q_hi / KT + 1;
  // Direct-to-LDS loads of a stage: load i = 0 .. NLD - 1 of this wavefront (K rows, then V rows).  Per-lane offsets
  // from the tile's first row, the same for every full tile; the last tile of the sequence, when cut off, re-reads
  // row L - 1 for the rows past it (prepare_tile switches the offsets once; fetches past the end repeat that tile).
  constexpr int CPR = DH / 8, RPL = 64 / CPR;
  uint32_t koff[NLT];
  auto set_offsets = [&](int rows) {
#pragma unroll
    for (int j = 0; j < NLT; ++j) {
      const int row = (wave * NLT + j) * RPL + lane / CPR;
      const int gch = (lane % CPR) ^ tile_swz<DH>(row);
      koff[j] = (uint32_t)((min(row, rows - 1) * ld + gch * 8) * 2);
    }
  };
  set_offsets(KT);
  const int last_rows = min(L - (nt - 1) * KT, KT);
  auto prepare_tile = [&](int t) {
    if (t >= nt - 1 && last_rows < KT) set_offsets(last_rows);
  };
  auto issue_one = [&](int t, auto i_) {
    constexpr int i = decltype(i_)::value, j = i % NLT;
    const int key0 = min(t, nt - 1) * KT;
    const uint32_t st = lds0 + (t % NS) * STAGE_B;
    if constexpr (i < NLT) dma16(kb + (long)key0 * ld, koff[j], st + (wave * NLT + j) * 1024);
    else dma16(vb + (long)key0 * ld, koff[j], st + TILE_B + (wave * NLT + j) * 1024);
  };
#pragma unroll
  for (int t = 0; t < NS - 1; ++t) {   // the tile loop refills a stage one tile after it was used
    prepare_tile(t);
    static_for<0, NLD>([&](auto i_) { issue_one(t, i_); });
  }

  // this wavefront's 32 queries: Q and dO fragments, all requested before the first is used
  V8 qf[KS], dof[KS];
  {
    u32x4 z0[KS], z1[KS];   // loaded by every lane, then cleared past the end: see the dK / dV kernel
    const int qc = min(q, L - 1);
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      z0[s] = *(const u32x4*)(qb + (long)qc * ld + s * 16 + hf * 8);
      z1[s] = *(const u32x4*)(dob + (long)qc * d + s * 16 + hf * 8);
    }
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      z0[s] = q < L ? z0[s] : u32x4{0u, 0u, 0u, 0u};
      z1[s] = q < L ? z1[s] : u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      qf[s] = __builtin_bit_cast(V8, z0[s]);
      dof[s] = __builtin_bit_cast(V8, z1[s]);
      pin_agpr(qf[s]);
      pin_agpr(dof[s]);
    }
  }
  float lse2 = INFINITY, dq_ = 0.f;
  if (q < L) {
    lse2 = lse2v[((long)b * L + q) * h + head];
    dq_ = dvec[((long)b * L + q) * h + head];
  }
  f32x16 acc[DT];
#pragma unroll
  for (int j = 0; j < DT; ++j) {
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
    pin_agpr(acc[j]);
  }
  // the Q / dO fragments were requested after the three stages: when they are here, so are the stages
  asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");

  // fragment n = 0 .. 31 of a tile's first products, in MFMA order: key block n / 16, k step (n % 16) / 2, K (S^T, even n)
  // or V (dP^T, odd n)
  V8 nf[8];
  auto read_frag = [&](auto n_) {
    constexpr int n = decltype(n_)::value;
    lds_read16<(n / 16) * 32 * (DH * 2) + (n % 2) * TILE_B>(nf[n % 8], nat[(n % 16) / 2]);
  };
  static_for<0, 8>([&](auto i_) { read_frag(i_); });
  TrFrag tf[8];
  f32x16 sacc0, pacc0, sacc1, pacc1;
  u32x4 dw[2][2];      // dS^T of a key block, 16 bits each: per 16-key step the B operand of the second product
  // transposed fragment for MFMA 32 + M, M = 8 c + m: 16-key step m / 4 of block c, head-dimension block j = m % 4
  auto read_tr = [&](auto M_, auto half_) {
    constexpr int M = decltype(M_)::value, half = decltype(half_)::value;
    constexpr int c = M / 8, m = M % 8, g = m / 4, j = m % 4;
    constexpr int imm = (c * 32 + g * 16) * (DH * 2);
    if constexpr (half == 0) lds_read_tr<imm>(tf[M % 8].lo, tr0[j]);
    else lds_read_tr<imm>(tf[M % 8].hi, tr1[j]);
  };

  auto tile = [&](auto masked_tag, int t) {
    constexpr bool MASKED = decltype(masked_tag)::value;
    const int key0 = t * KT;
    // element e of block c is key key0 + 32 c + 16 (e / 8) + 8 hf + e % 8, the lane's column is its query
    auto element = [&](auto c_, auto e_, f32x16& sacc, const f32x16& pacc) {
      constexpr int c = decltype(c_)::value, e = decltype(e_)::value, g = e >> 3, i = e & 7;
      float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[e], scale_log2, -lse2));
      if constexpr (MASKED) {
        if (key0 + 32 * c + 16 * g + 8 * hf + i > q) p = 0.f;
      }
      sacc[e] = p * (pacc[e] - dq_) * gsc;
      if constexpr (e & 1) {
        typedef T T2 __attribute__((ext_vector_type(2)));
        T2 a;
        a[0] = from_f<T>(sacc[e - 1]);
        a[1] = from_f<T>(sacc[e]);
        dw[c][g][i >> 1] = __builtin_bit_cast(uint32_t, a);
        if constexpr (i == 7) operand_ready(dw[c][g]);
      }
    };
    auto operand = [&](const u32x4& w) { return __builtin_bit_cast(V8, w); };

    static_for<0, 48>([&](auto g_) {
      constexpr int g = decltype(g_)::value;
      if constexpr (g < 44 && g % 2 == 0) lgkm_wait<DqPlan::wait(g)>();
      if constexpr (g < 32) {
        constexpr int s = (g % 16) / 2;
        if constexpr (g < 16) {
          if constexpr (g % 2 == 0) mma_to_vgpr<T, s == 0>(sacc0, nf[g % 8], qf[s]);
          else mma_to_vgpr<T, s == 0>(pacc0, nf[g % 8], dof[s]);
        } else {
          if constexpr (g % 2 == 0) mma_to_vgpr<T, s == 0>(sacc1, nf[g % 8], qf[s]);
          else mma_to_vgpr<T, s == 0>(pacc1, nf[g % 8], dof[s]);
        }
      } else {
        constexpr int M = g - 32, c = M / 8, m = M % 8, gq = m / 4, j = m % 4;
        mma_to_agpr<T>(acc[j], tr_value<T>(tf[M % 8]), operand(dw[c][gq]));
      }
      // LDS reads of this gap
      if constexpr (g < 24) read_frag(IC<g + 8>{});
      if constexpr (g >= 24 && g < 32) read_tr(IC<(g - 24) / 2>{}, IC<(g - 24) % 2>{});
      if constexpr (g >= 32 && g < 44) {
        read_tr(IC<g - 32 + 4>{}, IC<0>{});
        read_tr(IC<g - 32 + 4>{}, IC<1>{});
      }
      // direct-to-LDS loads of tile t + NS - 1 into the stage that tile t - 1 left
      if constexpr (g == 0) prepare_tile(t + NS - 1);
      if constexpr (g < 16 && g % 2 == 1) issue_one(t + NS - 1, IC<g / 2>{});
      // vector work of this gap
      if constexpr (g == 16) bwd_mfma_settle(sacc0);
      if constexpr (g == 32) bwd_mfma_settle(sacc1);
      if constexpr (g >= 16 && g < 32) element(IC<0>{}, IC<g - 16>{}, sacc0, pacc0);
      if constexpr (g >= 32 && g < 40) element(IC<1>{}, IC<g - 32>{}, sacc1, pacc1);
      if constexpr (g >= 40 && g < 44) {
        element(IC<1>{}, IC<8 + 2 * (g - 40)>{}, sacc1, pacc1);
        element(IC<1>{}, IC<9 + 2 * (g - 40)>{}, sacc1, pacc1);
      }
      // ring step and the first fragments of the next tile
      if constexpr (g == 43) {
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"((NS - 2) * NLD) : "memory");
        const int step = ((t + 1) % NS == 0) ? -(NS - 1) * STAGE_B : STAGE_B;
#pragma unroll
        for (int s = 0; s < KS; ++s) nat[s] += step;
#pragma unroll
        for (int jj = 0; jj < DT; ++jj) {
          tr0[jj] += step;
          tr1[jj] += step;
        }
      }
      if constexpr (g >= 44) {
        read_frag(IC<2 * (g - 44)>{});
        read_frag(IC<2 * (g - 44) + 1>{});
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    asm volatile("s_nop 15\n\ts_nop 7" : "+a"(acc[0]), "+a"(acc[1]), "+a"(acc[2]), "+a"(acc[3]));
  };

  // The key tiles that reach the diagonal of some query of the workgroup (the last two) need the mask.
  const int n_plain = max(0, min(nt, (qtile * BQ) / KT));
  int t = 0;
  for (; t < n_plain; ++t) tile(std::false_type{}, t);
  for (; t < nt; ++t) tile(std::true_type{}, t);
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");   // see the dK / dV kernel
  store_grad_rows_staged<T>(dqkv + ((long)b * L + wq0) * ld + (long)head * DH, ld, L - wq0, acc, scale / gsc, lane,
                            (rope && q < L) ? rope + (long)q * DH : nullptr, smem + wave * 8704);
}

// ---- forward (training layout) ---------------------------------------------------------------------
// flash_fwd_ring_kernel at head_dim 128 on the same scheme, software-pipelined over the key tiles.  A workgroup
// works on 128 queries at a time (32 per wavefront, Q fragments in the accumulator file) and takes one or several
// such query tiles of a head in a row (snake_tile, tiles_per_workgroup); K / V tiles of 64 keys come through
// the ring.  Iteration t holds the scores S^T(t) complete in registers and runs 32 MFMAs:
//   0..15  S^T(t + 1) = K(t + 1) Q^T (the two 32-key blocks alternating) beside the exponentials of the first 32
//          keys of tile t;
//   16..31 O^T += V(t)^T P(t)^T beside the exponentials of the second 32 keys (gaps 16..27) and the maximum of
//          S^T(t + 1) (gaps 28..31);
// then the running maximum moves if it has to (rarely: see below) - so neither product waits for the vector unit
// and the exponentials run in the shadow of MFMAs.  The eight direct-to-LDS loads of tile t + 3 go into the odd
// gaps 1..15, the ring step comes after gap 27 (it waits for tile t + 2, whose K the next iteration reads).
struct FwdPlan {
  static constexpr int tau(int gap) { return gap >= 28 ? gap - 28 : gap + 4; }
  static constexpr int reads_at(int t) {
    const int gap = t < 4 ? 28 + t : t - 4;
    if (gap >= 28) return 2;        // two K fragments of the tile after the next
    if (gap < 8) return 1;          // K fragment
    if (gap < 12) return 0;
    return 2;                       // transposed V fragment (gaps 12..27)
  }
  static constexpr int issued_through(int t) {
    int n = 0;
    for (int i = 0; i <= t; ++i) n += reads_at(i);
    return n;
  }
  static constexpr int newer(int gap, int tr, int pos) { return issued_through(tau(gap) - 1) - issued_through(tr - 1) - pos - 1; }
  static constexpr int need_tau(int g) {
    if (g < 8) return g / 2;
    if (g < 16) return g - 4;                       // issued in gap g - 8
    return g;                                       // transposed fragment of MFMA 16 + M: gap 12 + M
  }
  static constexpr int need_pos(int g) { return g < 8 ? g % 2 : g < 16 ? 0 : 1; }
  static constexpr int wait(int g) { return newer(g, need_tau(g + 1), need_pos(g + 1)); }
};

// The queries a workgroup owns: `ipw` tiles of 128 of one (sequence, head), taken in order, heaviest first.  The
// G = gridDim.y workgroups of a head deal the tiles out in a snake (workgroup y takes places y, 2G - 1 - y,
// 2G + y, ... of the list of tiles by decreasing weight), which gives every workgroup the same number of key
// tiles when the count divides; place k of workgroup y, or a negative number when the list has ended.
__host__ __device__ __forceinline__ int snake_tile(int k, int y, int G, int n_tiles) {
  return n_tiles - 1 - (k * G + ((k & 1) ? G - 1 - y : y));
}

// A wavefront's 32 rows (as store_grad_rows_staged takes them) through 4352 bytes of LDS of its own, sixteen rows
// at a time - for the kernels whose ring stays live under the store.
template <class T>
__device__ __forceinline__ void store_rows_staged16(T* out, long ld, int rows, const f32x16 (&acc)[4], float mul,
                                                    int lane, const float* tab, char* tile) {
  typedef typename Mma<T>::V4 V4;
  constexpr int DH = 128, DT = 4, RS = DH * 2 + 16;
  const int col = lane & 31, hf = lane >> 5;
  char* my = tile + (col & 15) * RS;
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    if ((col >> 4) == pass) {
      if (tab == nullptr) {
#pragma unroll
        for (int j = 0; j < DT; ++j)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            V4 v;
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = from_f<T>(acc[j][g * 4 + i] * mul);
            *(V4*)(my + (j * 32 + 8 * g + 4 * hf) * 2) = v;
          }
      } else {
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
            *(V4*)(my + i0 * 2) = lo;
            *(V4*)(my + (i0 + DH / 2) * 2) = hi;
          }
      }
    }
    // the LDS executes one wavefront's operations in order: the reads see the writes above, and the writes of the
    // second pass come after the reads of the first
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int r16 = it * 4 + (lane >> 4), r = pass * 16 + r16;
      const u32x4 v = *(const u32x4*)(tile + r16 * RS + (lane & 15) * 16);
      if (r < rows) *(u32x4*)(out + (long)r * ld + (lane & 15) * 8) = v;
    }
  }
}

// LDS of the kernel below: the ring, then the four wavefronts' row staging
constexpr int FWD128_LDS = 4 * 2 * KT * 128 * 2 + 4 * 4352;

template <class T>
__global__ __launch_bounds__(256) void flash_fwd128_kernel(const T* __restrict__ qkv, T* __restrict__ o,
                                                           float* __restrict__ lse, int L, int h, float scale_log2,
                                                           int ipw) {
  typedef typename Mma<T>::V8 V8;
  constexpr int DH = 128, BQ = 128, NS = 4, KS = DH / 16, DT = DH / 32;
  constexpr int TILE_B = KT * DH * 2;            // bytes of a K or V tile
  constexpr int STAGE_B = 2 * TILE_B;
  constexpr int NLT = TILE_B / 1024 / 4;         // wave loads per wavefront and tile
  constexpr int NLD = 2 * NLT;                   // loads per wavefront and stage
  static_assert(NLD == 8, "the refill of a stage takes the eight odd gaps 1 .. 15");
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  const int b = blockIdx.x / h, head = blockIdx.x % h;
  const int d = h * DH;
  const long ld = 3L * d;
  const int n_qt = (L + BQ - 1) / BQ;
  const T* qb = qkv + (long)b * L * ld + (long)head * DH;
  const T* kb = qb + d;
  const T* vb = qb + 2 * d;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int col = lane & 31, hf = lane >> 5;

  const uint32_t lds0 = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)smem;
  // K fragments and V^T fragments: the addresses below are those of ring stage pk and pv
  uint32_t nat[KS], tr0[DT], tr1[DT];
  int pk = 0, pv = 0;
  {
    const int row = pi_row(col);   // MFMA row r is key pi(r): a lane's 8 values per 16-key step are consecutive keys
#pragma unroll
    for (int s = 0; s < KS; ++s) nat[s] = lds0 + row * (DH * 2) + (((2 * s + hf) ^ tile_swz<DH>(row)) * 16);
    const int i16 = lane & 15, a = i16 >> 2, j4 = i16 & 3;
    const int k = 8 * (lane >> 5) + a;
#pragma unroll
    for (int j = 0; j < DT; ++j) {
      const int nb = j * 32 + 16 * ((lane >> 4) & 1) + 4 * j4;
      tr0[j] = lds0 + TILE_B + k * (DH * 2) + (((nb >> 3) ^ tile_swz<DH>(k)) * 16) + ((nb >> 2) & 1) * 8;
      tr1[j] = lds0 + TILE_B + (k + 4) * (DH * 2) + (((nb >> 3) ^ tile_swz<DH>(k + 4)) * 16) + ((nb >> 2) & 1) * 8;
    }
  }
  auto step_k = [&]() {   // K fragments: on to the next stage of the ring
    const int step = pk == NS - 1 ? -(NS - 1) * STAGE_B : STAGE_B;
    pk = pk == NS - 1 ? 0 : pk + 1;
#pragma unroll
    for (int s = 0; s < KS; ++s) nat[s] += step;
  };
  auto step_v = [&]() {
    const int step = pv == NS - 1 ? -(NS - 1) * STAGE_B : STAGE_B;
    pv = pv == NS - 1 ? 0 : pv + 1;
#pragma unroll
    for (int jj = 0; jj < DT; ++jj) {
      tr0[jj] += step;
      tr1[jj] += step;
    }
  };

  // ---- the direct-to-LDS loads of a key tile (K and V rows 64 kt ..) into a ring stage
  constexpr int CPR = DH / 8, RPL = 64 / CPR;
  uint32_t koff[NLT];
  int off_rows = 0;   // the row count koff was made for
  auto prepare_tile = [&](int kt) {
    const int rows = min(L - kt * KT, KT);
    if (rows != off_rows) {   // uniform; after the first tile only where a sequence ends inside a tile
      off_rows = rows;
#pragma unroll
      for (int j = 0; j < NLT; ++j) {
        const int row = (wave * NLT + j) * RPL + lane / CPR;
        const int gch = (lane % CPR) ^ tile_swz<DH>(row);
        koff[j] = (uint32_t)((min(row, rows - 1) * ld + gch * 8) * 2);
      }
    }
  };
  auto issue_one = [&](int stage, int kt, auto i_) {
    constexpr int i = decltype(i_)::value, j = i % NLT;
    const uint32_t st = lds0 + stage * STAGE_B;
    if constexpr (i < NLT) dma16(kb + (long)kt * KT * ld, koff[j], st + (wave * NLT + j) * 1024);
    else dma16(vb + (long)kt * KT * ld, koff[j], st + TILE_B + (wave * NLT + j) * 1024);
  };

  // ---- the workgroup's query tiles
  const int G = gridDim.y, y = blockIdx.y;
  struct Item {
    int qtile, nt, n_iter;
  };
  auto make_item = [&](int k) {
    Item it;
    it.qtile = k < ipw ? snake_tile(k, y, G, n_qt) : -1;
    const int q_hi = min(L, it.qtile * BQ + BQ) - 1;
    it.nt = q_hi / KT + 1;
    // an odd number of tiles (only when L is not a multiple of 128) is rounded up: see the loop below
    it.n_iter = it.nt + (it.nt & 1);
    return it;
  };
  auto load_q = [&](u32x4 (&z)[KS], int qtile) {   // by every lane, cleared past the end afterwards: see the dK / dV kernel
    const int qc = min(qtile * BQ + wave * 32 + col, L - 1);
#pragma unroll
    for (int s = 0; s < KS; ++s) z[s] = *(const u32x4*)(qb + (long)qc * ld + s * 16 + hf * 8);
  };

  int k_item = 0;
  Item cur = make_item(0);
  int gs = 0;   // ring stage of tile 0 of the current item
#pragma unroll
  for (int u = 0; u < NS - 1; ++u) {   // the tile loop refills a stage one tile after it was last used
    const int kt = min(u, cur.nt - 1);
    prepare_tile(kt);
    static_for<0, NLD>([&](auto i_) { issue_one(u, kt, i_); });
  }
  u32x4 z[KS];
  load_q(z, cur.qtile);

  V8 qf[KS];
  f32x16 oacc[DT];
  V8 nf[8];
  TrFrag tf[8];
  f32x16 sa[2], sb[2];   // the scores of the tile being normalised and of the tile being multiplied, alternately
  u32x4 pw[4];           // P^T of the tile, 16 bits each: the B operand of each 16-key step of the second product
  float m_run, l_run, m_ref;
  int wq0, q, t_plain;

  // K fragment n = 0 .. 15 of a tile, in MFMA order: k step n / 2, key block n % 2
  auto read_frag = [&](auto n_) {
    constexpr int n = decltype(n_)::value;
    lds_read16<(n % 2) * 32 * (DH * 2)>(nf[n % 8], nat[n / 2]);
  };
  // transposed fragment of V for MFMA 16 + M, M = 4 kk + j: 16-key step kk, head-dimension block j
  auto read_tr = [&](auto M_, auto half_) {
    constexpr int M = decltype(M_)::value, half = decltype(half_)::value;
    constexpr int kk = M / 4, j = M % 4;
    if constexpr (half == 0) lds_read_tr<kk * 16 * (DH * 2)>(tf[M % 8].lo, tr0[j]);
    else lds_read_tr<kk * 16 * (DH * 2)>(tf[M % 8].hi, tr1[j]);
  };
  // Mask and maximum of the scores of tile `tile` (element e of block c <-> key 64 tile + 32 c + 16 (e / 8) + 8 hf + e % 8),
  // then the reference of the exponentials: m_run follows the running maximum lazily - only when some query of the
  // wavefront exceeds it by more than 2^8 are the sum and the accumulators rescaled (exact either way; until then
  // p <= 256, far inside every format involved), which takes the rescaling out of all but the first tiles of a row.
  auto part_max = [&](bool masked, f32x16 (&sc)[2], int tile, auto c_, auto quarter_, float& mx) {
    constexpr int c = decltype(c_)::value, e0 = decltype(quarter_)::value * 8;
    if (masked) {   // uniform: the tile reaches the diagonal of some query of the wavefront
#pragma unroll
      for (int e = e0; e < e0 + 8; ++e) {
        const int key = tile * KT + c * 32 + 16 * (e >> 3) + 8 * hf + (e & 7);
        if (key > q) sc[c][e] = -INFINITY;
      }
    }
#pragma unroll
    for (int e = e0; e < e0 + 8; ++e) mx = fmaxf(mx, sc[c][e]);
  };
  auto new_reference = [&](float mx) {
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * scale_log2;
    if (__builtin_amdgcn_ballot_w64(mx > m_run + 8.f) != 0) {
      const float m_new = fmaxf(m_run, mx);
      const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m_run - m_new);
      l_run *= alpha;
      m_run = m_new;
#pragma unroll
      for (int j = 0; j < DT; ++j) {
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[j][e] *= alpha;
        pin_agpr(oacc[j]);
      }
    }
    m_ref = m_run == -INFINITY ? 0.f : m_run;   // a row with no visible key yet
  };

  Item nxt_item = make_item(1);
  // Iteration t of the current item: `cur_s` holds the scores of tile t, `nxt_s` receives those of tile t + 1.
  auto iteration = [&](int t, f32x16 (&cur_s)[2], f32x16 (&nxt_s)[2]) {
    const bool masked = t + 1 >= t_plain;
    float rs = 0.f, mx = -INFINITY;
    // the tile that goes into the stage tile t - 1 left: tile t + 3 of this item (its last tile again once it has
    // run out), and past its last iteration the first tiles of the workgroup's next item
    const int u = t + NS - 1;
    const int stage = (gs + u) % NS;
    const int kt = u < cur.n_iter ? min(u, cur.nt - 1) : nxt_item.qtile >= 0 ? min(u - cur.n_iter, nxt_item.nt - 1) : cur.nt - 1;
    auto exponential = [&](auto c_, auto e_) {
      constexpr int c = decltype(c_)::value, e = decltype(e_)::value, g = e >> 3, i = e & 7;
      const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(cur_s[c][e], scale_log2, -m_ref));
      rs += p;
      cur_s[c][e] = p;
      if constexpr (e & 1) {
        typedef T T2 __attribute__((ext_vector_type(2)));
        T2 a;
        a[0] = from_f<T>(cur_s[c][e - 1]);
        a[1] = from_f<T>(p);
        pw[c * 2 + g][i >> 1] = __builtin_bit_cast(uint32_t, a);
        if constexpr (i == 7) operand_ready(pw[c * 2 + g]);
      }
    };
    auto operand = [&](const u32x4& w) { return __builtin_bit_cast(V8, w); };
    static_for<0, 32>([&](auto g_) {
      constexpr int g = decltype(g_)::value;
      if constexpr (g < 28 && g % 2 == 0) lgkm_wait<FwdPlan::wait(g)>();
      if constexpr (g < 16) {
        mma_to_vgpr<T, (g / 2 == 0)>(nxt_s[g % 2], nf[g % 8], qf[g / 2]);
      } else {
        constexpr int M = g - 16, kk = M / 4, j = M % 4;
        mma_to_agpr<T>(oacc[j], tr_value<T>(tf[M % 8]), operand(pw[kk]));
      }
      // LDS reads
      if constexpr (g < 8) read_frag(IC<g + 8>{});
      if constexpr (g >= 12 && g < 16) {
        read_tr(IC<g - 12>{}, IC<0>{});
        read_tr(IC<g - 12>{}, IC<1>{});
      }
      if constexpr (g >= 16 && g < 28) {
        read_tr(IC<g - 16 + 4>{}, IC<0>{});
        read_tr(IC<g - 16 + 4>{}, IC<1>{});
      }
      // direct-to-LDS loads
      if constexpr (g == 0) prepare_tile(kt);
      if constexpr (g < 16 && g % 2 == 1) issue_one(stage, kt, IC<g / 2>{});
      // vector work
      if constexpr (g < 16) exponential(IC<0>{}, g_);
      if constexpr (g >= 16 && g < 24) exponential(IC<1>{}, IC<g - 16>{});
      if constexpr (g >= 24 && g < 28) {
        exponential(IC<1>{}, IC<8 + 2 * (g - 24)>{});
        exponential(IC<1>{}, IC<9 + 2 * (g - 24)>{});
      }
      if constexpr (g >= 28) part_max(masked, nxt_s, t + 1, IC<(g - 28) / 2>{}, IC<(g - 28) % 2>{}, mx);
      if constexpr (g == 27) {
        // every read of this iteration has been issued: when they have landed, and tile t + 2 too (only the loads of
        // this iteration outstanding), the stage of tile t is handed back; K moves on to tile t + 2, V to tile t + 1
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(NLD) : "memory");
        step_k();
        step_v();
      }
      if constexpr (g >= 28) {
        read_frag(IC<2 * (g - 28)>{});
        read_frag(IC<2 * (g - 28) + 1>{});
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    l_run += rs;
    asm volatile("s_nop 15\n\ts_nop 7" : "+a"(oacc[0]), "+a"(oacc[1]), "+a"(oacc[2]), "+a"(oacc[3]));
    new_reference(mx);
  };

  while (true) {
    // ---- start of an item: its Q fragments (loaded a while ago), empty accumulators
    wq0 = cur.qtile * BQ + wave * 32;
    q = wq0 + col;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      qf[s] = __builtin_bit_cast(V8, q < L ? z[s] : u32x4{0u, 0u, 0u, 0u});
      pin_agpr(qf[s]);
    }
#pragma unroll
    for (int j = 0; j < DT; ++j) {
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[j][e] = 0.f;
      pin_agpr(oacc[j]);
    }
    m_run = -INFINITY, l_run = 0.f, m_ref = 0.f;
    // The Q loads were issued after every direct-to-LDS load so far, with none in between, and loads return in
    // order: the compiler's own wait for them (it sits before the selects above) has also waited for the item's
    // first three tiles - while the stores of the previous item's rows, which came later, may still be on their way.
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");

    // ---- the scores of tile 0, their maximum, and the first K fragments of tile 1.  K fragments stand one stage
    // past the item's first after the previous item (or at it, for the first item); V fragments stand at it.
    if (pk != gs) {
      const int back = pk == 0 ? (NS - 1) * STAGE_B : -STAGE_B;
      pk = gs;
#pragma unroll
      for (int s = 0; s < KS; ++s) nat[s] += back;
    }
    static_for<0, 8>([&](auto i_) { read_frag(i_); });
    static_for<0, 16>([&](auto g_) {
      constexpr int g = decltype(g_)::value;
      lgkm_wait<(g < 8 ? 7 : 15 - g)>();   // fragments g + 1 .. g + 7 (up to the sixteenth) may still be on their way
      mma_to_vgpr<T, (g / 2 == 0)>(sa[g % 2], nf[g % 8], qf[g / 2]);
      if constexpr (g < 8) read_frag(IC<g + 8>{});
    });
    {
      step_k();
      static_for<0, 8>([&](auto i_) { read_frag(i_); });
      asm volatile("s_nop 10" : "+v"(sa[0]), "+v"(sa[1]));
      float mx = -INFINITY;
      static_for<0, 4>([&](auto k_) { part_max(true, sa, 0, IC<decltype(k_)::value / 2>{}, IC<decltype(k_)::value % 2>{}, mx); });
      new_reference(mx);
    }

    // Tiles entirely below the diagonal of the wavefront's first row need no mask; the rest are masked, and so is the
    // tile past the last one, whose scores the last iteration forms and nobody uses (a tile entirely above the last
    // row's diagonal adds zeros: all wavefronts make the same trips, so the barriers match).
    t_plain = min(cur.nt, max(0, (wq0 + 1) / KT));
    // The two score buffers change roles every iteration: one loop, two iterations per trip, so that every fragment
    // in flight across an iteration boundary is in the registers the next iteration expects (another loop would be
    // another register assignment, and the compiler would copy registers whose reads have not landed).  The extra
    // iteration of an odd tile count works on scores that are all masked, i.e. adds P = 0.
    for (int t = 0; t < cur.n_iter; t += 2) {
      iteration(t, sa, sb);
      iteration(t + 1, sb, sa);
    }
    // the fragments read ahead for a tile nobody multiplies land before their registers get another use
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");

    // ---- end of the item: ask for the next item's Q, store this item's rows (the ring stays live: its stages hold
    // or await the next item's first tiles)
    const bool more = nxt_item.qtile >= 0;
    if (more) load_q(z, nxt_item.qtile);
    const float l = l_run + __shfl_xor(l_run, 32, 64);
    store_rows_staged16<T>(o + ((long)b * L + wq0) * d + (long)head * DH, d, L - wq0, oacc, 1.0f / l, lane, nullptr,
                           smem + NS * STAGE_B + wave * 4352);
    if (lse && hf == 0 && q < L)
      lse[((long)b * L + q) * h + head] = (m_run + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
    if (!more) break;
    gs = (gs + cur.n_iter) % NS;
    cur = nxt_item;
    ++k_item;
    nxt_item = make_item(k_item + 1);
  }
  // no direct-to-LDS write may outlive the workgroup
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}
