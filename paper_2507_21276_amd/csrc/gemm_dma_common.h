// Shared by the two direct-to-LDS GEMM kernels (32x32x16 and 16x16x32 MFMA): launch arguments,
// the LDS tile layouts' load side, and the placement of memory instructions between MFMAs.
#pragma once
#include "common.h"

namespace {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

struct DmaArgs {
  int M, N, K;
  const void* A; long lda; int a_kmajor;
  const void* B; long ldb; int b_kmajor;
  void* C; long ldc; int c_dtype;
  const void* bias; int bias_dtype;
  const float* resid; long ldr;
  int accumulate;
  const float* alpha;
  int tiles_m, tiles_n;
  long split_stride;   // split-K launches (gridDim.y > 1, MODE 2): elements between the partial results
  // MODE 3 only: rotary embedding of the columns below rope_cols (heads of 128)
  const int32_t* rope_pos; const float* rope_table; int rope_cols;
  // MODE 5 only (16x16x32 kernel): the product is the gradient of a SwiGLU output; the saved (gate | up)
  // pre-activations [M, 2 N] and the gradient buffer of the same shape that the epilogue fills
  const void* glu_pre = nullptr; void* glu_grad = nullptr;
};

constexpr int TK = 64;  // k extent of a tile; a tile of ROWS rows is ROWS * 128 bytes = ROWS / 8 wave loads

// Direct-to-LDS loads of one operand tile of ROWS rows (256 or 128): ROWS / 32
// wave loads per wavefront.  The per-lane byte offsets inside the tile are fixed
// for the whole k loop (`off`, computed once); only the uniform tile base moves.
// K8: the chunk index of a k-strided tile is also XOR-permuted with 2 * ((k >> 3) & 1) (the 16x16x32 kernel,
// whose transposing reads put k and k + 8 into the same 32 lanes)
template <bool KMAJOR, int ROWS, bool K8 = false>
__device__ __forceinline__ void tile_offsets(uint32_t (&off)[ROWS / 32], long ld, int row0, int nrows, int wave,
                                             int lane) {
  constexpr int NL = ROWS / 32;         // wave loads per wavefront
  constexpr int LPR = ROWS / 8;         // lanes (16-byte chunks) per k row of a k-strided tile
#pragma unroll
  for (int j = 0; j < NL; ++j) {
    const int q = wave * NL + j;  // 1 KB block of the tile
    if (KMAJOR) {
      const int row = q * 8 + (lane >> 3);
      const int kc = (lane & 7) ^ ((row >> 1) & 7);
      int gr = row0 + row;
      gr = gr < nrows ? gr : nrows - 1;  // rows past the edge: any valid data, never stored
      off[j] = (uint32_t)(((long)(gr - row0) * ld + kc * 8) * 2);
    } else {
      const int krow = q * (64 / LPR) + lane / LPR;
      const int cl = (lane % LPR) ^ (4 * (krow & 3)) ^ (K8 ? 2 * ((krow >> 3) & 1) : 0);
      int gr = row0 + cl * 8;
      gr = gr + 8 <= nrows ? gr : nrows - 8;
      off[j] = (uint32_t)(((long)krow * ld + (gr - row0)) * 2);
    }
  }
}

// One direct-to-LDS wave load in the scalar-base form: address = uniform 64-bit base + per-lane 32-bit
// offset, LDS destination in M0.  Issued from assembly: the builtin takes a flat pointer, which the
// compiler forms with a 64-bit vector add per load (1 % of the GEMM leg).  The compiler therefore does not
// count these loads: every wait for them in this file is explicit (s_waitcnt with vmcnt(0)).
__device__ __forceinline__ void dma_load(const char* base, uint32_t off, const char* lds_dst) {
  const uint32_t l = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)lds_dst;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(l), "v"(off), "s"(base)
               : "memory", "m0");
}

template <int ROWS>
__device__ __forceinline__ void issue_tile(const char* tile_base, const uint32_t (&off)[ROWS / 32], char* lds_tile,
                                           int wave) {
  constexpr int NL = ROWS / 32;
#pragma unroll
  for (int j = 0; j < NL; ++j) dma_load(tile_base, off[j], lds_tile + (wave * NL + j) * 1024);
}

// load `l` (0 .. (BM + BN) / 32 - 1) of a wavefront's share of the A and B tiles
template <int BM, int BN>
__device__ __forceinline__ void issue_one(int l, const char* a_tile, const uint32_t (&a_off)[BM / 32],
                                          const char* b_tile, const uint32_t (&b_off)[BN / 32], char* lds_a,
                                          char* lds_b, int wave) {
  constexpr int NA = BM / 32, NB = BN / 32;
  if (l < NA) dma_load(a_tile, a_off[l], lds_a + (wave * NA + l) * 1024);
  else dma_load(b_tile, b_off[l - NA], lds_b + (wave * NB + l - NA) * 1024);
}

// Where in a k sub-step of NM MFMAs the other instructions go: one LDS fragment read or one
// direct-to-LDS load in the gap after an MFMA, instead of a chunk's reads and load together after
// every second MFMA (1.1 % on the GEMM leg).  Reads are spread over the first seven eighths of the
// sub-step (the rest covers the last one's latency; spreading them over three quarters or all of it
// measured 0.5 % slower, over half of it 2 % slower), loads take the gaps in between and at the end;
// with more loads than free gaps they share gaps from the first on.
template <int NM, int NF, int LPK>
struct GapPlan {
  int read_gap[NF];
  int load_gap[LPK > 0 ? LPK : 1];
  constexpr GapPlan() : read_gap{}, load_gap{} {
    const int span = NM * 7 / 8 > 0 ? NM * 7 / 8 : 1;
    for (int r = 0; r < NF; ++r) read_gap[r] = r * span / NF;
    int cnt = 0;
    for (int g = 0; g < NM && cnt < LPK; ++g) {
      bool taken = false;
      for (int r = 0; r < NF; ++r) taken = taken || read_gap[r] == g;
      if (!taken) load_gap[cnt++] = g;
    }
    for (int l = cnt; l < LPK; ++l) load_gap[l] = (l - cnt) % NM;
  }
};

typedef f32x4 __attribute__((may_alias)) f32x4_a;
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef u32x2_t __attribute__((may_alias)) u32x2_a;

}  // namespace
