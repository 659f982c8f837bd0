// Shared device/host helpers of the stage library (HIP, gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/lemix_kernels.h"
#include "../../include/lemix_stage.h"

typedef __bf16 bf16_t;
typedef _Float16 f16_t;

typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef f16_t f16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef f16_t f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define LS_WAVE 64

template <class T> struct vec8;
template <> struct vec8<bf16_t> { typedef bf16x8 type; };
template <> struct vec8<f16_t> { typedef f16x8 type; };

template <class T> __device__ __forceinline__ float to_f(T v) { return (float)v; }
template <class T> __device__ __forceinline__ T from_f(float v) { return (T)v; }

// element load/store by runtime dtype (LS_F32 / LS_BF16 / LS_F16)
__device__ __forceinline__ float load_as_f(const void* p, size_t i, int dtype) {
  if (dtype == LS_F32) return ((const float*)p)[i];
  if (dtype == LS_BF16) return (float)((const bf16_t*)p)[i];
  return (float)((const f16_t*)p)[i];
}
__device__ __forceinline__ void store_from_f(void* p, size_t i, int dtype, float v) {
  if (dtype == LS_F32) ((float*)p)[i] = v;
  else if (dtype == LS_BF16) ((bf16_t*)p)[i] = (bf16_t)v;
  else ((f16_t*)p)[i] = (f16_t)v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// block-wide sum for blockDim.x a multiple of 64, up to 1024; `red` has >= 16 floats
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += red[i];
  return t;
}

constexpr float kGeluC = 0.7978845608028654f;  // sqrt(2/pi)
__device__ __forceinline__ float gelu_f(float u, int kind) {
  if (kind == LS_ACT_GELU_TANH) return 0.5f * u * (1.f + tanhf(kGeluC * (u + 0.044715f * u * u * u)));
  return 0.5f * u * (1.f + erff(u * 0.70710678118654752f));
}

static inline size_t dtype_size(int dt) { return dt == LS_F32 ? 4 : 2; }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Launch timing by kind of kernel (lsk_timing_begin / lsk_timing_end, defined in stage.hip): while it is on,
// an LsTimed object at the top of an entry point records a HIP event on the stream before the entry point's
// launches and one after them; nested entry points count once, under the outermost kind.
struct LsTimed {
  LsTimed(int kind, void* stream);
  ~LsTimed();
  bool armed;
  void* stream;
};

// host-side error plumbing (defined in stage.hip)
void ls_set_error(const char* fmt, ...);
#define LS_CHECK_HIP(expr)                                                         \
  do {                                                                             \
    hipError_t e_ = (expr);                                                        \
    if (e_ != hipSuccess) {                                                        \
      ls_set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
      return LS_EHIP;                                                              \
    }                                                                              \
  } while (0)
#define LS_CHECK_LAUNCH() LS_CHECK_HIP(hipGetLastError())
#define LS_REQUIRE(cond, ...)                                                      \
  do {                                                                             \
    if (!(cond)) {                                                                 \
      ls_set_error(__VA_ARGS__);                                                   \
      return LS_EINVAL;                                                            \
    }                                                                              \
  } while (0)
#define LS_TRY(expr)                                                               \
  do {                                                                             \
    ls_status s_ = (expr);                                                         \
    if (s_ != LS_OK) return s_;                                                    \
  } while (0)
