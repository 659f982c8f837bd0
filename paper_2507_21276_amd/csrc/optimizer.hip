// Model update after a training task (Model Update Synchronization: a co-located instance
// applies its own updates, and later inference tasks on the stage are served from them).
// One bandwidth-bound pass per parameter tensor: gradient, both moments and the fp32 master
// weight are read once; the moments, the master weight, the parameter vector in its storage
// type and the matrix-core operand copy are written in the same pass.
//   SGD with momentum and L2 decay:  g' = g + wd w;  b <- mu b + g';  w <- w - lr b
//   AdamW (decoupled decay):         m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2
//                                    w <- w - lr (m / c1 / (sqrt(v / c2) + eps) + wd w),  c = 1 - beta^t
// Algorithmic bytes per parameter: 16 read (g, m, v, w) + 12 written + the two 16-bit copies.
#include "common.h"

namespace {

struct OptArgs {
  int kind;            // 0 SGD, 1 AdamW
  float lr, beta1, beta2, eps, wd, momentum, grad_scale;
  float inv_c1, inv_c2;   // 1 / (1 - beta1^t), 1 / (1 - beta2^t)
};

template <class TP, class TO>
__global__ __launch_bounds__(256) void optimizer_kernel(OptArgs a, size_t n, const float* __restrict__ g,
                                                        float* __restrict__ m, float* __restrict__ v,
                                                        float* master, TP* params, TO* params_op) {
  const size_t i4 = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i4 >= n) return;
  const int cnt = n - i4 < 4 ? (int)(n - i4) : 4;
  float gg[4], mm[4], vv[4], ww[4];
  if (cnt == 4) {
    const f32x4 g4 = *(const f32x4*)(g + i4), m4 = *(const f32x4*)(m + i4), w4 = *(const f32x4*)(master + i4);
    f32x4 v4 = {0.f, 0.f, 0.f, 0.f};
    if (a.kind == 1) v4 = *(const f32x4*)(v + i4);
#pragma unroll
    for (int e = 0; e < 4; ++e) { gg[e] = g4[e]; mm[e] = m4[e]; vv[e] = v4[e]; ww[e] = w4[e]; }
  } else {
    for (int e = 0; e < 4; ++e) {
      const bool ok = e < cnt;
      gg[e] = ok ? g[i4 + e] : 0.f;
      mm[e] = ok ? m[i4 + e] : 0.f;
      vv[e] = ok && a.kind == 1 ? v[i4 + e] : 0.f;
      ww[e] = ok ? master[i4 + e] : 0.f;
    }
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    float gi = gg[e] * a.grad_scale;
    if (a.kind == 0) {
      gi += a.wd * ww[e];
      mm[e] = a.momentum * mm[e] + gi;
      ww[e] -= a.lr * mm[e];
    } else {
      mm[e] = a.beta1 * mm[e] + (1.0f - a.beta1) * gi;
      vv[e] = a.beta2 * vv[e] + (1.0f - a.beta2) * gi * gi;
      const float mh = mm[e] * a.inv_c1, vh = vv[e] * a.inv_c2;
      ww[e] -= a.lr * (mh / (sqrtf(vh) + a.eps) + a.wd * ww[e]);
    }
  }
  if (cnt == 4) {
    *(f32x4*)(m + i4) = f32x4{mm[0], mm[1], mm[2], mm[3]};
    if (a.kind == 1) *(f32x4*)(v + i4) = f32x4{vv[0], vv[1], vv[2], vv[3]};
    *(f32x4*)(master + i4) = f32x4{ww[0], ww[1], ww[2], ww[3]};
  } else {
    for (int e = 0; e < cnt; ++e) {
      m[i4 + e] = mm[e];
      if (a.kind == 1) v[i4 + e] = vv[e];
      master[i4 + e] = ww[e];
    }
  }
  for (int e = 0; e < cnt; ++e) {
    // the 16-bit copies are rounded from the fp32 master weight, the operand copy from the
    // stored parameter (what ls_bind_params would produce from it)
    if ((const void*)params != (const void*)master) params[i4 + e] = from_f<TP>(ww[e]);
    if (params_op) params_op[i4 + e] = from_f<TO>(to_f(from_f<TP>(ww[e])));
  }
}

template <class TP, class TO>
ls_status launch(const OptArgs& a, size_t n, const float* g, float* m, float* v, float* master, void* params,
                 void* params_op, hipStream_t st) {
  const size_t wgs = (n + 1023) / 1024;
  optimizer_kernel<TP, TO><<<(unsigned)wgs, 256, 0, st>>>(a, n, g, m, v, master, (TP*)params, (TO*)params_op);
  LS_CHECK_LAUNCH();
  return LS_OK;
}

}  // namespace

// One tensor of n elements starting at the given pointers.  param_dtype: LS_F32 (params may be
// the master vector itself) or LS_BF16; op_dtype / params_op: the operand copy (LS_F16 or
// LS_BF16), or params_op == nullptr when the stage reads the parameter vector directly.
extern "C" ls_status lsk_optimizer(int kind, float lr, float beta1, float beta2, float eps, float weight_decay,
                                   float momentum, float grad_scale, int step, size_t n, const float* grad, float* m,
                                   float* v, float* master, void* params, int param_dtype, void* params_op,
                                   int op_dtype, void* stream) {
  LS_REQUIRE(kind == 0 || kind == 1, "optimizer: kind must be 0 (SGD) or 1 (AdamW)");
  LS_REQUIRE(grad && m && master && params && (kind == 0 || v), "optimizer: null argument");
  LS_REQUIRE(step >= 1, "optimizer: steps count from 1");
  LS_REQUIRE(param_dtype == LS_F32 || param_dtype == LS_BF16, "optimizer: parameters are fp32 or bf16");
  LS_REQUIRE(param_dtype != LS_F32 || !params_op, "optimizer: fp32 stages have no operand copy");
  LS_REQUIRE(!params_op || op_dtype == LS_F16 || op_dtype == LS_BF16, "optimizer: operand copy is fp16 or bf16");
  LS_REQUIRE(((uintptr_t)grad | (uintptr_t)m | (uintptr_t)master | (uintptr_t)(kind == 1 ? v : m)) % 16 == 0,
             "optimizer: fp32 vectors must be 16-byte aligned");
  if (n == 0) return LS_OK;
  OptArgs a{kind, lr, beta1, beta2, eps, weight_decay, momentum, grad_scale,
            (float)(1.0 / (1.0 - pow((double)beta1, step))), (float)(1.0 / (1.0 - pow((double)beta2, step)))};
  hipStream_t st = (hipStream_t)stream;
  if (param_dtype == LS_F32) return launch<float, f16_t>(a, n, grad, m, v, master, params, nullptr, st);
  if (!params_op || op_dtype == LS_BF16) return launch<bf16_t, bf16_t>(a, n, grad, m, v, master, params, params_op, st);
  return launch<bf16_t, f16_t>(a, n, grad, m, v, master, params, params_op, st);
}
