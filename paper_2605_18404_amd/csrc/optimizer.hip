// Optimizer step (the pipeline's "OS" instruction, Table 2): one AdamW update of the flat
// parameter vector, in place.  Element-wise and bound by HBM: 16 bytes read and 12 written per
// parameter, one pass, 16-byte accesses.
#include <cmath>

#include "common.h"

namespace {

struct AdamwConsts {
  float b1, one_minus_b1, b2, one_minus_b2;
  float c1, c2;  // bias corrections 1 / (1 - beta^t), formed in double on the host
  float lr, eps, wd, gscale;
};

__device__ __forceinline__ void adamw_one(float& th, float g, float& m, float& v, const AdamwConsts& k) {
  g *= k.gscale;
  m = k.b1 * m + k.one_minus_b1 * g;
  v = k.b2 * v + k.one_minus_b2 * (g * g);
  const float step = (m * k.c1) / (sqrtf(v * k.c2) + k.eps) + k.wd * th;
  th -= k.lr * step;
}

// VEC = 4: all four arrays are 16-byte aligned, thread t handles elements 4t..4t+3 (n4 groups) and
// the last n - 4 n4 elements are taken one each by the first threads.  VEC = 1: one element per thread.
template <int VEC>
__global__ void __launch_bounds__(256) k_adamw(float* __restrict__ theta, const float* __restrict__ grad, float* __restrict__ m,
                                               float* __restrict__ v, int64_t n, AdamwConsts k) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (VEC == 4) {
    const int64_t n4 = n >> 2;
    if (t < n4) {
      float4 th = reinterpret_cast<float4*>(theta)[t], mm = reinterpret_cast<float4*>(m)[t], vv = reinterpret_cast<float4*>(v)[t];
      const float4 g = reinterpret_cast<const float4*>(grad)[t];
      adamw_one(th.x, g.x, mm.x, vv.x, k);
      adamw_one(th.y, g.y, mm.y, vv.y, k);
      adamw_one(th.z, g.z, mm.z, vv.z, k);
      adamw_one(th.w, g.w, mm.w, vv.w, k);
      reinterpret_cast<float4*>(theta)[t] = th;
      reinterpret_cast<float4*>(m)[t] = mm;
      reinterpret_cast<float4*>(v)[t] = vv;
    }
    const int64_t i = (n4 << 2) + t;
    if (t < 3 && i < n) adamw_one(theta[i], grad[i], m[i], v[i], k);
  } else {
    if (t < n) adamw_one(theta[t], grad[t], m[t], v[t], k);
  }
}

}  // namespace

extern "C" int mlip_optimizer_step(mlip_ctx* ctx, int64_t n, float* params, const float* grad, float* m, float* v,
                                   int32_t step, const mlip_adamw* h) {
  if (!ctx) return MLIP_E_INVALID;
  if (!params || !grad || !m || !v || !h) MLIP_FAIL(ctx, MLIP_E_INVALID, "optimizer_step: null pointer");
  if (n < 0 || step < 1) MLIP_FAIL(ctx, MLIP_E_INVALID, "optimizer_step: n must be >= 0 and step >= 1");
  if (!std::isfinite(h->lr) || !(h->beta1 >= 0.f && h->beta1 < 1.f) || !(h->beta2 >= 0.f && h->beta2 < 1.f) || !(h->eps >= 0.f) ||
      !std::isfinite(h->eps) || !(h->weight_decay >= 0.f) || !std::isfinite(h->weight_decay) || !std::isfinite(h->grad_scale))
    MLIP_FAIL(ctx, MLIP_E_INVALID, "optimizer_step: hyper-parameters out of range");
  if (n == 0) return MLIP_OK;
  AdamwConsts k;
  k.b1 = h->beta1;
  k.b2 = h->beta2;
  k.one_minus_b1 = (float)(1.0 - (double)h->beta1);
  k.one_minus_b2 = (float)(1.0 - (double)h->beta2);
  k.c1 = (float)(1.0 / (1.0 - std::pow((double)h->beta1, (double)step)));
  k.c2 = (float)(1.0 / (1.0 - std::pow((double)h->beta2, (double)step)));
  k.lr = h->lr;
  k.eps = h->eps;
  k.wd = h->weight_decay;
  k.gscale = h->grad_scale;
  const uintptr_t bits = (uintptr_t)params | (uintptr_t)grad | (uintptr_t)m | (uintptr_t)v;
  if ((bits & 15) == 0) {
    const int64_t threads = std::max<int64_t>(n >> 2, 3);
    hipLaunchKernelGGL(k_adamw<4>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, ctx->stream, params, grad, m, v, n, k);
  } else {
    hipLaunchKernelGGL(k_adamw<1>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, ctx->stream, params, grad, m, v, n, k);
  }
  MLIP_HIP_CHECK(ctx, hipGetLastError());
  return MLIP_OK;
}
