// Optimiser step of the paper's Transformer runs (App. B, training configuration): Adam with bias
// correction, one fused pass over the flat parameter buffer.
//
//   m <- b1 m + (1-b1) g     v <- b2 v + (1-b2) g^2
//   w <- w - lr * (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps)
//
// HBM-bound: per parameter it reads g, m, v, w (16 B) and writes m, v, w (12 B), plus 2 B for the
// bf16 image of w in bf16 mode.  Four parameters per thread per pass (16-byte accesses), grid-stride.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "../../include/interlock.h"
#include "common.h"

namespace il {
namespace {

struct AdamScalars { float b1, b2, omb1, omb2, c1, c2, lr, eps; };

__device__ inline float adam_one(float g, float &m, float &v, float w, const AdamScalars &a) {
  m = a.b1 * m + a.omb1 * g;
  v = a.b2 * v + a.omb2 * g * g;
  return w - a.lr * (m * a.c1) / (sqrtf(v * a.c2) + a.eps);
}

// BF: also write the bf16 image of the updated fp32 weights.  Buffers are 16-byte aligned
// (8-byte for the bf16 image); the tail (< 4 elements) is handled by the last thread, element-wise.
template <bool BF>
__global__ __launch_bounds__(256) void adam_step_kernel(float *__restrict__ w, bf16_t *__restrict__ p,
                                                        const float *__restrict__ g, float *__restrict__ m,
                                                        float *__restrict__ v, size_t count, AdamScalars a) {
  const size_t n4 = count >> 2;
  const size_t stride = (size_t)gridDim.x * 256;
  // two independent 16-byte groups per thread and pass: more loads in flight per wavefront
  for (size_t i0 = (size_t)blockIdx.x * 256 + threadIdx.x; i0 < n4; i0 += 2 * stride) {
    const size_t i1 = i0 + stride;
    const bool two = i1 < n4;
    const float4 g0 = reinterpret_cast<const float4 *>(g)[i0];
    float4 m0 = reinterpret_cast<float4 *>(m)[i0], v0 = reinterpret_cast<float4 *>(v)[i0];
    float4 w0 = reinterpret_cast<float4 *>(w)[i0];
    float4 g1 = g0, m1 = m0, v1 = v0, w1 = w0;
    if (two) {
      g1 = reinterpret_cast<const float4 *>(g)[i1];
      m1 = reinterpret_cast<float4 *>(m)[i1];
      v1 = reinterpret_cast<float4 *>(v)[i1];
      w1 = reinterpret_cast<float4 *>(w)[i1];
    }
    auto update = [&](const float4 &gg, float4 &mm, float4 &vv, float4 &ww, size_t i) {
      ww.x = adam_one(gg.x, mm.x, vv.x, ww.x, a);
      ww.y = adam_one(gg.y, mm.y, vv.y, ww.y, a);
      ww.z = adam_one(gg.z, mm.z, vv.z, ww.z, a);
      ww.w = adam_one(gg.w, mm.w, vv.w, ww.w, a);
      reinterpret_cast<float4 *>(m)[i] = mm;
      reinterpret_cast<float4 *>(v)[i] = vv;
      reinterpret_cast<float4 *>(w)[i] = ww;
      if constexpr (BF) {
        uint2 q;
        q.x = pack_bf16x2(ww.x, ww.y);
        q.y = pack_bf16x2(ww.z, ww.w);
        reinterpret_cast<uint2 *>(p)[i] = q;
      }
    };
    update(g0, m0, v0, w0, i0);
    if (two) update(g1, m1, v1, w1, i1);
  }
  if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 255)
    for (size_t i = n4 << 2; i < count; ++i) {
      float mm = m[i], vv = v[i];
      const float ww = adam_one(g[i], mm, vv, w[i], a);
      m[i] = mm; v[i] = vv; w[i] = ww;
      if constexpr (BF) p[i] = f32_to_bf16(ww);
    }
}

}  // namespace
}  // namespace il

extern "C" {

double il_lr_schedule(int64_t step, int32_t d_model, int32_t warmup_steps) {
  if (step < 1 || d_model < 1 || warmup_steps < 1) return 0.0;
  const double s = (double)step, w = (double)warmup_steps;
  return std::pow((double)d_model, -0.5) * std::fmin(std::pow(s, -0.5), s * std::pow(w, -1.5));
}

int il_adam_step(int32_t dtype, void *params, float *master, const float *grads, float *m, float *v,
                 size_t count, int64_t step, float lr, float beta1, float beta2, float eps, void *stream) {
  using namespace il;
  if (dtype != IL_F32 && dtype != IL_BF16) return IL_E_ARG;
  if (!params || !grads || !m || !v || step < 1) return IL_E_ARG;
  if ((dtype == IL_BF16) != (master != nullptr)) return IL_E_ARG;
  if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f) || !(lr >= 0.f))
    return IL_E_ARG;
  float *w = dtype == IL_BF16 ? master : (float *)params;
  if (((uintptr_t)w | (uintptr_t)grads | (uintptr_t)m | (uintptr_t)v) & 15) return IL_E_SHAPE;
  if (dtype == IL_BF16 && ((uintptr_t)params & 7)) return IL_E_SHAPE;
  if (count == 0) return IL_OK;
  AdamScalars a;
  a.b1 = beta1; a.b2 = beta2; a.omb1 = 1.f - beta1; a.omb2 = 1.f - beta2;
  a.c1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)step)));   // bias corrections in double
  a.c2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)step)));
  a.lr = lr; a.eps = eps;
  size_t blocks = ((count >> 2) + 255) / 256;
  if (blocks < 1) blocks = 1;
  if (blocks > 8192) blocks = 8192;  // 32 workgroups per CU, grid-stride beyond that
  hipStream_t s = (hipStream_t)stream;
  if (dtype == IL_BF16)
    hipLaunchKernelGGL(adam_step_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, w, (bf16_t *)params, grads,
                       m, v, count, a);
  else
    hipLaunchKernelGGL(adam_step_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, w, (bf16_t *)nullptr, grads,
                       m, v, count, a);
  return hipGetLastError() == hipSuccess ? IL_OK : IL_E_HIP;
}

}  // extern "C"
