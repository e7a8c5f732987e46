// Causal attention without matrix cores: the true-fp32 path (IL_F32) and head widths
// the MFMA kernels do not cover.  One thread per query row (forward, dQ) or per key row
// (dK, dV); online softmax in fp32; probabilities are recomputed from the saved
// log-sum-exp in the backward.
#include "common.h"

namespace il {
namespace {

// grid (ceil(T/64), B*H); thread = query position t
template <typename T, int DH>
__global__ __launch_bounds__(64) void attn_fwd_simt(const T *__restrict__ qkv, int Tn, int H,
                                                    T *__restrict__ o, float *__restrict__ lse) {
  const int t = blockIdx.x * 64 + threadIdx.x;
  const int b = blockIdx.y / H, h = blockIdx.y % H;
  if (t >= Tn) return;
  const int d = H * DH;
  const size_t ld3 = 3 * (size_t)d;
  const T *qp = qkv + ((size_t)b * Tn + t) * ld3 + h * DH;
  const float scale = rsqrtf((float)DH);
  float q[DH], acc[DH];
#pragma unroll
  for (int i = 0; i < DH; ++i) { q[i] = ld<T>(qp + i) * scale; acc[i] = 0.f; }
  float m = -INFINITY, l = 0.f;
  for (int u = 0; u <= t; ++u) {
    const T *kp = qkv + ((size_t)b * Tn + u) * ld3 + d + h * DH;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < DH; ++i) s = fmaf(q[i], ld<T>(kp + i), s);
    float mn = fmaxf(m, s);
    float c = __expf(m - mn), p = __expf(s - mn);
    l = l * c + p;
    const T *vp = kp + d;
#pragma unroll
    for (int i = 0; i < DH; ++i) acc[i] = acc[i] * c + p * ld<T>(vp + i);
    m = mn;
  }
  const float inv = 1.f / l;
  T *op = o + ((size_t)b * Tn + t) * d + h * DH;
#pragma unroll
  for (int i = 0; i < DH; ++i) st<T>(op + i, acc[i] * inv);
  lse[((size_t)b * H + h) * Tn + t] = m + __logf(l);
}

// dsum[s][b][h][t] = sum_i dO*O ; grid (ceil(T/64), B*H, nstreams)
template <typename T, int DH>
__global__ __launch_bounds__(64) void attn_dsum_simt(const T *__restrict__ o, const T *__restrict__ d_o, int Tn,
                                                     int H, int B, float *__restrict__ dsum) {
  const int t = blockIdx.x * 64 + threadIdx.x;
  const int b = blockIdx.y / H, h = blockIdx.y % H, sidx = blockIdx.z;
  if (t >= Tn) return;
  const int d = H * DH;
  const size_t N = (size_t)B * Tn;
  const T *op = o + ((size_t)b * Tn + t) * d + h * DH;
  const T *dp = d_o + (sidx * N + (size_t)b * Tn + t) * d + h * DH;
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < DH; ++i) s = fmaf(ld<T>(op + i), ld<T>(dp + i), s);
  dsum[(sidx * (size_t)B * H + blockIdx.y) * Tn + t] = s;
}

// dQ: thread = query row; grid (ceil(T/64), B*H, nstreams)
template <typename T, int DH>
__global__ __launch_bounds__(64) void attn_dq_simt(const T *__restrict__ qkv, const T *__restrict__ d_o,
                                                   const float *__restrict__ lse, const float *__restrict__ dsum,
                                                   int Tn, int H, int B, T *__restrict__ dqkv) {
  const int t = blockIdx.x * 64 + threadIdx.x;
  const int b = blockIdx.y / H, h = blockIdx.y % H, sidx = blockIdx.z;
  if (t >= Tn) return;
  const int d = H * DH;
  const size_t ld3 = 3 * (size_t)d, N = (size_t)B * Tn;
  const float scale = rsqrtf((float)DH);
  const T *qp = qkv + ((size_t)b * Tn + t) * ld3 + h * DH;
  const T *dop = d_o + (sidx * N + (size_t)b * Tn + t) * d + h * DH;
  float q[DH], g[DH], dq[DH];
#pragma unroll
  for (int i = 0; i < DH; ++i) { q[i] = ld<T>(qp + i) * scale; g[i] = ld<T>(dop + i); dq[i] = 0.f; }
  const float L = lse[((size_t)b * H + h) * Tn + t];
  const float D = dsum[(sidx * (size_t)B * H + blockIdx.y) * Tn + t];
  for (int u = 0; u <= t; ++u) {
    const T *kp = qkv + ((size_t)b * Tn + u) * ld3 + d + h * DH;
    const T *vp = kp + d;
    float s = 0.f, dp = 0.f;
#pragma unroll
    for (int i = 0; i < DH; ++i) { s = fmaf(q[i], ld<T>(kp + i), s); dp = fmaf(g[i], ld<T>(vp + i), dp); }
    float ds = __expf(s - L) * (dp - D);
#pragma unroll
    for (int i = 0; i < DH; ++i) dq[i] = fmaf(ds, ld<T>(kp + i), dq[i]);
  }
  T *out = dqkv + (sidx * N + (size_t)b * Tn + t) * ld3 + h * DH;
#pragma unroll
  for (int i = 0; i < DH; ++i) st<T>(out + i, dq[i] * scale);
}

// dK, dV: thread = key row u, loops over queries t >= u
template <typename T, int DH>
__global__ __launch_bounds__(64) void attn_dkv_simt(const T *__restrict__ qkv, const T *__restrict__ d_o,
                                                    const float *__restrict__ lse, const float *__restrict__ dsum,
                                                    int Tn, int H, int B, T *__restrict__ dqkv) {
  const int u = blockIdx.x * 64 + threadIdx.x;
  const int b = blockIdx.y / H, h = blockIdx.y % H, sidx = blockIdx.z;
  if (u >= Tn) return;
  const int d = H * DH;
  const size_t ld3 = 3 * (size_t)d, N = (size_t)B * Tn;
  const float scale = rsqrtf((float)DH);
  const T *kp = qkv + ((size_t)b * Tn + u) * ld3 + d + h * DH;
  float k[DH], v[DH], dk[DH], dv[DH];
#pragma unroll
  for (int i = 0; i < DH; ++i) { k[i] = ld<T>(kp + i); v[i] = ld<T>(kp + d + i); dk[i] = 0.f; dv[i] = 0.f; }
  for (int t = u; t < Tn; ++t) {
    const T *qp = qkv + ((size_t)b * Tn + t) * ld3 + h * DH;
    const T *dop = d_o + (sidx * N + (size_t)b * Tn + t) * d + h * DH;
    float s = 0.f, dp = 0.f;
#pragma unroll
    for (int i = 0; i < DH; ++i) { s = fmaf(ld<T>(qp + i), k[i], s); dp = fmaf(ld<T>(dop + i), v[i], dp); }
    const float p = __expf(s * scale - lse[((size_t)b * H + h) * Tn + t]);
    const float ds = p * (dp - dsum[(sidx * (size_t)B * H + blockIdx.y) * Tn + t]) * scale;
#pragma unroll
    for (int i = 0; i < DH; ++i) { dv[i] = fmaf(p, ld<T>(dop + i), dv[i]); dk[i] = fmaf(ds, ld<T>(qp + i), dk[i]); }
  }
  T *out = dqkv + (sidx * N + (size_t)b * Tn + u) * ld3 + d + h * DH;
#pragma unroll
  for (int i = 0; i < DH; ++i) { st<T>(out + i, dk[i]); st<T>(out + d + i, dv[i]); }
}

template <typename T, int DH>
hipError_t fwd_t(const void *qkv, int B, int Tn, int H, void *o, float *lse, hipStream_t s) {
  hipLaunchKernelGGL((attn_fwd_simt<T, DH>), dim3((Tn + 63) / 64, B * H), dim3(64), 0, s, (const T *)qkv, Tn, H,
                     (T *)o, lse);
  return hipGetLastError();
}
template <typename T, int DH>
hipError_t bwd_t(const void *qkv, const void *o, const void *d_o, const float *lse, int ns, int B, int Tn, int H,
                 void *dqkv, float *dsum, hipStream_t s) {
  dim3 grid((Tn + 63) / 64, B * H, ns);
  hipLaunchKernelGGL((attn_dsum_simt<T, DH>), grid, dim3(64), 0, s, (const T *)o, (const T *)d_o, Tn, H, B, dsum);
  hipLaunchKernelGGL((attn_dq_simt<T, DH>), grid, dim3(64), 0, s, (const T *)qkv, (const T *)d_o, lse, dsum, Tn,
                     H, B, (T *)dqkv);
  hipLaunchKernelGGL((attn_dkv_simt<T, DH>), grid, dim3(64), 0, s, (const T *)qkv, (const T *)d_o, lse, dsum, Tn,
                     H, B, (T *)dqkv);
  return hipGetLastError();
}

}  // namespace

#define IL_DISPATCH_DH(CALL)            \
  switch (dh) {                         \
    case 16: return CALL(16);           \
    case 32: return CALL(32);           \
    case 64: return CALL(64);           \
    case 128: return CALL(128);         \
    default: return hipErrorInvalidValue; \
  }

hipError_t attention_forward_simt(int dtype, const void *qkv, int B, int T, int H, int dh, void *o, float *lse,
                                  hipStream_t s) {
#define F32(D) fwd_t<float, D>(qkv, B, T, H, o, lse, s)
#define B16(D) fwd_t<bf16_t, D>(qkv, B, T, H, o, lse, s)
  if (dtype == 0) { IL_DISPATCH_DH(F32) } else { IL_DISPATCH_DH(B16) }
#undef F32
#undef B16
}

hipError_t attention_backward_simt(int dtype, const void *qkv, const void *o, const void *d_o, const float *lse,
                                   int ns, int B, int T, int H, int dh, void *dqkv, float *dsum, hipStream_t s) {
#define F32(D) bwd_t<float, D>(qkv, o, d_o, lse, ns, B, T, H, dqkv, dsum, s)
#define B16(D) bwd_t<bf16_t, D>(qkv, o, d_o, lse, ns, B, T, H, dqkv, dsum, s)
  if (dtype == 0) { IL_DISPATCH_DH(F32) } else { IL_DISPATCH_DH(B16) }
#undef F32
#undef B16
}

hipError_t attention_forward_mfma(const void *qkv, int B, int T, int H, int dh, void *o, float *lse,
                                  hipStream_t s);

hipError_t attention_backward_mfma(const void *qkv, const void *o, const void *d_o, const float *lse, int ns,
                                   int B, int T, int H, int dh, void *dqkv, float *dsum, hipStream_t s);

// Front ends used by the step: bf16 with head width 64 or 128 runs on the matrix cores,
// everything else (fp32; bf16 with head width 16 or 32) on the kernels above.
hipError_t attention_forward(int dtype, const void *qkv, int B, int T, int H, int dh, void *o, float *lse,
                             hipStream_t s) {
  if (dtype == 1 && (dh == 64 || dh == 128 || dh == 256)) return attention_forward_mfma(qkv, B, T, H, dh, o, lse, s);
  return attention_forward_simt(dtype, qkv, B, T, H, dh, o, lse, s);
}
hipError_t attention_backward(int dtype, const void *qkv, const void *o, const void *d_o, const float *lse,
                              int ns, int B, int T, int H, int dh, void *dqkv, float *dsum, hipStream_t s) {
  if (dtype == 1 && (dh == 64 || dh == 128 || dh == 256))
    return attention_backward_mfma(qkv, o, d_o, lse, ns, B, T, H, dh, dqkv, dsum, s);
  return attention_backward_simt(dtype, qkv, o, d_o, lse, ns, B, T, H, dh, dqkv, dsum, s);
}

}  // namespace il
