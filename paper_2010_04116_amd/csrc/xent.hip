// Softmax cross-entropy over one tile of logits rows, in place: the row's loss and
// dlogits = (softmax - onehot)/N replace the logits, so probabilities never exist
// outside the [head_chunk, V] tile the head GEMMs work on.  One 256-thread block per
// row.  fp32: max / sum-exp reductions over the row by wavefront shuffles then LDS across
// the 4 waves.  bf16: the row statistics arrive with the tile, taken from the logits
// GEMM's fp32 accumulators group by group; the kernel merges them and makes one pass.
#include "common.h"

namespace il {
namespace {

__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

template <typename T>
__global__ __launch_bounds__(256) void xent_rows_kernel(T *z, const int32_t *__restrict__ targets, int V,
                                                        float inv_n, float *__restrict__ rowloss) {
  __shared__ float red[4];
  const int row = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  T *zr = z + (size_t)row * V;
  float mx = -INFINITY;
  for (int c = threadIdx.x; c < V; c += 256) mx = fmaxf(mx, ld<T>(zr + c));
  mx = wave_max(mx);
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float se = 0.f;
  for (int c = threadIdx.x; c < V; c += 256) se += __expf(ld<T>(zr + c) - mx);
  se = wave_sum(se);
  if (lane == 0) red[wave] = se;
  __syncthreads();
  se = (red[0] + red[1]) + (red[2] + red[3]);
  const float lse = mx + __logf(se);
  const int tgt = targets[row];
  if (tgt < 0 || tgt >= V) {  // ignored position: no loss, no gradient, nothing read out of bounds
    if (threadIdx.x == 0) rowloss[row] = 0.f;
    for (int c = threadIdx.x; c < V; c += 256) st<T>(zr + c, 0.f);
    return;
  }
  if (threadIdx.x == 0) rowloss[row] = lse - ld<T>(zr + tgt);
  __syncthreads();  // the target logit is read before anyone overwrites it
  for (int c = threadIdx.x; c < V; c += 256) {
    float p = __expf(ld<T>(zr + c) - lse);
    st<T>(zr + c, (p - (c == tgt ? 1.f : 0.f)) * inv_n);
  }
}

// One pass over a tile of half logits whose per-group statistics came with it from the logits GEMM:
// 256 threads per row merge the (max, sum-exp) pairs of the row's 64-column groups into its
// log-sum-exp, then stream the row once: dz = (exp(z - lse) - onehot) * inv_n, written back as bf16.
__global__ __launch_bounds__(256) void xent_from_stats_kernel(bf16_t *z, const float *__restrict__ stats,
                                                              const float *__restrict__ ztgt,
                                                              const int32_t *__restrict__ targets, int V, int ngrp,
                                                              float inv_n, float *__restrict__ rowloss) {
  __shared__ float red[4];
  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  bf16_t *zr = z + (size_t)row * V;
  const int nvec = V >> 3;
  const int tgt = targets[row];
  if (tgt < 0 || tgt >= V) {  // ignored position (uniform over the workgroup): zero loss, zero gradient
    if (tid == 0) rowloss[row] = 0.f;
    for (int v = tid; v < nvec; v += 256) *reinterpret_cast<uint4 *>(zr + v * 8) = uint4{0u, 0u, 0u, 0u};
    return;
  }
  const float2 *sr = reinterpret_cast<const float2 *>(stats) + (size_t)row * ngrp;
  float mx = -INFINITY;
  for (int i = tid; i < ngrp; i += 256) mx = fmaxf(mx, sr[i].x);
  mx = wave_max(mx);
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float se = 0.f;
  for (int i = tid; i < ngrp; i += 256) {
    const float2 p = sr[i];
    se += p.y * __builtin_amdgcn_exp2f((p.x - mx) * 1.4426950408889634f);
  }
  se = wave_sum(se);
  if (lane == 0) red[wave] = se;
  __syncthreads();
  se = (red[0] + red[1]) + (red[2] + red[3]);
  const float lse = mx + __logf(se);
  const float lse2 = lse * 1.4426950408889634f;
  if (tid == 0) rowloss[row] = lse - ztgt[row];
  constexpr int U = 4;  // 16-byte vectors in flight per thread
  for (int v0 = tid; v0 < nvec; v0 += 256 * U) {
    uint4 q[U];
#pragma unroll
    for (int k = 0; k < U; ++k)
      if (v0 + 256 * k < nvec) q[k] = *reinterpret_cast<const uint4 *>(zr + (v0 + 256 * k) * 8);
#pragma unroll
    for (int k = 0; k < U; ++k) {
      const int v = v0 + 256 * k;
      if (v >= nvec) break;
      const uint32_t u[4] = {q[k].x, q[k].y, q[k].z, q[k].w};
      float p[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        p[2 * e] = __builtin_amdgcn_exp2f(f16_to_f32((uint16_t)(u[e] & 0xFFFF)) * 1.4426950408889634f - lse2);
        p[2 * e + 1] = __builtin_amdgcn_exp2f(f16_to_f32((uint16_t)(u[e] >> 16)) * 1.4426950408889634f - lse2);
      }
      const int c0 = v * 8;
      if (tgt >= c0 && tgt < c0 + 8) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (c0 + e == tgt) p[e] -= 1.f;
      }
      uint4 o;
      o.x = pack_bf16x2(p[0] * inv_n, p[1] * inv_n);
      o.y = pack_bf16x2(p[2] * inv_n, p[3] * inv_n);
      o.z = pack_bf16x2(p[4] * inv_n, p[5] * inv_n);
      o.w = pack_bf16x2(p[6] * inv_n, p[7] * inv_n);
      *reinterpret_cast<uint4 *>(zr + c0) = o;
    }
  }
}

}  // namespace

hipError_t xent_rows_from_stats(void *z, const float *stats, const float *ztgt, const int32_t *targets, int rows,
                                int V, float inv_n, float *rowloss, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if ((V & 7) || !stats || !ztgt) return hipErrorInvalidValue;
  hipLaunchKernelGGL(xent_from_stats_kernel, dim3(rows), dim3(256), 0, s, (bf16_t *)z, stats, ztgt, targets, V,
                     (V + kStatGroup - 1) / kStatGroup, inv_n, rowloss);
  return hipGetLastError();
}

hipError_t xent_rows(int dtype, void *z, const int32_t *targets, int rows, int V, float inv_n, float *rowloss,
                     hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (dtype != 0) return hipErrorInvalidValue;  // bf16 runs take xent_rows_from_stats
  hipLaunchKernelGGL(xent_rows_kernel<float>, dim3(rows), dim3(256), 0, s, (float *)z, targets, V, inv_n, rowloss);
  return hipGetLastError();
}

}  // namespace il
