// Softmax cross-entropy over one tile of logits rows, in place: the row's loss and
// dlogits = (softmax - onehot)/N replace the logits, so probabilities never exist
// outside the [head_chunk, V] tile the head GEMMs work on.  One 256-thread block per
// row; max / sum-exp reductions by wavefront shuffles then LDS across the 4 waves.
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
  if (threadIdx.x == 0) rowloss[row] = lse - ld<T>(zr + tgt);
  __syncthreads();  // the target logit is read before anyone overwrites it
  for (int c = threadIdx.x; c < V; c += 256) {
    float p = __expf(ld<T>(zr + c) - lse);
    st<T>(zr + c, (p - (c == tgt ? 1.f : 0.f)) * inv_n);
  }
}

}  // namespace

hipError_t xent_rows(int dtype, void *z, const int32_t *targets, int rows, int V, float inv_n, float *rowloss,
                     hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (dtype == 0)
    hipLaunchKernelGGL(xent_rows_kernel<float>, dim3(rows), dim3(256), 0, s, (float *)z, targets, V, inv_n,
                       rowloss);
  else
    hipLaunchKernelGGL(xent_rows_kernel<bf16_t>, dim3(rows), dim3(256), 0, s, (bf16_t *)z, targets, V, inv_n,
                       rowloss);
  return hipGetLastError();
}

}  // namespace il
