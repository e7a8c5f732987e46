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

// bf16 rows up to NT*8*J columns: the whole row stays in registers (16-byte vectors strided
// over the NT threads of the workgroup), so the logits tile is read once and written once.
// The exponentials go straight to the hardware instruction: every argument is <= 0 up to
// rounding, and a result below 2^-126 may flush to zero.
// F16IN: the logits are IEEE half (the logits GEMM's fp32 accumulators rounded to 11 significant bits instead
// of bfloat16's 8: the softmax takes exp of them, so their absolute error is the relative error of every
// probability); the dlogits written back over them are bf16, the operand type of the GEMMs that follow.
template <int J, int NT, bool F16IN>
__global__ __launch_bounds__(NT) void xent_rows_reg_kernel(bf16_t *z, const int32_t *__restrict__ targets, int V,
                                                            float inv_n, float *__restrict__ rowloss) {
  auto cvt = [](uint32_t h) { return F16IN ? f16_to_f32((uint16_t)h) : bf16_to_f32((bf16_t)h); };
  constexpr int NW = NT / 64;
  __shared__ float red[NW];
  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  bf16_t *zr = z + (size_t)row * V;
  const int nvec = V >> 3;
  const int tgt = targets[row];
  if (tgt < 0 || tgt >= V) {  // ignored position (uniform over the workgroup): zero loss, zero gradient
    if (tid == 0) rowloss[row] = 0.f;
    for (int v = tid; v < nvec; v += NT) *reinterpret_cast<uint4 *>(zr + v * 8) = uint4{0u, 0u, 0u, 0u};
    return;
  }
  const float ztgt = cvt(zr[tgt]);  // read before any thread overwrites the row (barriers below)
  uint4 q[J];
  float mx = -INFINITY;
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int v = tid + NT * j;
    if (v < nvec) {
      q[j] = *reinterpret_cast<const uint4 *>(zr + v * 8);
      const uint32_t u[4] = {q[j].x, q[j].y, q[j].z, q[j].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        mx = fmaxf(mx, cvt(u[e] & 0xFFFF));
        mx = fmaxf(mx, cvt(u[e] >> 16));
      }
    }
  }
  mx = wave_max(mx);
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  mx = red[0];
#pragma unroll
  for (int i = 1; i < NW; ++i) mx = fmaxf(mx, red[i]);
  __syncthreads();
  const float mx2 = mx * 1.4426950408889634f;
  float se = 0.f;
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int v = tid + NT * j;
    if (v < nvec) {
      const uint32_t u[4] = {q[j].x, q[j].y, q[j].z, q[j].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        se += __builtin_amdgcn_exp2f(cvt(u[e] & 0xFFFF) * 1.4426950408889634f - mx2);
        se += __builtin_amdgcn_exp2f(cvt(u[e] >> 16) * 1.4426950408889634f - mx2);
      }
    }
  }
  se = wave_sum(se);
  if (lane == 0) red[wave] = se;
  __syncthreads();
  se = 0.f;
#pragma unroll
  for (int i = 0; i < NW; i += 4) se += (red[i] + red[i + 1]) + (red[i + 2] + red[i + 3]);
  const float lse = mx + __logf(se);
  const float lse2 = lse * 1.4426950408889634f;
  if (tid == 0) rowloss[row] = lse - ztgt;
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int v = tid + NT * j;
    if (v < nvec) {
      const uint32_t u[4] = {q[j].x, q[j].y, q[j].z, q[j].w};
      float p[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        p[2 * e] = __builtin_amdgcn_exp2f(cvt(u[e] & 0xFFFF) * 1.4426950408889634f - lse2);
        p[2 * e + 1] = __builtin_amdgcn_exp2f(cvt(u[e] >> 16) * 1.4426950408889634f - lse2);
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

hipError_t xent_rows(int dtype, void *z, const int32_t *targets, int rows, int V, float inv_n, float *rowloss,
                     hipStream_t s, int z_is_f16) {
  if (rows <= 0) return hipSuccess;
  const bool reg = (V & 7) == 0 && V <= 1024 * 8 * 8;
  if (z_is_f16 && (dtype == 0 || !reg)) return hipErrorInvalidValue;  // half logits: only the in-register kernels
  if (dtype == 0)
    hipLaunchKernelGGL(xent_rows_kernel<float>, dim3(rows), dim3(256), 0, s, (float *)z, targets, V, inv_n,
                       rowloss);
  else if (reg && V <= 512 * 8 * 8) {
    if (z_is_f16)
      hipLaunchKernelGGL((xent_rows_reg_kernel<8, 512, true>), dim3(rows), dim3(512), 0, s, (bf16_t *)z, targets, V,
                         inv_n, rowloss);
    else
      hipLaunchKernelGGL((xent_rows_reg_kernel<8, 512, false>), dim3(rows), dim3(512), 0, s, (bf16_t *)z, targets, V,
                         inv_n, rowloss);
  } else if (reg) {  // wider rows: twice the threads rather than twice the registers
    if (z_is_f16)
      hipLaunchKernelGGL((xent_rows_reg_kernel<8, 1024, true>), dim3(rows), dim3(1024), 0, s, (bf16_t *)z, targets, V,
                         inv_n, rowloss);
    else
      hipLaunchKernelGGL((xent_rows_reg_kernel<8, 1024, false>), dim3(rows), dim3(1024), 0, s, (bf16_t *)z, targets, V,
                         inv_n, rowloss);
  } else
    hipLaunchKernelGGL(xent_rows_kernel<bf16_t>, dim3(rows), dim3(256), 0, s, (bf16_t *)z, targets, V, inv_n,
                       rowloss);
  return hipGetLastError();
}

}  // namespace il
