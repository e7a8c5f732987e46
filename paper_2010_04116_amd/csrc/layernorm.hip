// LayerNorm forward and backward for the pre-LN block.  One 64-lane wavefront owns a
// row; row reductions are wavefront shuffles (no LDS), statistics are fp32.  The
// backward is fused with the residual-gradient add (the gradient stream G is updated in
// place) and with the first stage of the gamma/beta column reductions.
#include "common.h"

namespace il {
namespace {

constexpr int kWaves = 4;         // rows in flight per 256-thread block
constexpr int kMaxJ = 32;         // lane owns columns lane + 64*j, j < kMaxJ  (d <= 2048)
constexpr int kLnBwdBlocks = 1024;

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

template <typename T>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const float *__restrict__ x, const T *__restrict__ gamma,
                                                     const T *__restrict__ beta, float eps, int rows, int d,
                                                     T *__restrict__ y, float *__restrict__ stats,
                                                     float *__restrict__ xcopy) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = blockIdx.x * kWaves + wave;
  if (row >= rows) return;
  const float *xr = x + (size_t)row * d;
  float v[kMaxJ];
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < kMaxJ; ++j) {
    int c = lane + 64 * j;
    v[j] = (c < d) ? xr[c] : 0.f;
    s += v[j];
  }
  const float mean = wave_sum(s) / d;
  float q = 0.f;
#pragma unroll
  for (int j = 0; j < kMaxJ; ++j) {
    int c = lane + 64 * j;
    float t = (c < d) ? v[j] - mean : 0.f;
    q += t * t;
  }
  const float rstd = rsqrtf(wave_sum(q) / d + eps);
#pragma unroll
  for (int j = 0; j < kMaxJ; ++j) {
    int c = lane + 64 * j;
    if (c < d) {
      st<T>(y + (size_t)row * d + c, (v[j] - mean) * rstd * ld<T>(gamma + c) + ld<T>(beta + c));
      if (xcopy) xcopy[(size_t)row * d + c] = v[j];
    }
  }
  if (lane == 0) {
    stats[2 * row] = mean;
    stats[2 * row + 1] = rstd;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void ln_bwd_kernel(const T *__restrict__ dy, const float *__restrict__ x,
                                                     const float *__restrict__ stats,
                                                     const T *__restrict__ gamma, int rows, int N, int d,
                                                     float *G, T *Gb,
                                                     StreamWeights sw, float *__restrict__ partials) {
  __shared__ float red[kWaves][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float dg[kMaxJ], db[kMaxJ], gm[kMaxJ];
#pragma unroll
  for (int j = 0; j < kMaxJ; ++j) {
    int c = lane + 64 * j;
    dg[j] = 0.f;
    db[j] = 0.f;
    gm[j] = (c < d) ? ld<T>(gamma + c) : 0.f;
  }
  for (int row = blockIdx.x * kWaves + wave; row < rows; row += gridDim.x * kWaves) {
    const int tok = row % N;
    const float w = sw.w[row / N];
    const float mean = stats[2 * tok], rstd = stats[2 * tok + 1];
    const float *xr = x + (size_t)tok * d;
    const T *dyr = dy + (size_t)row * d;
    float xh[kMaxJ], dxh[kMaxJ];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int j = 0; j < kMaxJ; ++j) {
      int c = lane + 64 * j;
      if (c < d) {
        float dyv = ld<T>(dyr + c);
        xh[j] = (xr[c] - mean) * rstd;
        dxh[j] = dyv * gm[j];
        s1 += dxh[j];
        s2 += dxh[j] * xh[j];
        dg[j] += w * dyv * xh[j];
        db[j] += w * dyv;
      } else {
        xh[j] = 0.f;
        dxh[j] = 0.f;
      }
    }
    const float m1 = wave_sum(s1) / d, m2 = wave_sum(s2) / d;
    float *gr = G + (size_t)row * d;
    T *gbr = Gb + (size_t)row * d;
#pragma unroll
    for (int j = 0; j < kMaxJ; ++j) {
      int c = lane + 64 * j;
      if (c < d) {
        float v = gr[c] + rstd * (dxh[j] - m1 - xh[j] * m2);
        gr[c] = v;
        st<T>(gbr + c, v);
      }
    }
  }
  // block-level column sums: waves 1..3 hand their registers to wave 0 through LDS
  float *pg = partials + (size_t)blockIdx.x * 2 * d;
#pragma unroll
  for (int j = 0; j < kMaxJ; ++j) {
    if (64 * j >= d) continue;  // uniform across the block
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      __syncthreads();
      red[wave][lane] = pass ? db[j] : dg[j];
      __syncthreads();
      if (wave == 0) {
        int c = lane + 64 * j;
        float v = red[0][lane] + red[1][lane] + red[2][lane] + red[3][lane];
        if (c < d) pg[pass * d + c] = v;
      }
    }
  }
}

}  // namespace

int ln_backward_max_blocks() { return kLnBwdBlocks; }

hipError_t ln_forward(int dtype, const float *x, const void *gamma, const void *beta, float eps, int rows,
                      int d, void *y, float *stats, float *xcopy, hipStream_t s) {
  dim3 grid((rows + kWaves - 1) / kWaves);
  if (dtype == 0)
    hipLaunchKernelGGL(ln_fwd_kernel<float>, grid, dim3(256), 0, s, x, (const float *)gamma,
                       (const float *)beta, eps, rows, d, (float *)y, stats, xcopy);
  else
    hipLaunchKernelGGL(ln_fwd_kernel<bf16_t>, grid, dim3(256), 0, s, x, (const bf16_t *)gamma,
                       (const bf16_t *)beta, eps, rows, d, (bf16_t *)y, stats, xcopy);
  return hipGetLastError();
}

hipError_t ln_backward_residual(int dtype, const void *dy, const float *x, const float *stats,
                                const void *gamma, int rows, int N, int d, float *G, void *Gb,
                                StreamWeights sw, float *partials, int *nblk, hipStream_t s) {
  int blocks = (rows + kWaves - 1) / kWaves;
  if (blocks > kLnBwdBlocks) blocks = kLnBwdBlocks;
  *nblk = blocks;
  if (dtype == 0)
    hipLaunchKernelGGL(ln_bwd_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float *)dy, x, stats,
                       (const float *)gamma, rows, N, d, G, (float *)Gb, sw, partials);
  else
    hipLaunchKernelGGL(ln_bwd_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, (const bf16_t *)dy, x, stats,
                       (const bf16_t *)gamma, rows, N, d, G, (bf16_t *)Gb, sw, partials);
  return hipGetLastError();
}

}  // namespace il
