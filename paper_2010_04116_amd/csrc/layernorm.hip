// LayerNorm forward and backward for the pre-LN block.  One 64-lane wavefront owns a
// row; row reductions are wavefront shuffles (no LDS), statistics are fp32.  The
// backward is fused with the residual-gradient add (the gradient stream G is updated in
// place) and with the first stage of the gamma/beta column reductions.
#include "common.h"

namespace il {
namespace {

constexpr int kWaves = 4;         // rows in flight per 256-thread block
constexpr int kMaxJ = 32;         // lane owns columns lane + 64*j, j < kMaxJ  (d <= 2048)
constexpr int kLnBwdBlocks = 512;

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

// Vector access helpers: V consecutive elements per lane (V = 4 when d % 256 == 0, else 1).
template <typename T, int V> struct Vec;
template <> struct Vec<float, 4> {
  static __device__ inline void load(const float *p, float (&o)[4]) {
    const float4 v = *reinterpret_cast<const float4 *>(p);
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  }
  static __device__ inline void store(float *p, const float (&o)[4]) {
    *reinterpret_cast<float4 *>(p) = make_float4(o[0], o[1], o[2], o[3]);
  }
};
template <> struct Vec<bf16_t, 4> {
  static __device__ inline void load(const bf16_t *p, float (&o)[4]) {
    const uint2 v = *reinterpret_cast<const uint2 *>(p);
    o[0] = bf16_to_f32((bf16_t)(v.x & 0xFFFF)); o[1] = bf16_to_f32((bf16_t)(v.x >> 16));
    o[2] = bf16_to_f32((bf16_t)(v.y & 0xFFFF)); o[3] = bf16_to_f32((bf16_t)(v.y >> 16));
  }
  static __device__ inline void store(bf16_t *p, const float (&o)[4]) {
    uint2 v;
    v.x = pack_bf16x2(o[0], o[1]);
    v.y = pack_bf16x2(o[2], o[3]);
    *reinterpret_cast<uint2 *>(p) = v;
  }
};
template <typename T> struct Vec<T, 1> {
  static __device__ inline void load(const T *p, float (&o)[1]) { o[0] = ld<T>(p); }
  static __device__ inline void store(T *p, const float (&o)[1]) { st<T>(p, o[0]); }
};

// Forward with 16-byte accesses for d = 256 J: a lane owns columns (lane + 64 j) * 4 + (0..3), j < J.
template <typename T, int J>
__global__ __launch_bounds__(256) void ln_fwd_vec_kernel(const float *__restrict__ x, const T *__restrict__ gamma,
                                                         const T *__restrict__ beta, float eps, int rows,
                                                         T *__restrict__ y, float *__restrict__ stats,
                                                         float *__restrict__ xcopy) {
  constexpr int d = 256 * J;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = blockIdx.x * kWaves + wave;
  if (row >= rows) return;
  const float *xr = x + (size_t)row * d;
  float v[J][4];
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < J; ++j) {
    Vec<float, 4>::load(xr + (lane + 64 * j) * 4, v[j]);
    s += (v[j][0] + v[j][1]) + (v[j][2] + v[j][3]);
  }
  const float mean = wave_sum(s) * (1.f / d);
  float q = 0.f;
#pragma unroll
  for (int j = 0; j < J; ++j)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float t = v[j][e] - mean;
      q += t * t;
    }
  const float rstd = rsqrtf(wave_sum(q) * (1.f / d) + eps);
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int c = (lane + 64 * j) * 4;
    float g[4], b[4], o[4];
    Vec<T, 4>::load(gamma + c, g);
    Vec<T, 4>::load(beta + c, b);
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (v[j][e] - mean) * rstd * g[e] + b[e];
    Vec<T, 4>::store(y + (size_t)row * d + c, o);
    if (xcopy) Vec<float, 4>::store(xcopy + (size_t)row * d + c, v[j]);
  }
  if (lane == 0) {
    stats[2 * row] = mean;
    stats[2 * row + 1] = rstd;
  }
}

// Lane owns columns (lane + 64 j) * V + (0..V-1), j < J.
template <typename T, int V, int J>
__global__ __launch_bounds__(256) void ln_bwd_kernel(const T *__restrict__ dy, const float *__restrict__ x,
                                                     const float *__restrict__ stats,
                                                     const T *__restrict__ gamma, int rows, int N, int d,
                                                     float *G, T *Gb, StreamWeights sw,
                                                     float *__restrict__ partials) {
  __shared__ float red[kWaves][64 * V];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float dg[J][V], db[J][V], gm[J][V];
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int c = (lane + 64 * j) * V;
#pragma unroll
    for (int e = 0; e < V; ++e) { dg[j][e] = 0.f; db[j][e] = 0.f; gm[j][e] = 0.f; }
    if (c < d) Vec<T, V>::load(gamma + c, gm[j]);
  }
  const float invd = 1.f / d;
  for (int row = blockIdx.x * kWaves + wave; row < rows; row += gridDim.x * kWaves) {
    const int tok = row % N;
    const float w = sw.w[row / N];
    const float mean = stats[2 * tok], rstd = stats[2 * tok + 1];
    const float *xr = x + (size_t)tok * d;
    const T *dyr = dy + (size_t)row * d;
    float *gr = G + (size_t)row * d;
    T *gbr = Gb + (size_t)row * d;
    float xh[J][V], dxh[J][V], gv[J][V];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int j = 0; j < J; ++j) {
      const int c = (lane + 64 * j) * V;
      if (c < d) {
        float dyv[V];
        Vec<T, V>::load(dyr + c, dyv);
        Vec<float, V>::load(xr + c, xh[j]);
        Vec<float, V>::load(gr + c, gv[j]);
#pragma unroll
        for (int e = 0; e < V; ++e) {
          xh[j][e] = (xh[j][e] - mean) * rstd;
          dxh[j][e] = dyv[e] * gm[j][e];
          s1 += dxh[j][e];
          s2 += dxh[j][e] * xh[j][e];
          dg[j][e] += w * dyv[e] * xh[j][e];
          db[j][e] += w * dyv[e];
        }
      } else {
#pragma unroll
        for (int e = 0; e < V; ++e) { xh[j][e] = 0.f; dxh[j][e] = 0.f; gv[j][e] = 0.f; }
      }
    }
    const float m1 = wave_sum(s1) * invd, m2 = wave_sum(s2) * invd;
#pragma unroll
    for (int j = 0; j < J; ++j) {
      const int c = (lane + 64 * j) * V;
      if (c < d) {
#pragma unroll
        for (int e = 0; e < V; ++e) gv[j][e] += rstd * (dxh[j][e] - m1 - xh[j][e] * m2);
        Vec<float, V>::store(gr + c, gv[j]);
        if ((const void *)Gb != (const void *)G) Vec<T, V>::store(gbr + c, gv[j]);
      }
    }
  }
  // block-level column sums: the four wavefronts combine through LDS, fixed order
  float *pg = partials + (size_t)blockIdx.x * 2 * d;
#pragma unroll
  for (int j = 0; j < J; ++j) {
    if (64 * j * V >= d) continue;  // uniform across the block
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      __syncthreads();
#pragma unroll
      for (int e = 0; e < V; ++e) red[wave][lane * V + e] = pass ? db[j][e] : dg[j][e];
      __syncthreads();
      if (wave == 0) {
        const int c = (lane + 64 * j) * V;
#pragma unroll
        for (int e = 0; e < V; ++e) {
          const int i = lane * V + e;
          if (c + e < d) pg[pass * d + c + e] = (red[0][i] + red[1][i]) + (red[2][i] + red[3][i]);
        }
      }
    }
  }
}

template <typename T>
void launch_ln_bwd(int blocks, hipStream_t s, const void *dy, const float *x, const float *stats, const void *gamma,
                   int rows, int N, int d, float *G, void *Gb, StreamWeights sw, float *partials) {
#define IL_LN_BWD(V, J)                                                                                          \
  hipLaunchKernelGGL((ln_bwd_kernel<T, V, J>), dim3(blocks), dim3(256), 0, s, (const T *)dy, x, stats,          \
                     (const T *)gamma, rows, N, d, G, (T *)Gb, sw, partials)
  if (d % 256 == 0 && d <= 512) IL_LN_BWD(4, 2);
  else if (d % 256 == 0 && d <= 1024) IL_LN_BWD(4, 4);
  else if (d % 256 == 0 && d <= 2048) IL_LN_BWD(4, 8);
  else if (d <= 256) IL_LN_BWD(1, 4);
  else IL_LN_BWD(1, 32);
#undef IL_LN_BWD
}

}  // namespace

int ln_backward_max_blocks() { return kLnBwdBlocks; }

hipError_t ln_forward(int dtype, const float *x, const void *gamma, const void *beta, float eps, int rows,
                      int d, void *y, float *stats, float *xcopy, hipStream_t s) {
  dim3 grid((rows + kWaves - 1) / kWaves);
#define IL_LN_FWD_VEC(T, J)                                                                                   \
  hipLaunchKernelGGL((ln_fwd_vec_kernel<T, J>), grid, dim3(256), 0, s, x, (const T *)gamma, (const T *)beta, \
                     eps, rows, (T *)y, stats, xcopy)
  if (dtype != 0 && (d == 256 || d == 512 || d == 1024 || d == 2048)) {
    switch (d / 256) {
      case 1: IL_LN_FWD_VEC(bf16_t, 1); break;
      case 2: IL_LN_FWD_VEC(bf16_t, 2); break;
      case 4: IL_LN_FWD_VEC(bf16_t, 4); break;
      default: IL_LN_FWD_VEC(bf16_t, 8); break;
    }
  } else if (dtype == 0 && (d == 256 || d == 512 || d == 1024 || d == 2048)) {
    switch (d / 256) {
      case 1: IL_LN_FWD_VEC(float, 1); break;
      case 2: IL_LN_FWD_VEC(float, 2); break;
      case 4: IL_LN_FWD_VEC(float, 4); break;
      default: IL_LN_FWD_VEC(float, 8); break;
    }
  } else if (dtype == 0) {
    hipLaunchKernelGGL(ln_fwd_kernel<float>, grid, dim3(256), 0, s, x, (const float *)gamma,
                       (const float *)beta, eps, rows, d, (float *)y, stats, xcopy);
  } else {
    hipLaunchKernelGGL(ln_fwd_kernel<bf16_t>, grid, dim3(256), 0, s, x, (const bf16_t *)gamma,
                       (const bf16_t *)beta, eps, rows, d, (bf16_t *)y, stats, xcopy);
  }
#undef IL_LN_FWD_VEC
  return hipGetLastError();
}

hipError_t ln_backward_residual(int dtype, const void *dy, const float *x, const float *stats,
                                const void *gamma, int rows, int N, int d, float *G, void *Gb,
                                StreamWeights sw, float *partials, int *nblk, hipStream_t s) {
  int blocks = (rows + kWaves - 1) / kWaves;
  if (blocks > kLnBwdBlocks) blocks = kLnBwdBlocks;
  *nblk = blocks;
  if (dtype == 0)
    launch_ln_bwd<float>(blocks, s, dy, x, stats, gamma, rows, N, d, G, Gb, sw, partials);
  else
    launch_ln_bwd<bf16_t>(blocks, s, dy, x, stats, gamma, rows, N, d, G, Gb, sw, partials);
  return hipGetLastError();
}

}  // namespace il
