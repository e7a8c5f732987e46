// Small bandwidth-bound helpers: deterministic two-stage column sums (bias gradients,
// LayerNorm gain/bias gradients), gradient-stream injection / combination, fp32 -> T
// conversion.  No float atomics anywhere: every reduction has a fixed order.
#include "common.h"

namespace il {
namespace {

constexpr int kColBlocksY = 64;   // row splits of the first stage

// First stage, fused with the weighted sum over gradient streams.  Y holds `ns` stacked
// streams of N rows; for every token row the kernel forms ysum = sum_s w[s] * Y[s*N + row] in
// fp32, optionally stores it (rounded to T) for the weight-gradient GEMM, and accumulates its
// column sums (the bias gradient).  V = 8: grid (ceil(cols/256), nby), block = 32 column groups
// of 8 x 8 row lanes, 16-byte accesses (cols % 8 == 0).  V = 1: block = 64 columns x 4 row lanes.
template <typename T, int V>
__global__ __launch_bounds__(256) void sum_colsum_kernel(SumColsumJobs jobs) {
  constexpr int CG = V == 8 ? 32 : 64, RL = 256 / CG;
  __shared__ float red[RL][CG * V];
  const SumColsumJob &jb = jobs.job[blockIdx.z];   // grid.z selects the job
  const T *__restrict__ Y = (const T *)jb.Y;
  T *__restrict__ ysum = (T *)jb.ysum;
  float *__restrict__ partials = jb.partials;
  const int N = jb.N, cols = jb.cols, ldy = jb.ldy, ns = jb.ns;
  const StreamWeights &sw = jb.sw;
  if ((int)blockIdx.x * CG * V >= cols) return;  // uniform: this job is narrower than the widest one
  const int tx = threadIdx.x % CG, ty = threadIdx.x / CG;
  const int c = (blockIdx.x * CG + tx) * V;
  const int per = (N + gridDim.y - 1) / gridDim.y;
  const int r0 = blockIdx.y * per, r1 = min(N, r0 + per);
  float acc[V];
#pragma unroll
  for (int e = 0; e < V; ++e) acc[e] = 0.f;
  if (c < cols)
    for (int r = r0 + ty; r < r1; r += RL) {
      float v[V];
#pragma unroll
      for (int e = 0; e < V; ++e) v[e] = 0.f;
      for (int si = 0; si < ns; ++si) {
        const float w = sw.w[si];
        if (w == 0.f) continue;
        const T *src = Y + ((size_t)si * N + r) * ldy + c;
        if constexpr (V == 8) {
          const uint4 q = *reinterpret_cast<const uint4 *>(src);
          const uint32_t u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v[2 * e] += w * bf16_to_f32((bf16_t)(u[e] & 0xFFFF));
            v[2 * e + 1] += w * bf16_to_f32((bf16_t)(u[e] >> 16));
          }
        } else {
          v[0] += w * ld<T>(src);
        }
      }
      if (ysum) {
        if constexpr (V == 8) {
          uint4 q;
          q.x = pack_bf16x2(v[0], v[1]);
          q.y = pack_bf16x2(v[2], v[3]);
          q.z = pack_bf16x2(v[4], v[5]);
          q.w = pack_bf16x2(v[6], v[7]);
          *reinterpret_cast<uint4 *>(ysum + (size_t)r * cols + c) = q;
        } else {
          st<T>(ysum + (size_t)r * cols + c, v[0]);
        }
      }
#pragma unroll
      for (int e = 0; e < V; ++e) acc[e] += v[e];
    }
#pragma unroll
  for (int e = 0; e < V; ++e) red[ty][tx * V + e] = acc[e];
  __syncthreads();
  for (int i = threadIdx.x; i < CG * V; i += 256) {
    const int cc = blockIdx.x * CG * V + i;
    if (cc < cols) {
      float v = 0.f;
#pragma unroll
      for (int y = 0; y < RL; ++y) v += red[y][i];
      partials[(size_t)blockIdx.y * cols + cc] = v;
    }
  }
}

// Second stage: block = 16 columns x 16 partial lanes; fixed summation order.
__global__ __launch_bounds__(256) void colsum_final_kernel(const float *__restrict__ partials, int nblk, int cols,
                                                           float *__restrict__ out, int accumulate) {
  __shared__ float red[16][17];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + tx;
  float acc = 0.f;
  if (c < cols)
    for (int p = ty; p < nblk; p += 16) acc += partials[(size_t)p * cols + c];
  red[ty][tx] = acc;
  __syncthreads();
  if (ty == 0 && c < cols) {
    float v = accumulate ? out[c] : 0.f;
#pragma unroll
    for (int y = 0; y < 16; ++y) v += red[y][tx];
    out[c] = v;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void inject_kernel(const float *__restrict__ src, float *G, T *Gb, size_t count,
                                                     int accumulate) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t step = (size_t)gridDim.x * 256;
  for (; i < count; i += step) {
    float v = src[i] + (accumulate ? G[i] : 0.f);
    G[i] = v;
    st<T>(Gb + i, v);
  }
}

__global__ __launch_bounds__(256) void combine_kernel(const float *__restrict__ G, size_t stride, int nstreams,
                                                      StreamWeights sw, float *__restrict__ out, size_t count,
                                                      int accumulate) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t step = (size_t)gridDim.x * 256;
  for (; i < count; i += step) {
    float v = accumulate ? out[i] : 0.f;
    for (int j = 0; j < nstreams; ++j) v += sw.w[j] * G[(size_t)j * stride + i];
    out[i] = v;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void convert_kernel(const float *__restrict__ src, T *__restrict__ dst,
                                                      size_t count) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t step = (size_t)gridDim.x * 256;
  for (; i < count; i += step) st<T>(dst + i, src[i]);
}

__global__ __launch_bounds__(256) void sum_scalar_kernel(const float *__restrict__ v, int n, float scale,
                                                         float *__restrict__ out) {
  __shared__ float red[256];
  float acc = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) acc += v[i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = red[0] * scale;
}

inline int grid_for(size_t count) {
  size_t b = (count + 255) / 256;
  return (int)(b > 4096 ? 4096 : (b ? b : 1));
}

}  // namespace

int colsum_max_blocks() { return kColBlocksY; }
hipError_t sum_colsum_multi(int dtype, const SumColsumJobs &jobs, int *nblk, hipStream_t s) {
  if (jobs.count < 1 || jobs.count > kMaxSumColsumJobs) return hipErrorInvalidValue;
  const int N = jobs.job[0].N;
  int nby = (N + 63) / 64;
  if (nby > kColBlocksY) nby = kColBlocksY;
  if (nby < 1) nby = 1;
  *nblk = nby;
  int maxc = 0;
  bool vec = dtype != 0;
  for (int i = 0; i < jobs.count; ++i) {
    const SumColsumJob &j = jobs.job[i];
    if (j.N != N) return hipErrorInvalidValue;  // the jobs of one launch share the row split
    maxc = j.cols > maxc ? j.cols : maxc;
    vec = vec && (j.cols & 7) == 0 && (j.ldy & 7) == 0;
  }
  if (dtype == 0)
    hipLaunchKernelGGL((sum_colsum_kernel<float, 1>), dim3((maxc + 63) / 64, nby, jobs.count), dim3(256), 0, s, jobs);
  else if (vec)
    hipLaunchKernelGGL((sum_colsum_kernel<bf16_t, 8>), dim3((maxc + 255) / 256, nby, jobs.count), dim3(256), 0, s,
                       jobs);
  else
    hipLaunchKernelGGL((sum_colsum_kernel<bf16_t, 1>), dim3((maxc + 63) / 64, nby, jobs.count), dim3(256), 0, s, jobs);
  return hipGetLastError();
}

hipError_t sum_colsum(int dtype, const void *Y, int N, int cols, int ldy, int ns, StreamWeights sw, void *ysum,
                      float *partials, int *nblk, hipStream_t s) {
  SumColsumJobs jobs;
  jobs.count = 1;
  jobs.job[0] = SumColsumJob{Y, N, cols, ldy, ns, sw, ysum, partials};
  return sum_colsum_multi(dtype, jobs, nblk, s);
}

// Several second stages in one launch: grid.y selects the job.
__global__ __launch_bounds__(256) void colsum_final_multi_kernel(ColsumJobs jobs) {
  __shared__ float red[16][17];
  const ColsumJob &jb = jobs.job[blockIdx.y];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + tx;
  if (blockIdx.x * 16 >= jb.cols) return;  // uniform across the block
  float acc = 0.f;
  if (c < jb.cols)
    for (int p = ty; p < jb.nblk; p += 16) acc += jb.partials[(size_t)p * jb.cols + c];
  red[ty][tx] = acc;
  __syncthreads();
  if (ty == 0 && c < jb.cols) {
    float v = jb.accumulate ? jb.out[c] : 0.f;
#pragma unroll
    for (int y = 0; y < 16; ++y) v += red[y][tx];
    jb.out[c] = v;
  }
}

hipError_t colsum_final_multi(const ColsumJobs &jobs, hipStream_t s) {
  if (jobs.count < 1) return hipSuccess;
  int maxc = 0;
  for (int i = 0; i < jobs.count; ++i) maxc = jobs.job[i].cols > maxc ? jobs.job[i].cols : maxc;
  hipLaunchKernelGGL(colsum_final_multi_kernel, dim3((maxc + 15) / 16, jobs.count), dim3(256), 0, s, jobs);
  return hipGetLastError();
}

hipError_t colsum_final(const float *partials, int nblk, int cols, float *out, int accumulate, hipStream_t s) {
  hipLaunchKernelGGL(colsum_final_kernel, dim3((cols + 15) / 16), dim3(256), 0, s, partials, nblk, cols, out,
                     accumulate);
  return hipGetLastError();
}

hipError_t stream_inject(int dtype, const float *src, float *G, void *Gb, size_t count, int accumulate,
                         hipStream_t s) {
  if (dtype == 0)
    hipLaunchKernelGGL(inject_kernel<float>, dim3(grid_for(count)), dim3(256), 0, s, src, G, (float *)Gb, count,
                       accumulate);
  else
    hipLaunchKernelGGL(inject_kernel<bf16_t>, dim3(grid_for(count)), dim3(256), 0, s, src, G, (bf16_t *)Gb,
                       count, accumulate);
  return hipGetLastError();
}

hipError_t stream_combine(const float *G, size_t stride, int nstreams, StreamWeights sw, float *out,
                          size_t count, int accumulate, hipStream_t s) {
  hipLaunchKernelGGL(combine_kernel, dim3(grid_for(count)), dim3(256), 0, s, G, stride, nstreams, sw, out,
                     count, accumulate);
  return hipGetLastError();
}

hipError_t convert_f32(int dtype, const float *src, void *dst, size_t count, hipStream_t s) {
  if (dtype == 0)
    hipLaunchKernelGGL(convert_kernel<float>, dim3(grid_for(count)), dim3(256), 0, s, src, (float *)dst, count);
  else
    hipLaunchKernelGGL(convert_kernel<bf16_t>, dim3(grid_for(count)), dim3(256), 0, s, src, (bf16_t *)dst,
                       count);
  return hipGetLastError();
}

hipError_t sum_scalar(const float *rowloss, int rows, float scale, float *loss_out, hipStream_t s) {
  hipLaunchKernelGGL(sum_scalar_kernel, dim3(1), dim3(256), 0, s, rowloss, rows, scale, loss_out);
  return hipGetLastError();
}

}  // namespace il
