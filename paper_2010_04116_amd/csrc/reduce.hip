// Small bandwidth-bound helpers: deterministic two-stage column sums (bias gradients,
// LayerNorm gain/bias gradients), gradient-stream injection / combination, fp32 -> T
// conversion.  No float atomics anywhere: every reduction has a fixed order.
#include "common.h"

namespace il {
namespace {

constexpr int kColBlocksY = 64;   // row splits of the first stage

// grid (ceil(cols/64), nby); block 256 = 64 columns x 4 row lanes
template <typename T>
__global__ __launch_bounds__(256) void colsum_partial_kernel(const T *__restrict__ Y, int rows, int N, int cols,
                                                             int ldy, StreamWeights sw,
                                                             float *__restrict__ partials) {
  __shared__ float red[4][64];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + tx;
  const int per = (rows + gridDim.y - 1) / gridDim.y;
  const int r0 = blockIdx.y * per, r1 = min(rows, r0 + per);
  float acc = 0.f;
  if (c < cols)
    for (int r = r0 + ty; r < r1; r += 4) acc += sw.w[r / N] * ld<T>(Y + (size_t)r * ldy + c);
  red[ty][tx] = acc;
  __syncthreads();
  if (ty == 0 && c < cols)
    partials[(size_t)blockIdx.y * cols + c] = red[0][tx] + red[1][tx] + red[2][tx] + red[3][tx];
}

__global__ __launch_bounds__(256) void colsum_final_kernel(const float *__restrict__ partials, int nblk, int cols,
                                                           float *__restrict__ out, int accumulate) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= cols) return;
  float acc = accumulate ? out[c] : 0.f;
  for (int p = 0; p < nblk; ++p) acc += partials[(size_t)p * cols + c];
  out[c] = acc;
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

hipError_t colsum_partial(int dtype, const void *Y, int rows, int N, int cols, int ldy, StreamWeights sw,
                          float *partials, int *nblk, hipStream_t s) {
  int nby = (rows + 63) / 64;
  if (nby > kColBlocksY) nby = kColBlocksY;
  if (nby < 1) nby = 1;
  *nblk = nby;
  dim3 grid((cols + 63) / 64, nby);
  if (dtype == 0)
    hipLaunchKernelGGL(colsum_partial_kernel<float>, grid, dim3(256), 0, s, (const float *)Y, rows, N, cols,
                       ldy, sw, partials);
  else
    hipLaunchKernelGGL(colsum_partial_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t *)Y, rows, N, cols,
                       ldy, sw, partials);
  return hipGetLastError();
}

hipError_t colsum_final(const float *partials, int nblk, int cols, float *out, int accumulate, hipStream_t s) {
  hipLaunchKernelGGL(colsum_final_kernel, dim3((cols + 255) / 256), dim3(256), 0, s, partials, nblk, cols, out,
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
