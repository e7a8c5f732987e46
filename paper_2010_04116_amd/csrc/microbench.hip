// Measured peaks of the board, reported beside the nominal ones: a matrix-unit-only loop
// (v_mfma_f32_32x32x16_bf16 on register operands, no memory traffic) and a streaming copy of
// known size in two forms - 16 bytes per lane, grid-stride, plain loads and stores; and four such
// vectors in flight per lane with non-temporal loads and stores, which is the fastest copy found on
// this part (5.9-6.3 TB/s against 4.6-5.1) - of which the better rate is reported.  The plain copy
// also serves as the kernel of known HBM traffic against which the profiler's FETCH_SIZE /
// WRITE_SIZE counters are scaled.
#include "../../include/interlock.h"
#include "../../include/interlock_test.h"

#include <algorithm>

#include "common.h"

namespace il {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr int kAcc = 4;  // independent accumulators per wavefront: back-to-back issue without dependence stalls

__global__ __launch_bounds__(256) void mfma_only_kernel(float *out, int iters) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(float)((threadIdx.x + i) & 7);
    b[i] = (__bf16)(float)(i + 1);
  }
  floatx16 acc[kAcc];
#pragma unroll
  for (int j = 0; j < kAcc; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < kAcc; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < kAcc; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[j][r];
  if (s == 12345.678f) out[threadIdx.x] = s;  // keeps the loop alive; never true for these operands
}

__global__ __launch_bounds__(256) void stream_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                                          size_t n16) {
  const size_t step = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += step) dst[i] = src[i];
}

typedef unsigned int u32x4v __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void stream_copy4_kernel(const u32x4v *__restrict__ src, u32x4v *__restrict__ dst,
                                                           size_t n16) {
  constexpr int U = 4;
  const size_t step = (size_t)gridDim.x * 256 * U;
  for (size_t i = (size_t)blockIdx.x * 256 * U + threadIdx.x; i < n16; i += step) {
    u32x4v v[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (i + u * 256 < n16) v[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (i + u * 256 < n16) __builtin_nontemporal_store(v[u], dst + i + u * 256);
  }
}

struct Timer {
  hipEvent_t e0 = nullptr, e1 = nullptr;
  bool ok() { return hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess; }
  ~Timer() {
    if (e0) hipEventDestroy(e0);
    if (e1) hipEventDestroy(e1);
  }
};

}  // namespace
}  // namespace il

using namespace il;

extern "C" {

int il_measure_mfma_peak(float *scratch, int32_t iters, void *stream, double *tflops_out) {
  if (!scratch || !tflops_out || iters < 1 || iters > (1 << 22)) return IL_E_ARG;
  hipStream_t s = (hipStream_t)stream;
  Timer t;
  if (!t.ok()) return IL_E_HIP;
  const int wgs = 256 * 2;  // two workgroups of four wavefronts per CU: two wavefronts per SIMD
  hipLaunchKernelGGL(mfma_only_kernel, dim3(wgs), dim3(256), 0, s, scratch, iters / 8 + 1);  // warm-up
  if (hipEventRecord(t.e0, s) != hipSuccess) return IL_E_HIP;
  hipLaunchKernelGGL(mfma_only_kernel, dim3(wgs), dim3(256), 0, s, scratch, iters);
  if (hipGetLastError() != hipSuccess || hipEventRecord(t.e1, s) != hipSuccess) return IL_E_HIP;
  if (hipEventSynchronize(t.e1) != hipSuccess) return IL_E_HIP;
  float ms = 0.f;
  if (hipEventElapsedTime(&ms, t.e0, t.e1) != hipSuccess || !(ms > 0.f)) return IL_E_HIP;
  *tflops_out = (double)wgs * 4 * iters * kAcc * (2.0 * 32 * 32 * 16) / (ms * 1e-3) / 1e12;
  return IL_OK;
}

int il_measure_copy_peak(void *dst, const void *src, size_t bytes, int32_t reps, void *stream, double *gbs_out) {
  if (!dst || !src || !gbs_out || bytes < 16 || reps < 1 || reps > 1000) return IL_E_ARG;
  if (((uintptr_t)dst & 15) || ((uintptr_t)src & 15) || (bytes & 15)) return IL_E_SHAPE;
  hipStream_t s = (hipStream_t)stream;
  Timer t;
  if (!t.ok()) return IL_E_HIP;
  const size_t n16 = bytes / 16;
  const unsigned grid = (unsigned)std::min<size_t>((n16 + 255) / 256, 256 * 32);
  const unsigned grid4 = (unsigned)std::min<size_t>((n16 + 1023) / 1024, 256 * 128);
  double best = 0.0;
  for (int form = 0; form < 2; ++form) {
    auto launch = [&]() {
      if (form == 0)
        hipLaunchKernelGGL(stream_copy_kernel, dim3(grid), dim3(256), 0, s, (const uint4 *)src, (uint4 *)dst, n16);
      else
        hipLaunchKernelGGL(stream_copy4_kernel, dim3(grid4), dim3(256), 0, s, (const u32x4v *)src, (u32x4v *)dst, n16);
    };
    launch();
    if (hipEventRecord(t.e0, s) != hipSuccess) return IL_E_HIP;
    for (int i = 0; i < reps; ++i) launch();
    if (hipGetLastError() != hipSuccess || hipEventRecord(t.e1, s) != hipSuccess) return IL_E_HIP;
    if (hipEventSynchronize(t.e1) != hipSuccess) return IL_E_HIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, t.e0, t.e1) != hipSuccess || !(ms > 0.f)) return IL_E_HIP;
    best = std::max(best, 2.0 * (double)bytes * reps / (ms * 1e-3) / 1e9);  // bytes read + bytes written
  }
  *gbs_out = best;
  return IL_OK;
}

}  // extern "C"
