// Plain-FMA tiled GEMM with the library's fused epilogues.  This is the true-fp32
// path (no matrix cores, no reduced-precision shortcuts) used when il_config.dtype is
// IL_F32; sizes there are small, so the kernel favours generality over speed:
// arbitrary M, N, K, both operand layouts.
#include "common.h"

namespace il {
namespace {

constexpr int TM = 64, TN = 64, TK = 16;

template <typename T>
__global__ __launch_bounds__(256) void gemm_simt_kernel(GemmArgs g) {
  __shared__ float As[TK][TM + 1];
  __shared__ float Bs[TK][TN + 1];
  const T *A = (const T *)g.A;
  const T *B = (const T *)g.B;
  const int t = threadIdx.x;
  const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
  const int tx = t % 16, ty = t / 16;
  float acc[4][4] = {};

  for (int k0 = 0; k0 < g.K; k0 += TK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int idx = t + 256 * i;
      int kk, mm;
      if (g.a_kmajor) { mm = idx % TM; kk = idx / TM; } else { kk = idx % TK; mm = idx / TK; }
      int gk = k0 + kk, gm = m0 + mm;
      float v = 0.f;
      if (gk < g.K && gm < g.M) {
        if (g.a_kmajor) {
          v = ld<T>(A + (size_t)gk * g.lda + gm);
        } else {
          v = ld<T>(A + (size_t)gm * g.lda + gk);
        }
      }
      As[kk][mm] = v;
      int nn;
      if (g.b_kmajor) { nn = idx % TN; kk = idx / TN; } else { kk = idx % TK; nn = idx / TK; }
      gk = k0 + kk;
      int gn = n0 + nn;
      v = 0.f;
      if (gk < g.K && gn < g.N) {
        if (g.b_kmajor) {
          v = ld<T>(B + (size_t)gk * g.ldb + gn);
        } else {
          v = ld<T>(B + (size_t)gn * g.ldb + gk);
        }
      }
      Bs[kk][nn] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }

  const T *bias = (const T *)g.bias;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int row = m0 + ty * 4 + i;
    if (row >= g.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int col = n0 + tx * 4 + j;
      if (col >= g.N) continue;
      size_t o = (size_t)row * g.ldc + col;
      float v = acc[i][j];
      switch (g.epi) {
        case EPI_STORE: st<T>((T *)g.C + o, v); break;
        case EPI_BIAS: st<T>((T *)g.C + o, v + ld<T>(bias + col)); break;
        case EPI_BIAS_GELU: {
          v += ld<T>(bias + col);
          st<T>((T *)g.C + o, v);
          // the activation is taken of the stored (rounded) pre-activation so that the
          // backward, which only has the stored value, differentiates the same function
          float us = ld<T>((T *)g.C + o);
          st<T>((T *)g.C2 + o, gelu_f(us));
          break;
        }
        case EPI_BIAS_RES: ((float *)g.C)[o] = v + ld<T>(bias + col) + g.res[o]; break;
        case EPI_GELU_BWD: {
          float u = ld<T>((const T *)g.aux + (size_t)(row % g.aux_wrap) * g.ldc + col);
          st<T>((T *)g.C + o, v * gelu_grad_f(u));
          break;
        }
        case EPI_STORE_F32: ((float *)g.C)[o] = v; break;
        case EPI_WGRAD: {
          float *c = (float *)g.C + o;
          *c = g.scale * v + (g.beta ? *c : 0.f);
          break;
        }
      }
    }
  }
}

}  // namespace

hipError_t gemm_simt(int dtype, const GemmArgs &g, hipStream_t s) {
  dim3 grid((g.N + TN - 1) / TN, (g.M + TM - 1) / TM);
  if (dtype == 0)
    hipLaunchKernelGGL(gemm_simt_kernel<float>, grid, dim3(256), 0, s, g);
  else
    hipLaunchKernelGGL(gemm_simt_kernel<bf16_t>, grid, dim3(256), 0, s, g);
  return hipGetLastError();
}

hipError_t gemm_f32(const GemmArgs &g, hipStream_t s) { return gemm_simt(0, g, s); }

}  // namespace il
