// Input embedding of the first module (App. B: an embedding matrix in front of the Transformer
// blocks) and its gradient.
//
//   forward :  x0[i, :]   = wte[tokens[i], :] + wpe[i % T, :]                      (fp32 out)
//   backward:  dwpe[t, :] = sum_b dx0[b*T + t, :]
//              dwte[v, :] = sum over the positions i with tokens[i] == v of dx0[i, :]
//
// The token gradient is a scatter-add.  It is done without atomics and with a fixed summation
// order: a workgroup owns kRows consecutive vocabulary rows, clears them, scans the whole token
// array for positions that hit its rows (the array is a few KB and stays in L2) and adds those
// rows of dx0 in ascending position order.  Every element of dwte and dwpe is written exactly
// once per call by a plain store of its final value; a token outside [0, vocab) embeds as zero
// and receives no gradient.  All three kernels are HBM-bound.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/interlock.h"
#include "common.h"

namespace il {
namespace {

constexpr int kRows = 32;        // vocabulary rows per workgroup in the token-gradient kernel
constexpr int kListCap = 1024;   // matches kept per scan pass (a pass ends early when the list is full)

template <typename T>
__global__ __launch_bounds__(256) void embed_fwd_kernel(const T *__restrict__ wte, const T *__restrict__ wpe,
                                                        const int32_t *__restrict__ tokens, int N, int Tn, int d,
                                                        int V, float *__restrict__ x0) {
  // one row per wavefront pass, 4 columns per lane
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = blockIdx.x * 4 + wave; i < N; i += gridDim.x * 4) {
    const int tok = tokens[i];
    const bool ok = tok >= 0 && tok < V;
    const T *te = wte + (size_t)(ok ? tok : 0) * d, *pe = wpe + (size_t)(i % Tn) * d;
    float *o = x0 + (size_t)i * d;
    for (int c = lane * 4; c < d; c += 256) {
      if (c + 3 < d) {
        float4 r;
        r.x = (ok ? ld<T>(te + c) : 0.f) + ld<T>(pe + c);
        r.y = (ok ? ld<T>(te + c + 1) : 0.f) + ld<T>(pe + c + 1);
        r.z = (ok ? ld<T>(te + c + 2) : 0.f) + ld<T>(pe + c + 2);
        r.w = (ok ? ld<T>(te + c + 3) : 0.f) + ld<T>(pe + c + 3);
        if ((d & 3) == 0) {
          *reinterpret_cast<float4 *>(o + c) = r;
        } else {
          o[c] = r.x; o[c + 1] = r.y; o[c + 2] = r.z; o[c + 3] = r.w;
        }
      } else {
        for (int e = c; e < d; ++e) o[e] = (ok ? ld<T>(te + e) : 0.f) + ld<T>(pe + e);
      }
    }
  }
}

// dwpe[t, c] = sum_b dx0[b*T + t, c], b ascending
__global__ __launch_bounds__(256) void embed_bwd_pos_kernel(const float *__restrict__ dx0, int B, int Tn, int d,
                                                            float *__restrict__ dwpe) {
  const size_t total = (size_t)Tn * d;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    float s = 0.f;
    for (int b = 0; b < B; ++b) s += dx0[(size_t)b * total + i];
    dwpe[i] = s;
  }
}

// Workgroup blockIdx.x owns vocabulary rows [v0, v0 + kRows).
__global__ __launch_bounds__(256) void embed_bwd_tok_kernel(const float *__restrict__ dx0,
                                                            const int32_t *__restrict__ tokens, int N, int d, int V,
                                                            float *__restrict__ dwte) {
  __shared__ int list_pos[kListCap];
  __shared__ int wave_cnt[4];
  __shared__ int list_len, next_start;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int v0 = blockIdx.x * kRows, v1 = min(V, v0 + kRows);
  float *rows = dwte + (size_t)v0 * d;
  const size_t nel = (size_t)(v1 - v0) * d;
  for (size_t i = t; i < nel; i += 256) rows[i] = 0.f;
  __syncthreads();  // (workgroup-scope release/acquire: the adds below see the zeros)

  int start = 0;
  while (start < N) {
    // scan up to kListCap / 256 chunks of 256 positions; matches are appended in position order
    if (t == 0) { list_len = 0; next_start = N; }
    __syncthreads();
    int len = 0;
    for (int base = start; base < N; base += 256) {
      if (len + 256 > kListCap) { if (t == 0) next_start = base; break; }   // uniform: len is uniform
      const int i = base + t;
      const int tok = i < N ? tokens[i] : -1;
      const bool hit = tok >= v0 && tok < v1;
      const unsigned long long m = __ballot(hit);
      if (lane == 0) wave_cnt[wave] = __popcll(m);
      __syncthreads();
      int off = len;
      for (int w2 = 0; w2 < wave; ++w2) off += wave_cnt[w2];
      if (hit) list_pos[off + __popcll(m & ((1ull << lane) - 1ull))] = i;
      len += wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
      __syncthreads();
    }
    if (t == 0) list_len = len;
    __syncthreads();
    const int n = list_len;
    // ascending position order: each column is owned by one thread, so its adds are sequential
    for (int e = 0; e < n; ++e) {
      const int i = list_pos[e];
      const float *src = dx0 + (size_t)i * d;
      float *dst = dwte + (size_t)tokens[i] * d;
      for (int c = t; c < d; c += 256) dst[c] += src[c];
    }
    start = next_start;
    __syncthreads();
  }
}

}  // namespace
}  // namespace il

extern "C" {

int il_embed_forward(int32_t dtype, const void *wte, const void *wpe, const int32_t *tokens, int32_t batch,
                     int32_t seq, int32_t d_model, int32_t vocab, float *x0, void *stream) {
  using namespace il;
  if (dtype != IL_F32 && dtype != IL_BF16) return IL_E_ARG;
  if (!wte || !wpe || !tokens || !x0 || batch < 1 || seq < 1 || d_model < 1 || vocab < 1) return IL_E_ARG;
  const long long N = (long long)batch * seq;
  if (N > (1 << 24) || vocab > (1 << 24)) return IL_E_SHAPE;
  if ((d_model & 3) == 0 && ((uintptr_t)x0 & 15)) return IL_E_SHAPE;
  const int blocks = (int)((N + 3) / 4 < 4096 ? (N + 3) / 4 : 4096);
  hipStream_t s = (hipStream_t)stream;
  if (dtype == IL_F32)
    hipLaunchKernelGGL(embed_fwd_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float *)wte,
                       (const float *)wpe, tokens, (int)N, seq, d_model, vocab, x0);
  else
    hipLaunchKernelGGL(embed_fwd_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, (const bf16_t *)wte,
                       (const bf16_t *)wpe, tokens, (int)N, seq, d_model, vocab, x0);
  return hipGetLastError() == hipSuccess ? IL_OK : IL_E_HIP;
}

int il_embed_backward(const float *dx0, const int32_t *tokens, int32_t batch, int32_t seq, int32_t d_model,
                      int32_t vocab, float *dwte, float *dwpe, void *stream) {
  using namespace il;
  if (!dx0 || !tokens || !dwte || !dwpe || batch < 1 || seq < 1 || d_model < 1 || vocab < 1) return IL_E_ARG;
  const long long N = (long long)batch * seq;
  if (N > (1 << 24) || vocab > (1 << 24)) return IL_E_SHAPE;
  hipStream_t s = (hipStream_t)stream;
  const size_t total = (size_t)seq * d_model;
  const int pblocks = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
  hipLaunchKernelGGL(embed_bwd_pos_kernel, dim3(pblocks), dim3(256), 0, s, dx0, batch, seq, d_model, dwpe);
  hipLaunchKernelGGL(embed_bwd_tok_kernel, dim3((vocab + kRows - 1) / kRows), dim3(256), 0, s, dx0, tokens, (int)N,
                     d_model, vocab, dwte);
  return hipGetLastError() == hipSuccess ? IL_OK : IL_E_HIP;
}

}  // extern "C"
