// Internal declarations shared by the HIP sources of libinterlock (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace il {

typedef unsigned short bf16_t;  // raw bfloat16 bits

__host__ __device__ inline float bf16_to_f32(bf16_t h) {
  union { uint32_t u; float f; } c;
  c.u = ((uint32_t)h) << 16;
  return c.f;
}
// float -> bfloat16, round to nearest even.  On the device this is the hardware conversion
// (v_cvt_pk_bf16_f32); the host version does the same rounding in integer arithmetic.
__host__ __device__ inline bf16_t f32_to_bf16(float f) {
#if defined(__HIP_DEVICE_COMPILE__)
  const __bf16 b = (__bf16)f;
  return __builtin_bit_cast(bf16_t, b);
#else
  union { uint32_t u; float f; } c;
  c.f = f;
  uint32_t u = c.u;
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
#endif
}
// two floats -> packed bf16 pair (a in the low half)
__device__ inline uint32_t pack_bf16x2(float a, float b) {
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
  bf16x2_t v;
  v[0] = (__bf16)a;
  v[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, v);
}

// IEEE half <-> float (hardware conversions)
__device__ inline float f16_to_f32(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }
__device__ inline uint32_t pack_f16x2(float a, float b) {  // a in the low half; round to nearest even, clamped to the finite range
  const float lim = 65504.f;
  typedef __attribute__((__vector_size__(2 * sizeof(_Float16)))) _Float16 f16x2_t;
  f16x2_t v;
  v[0] = (_Float16)fminf(fmaxf(a, -lim), lim);
  v[1] = (_Float16)fminf(fmaxf(b, -lim), lim);
  return __builtin_bit_cast(uint32_t, v);
}

template <typename T> __device__ inline float ld(const T *p);
template <> __device__ inline float ld<float>(const float *p) { return *p; }
template <> __device__ inline float ld<bf16_t>(const bf16_t *p) { return bf16_to_f32(*p); }
template <typename T> __device__ inline void st(T *p, float v);
template <> __device__ inline void st<float>(float *p, float v) { *p = v; }
template <> __device__ inline void st<bf16_t>(bf16_t *p, float v) { *p = f32_to_bf16(v); }

// tanh-form GELU and its derivative, fp32, written through the logistic function: with
// y = sqrt(2/pi) (u + 0.044715 u^3) and s = 1 / (1 + exp(-2y)), tanh(y) = 2s - 1, so
//   gelu(u)  = u s,      gelu'(u) = s + s (1 - s) * 2 sqrt(2/pi) u (1 + 3 * 0.044715 u^2).
// exp and the reciprocal are the hardware instructions (relative error ~1e-6, far inside the fp32
// tolerance; both ends saturate correctly: s -> 0 or 1).  These sit in the epilogue of every MLP GEMM,
// where the two wavefronts of a SIMD share one vector ALU: the derivative costs eight plain and two
// transcendental instructions per element in this form.
__device__ inline float gelu_sigmoid(float u, float u2) {
  const float y = u * __builtin_fmaf(0.044715f, u2, 1.0f);
  const float e = __builtin_amdgcn_exp2f(y * -2.3022081715f);  // exp(-2 sqrt(2/pi) y'), -2 * 0.79788456 * log2(e)
  return __builtin_amdgcn_rcpf(e + 1.0f);
}
__device__ inline float gelu_f(float u) { return u * gelu_sigmoid(u, u * u); }
__device__ inline float gelu_grad_f(float u) {
  const float u2 = u * u;
  const float s = gelu_sigmoid(u, u2);
  const float w = u * __builtin_fmaf(0.2140644488f, u2, 1.5957691216f);  // 2 sqrt(2/pi) u (1 + 0.134145 u^2)
  const float t = __builtin_fmaf(-w, s, w);                              // w (1 - s)
  return __builtin_fmaf(s, t, s);
}

// Up to 16 gradient streams are stacked along the row dimension of the backward
// operands; stream i occupies rows [i*N, (i+1)*N).
constexpr int kMaxStreams = 16;
struct StreamWeights {
  float w[kMaxStreams];
};

// ---- GEMM front ends (implemented in gemm_simt.hip / gemm_mfma.hip) ----------------
enum Epi {
  EPI_STORE = 0,      // C = acc                                  (T out)
  EPI_BIAS = 1,       // C = acc + bias[col]                      (T out)
  EPI_BIAS_GELU = 2,  // C = acc + bias (pre-activation, T), C2 = gelu(C) (T)
  EPI_BIAS_RES = 3,   // Cf = acc + bias + res[row, col]          (fp32 out, fp32 residual)
  EPI_GELU_BWD = 4,   // C = acc * gelu'(aux[row mod wrap, col])  (T out, T aux)
  EPI_STORE_F32 = 5,  // Cf = acc                                 (fp32 out)
  EPI_WGRAD = 6,      // Cf = scale*acc (+ Cf if beta)            (fp32 out)
  EPI_LOGITS = 7      // the head's logits tile (bf16 operands only): C = acc as IEEE half, clamped to +-65504 (the
                      // softmax wants the three extra mantissa bits and never the range); and, when row_stats is
                      // set, softmax statistics straight from the fp32 accumulators: for every row and every
                      // group of 64 columns (max, sum of exp(z - max)), and the row's target logit
};
constexpr int kStatGroup = 64;  // columns per statistics group of EPI_LOGITS

struct GemmArgs {
  // C[M,N] = sum_k A(m,k) B(k,n); operand storage:
  //   a_kmajor == 0: A stored [M, K] row-major (lda);  1: A stored [K, M] row-major (lda)
  //   b_kmajor == 0: B stored [N, K] row-major (ldb);  1: B stored [K, N] row-major (ldb)
  const void *A;
  const void *B;
  int M, N, K;
  int lda, ldb;
  int a_kmajor, b_kmajor;
  int epi;
  void *C;        // T or fp32 depending on epi
  void *C2;       // EPI_BIAS_GELU second output
  int ldc;
  const void *bias;   // T [N]
  const float *res;   // fp32 [M, ldc]
  const void *aux;    // T, EPI_GELU_BWD
  int aux_wrap;       // rows of aux (row index taken modulo this)
  float scale;        // EPI_WGRAD
  uint32_t a_bytes, b_bytes;  // operand extents in bytes (filled by the bf16 front end)
  int k_begin, k_end; // reduction range [k_begin, k_end); both 0 = all of K (used by split-K)
  int tile;           // bf16: 0 = choose by shape, 1 = 256x256, 2 / 3 = 128x128 with 2 / 4 stages, 4 / 5 = 64x64 with 2 / 4,
                      // 6 = 256x128, 7 = 128x256 (three stages), 8 = 256x256 persistent
  int beta;           // EPI_WGRAD: accumulate into C
  // EPI_LOGITS, all optional together: row_stats [M][ceil(N / kStatGroup)][2] fp32, row_targets [M] int32,
  // row_ztgt [M] fp32 (written for rows whose target lies in [0, N))
  float *row_stats;
  const int32_t *row_targets;
  float *row_ztgt;
};

// Events attached to ONE kernel dispatch (hipExtLaunchKernelGGL): elapsed(start, stop) is that
// kernel's own execution time, the figure a kernel trace reports, without the gaps that events
// recorded between launches add.  gemm_time_next() arms the calling thread's next bf16 GEMM
// kernel launch; the launch disarms it.  Returns the timer that was still armed (nullptr if none).
struct KernelTimer { hipEvent_t start, stop; };
const KernelTimer *gemm_time_next(const KernelTimer *t);

hipError_t gemm_f32(const GemmArgs &g, hipStream_t s);    // T = float, SIMT
hipError_t gemm_bf16(const GemmArgs &g, hipStream_t s);   // T = bf16, MFMA
// Up to kMaxBatch independent GEMMs with the same operand layouts and epilogue in ONE launch
// (their tiles share the grid, so small problems fill the chip together).
constexpr int kMaxBatch = 8;
hipError_t gemm_bf16_batch(const GemmArgs *list, int count, hipStream_t s);
// Split-K for fp32-output epilogues (EPI_STORE_F32, EPI_WGRAD): `splits` partial products over
// disjoint K ranges go to ws ([splits][M][N] fp32) in one launch, then a reduction applies the
// epilogue.  Deterministic (fixed summation order).
hipError_t gemm_bf16_splitk(const GemmArgs &g, int splits, float *ws, hipStream_t s);
// out[i] = scale * sum_p part[p*stride + i] (+ out[i] if beta), rows x cols with pitch ldc
hipError_t splitk_reduce(const float *part, int splits, size_t stride, int rows, int cols, float *out, int ldc,
                         float scale, int beta, hipStream_t s);

// ---- row-wise kernels (layernorm.hip) -----------------------------------------------
// y = LN(x)*gamma+beta -> T; stats[row] = (mean, rstd); optional fp32 copy of x.
hipError_t ln_forward(int dtype, const float *x, const void *gamma, const void *beta, float eps,
                      int rows, int d, void *y, float *stats, float *xcopy, hipStream_t s);
// For each stacked row r (stream r / N, token r % N): G[r] += LN'(x)^T dy[r]; Gb[r] = T(G[r]);
// partial column sums of w*dy*xhat and w*dy go to `partials` ([nblk][2*d]); returns nblk.
hipError_t ln_backward_residual(int dtype, const void *dy, const float *x, const float *stats,
                                const void *gamma, int rows, int N, int d, float *G, void *Gb,
                                StreamWeights sw, float *partials, int *nblk, hipStream_t s);
int ln_backward_max_blocks();

// ---- reductions / elementwise (reduce.hip) --------------------------------------------
// out[c] = sum over blocks p of partials[p][c], c < cols (fp32 out, deterministic order)
hipError_t colsum_final(const float *partials, int nblk, int cols, float *out, int accumulate, hipStream_t s);
// ysum[r][c] = sum_s w[s] * Y[s*N + r][c] (stored in T when ysum != NULL, pitch = cols);
struct ColsumJob { const float *partials; int nblk, cols; float *out; int accumulate; };
constexpr int kMaxColsumJobs = 8;
struct ColsumJobs { int count; ColsumJob job[kMaxColsumJobs]; };
// all second stages of one block's backward in a single launch
hipError_t colsum_final_multi(const ColsumJobs &jobs, hipStream_t s);
// partials[p][c] = column sums of ysum over the rows of block p; returns nblk.  (The second
// stage stays a separate launch: a same-launch hand-over between workgroups needs a device-scope
// fence, which on this multi-XCD part writes back the L2 and costs far more than a launch.)
hipError_t sum_colsum(int dtype, const void *Y, int N, int cols, int ld, int ns, StreamWeights sw, void *ysum,
                      float *partials, int *nblk, hipStream_t s);
// Several such reductions over the same number of rows in one launch (grid.z selects the job).
struct SumColsumJob { const void *Y; int N, cols, ldy, ns; StreamWeights sw; void *ysum; float *partials; };
constexpr int kMaxSumColsumJobs = 2;
struct SumColsumJobs { int count; SumColsumJob job[kMaxSumColsumJobs]; };
hipError_t sum_colsum_multi(int dtype, const SumColsumJobs &jobs, int *nblk, hipStream_t s);
int colsum_max_blocks();
// G[i] = (accumulate ? G[i] : 0) + src[i]; Gb[i] = T(G[i])
hipError_t stream_inject(int dtype, const float *src, float *G, void *Gb, size_t count, int accumulate,
                         hipStream_t s);
// out[i] = (accumulate ? out[i] : 0) + sum_j w[j] * G[j*stride + i]
hipError_t stream_combine(const float *G, size_t stride, int nstreams, StreamWeights sw, float *out,
                          size_t count, int accumulate, hipStream_t s);
// dst = T(src)
hipError_t convert_f32(int dtype, const float *src, void *dst, size_t count, hipStream_t s);

// ---- attention (attention_*.hip) --------------------------------------------------------
// qkv: T [N, 3d] (Q|K|V, heads contiguous); o: T [N, d]; lse: fp32 [B, H, T]
hipError_t attention_forward(int dtype, const void *qkv, int B, int T, int H, int dh, void *o, float *lse,
                             hipStream_t s);
// d_o: T [nstreams*N, d]; dqkv: T [nstreams*N, 3d]; dsum: fp32 scratch [nstreams*N*H]
hipError_t attention_backward(int dtype, const void *qkv, const void *o, const void *d_o, const float *lse,
                              int nstreams, int B, int T, int H, int dh, void *dqkv, float *dsum,
                              hipStream_t s);

// ---- cross-entropy rows (xent.hip) --------------------------------------------------------
// For each of `rows` logit rows z (T, [rows, V], in place): rowloss = lse - z[target];
// z <- (softmax(z) - onehot(target)) * inv_n.
hipError_t xent_rows(int dtype, void *z, const int32_t *targets, int rows, int V, float inv_n,
                     float *rowloss, hipStream_t s);
// The same for a tile of IEEE-half logits whose row statistics the logits GEMM left behind (EPI_LOGITS):
// stats [rows][ceil(V / kStatGroup)][2] = (max, sum-exp) per 64-column group, ztgt [rows] = target logit.
// One pass over the tile: the groups are merged into the row's log-sum-exp, rowloss = lse - ztgt, and
// z (half) <- bf16((exp(z - lse) - onehot) * inv_n).  Any V that is a multiple of 8.
hipError_t xent_rows_from_stats(void *z, const float *stats, const float *ztgt, const int32_t *targets, int rows,
                                int V, float inv_n, float *rowloss, hipStream_t s);
// loss_out[0] = scale * sum(rowloss[0..rows))
hipError_t sum_scalar(const float *rowloss, int rows, float scale, float *loss_out, hipStream_t s);

}  // namespace il
