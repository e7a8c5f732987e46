// Causal attention forward / backward on the gfx950 matrix cores for bf16 and head
// widths 64 and 128.  K/V (forward, dQ) or Q/dO (dK, dV) tiles are LDS-resident and double
// buffered; scores are never written to memory.
//
// Orientation.  Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16:
// a lane then owns ONE query column (lane & 31) and holds 16 key rows per 32x32 tile in its
// accumulator registers.  Row max / row sum of the softmax are therefore in-register
// reductions plus one exchange with lane ^ 32, and the probabilities go straight from the
// accumulators into the B operand of the second product O^T = V^T P^T without touching LDS:
// the MFMA's k index is only a summation label, so the key order a lane happens to hold
// (rows 4h..4h+3 and 8+4h..8+4h+3 of each 16-key group, h = lane >> 5) is used as is and the
// A operand (V^T, staged transposed in LDS) is read in the same order.
//
// The backward recomputes the probabilities from the saved log-sum-exp in two kernels with
// fixed reduction order (no atomics): one owns a key/value tile and accumulates dK, dV over
// the query tiles at or below the diagonal, the other owns a query tile and accumulates dQ.
#include "common.h"

namespace il {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;

// byte offset of 16-byte chunk `chunk` of row `row` in an LDS tile with `rowb` bytes per row
__device__ inline int swz(int row, int chunk, int rowb) {
  return row * rowb + ((chunk ^ ((row ^ (row >> 3)) & 7)) << 4);
}
__device__ inline uint4 ldg16(const bf16_t *p) { return *reinterpret_cast<const uint4 *>(p); }

__device__ inline void transpose8x8(const uint4 (&in)[8], uint4 (&out)[8]) {
  const uint32_t *s = reinterpret_cast<const uint32_t *>(in);
  uint32_t *o = reinterpret_cast<uint32_t *>(out);
#pragma unroll
  for (int w = 0; w < 4; ++w)
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      uint32_t a = s[(2 * p) * 4 + w], b = s[(2 * p + 1) * 4 + w];
      o[(2 * w) * 4 + p] = (a & 0xFFFFu) | (b << 16);
      o[(2 * w + 1) * 4 + p] = (a >> 16) | (b & 0xFFFF0000u);
    }
}

__device__ inline uint32_t pack2(float a, float b) {
  return (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16);
}
union Frag {
  bf16x8 v;
  uint4 q;
  uint2 h[2];
  uint32_t u[4];
};

// A [ROWS x DH] tile of rows `row0..` of a token-major matrix (row stride ld), staged as is
// ([row][dh], dh contiguous).  Rows >= row_end are zero.
template <int ROWS, int DH>
struct RowTile {
  static constexpr int NCH = ROWS * DH / 8 / 256;
  static_assert(NCH >= 1, "tile too small for 256 threads");
  uint4 r[NCH];
  __device__ inline void fetch(const bf16_t *base, size_t ld, int row0, int row_end, int t) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = t + 256 * i, row = c / (DH / 8), ch = c % (DH / 8);
      r[i] = (row0 + row < row_end) ? ldg16(base + (size_t)(row0 + row) * ld + ch * 8) : make_uint4(0, 0, 0, 0);
    }
  }
  __device__ inline void store(char *lds, int t) const {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = t + 256 * i, row = c / (DH / 8), ch = c % (DH / 8);
      *reinterpret_cast<uint4 *>(lds + swz(row, ch, DH * 2)) = r[i];
    }
  }
};

// The same [ROWS x DH] tile staged transposed: LDS row = dh index, ROWS token columns.
template <int ROWS, int DH>
struct ColTile {
  static constexpr int NBLK = (ROWS / 8) * (DH / 8);  // 8x8 blocks
  static constexpr int PER = (NBLK + 255) / 256;
  uint4 r[PER][8];
  __device__ inline void fetch(const bf16_t *base, size_t ld, int row0, int row_end, int t) {
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      const int blk = t + 256 * j;
      const int db = blk % (DH / 8), rb = blk / (DH / 8);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int row = row0 + rb * 8 + i;
        r[j][i] = (blk < NBLK && row < row_end) ? ldg16(base + (size_t)row * ld + db * 8) : make_uint4(0, 0, 0, 0);
      }
    }
  }
  __device__ inline void store(char *lds, int t) const {
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      const int blk = t + 256 * j;
      if (blk < NBLK) {
        const int db = blk % (DH / 8), rb = blk / (DH / 8);
        uint4 o[8];
        transpose8x8(r[j], o);
#pragma unroll
        for (int c = 0; c < 8; ++c) *reinterpret_cast<uint4 *>(lds + swz(db * 8 + c, rb, ROWS * 2)) = o[c];
      }
    }
  }
};

// MFMA A operand for a product whose k index runs over 16 token columns of a transposed
// tile, in the order a lane holds them in a 32x32 accumulator: columns c0*8 + 4h + (0..3) and
// c0*8 + 8 + 4h + (0..3).
__device__ inline bf16x8 read_tr_frag(const char *lds, int row, int c0, int hh, int rowb) {
  Frag f;
  f.h[0] = *reinterpret_cast<const uint2 *>(lds + swz(row, c0, rowb) + 8 * hh);
  f.h[1] = *reinterpret_cast<const uint2 *>(lds + swz(row, c0 + 1, rowb) + 8 * hh);
  return f.v;
}

// ------------------------------------------------------------------ forward -------------
// grid (ceil(T/128), B*H); 4 wavefronts, each owns 32 queries; key tiles of 64.
template <int DH>
__global__ __launch_bounds__(256) void attn_fwd_mfma(const bf16_t *__restrict__ qkv, int T, int H,
                                                     bf16_t *__restrict__ o, float *__restrict__ lse) {
  constexpr int BQ = 128, BKV = 64;
  constexpr int KT = BKV * DH * 2, VT = DH * BKV * 2, STAGE = KT + VT;
  __shared__ __attribute__((aligned(16))) char smem[2 * STAGE];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6, hh = lane >> 5, lq = lane & 31;
  const int qt = gridDim.x - 1 - blockIdx.x;  // long rows first
  const int b = blockIdx.y / H, h = blockIdx.y % H;
  const int d = H * DH;
  const size_t ld3 = 3 * (size_t)d;
  const bf16_t *qbase = qkv + (size_t)b * T * ld3 + h * DH;
  const bf16_t *kbase = qbase + d, *vbase = qbase + 2 * d;
  const int q0 = qt * BQ, qw0 = q0 + 32 * wave, q = qw0 + lq;
  const int kv_end = min(T, q0 + BQ);
  const int nkv = (kv_end + BKV - 1) / BKV;

  Frag qf[DH / 16];
#pragma unroll
  for (int ks = 0; ks < DH / 16; ++ks)
    qf[ks].q = (q < T) ? ldg16(qbase + (size_t)q * ld3 + 16 * ks + 8 * hh) : make_uint4(0, 0, 0, 0);

  floatx16 oacc[DH / 32];
#pragma unroll
  for (int i = 0; i < DH / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
  float m = kNegBig, l = 0.f;
  const float sc = rsqrtf((float)DH) * kLog2e;

  RowTile<BKV, DH> lk;
  ColTile<BKV, DH> lv;
  lk.fetch(kbase, ld3, 0, T, t);
  lv.fetch(vbase, ld3, 0, T, t);
  lk.store(smem, t);
  lv.store(smem + KT, t);
  __syncthreads();

  for (int kt = 0; kt < nkv; ++kt) {
    const char *sk = smem + (kt & 1) * STAGE, *sv = sk + KT;
    const int kv0 = kt * BKV;
    if (kt + 1 < nkv) {
      lk.fetch(kbase, ld3, kv0 + BKV, T, t);
      lv.fetch(vbase, ld3, kv0 + BKV, T, t);
    }
    if (kv0 <= qw0 + 31) {  // some key of the tile is visible to some query of this wavefront
      floatx16 s[2];
#pragma unroll
      for (int a = 0; a < 2; ++a) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[a][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < DH / 16; ++ks) {
          const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(sk + swz(32 * a + lq, 2 * ks + hh, DH * 2));
          s[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks].v, s[a], 0, 0, 0);
        }
      }
      const bool diag = kv0 + BKV - 1 > qw0 || kv0 + BKV > T;
      float mx = kNegBig;
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float v = s[a][r] * sc;
          if (diag) {
            const int kv = kv0 + 32 * a + 8 * (r >> 2) + 4 * hh + (r & 3);
            if (kv > q || kv >= T) v = kNegBig;
          }
          s[a][r] = v;
          mx = fmaxf(mx, v);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float mnew = fmaxf(m, mx);
      const float alpha = exp2f(m - mnew);
      float rs = 0.f;
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = exp2f(s[a][r] - mnew);
          s[a][r] = p;
          rs += p;
        }
      l = l * alpha + rs;
      m = mnew;
#pragma unroll
      for (int i = 0; i < DH / 32; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int bq = 0; bq < 2; ++bq) {
          Frag pf;
#pragma unroll
          for (int e = 0; e < 4; ++e) pf.u[e] = pack2(s[a][8 * bq + 2 * e], s[a][8 * bq + 2 * e + 1]);
#pragma unroll
          for (int dt = 0; dt < DH / 32; ++dt) {
            const bf16x8 vf = read_tr_frag(sv, dt * 32 + lq, 4 * a + 2 * bq, hh, BKV * 2);
            oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf.v, oacc[dt], 0, 0, 0);
          }
        }
    }
    if (kt + 1 < nkv) {
      char *nk = smem + ((kt + 1) & 1) * STAGE;
      lk.store(nk, t);
      lv.store(nk + KT, t);
    }
    __syncthreads();
  }

  l += __shfl_xor(l, 32, 64);
  if (q < T) {
    const float inv = 1.f / l;
    bf16_t *op = o + ((size_t)b * T + q) * d + h * DH;
#pragma unroll
    for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 v;
        v.x = pack2(oacc[dt][4 * g] * inv, oacc[dt][4 * g + 1] * inv);
        v.y = pack2(oacc[dt][4 * g + 2] * inv, oacc[dt][4 * g + 3] * inv);
        *reinterpret_cast<uint2 *>(op + dt * 32 + 8 * g + 4 * hh) = v;
      }
    if (hh == 0) lse[((size_t)b * H + h) * T + q] = (m + log2f(l)) * kLn2;
  }
}

}  // namespace

hipError_t attention_forward_mfma(const void *qkv, int B, int T, int H, int dh, void *o, float *lse,
                                  hipStream_t s) {
  dim3 grid((T + 127) / 128, B * H);
  if (dh == 64)
    hipLaunchKernelGGL(attn_fwd_mfma<64>, grid, dim3(256), 0, s, (const bf16_t *)qkv, T, H, (bf16_t *)o, lse);
  else if (dh == 128)
    hipLaunchKernelGGL(attn_fwd_mfma<128>, grid, dim3(256), 0, s, (const bf16_t *)qkv, T, H, (bf16_t *)o, lse);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace il
