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


// ------------------------------------------------------------------ backward: dQ --------
// grid (ceil(T/128), B*H, streams).  Same walk as the forward.  Also writes
// dsum[q] = sum_i dO[q,i] O[q,i] for the dK/dV kernel.
template <int DH>
__global__ __launch_bounds__(256) void attn_bwd_dq_mfma(const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ o,
                                                        const bf16_t *__restrict__ d_o,
                                                        const float *__restrict__ lse, int B, int T, int H,
                                                        bf16_t *__restrict__ dqkv, float *__restrict__ dsum) {
  constexpr int BQ = 128, BKV = 64;
  constexpr int KT = BKV * DH * 2, STAGE = 3 * KT;  // K, V as stored, K transposed
  __shared__ __attribute__((aligned(16))) char smem[2 * STAGE];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6, hh = lane >> 5, lq = lane & 31;
  const int qt = gridDim.x - 1 - blockIdx.x;
  const int b = blockIdx.y / H, h = blockIdx.y % H, sidx = blockIdx.z;
  const int d = H * DH;
  const size_t ld3 = 3 * (size_t)d, N = (size_t)B * T;
  const bf16_t *qbase = qkv + (size_t)b * T * ld3 + h * DH;
  const bf16_t *kbase = qbase + d, *vbase = qbase + 2 * d;
  const int q0 = qt * BQ, qw0 = q0 + 32 * wave, q = qw0 + lq;
  const int kv_end = min(T, q0 + BQ);
  const int nkv = (kv_end + BKV - 1) / BKV;
  const size_t tok = (size_t)b * T + q;

  Frag qf[DH / 16], gf[DH / 16];
  float dsv = 0.f;
#pragma unroll
  for (int ks = 0; ks < DH / 16; ++ks) {
    Frag of;
    if (q < T) {
      qf[ks].q = ldg16(qbase + (size_t)q * ld3 + 16 * ks + 8 * hh);
      gf[ks].q = ldg16(d_o + (sidx * N + tok) * d + h * DH + 16 * ks + 8 * hh);
      of.q = ldg16(o + tok * d + h * DH + 16 * ks + 8 * hh);
    } else {
      qf[ks].q = make_uint4(0, 0, 0, 0);
      gf[ks].q = make_uint4(0, 0, 0, 0);
      of.q = make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      dsv += bf16_to_f32((bf16_t)(gf[ks].u[e] & 0xFFFF)) * bf16_to_f32((bf16_t)(of.u[e] & 0xFFFF));
      dsv += bf16_to_f32((bf16_t)(gf[ks].u[e] >> 16)) * bf16_to_f32((bf16_t)(of.u[e] >> 16));
    }
  }
  dsv += __shfl_xor(dsv, 32, 64);
  const size_t sidx_row = (sidx * (size_t)B * H + blockIdx.y) * T;
  if (q < T && hh == 0) dsum[sidx_row + q] = dsv;
  const float sc = rsqrtf((float)DH);
  const float sc2 = sc * kLog2e;
  const float lq2 = (q < T) ? lse[((size_t)b * H + h) * T + q] * kLog2e : 0.f;

  floatx16 dq[DH / 32];
#pragma unroll
  for (int i = 0; i < DH / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[i][r] = 0.f;

  RowTile<BKV, DH> lk, lv;
  ColTile<BKV, DH> lkt;
  lk.fetch(kbase, ld3, 0, T, t);
  lv.fetch(vbase, ld3, 0, T, t);
  lkt.fetch(kbase, ld3, 0, T, t);
  lk.store(smem, t);
  lv.store(smem + KT, t);
  lkt.store(smem + 2 * KT, t);
  __syncthreads();

  for (int kt = 0; kt < nkv; ++kt) {
    const char *sk = smem + (kt & 1) * STAGE, *sv = sk + KT, *skt = sk + 2 * KT;
    const int kv0 = kt * BKV;
    if (kt + 1 < nkv) {
      lk.fetch(kbase, ld3, kv0 + BKV, T, t);
      lv.fetch(vbase, ld3, kv0 + BKV, T, t);
      lkt.fetch(kbase, ld3, kv0 + BKV, T, t);
    }
    if (kv0 <= qw0 + 31) {
      const bool diag = kv0 + BKV - 1 > qw0 || kv0 + BKV > T;
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        floatx16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < DH / 16; ++ks) {
          const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(sk + swz(32 * a + lq, 2 * ks + hh, DH * 2));
          const bf16x8 vf = *reinterpret_cast<const bf16x8 *>(sv + swz(32 * a + lq, 2 * ks + hh, DH * 2));
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks].v, s, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, gf[ks].v, dp, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float p = exp2f(s[r] * sc2 - lq2);
          if (diag) {
            const int kv = kv0 + 32 * a + 8 * (r >> 2) + 4 * hh + (r & 3);
            if (kv > q || kv >= T) p = 0.f;
          }
          s[r] = p * (dp[r] - dsv) * sc;  // dS^T
        }
#pragma unroll
        for (int bq = 0; bq < 2; ++bq) {
          Frag pf;
#pragma unroll
          for (int e = 0; e < 4; ++e) pf.u[e] = pack2(s[8 * bq + 2 * e], s[8 * bq + 2 * e + 1]);
#pragma unroll
          for (int dt = 0; dt < DH / 32; ++dt) {
            const bf16x8 kf = read_tr_frag(skt, dt * 32 + lq, 4 * a + 2 * bq, hh, BKV * 2);
            dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, pf.v, dq[dt], 0, 0, 0);
          }
        }
      }
    }
    if (kt + 1 < nkv) {
      char *nk = smem + ((kt + 1) & 1) * STAGE;
      lk.store(nk, t);
      lv.store(nk + KT, t);
      lkt.store(nk + 2 * KT, t);
    }
    __syncthreads();
  }
  if (q < T) {
    bf16_t *op = dqkv + (sidx * N + tok) * ld3 + h * DH;
#pragma unroll
    for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 v;
        v.x = pack2(dq[dt][4 * g], dq[dt][4 * g + 1]);
        v.y = pack2(dq[dt][4 * g + 2], dq[dt][4 * g + 3]);
        *reinterpret_cast<uint2 *>(op + dt * 32 + 8 * g + 4 * hh) = v;
      }
  }
}

// ------------------------------------------------------------------ backward: dK, dV ----
// grid (ceil(T/128), B*H, streams); 4 wavefronts, each owns 32 keys (a lane owns one key
// column); query tiles of 64 from the diagonal to the end of the sequence.  Scores are
// computed as S = Q K^T with the query index in the accumulator rows, so P and dS feed the
// products dV^T = dO^T P and dK^T = Q^T dS directly from registers.
template <int DH>
__global__ __launch_bounds__(256) void attn_bwd_dkv_mfma(const bf16_t *__restrict__ qkv,
                                                         const bf16_t *__restrict__ d_o,
                                                         const float *__restrict__ lse,
                                                         const float *__restrict__ dsum, int B, int T, int H,
                                                         bf16_t *__restrict__ dqkv) {
  constexpr int BKV = 128, BQ = 64;
  constexpr int QT = BQ * DH * 2;                 // one staged tile
  constexpr int STAGE = 4 * QT + 2 * BQ * 4;      // Q, dO, Q^T, dO^T, lse, dsum
  __shared__ __attribute__((aligned(16))) char smem[2 * STAGE];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6, hh = lane >> 5, lk_ = lane & 31;
  const int b = blockIdx.y / H, h = blockIdx.y % H, sidx = blockIdx.z;
  const int d = H * DH;
  const size_t ld3 = 3 * (size_t)d, N = (size_t)B * T;
  const bf16_t *qbase = qkv + (size_t)b * T * ld3 + h * DH;
  const bf16_t *kbase = qbase + d, *vbase = qbase + 2 * d;
  const bf16_t *gbase = d_o + (sidx * N + (size_t)b * T) * d + h * DH;
  const float *lrow = lse + ((size_t)b * H + h) * T;
  const float *drow = dsum + (sidx * (size_t)B * H + blockIdx.y) * T;
  const int kv0 = blockIdx.x * BKV, kvw0 = kv0 + 32 * wave, kv = kvw0 + lk_;
  const int qt0 = kv0 / BQ, nqt = (T + BQ - 1) / BQ;

  Frag kf[DH / 16], vf[DH / 16];
#pragma unroll
  for (int ks = 0; ks < DH / 16; ++ks) {
    if (kv < T) {
      kf[ks].q = ldg16(kbase + (size_t)kv * ld3 + 16 * ks + 8 * hh);
      vf[ks].q = ldg16(vbase + (size_t)kv * ld3 + 16 * ks + 8 * hh);
    } else {
      kf[ks].q = make_uint4(0, 0, 0, 0);
      vf[ks].q = make_uint4(0, 0, 0, 0);
    }
  }
  floatx16 dk[DH / 32], dv[DH / 32];
#pragma unroll
  for (int i = 0; i < DH / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dk[i][r] = 0.f; dv[i][r] = 0.f; }
  const float sc = rsqrtf((float)DH);
  const float sc2 = sc * kLog2e;

  RowTile<BQ, DH> lq, lg;
  ColTile<BQ, DH> lqt, lgt;
  float pl = 0.f, pd = 0.f;  // lse / dsum prefetch (threads 0..63)
  auto fetch = [&](int qt) {
    const int r0 = qt * BQ;
    lq.fetch(qbase, ld3, r0, T, t);
    lg.fetch(gbase, d, r0, T, t);
    lqt.fetch(qbase, ld3, r0, T, t);
    lgt.fetch(gbase, d, r0, T, t);
    if (t < BQ) {
      const bool in = r0 + t < T;
      pl = in ? lrow[r0 + t] * kLog2e : 0.f;
      pd = in ? drow[r0 + t] : 0.f;
    }
  };
  auto stage = [&](char *base) {
    lq.store(base, t);
    lg.store(base + QT, t);
    lqt.store(base + 2 * QT, t);
    lgt.store(base + 3 * QT, t);
    if (t < BQ) {
      reinterpret_cast<float *>(base + 4 * QT)[t] = pl;
      reinterpret_cast<float *>(base + 4 * QT + BQ * 4)[t] = pd;
    }
  };
  if (qt0 < nqt) {
    fetch(qt0);
    stage(smem);
  }
  __syncthreads();

  for (int qt = qt0; qt < nqt; ++qt) {
    const int it = qt - qt0;
    const char *sq = smem + (it & 1) * STAGE, *sg = sq + QT, *sqt = sq + 2 * QT, *sgt = sq + 3 * QT;
    const float *sl = reinterpret_cast<const float *>(sq + 4 * QT), *sd = sl + BQ;
    const int qb0 = qt * BQ;
    if (qt + 1 < nqt) fetch(qt + 1);
#pragma unroll
    for (int a = 0; a < BQ / 32; ++a) {
      const int qa0 = qb0 + 32 * a;
      if (qa0 + 31 < kvw0 || qa0 >= T) continue;  // every query of the sub-tile precedes every key
      floatx16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < DH / 16; ++ks) {
        const bf16x8 qf = *reinterpret_cast<const bf16x8 *>(sq + swz(32 * a + lk_, 2 * ks + hh, DH * 2));
        const bf16x8 gf = *reinterpret_cast<const bf16x8 *>(sg + swz(32 * a + lk_, 2 * ks + hh, DH * 2));
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kf[ks].v, s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gf, vf[ks].v, dp, 0, 0, 0);
      }
      const bool diag = qa0 < kvw0 + 31 || qa0 + 32 > T;
      floatx16 pr;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 l4 = *reinterpret_cast<const float4 *>(sl + 32 * a + 8 * g + 4 * hh);
        const float4 d4 = *reinterpret_cast<const float4 *>(sd + 32 * a + 8 * g + 4 * hh);
        const float lv4[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = 4 * g + e;
          float p = exp2f(s[r] * sc2 - lv4[e]);
          if (diag) {
            const int qq = qa0 + 8 * g + 4 * hh + e;
            if (kv > qq || qq >= T) p = 0.f;
          }
          pr[r] = p;
          s[r] = p * (dp[r] - dv4[e]) * sc;  // dS
        }
      }
#pragma unroll
      for (int bq = 0; bq < 2; ++bq) {
        Frag pf, sf;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          pf.u[e] = pack2(pr[8 * bq + 2 * e], pr[8 * bq + 2 * e + 1]);
          sf.u[e] = pack2(s[8 * bq + 2 * e], s[8 * bq + 2 * e + 1]);
        }
#pragma unroll
        for (int dt = 0; dt < DH / 32; ++dt) {
          const bf16x8 gt = read_tr_frag(sgt, dt * 32 + lk_, 4 * a + 2 * bq, hh, BQ * 2);
          const bf16x8 qtf = read_tr_frag(sqt, dt * 32 + lk_, 4 * a + 2 * bq, hh, BQ * 2);
          dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gt, pf.v, dv[dt], 0, 0, 0);
          dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qtf, sf.v, dk[dt], 0, 0, 0);
        }
      }
    }
    if (qt + 1 < nqt) stage(smem + ((it + 1) & 1) * STAGE);
    __syncthreads();
  }
  if (kv < T) {
    bf16_t *kp = dqkv + (sidx * N + (size_t)b * T + kv) * ld3 + d + h * DH;
#pragma unroll
    for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 v;
        v.x = pack2(dk[dt][4 * g], dk[dt][4 * g + 1]);
        v.y = pack2(dk[dt][4 * g + 2], dk[dt][4 * g + 3]);
        *reinterpret_cast<uint2 *>(kp + dt * 32 + 8 * g + 4 * hh) = v;
        v.x = pack2(dv[dt][4 * g], dv[dt][4 * g + 1]);
        v.y = pack2(dv[dt][4 * g + 2], dv[dt][4 * g + 3]);
        *reinterpret_cast<uint2 *>(kp + d + dt * 32 + 8 * g + 4 * hh) = v;
      }
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

hipError_t attention_backward_mfma(const void *qkv, const void *o, const void *d_o, const float *lse, int ns,
                                   int B, int T, int H, int dh, void *dqkv, float *dsum, hipStream_t s) {
  dim3 grid((T + 127) / 128, B * H, ns);
  if (dh == 64) {
    hipLaunchKernelGGL(attn_bwd_dq_mfma<64>, grid, dim3(256), 0, s, (const bf16_t *)qkv, (const bf16_t *)o,
                       (const bf16_t *)d_o, lse, B, T, H, (bf16_t *)dqkv, dsum);
    hipLaunchKernelGGL(attn_bwd_dkv_mfma<64>, grid, dim3(256), 0, s, (const bf16_t *)qkv, (const bf16_t *)d_o, lse,
                       dsum, B, T, H, (bf16_t *)dqkv);
  } else if (dh == 128) {
    hipLaunchKernelGGL(attn_bwd_dq_mfma<128>, grid, dim3(256), 0, s, (const bf16_t *)qkv, (const bf16_t *)o,
                       (const bf16_t *)d_o, lse, B, T, H, (bf16_t *)dqkv, dsum);
    hipLaunchKernelGGL(attn_bwd_dkv_mfma<128>, grid, dim3(256), 0, s, (const bf16_t *)qkv, (const bf16_t *)d_o, lse,
                       dsum, B, T, H, (bf16_t *)dqkv);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace il
