// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulate,
// with the library's fused epilogues.
//
// Tiling.  A 256-thread workgroup (4 wavefronts in a 2x2 arrangement) owns a BM x BN tile
// of C and walks K in steps of 64.  Each wavefront owns (BM/2) x (BN/2) = MI x NI MFMA
// tiles of 32x32, all held in accumulator registers.  Both operand tiles are staged in LDS
// as [row][64 k] bf16 with k contiguous (128 B per row), double buffered; the next K step
// is fetched from HBM into registers while the current one is multiplied.
//
// Operand layouts.  An operand is either "k-contiguous" ([rows, K] row-major: activations
// in forward / dgrad, weights in dgrad) or "k-major" ([K, rows] row-major: weights in
// forward, both operands of a weight gradient).  K-major tiles are transposed on the way
// into LDS: a thread loads an 8(k) x 8(row) block as eight 16-byte rows, transposes it in
// registers and writes eight 16-byte k-vectors, so the MFMA operand fetch from LDS is one
// ds_read_b128 per 32x16 fragment in every case.
//
// LDS swizzle.  The 16-byte chunk c of row r lives at chunk c ^ ((r ^ (r >> 3)) & 7): eight
// consecutive rows (operand fetch, k-contiguous fill) and eight rows 8 apart (transposing
// fill) both spread over all eight chunk positions, so neither side bank-conflicts.
//
// The grid is one-dimensional; tile ids are regrouped so that the workgroups that land on
// one XCD (id mod 8) work on neighbouring tiles and share their operands in that XCD's L2.
#include "common.h"

namespace il {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr int BK = 64;           // K step, bf16 elements
constexpr int ROWB = BK * 2;     // bytes per LDS row

__device__ inline int swz(int row, int chunk) { return row * ROWB + ((chunk ^ ((row ^ (row >> 3)) & 7)) << 4); }

__device__ inline uint4 ldg16(const bf16_t *p) { return *reinterpret_cast<const uint4 *>(p); }

// 8x8 transpose of 16-bit elements: in[r] holds row r (8 elements), out[c] column c.
__device__ inline void transpose8x8(const uint4 (&in)[8], uint4 (&out)[8]) {
  const uint32_t *s = reinterpret_cast<const uint32_t *>(in);   // s[r*4 + w]
  uint32_t *o = reinterpret_cast<uint32_t *>(out);              // o[c*4 + w]
#pragma unroll
  for (int w = 0; w < 4; ++w)      // source dword = columns 2w, 2w+1
#pragma unroll
    for (int p = 0; p < 4; ++p) {  // row pair 2p, 2p+1 -> destination dword p
      uint32_t a = s[(2 * p) * 4 + w], b = s[(2 * p + 1) * 4 + w];
      o[(2 * w) * 4 + p] = (a & 0xFFFFu) | (b << 16);
      o[(2 * w + 1) * 4 + p] = (a >> 16) | (b & 0xFFFF0000u);
    }
}

// One operand tile of ROWS rows x 64 k, fetched by the whole workgroup.
template <int ROWS, bool KMAJOR>
struct TileLoader {
  static constexpr int NCH = KMAJOR ? 8 : ROWS / 32;  // 16-byte registers per thread
  uint4 r[NCH];

  // base: operand origin; row0: first tile row; rows: operand rows (bound);
  // k0: first k of this step in operand coordinates; kend: bound on k; ld: leading dimension
  __device__ inline void fetch(const bf16_t *base, int row0, int rows, long k0, long kend, int ld, int t) {
    if constexpr (!KMAJOR) {
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = t + 256 * i, row = c >> 3, kc = c & 7;
        const long k = k0 + kc * 8;
        r[i] = (row0 + row < rows && k < kend) ? ldg16(base + (size_t)(row0 + row) * ld + k)
                                                : make_uint4(0, 0, 0, 0);
      }
    } else {
      const int mb = t % (ROWS / 8), kb = t / (ROWS / 8);
      const bool on = (ROWS >= 256 || t < ROWS) && (row0 + mb * 8 < rows);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const long k = k0 + kb * 8 + i;
        r[i] = (on && k < kend) ? ldg16(base + (size_t)k * ld + row0 + mb * 8) : make_uint4(0, 0, 0, 0);
      }
    }
  }

  __device__ inline void store(char *lds, int t) const {
    if constexpr (!KMAJOR) {
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = t + 256 * i, row = c >> 3, kc = c & 7;
        *reinterpret_cast<uint4 *>(lds + swz(row, kc)) = r[i];
      }
    } else {
      if (ROWS >= 256 || t < ROWS) {
        const int mb = t % (ROWS / 8), kb = t / (ROWS / 8);
        uint4 o[8];
        transpose8x8(r, o);
#pragma unroll
        for (int c = 0; c < 8; ++c) *reinterpret_cast<uint4 *>(lds + swz(mb * 8 + c, kb)) = o[c];
      }
    }
  }
};

template <int BM, int BN, bool AKM, bool BKM, int EPI>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmArgs g) {
  constexpr int WTM = BM / 2, WTN = BN / 2;   // wavefront tile
  constexpr int MI = WTM / 32, NI = WTN / 32; // MFMA tiles per wavefront
  constexpr int STAGE = (BM + BN) * ROWB;
  __shared__ __attribute__((aligned(16))) char smem[2 * STAGE];

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // ---- tile id: XCD regrouping, then groups of 8 tile rows ----
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  const int total = tiles_m * tiles_n;
  int pid = blockIdx.x;
  if ((total & 7) == 0) pid = (pid & 7) * (total >> 3) + (pid >> 3);
  constexpr int GM = 8;
  const int per_group = GM * tiles_n;
  const int group = pid / per_group, first_m = group * GM;
  const int gsize = min(tiles_m - first_m, GM);
  const int tm = first_m + (pid % per_group) % gsize, tn = (pid % per_group) / gsize;
  const int m0 = tm * BM, n0 = tn * BN;

  const bf16_t *A = (const bf16_t *)g.A;
  const bf16_t *B = (const bf16_t *)g.B;
  TileLoader<BM, AKM> la;
  TileLoader<BN, BKM> lb;
  const int nk = (g.K + BK - 1) / BK;
  const bool seg = AKM && BKM && g.segs.nseg > 0;

  auto fetch = [&](int kt) {
    long ka = (long)kt * BK, kb = ka, kenda = g.K, kendb = g.K;
    if (seg) {  // segmented reduction: a K step never straddles two segments
      const int s = (int)(ka / g.seg_len), r = (int)(ka % g.seg_len);
      ka = r; kenda = g.seg_len;
      kb = g.segs.row0[s] + r; kendb = g.segs.row0[s] + g.seg_len;
    }
    la.fetch(A, m0, g.M, ka, kenda, g.lda, t);
    lb.fetch(B, n0, g.N, kb, kendb, g.ldb, t);
  };

  floatx16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  fetch(0);
  la.store(smem, t);
  lb.store(smem + BM * ROWB, t);
  __syncthreads();

  const int frow = lane & 31, fchunk = lane >> 5;
  for (int kt = 0; kt < nk; ++kt) {
    const char *sa = smem + (kt & 1) * STAGE;
    const char *sb = sa + BM * ROWB;
    if (kt + 1 < nk) fetch(kt + 1);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[MI], bfr[NI];
#pragma unroll
      for (int i = 0; i < MI; ++i)
        af[i] = *reinterpret_cast<const bf16x8 *>(sa + swz(wm * WTM + i * 32 + frow, 2 * ks + fchunk));
#pragma unroll
      for (int j = 0; j < NI; ++j)
        bfr[j] = *reinterpret_cast<const bf16x8 *>(sb + swz(wn * WTN + j * 32 + frow, 2 * ks + fchunk));
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
      char *na = smem + ((kt + 1) & 1) * STAGE;
      la.store(na, t);
      lb.store(na + BM * ROWB, t);
    }
    __syncthreads();
  }

  // ---- epilogue: lane holds column (lane & 31), rows 8*(r/4) + 4*(lane>>5) + (r&3) of each tile ----
  const bf16_t *bias = (const bf16_t *)g.bias;
#pragma unroll
  for (int j = 0; j < NI; ++j) {
    const int col = n0 + wn * WTN + j * 32 + (lane & 31);
    if (col >= g.N) continue;
    float bv = 0.f;
    if constexpr (EPI == EPI_BIAS || EPI == EPI_BIAS_GELU || EPI == EPI_BIAS_RES) bv = bf16_to_f32(bias[col]);
#pragma unroll
    for (int i = 0; i < MI; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * WTM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row >= g.M) continue;
        const size_t o = (size_t)row * g.ldc + col;
        float v = acc[i][j][r];
        if constexpr (EPI == EPI_STORE) {
          ((bf16_t *)g.C)[o] = f32_to_bf16(v);
        } else if constexpr (EPI == EPI_BIAS) {
          ((bf16_t *)g.C)[o] = f32_to_bf16(v + bv);
        } else if constexpr (EPI == EPI_BIAS_GELU) {
          const bf16_t u = f32_to_bf16(v + bv);
          ((bf16_t *)g.C)[o] = u;
          ((bf16_t *)g.C2)[o] = f32_to_bf16(gelu_f(bf16_to_f32(u)));
        } else if constexpr (EPI == EPI_BIAS_RES) {
          ((float *)g.C)[o] = v + bv + g.res[o];
        } else if constexpr (EPI == EPI_GELU_BWD) {
          const float u = bf16_to_f32(((const bf16_t *)g.aux)[(size_t)(row % g.aux_wrap) * g.ldc + col]);
          ((bf16_t *)g.C)[o] = f32_to_bf16(v * gelu_grad_f(u));
        } else if constexpr (EPI == EPI_STORE_F32) {
          ((float *)g.C)[o] = v;
        } else {  // EPI_WGRAD
          float *c = (float *)g.C + o;
          *c = g.scale * v + (g.beta ? *c : 0.f);
        }
      }
    }
  }
}

template <int BM, int BN, bool AKM, bool BKM, int EPI>
hipError_t launch(const GemmArgs &g, hipStream_t s) {
  const int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  hipLaunchKernelGGL((gemm_mfma_kernel<BM, BN, AKM, BKM, EPI>), dim3(tiles), dim3(256), 0, s, g);
  return hipGetLastError();
}

template <bool AKM, bool BKM, int EPI>
hipError_t pick_tile(const GemmArgs &g, hipStream_t s) {
  auto tiles = [&](int bm, int bn) { return (long)((g.M + bm - 1) / bm) * ((g.N + bn - 1) / bn); };
  if (tiles(256, 256) >= 200) return launch<256, 256, AKM, BKM, EPI>(g, s);
  if (tiles(256, 128) >= 200) return launch<256, 128, AKM, BKM, EPI>(g, s);
  return launch<128, 128, AKM, BKM, EPI>(g, s);
}

}  // namespace

// The step uses exactly these (layout, epilogue) combinations; anything else is a
// programming error in the caller and is reported instead of silently taking another path.
hipError_t gemm_bf16(const GemmArgs &g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipErrorInvalidValue;
  if ((g.lda & 7) || (g.ldb & 7) || ((uintptr_t)g.A & 15) || ((uintptr_t)g.B & 15)) return hipErrorInvalidValue;
  if (g.a_kmajor && (g.M & 7)) return hipErrorInvalidValue;
  if (g.b_kmajor && (g.N & 7)) return hipErrorInvalidValue;
  if (!g.a_kmajor && (g.K & 7)) return hipErrorInvalidValue;
  if (!g.b_kmajor && (g.K & 7)) return hipErrorInvalidValue;
  if (g.segs.nseg > 0 && (!g.a_kmajor || !g.b_kmajor || g.seg_len % BK || g.K != g.segs.nseg * g.seg_len))
    return hipErrorInvalidValue;
  const int lay = g.a_kmajor * 2 + g.b_kmajor;
  switch (lay) {
    case 1:  // activations x weights[K,N]: forward linears, head logits
      switch (g.epi) {
        case EPI_STORE: return pick_tile<false, true, EPI_STORE>(g, s);
        case EPI_BIAS: return pick_tile<false, true, EPI_BIAS>(g, s);
        case EPI_BIAS_GELU: return pick_tile<false, true, EPI_BIAS_GELU>(g, s);
        case EPI_BIAS_RES: return pick_tile<false, true, EPI_BIAS_RES>(g, s);
        default: return hipErrorInvalidValue;
      }
    case 0:  // dY x W^T with W stored [N,K]: data gradients
      switch (g.epi) {
        case EPI_STORE: return pick_tile<false, false, EPI_STORE>(g, s);
        case EPI_GELU_BWD: return pick_tile<false, false, EPI_GELU_BWD>(g, s);
        case EPI_STORE_F32: return pick_tile<false, false, EPI_STORE_F32>(g, s);
        default: return hipErrorInvalidValue;
      }
    case 3:  // X^T dY: weight gradients
      if (g.epi == EPI_WGRAD) return pick_tile<true, true, EPI_WGRAD>(g, s);
      return hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
  }
}

}  // namespace il
