// Causal attention forward / backward on the gfx950 matrix cores for bf16 and head
// widths 64 and 128.  K/V (forward, dQ) or Q/dO (dK, dV) tiles are LDS-resident, double
// buffered and filled by direct HBM -> LDS loads; scores are never written to memory.
//
// Orientation.  Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16:
// a lane then owns ONE query column (lane & 31) and holds 16 key rows per 32x32 tile in its
// accumulator registers.  Row max / row sum of the softmax are therefore in-register
// reductions plus one exchange with lane ^ 32, and the probabilities go straight from the
// accumulators into the B operand of the second product O^T = V^T P^T without touching LDS:
// the MFMA's k index is only a summation label, so the key order a lane happens to hold
// (rows 4h..4h+3 and 8+4h..8+4h+3 of each 16-key group, h = lane >> 5) is used as is and the
// A operand V^T is fetched in the same order from the [key][dh] tile with the LDS transposing
// read (each source lane may point at any row, so no transposed copy is staged).
//
// The backward recomputes the probabilities from the saved log-sum-exp in two kernels with
// fixed reduction order (no atomics): one owns a key/value tile and accumulates dK, dV over
// the query tiles at or below the diagonal, the other owns a query tile and accumulates dQ.
#include "common.h"
#include "lds_dma.h"
#include <type_traits>

namespace il {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short short4v;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;
constexpr floatx16 kZero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

__device__ inline uint4 ldg16(const bf16_t *p) { return *reinterpret_cast<const uint4 *>(p); }
__device__ inline uint32_t pack2(float a, float b) {
  return pack_bf16x2(a, b);
}
union Frag {
  bf16x8 v;
  uint4 q;
  uint2 h[2];
  uint32_t u[4];
  short4v s[2];
};

// A [ROWS tokens] x [DH] tile of a token-major matrix, staged as is ([token][dh]) by direct
// loads (256 threads, 16 bytes each per round).  The 16-byte chunk c of row r sits at chunk
// position c ^ h(r).  LDS has 64 banks of 4 bytes: a ds_read_b128 serves 16 lanes (16 rows x 16
// bytes) per cycle and a transposing ds_read_b64_tr_b16 32 lanes (4 rows x 64 bytes), so h must
// send 16 consecutive rows to 16 different 16-byte positions of the 256-byte bank span and 4
// consecutive rows to 4 different 64-byte quarters of it.  Rows of 256 bytes or more all start at
// bank 0: h(r) = (r & 3) << 2 | (r >> 2) & 3.  Rows of 128 bytes alternate between the two halves
// of the span by themselves (bit 0 of r): h(r) = bit 1 of r << 2 | bit 2 << 1 | bit 3.  (With the
// earlier three-bit h(r) = (r & 3) << 1 | (r >> 2) & 1 the LDS counters showed every second cycle
// of these kernels' LDS activity as a bank conflict.)
template <int ROWS, int DH>
struct TokTile {
  static constexpr int RB = DH * 2, CPR = DH / 8, BYTES = ROWS * RB, NLD = BYTES / (256 * 16);
  static_assert(BYTES % (256 * 16) == 0 && NLD >= 1, "tile must divide over 256 threads");
  uint32_t voff[NLD];
  int radd[NLD];
  uint32_t rstride;
  __device__ static inline int h(int r) {
    if constexpr (DH >= 128) return ((r & 3) << 2) | ((r >> 2) & 3);
    return (((r >> 1) & 1) << 2) | (((r >> 2) & 1) << 1) | ((r >> 3) & 1);
  }
  // col0: first element column of this head; ld: elements per token row
  __device__ inline void init(int col0, int ld, int t) {
    rstride = (uint32_t)ld * 2u;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int p = i * 256 + t, row = p / CPR, chunk = (p % CPR) ^ h(row);
      radd[i] = row;
      voff[i] = ((uint32_t)row * ld + col0 + chunk * 8) * 2u;
    }
  }
  // rows [row0, row0 + ROWS) of the matrix; rows >= row_end read as zero
  __device__ inline void issue(BufRsrc rs, char *lds, int wave, int row0, int row_end) const {
    const uint32_t adv = (uint32_t)row0 * rstride;
    const uint32_t base = lds_address(lds) + wave * 1024;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const bool ok = row0 + radd[i] < row_end;
      dma16(rs, base + i * 4096, ok ? voff[i] + adv : kOob);
    }
  }
  // MFMA operand with the tile's rows as matrix rows and dh as k: rows rbase + (lane & 31),
  // dh slice [16 ks, 16 ks + 16)
  __device__ static inline bf16x8 rowfrag(const char *lds, int rbase, int ks, int lane) {
    const int row = rbase + (lane & 31), chunk = 2 * ks + (lane >> 5);
    return *reinterpret_cast<const bf16x8 *>(lds + row * RB + ((chunk ^ h(row)) << 4));
  }
  // MFMA A operand with dh as matrix rows (dt*32 + (lane & 31)) and 16 tokens as k, in the
  // order a lane holds them in a 32x32 accumulator: tokens tok0 + 4h + (0..3), tok0 + 8 + 4h + (0..3).
  __device__ static inline bf16x8 trfrag(const char *lds, int tok0, int dt, int lane) {
    const int g16 = lane >> 4, i = lane & 15;
    const int dcol = dt * 32 + 16 * (g16 & 1) + 4 * (i & 3);
    const int row = tok0 + 4 * (g16 >> 1) + (i >> 2);
    const int sub = ((dcol >> 2) & 1) * 8;
    Frag f;
    f.s[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v *)(
        lds + row * RB + (((dcol >> 3) ^ h(row)) << 4) + sub));
    f.s[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v *)(
        lds + (row + 8) * RB + (((dcol >> 3) ^ h(row + 8)) << 4) + sub));
    return f.v;
  }
};


// Which causal tile a workgroup takes.  Tiles differ in length (rank 0 = longest, rank nx-1 =
// shortest, lengths in the ratio nx : nx-1 : ... : 1) while the hardware hands workgroups to the
// chip's 8 XCDs round-robin by linear id and, inside an XCD, to its 32 CUs round-robin - the
// natural (x, y) order would give one XCD all the longest tiles and put two of them on each of
// its CUs.  Here every XCD receives the same mix of lengths, the 32 workgroups that start first
// on an XCD are its longest and the 32 that join them on the same CUs its shortest, in opposite
// order, so the two workgroups that share a CU add up to the same work everywhere; later rounds
// likewise.  Only the assignment of work to workgroups changes, never the result.
struct CausalTile {
  int rank, y;
};
__device__ inline CausalTile causal_tile() {
  const int nx = gridDim.x, ny = gridDim.y;
  const int L = blockIdx.x + nx * blockIdx.y;
  if ((ny & 7) != 0) return {(int)blockIdx.x, (int)blockIdx.y};
  const int j = L & 7, s = L >> 3, c = ny >> 3, P = nx * c;  // XCD, slot in the XCD, tiles per length and per XCD
  const int full = P & ~63, rho = s >> 6, w = s & 63;
  int i;  // position in the XCD's list of tiles sorted by decreasing length
  if (s < full)
    i = w < 32 ? 32 * rho + w : P - 1 - (32 * rho + (w - 32));
  else
    i = (full >> 1) + (s - full);
  return {i / c, j + 8 * (i % c)};
}

// ------------------------------------------------------------------ forward -------------
// grid (ceil(T/128), B*H); 4 wavefronts, each owns 32 queries; key tiles of 64.
template <int DH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(DH > 128 ? 1 : 2, DH > 128 ? 1 : 2))) void attn_fwd_mfma(const bf16_t *__restrict__ qkv, int T, int H,
                                                     bf16_t *__restrict__ o, float *__restrict__ lse) {
  constexpr int BQ = 128, BKV = DH > 128 ? 32 : 64, NA = BKV / 32;
  constexpr bool HOIST = DH <= 64;  // the wider head has no registers to spare for a whole tile of fragments
  constexpr int KT = BKV * DH * 2, STAGE = 2 * KT;
  typedef TokTile<BKV, DH> Tile;
  __shared__ __attribute__((aligned(16))) char smem[2 * STAGE];
  const int t = threadIdx.x, lane = t & 63, hh = lane >> 5, lq = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const CausalTile ct = causal_tile();
  const int qt = gridDim.x - 1 - ct.rank;  // the last query tile is the longest
  const int b = ct.y / H, h = ct.y % H;
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

  const BufRsrc rs = make_rsrc(qbase, (size_t)T * ld3 * 2 - (size_t)h * DH * 2);
  Tile lk, lv;
  lk.init(d, (int)ld3, t);
  lv.init(2 * d, (int)ld3, t);
  lk.issue(rs, smem, wave, 0, T);
  lv.issue(rs, smem + KT, wave, 0, T);

  for (int kt = 0; kt < nkv; ++kt) {
    const char *sk = smem + (kt & 1) * STAGE, *sv = sk + KT;
    const int kv0 = kt * BKV;
    wait_vmcnt<0>();
    __syncthreads();  // tile kt is complete; every wavefront is done with tile kt-1
    // A wavefront's LDS operations complete in issue order and a direct load is one of them:
    // every fragment of tile kt is requested before the loads of tile kt+1 are issued, so the
    // reads do not wait for data that is still on its way from memory.
    const bool live = kv0 <= qw0 + 31;  // some key of the tile is visible to some query of this wavefront
    bf16x8 kf[HOIST ? NA : 1][HOIST ? DH / 16 : 1], vf[HOIST ? NA : 1][2][HOIST ? DH / 32 : 1];
    auto fetch = [&]() {
      if constexpr (!HOIST) return;  // fragments are read where they are used
      if (live) {
#pragma unroll
        for (int a = 0; a < NA; ++a)
#pragma unroll
          for (int ks = 0; ks < DH / 16; ++ks) kf[a][ks] = Tile::rowfrag(sk, 32 * a, ks, lane);
#pragma unroll
        for (int a = 0; a < NA; ++a)
#pragma unroll
          for (int bq = 0; bq < 2; ++bq)
#pragma unroll
            for (int dt = 0; dt < DH / 32; ++dt) vf[a][bq][dt] = Tile::trfrag(sv, 32 * a + 16 * bq, dt, lane);
      }
    };
    auto prefetch = [&]() {
      if (kt + 1 < nkv) {
        char *nk = smem + ((kt + 1) & 1) * STAGE;
        lk.issue(rs, nk, wave, kv0 + BKV, T);
        lv.issue(rs, nk + KT, wave, kv0 + BKV, T);
      }
    };
    if constexpr (HOIST) { fetch(); prefetch(); } else { prefetch(); }
    if (live) {
      floatx16 s[NA];
#pragma unroll
      for (int a = 0; a < NA; ++a) {
        s[a] = kZero16;
#pragma unroll
        for (int ks = 0; ks < DH / 16; ++ks)
          s[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(HOIST ? kf[HOIST ? a : 0][HOIST ? ks : 0] : Tile::rowfrag(sk, 32 * a, ks, lane),
                                                         qf[ks].v, s[a], 0, 0, 0);
      }
      const bool diag = kv0 + BKV - 1 > qw0 || kv0 + BKV > T;
      float mx = kNegBig;
      // the causal / end-of-sequence mask is compiled into the diagonal tiles' path only
      auto scale_mask_max = [&](auto masked) {
#pragma unroll
        for (int a = 0; a < NA; ++a)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float v = s[a][r] * sc;
            if constexpr (decltype(masked)::value) {
              const int kv = kv0 + 32 * a + 8 * (r >> 2) + 4 * hh + (r & 3);
              if (kv > q || kv >= T) v = kNegBig;
            }
            s[a][r] = v;
            mx = fmaxf(mx, v);
          }
      };
      if (DH > 128 || diag)  // (at head width 256 a second copy of the loop costs more in registers than it saves)
        scale_mask_max(std::true_type{});
      else
        scale_mask_max(std::false_type{});
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float mnew = fmaxf(m, mx);
      const float alpha = __builtin_amdgcn_exp2f(m - mnew);
      float rs = 0.f;
#pragma unroll
      for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(s[a][r] - mnew);
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
      for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int bq = 0; bq < 2; ++bq) {
          Frag pf;
#pragma unroll
          for (int e = 0; e < 4; ++e) pf.u[e] = pack2(s[a][8 * bq + 2 * e], s[a][8 * bq + 2 * e + 1]);
#pragma unroll
          for (int dt = 0; dt < DH / 32; ++dt)
            oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                HOIST ? vf[HOIST ? a : 0][bq][HOIST ? dt : 0] : Tile::trfrag(sv, 32 * a + 16 * bq, dt, lane), pf.v, oacc[dt], 0,
                0, 0);
        }
    }
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
__device__ __forceinline__ void attn_bwd_dq_body(const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ o,
                                                 const bf16_t *__restrict__ d_o, const float *__restrict__ lse, int B,
                                                 int T, int H, bf16_t *__restrict__ dqkv, float *__restrict__ dsum) {
  constexpr int BQ = 128, BKV = 64;
  constexpr int KT = BKV * DH * 2, STAGE = 2 * KT;  // K and V tiles as stored
  typedef TokTile<BKV, DH> Tile;
  __shared__ __attribute__((aligned(16))) char smem[2 * STAGE];
  const int t = threadIdx.x, lane = t & 63, hh = lane >> 5, lq = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const CausalTile ct = causal_tile();
  const int qt = gridDim.x - 1 - ct.rank;
  const int b = ct.y / H, h = ct.y % H, sidx = blockIdx.z;
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
  const size_t sidx_row = (sidx * (size_t)B * H + ct.y) * T;
  if (q < T && hh == 0) dsum[sidx_row + q] = dsv;
  const float sc = rsqrtf((float)DH);
  const float sc2 = sc * kLog2e;
  const float lq2 = (q < T) ? lse[((size_t)b * H + h) * T + q] * kLog2e : 0.f;
  const float dsv_sc = dsv * sc;

  floatx16 dq[DH / 32];
#pragma unroll
  for (int i = 0; i < DH / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[i][r] = 0.f;

  const BufRsrc rs = make_rsrc(qbase, (size_t)T * ld3 * 2 - (size_t)h * DH * 2);
  Tile lk, lv;
  lk.init(d, (int)ld3, t);
  lv.init(2 * d, (int)ld3, t);
  lk.issue(rs, smem, wave, 0, T);
  lv.issue(rs, smem + KT, wave, 0, T);

  for (int kt = 0; kt < nkv; ++kt) {
    const char *sk = smem + (kt & 1) * STAGE, *sv = sk + KT;
    const int kv0 = kt * BKV;
    wait_vmcnt<0>();
    __syncthreads();
    if (kt + 1 < nkv) {
      char *nk = smem + ((kt + 1) & 1) * STAGE;
      lk.issue(rs, nk, wave, kv0 + BKV, T);
      lv.issue(rs, nk + KT, wave, kv0 + BKV, T);
    }
    if (kv0 <= qw0 + 31) {
      const bool diag = kv0 + BKV - 1 > qw0 || kv0 + BKV > T;
#pragma unroll(DH > 64 ? 1 : 2)
      for (int a = 0; a < 2; ++a) {
        floatx16 s = kZero16, dp = kZero16;  // a constant accumulator input costs no registers to clear
#pragma unroll
        for (int ks = 0; ks < DH / 16; ++ks) {
          const bf16x8 kf = Tile::rowfrag(sk, 32 * a, ks, lane);
          const bf16x8 vf = Tile::rowfrag(sv, 32 * a, ks, lane);
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks].v, s, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, gf[ks].v, dp, 0, 0, 0);
        }
        auto probs = [&](auto masked) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float p = __builtin_amdgcn_exp2f(s[r] * sc2 - lq2);
            if constexpr (decltype(masked)::value) {
              const int kv = kv0 + 32 * a + 8 * (r >> 2) + 4 * hh + (r & 3);
              if (kv > q || kv >= T) p = 0.f;
            }
            s[r] = p * (dp[r] * sc - dsv_sc);  // dS^T
          }
        };
        if (DH > 128 || diag)
          probs(std::true_type{});
        else
          probs(std::false_type{});
#pragma unroll
        for (int bq = 0; bq < 2; ++bq) {
          Frag pf;
#pragma unroll
          for (int e = 0; e < 4; ++e) pf.u[e] = pack2(s[8 * bq + 2 * e], s[8 * bq + 2 * e + 1]);
#pragma unroll
          for (int dt = 0; dt < DH / 32; ++dt) {
            const bf16x8 kf = Tile::trfrag(sk, 32 * a + 16 * bq, dt, lane);
            dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, pf.v, dq[dt], 0, 0, 0);
          }
        }
      }
    }
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
// grid (ceil(T/128), B*H, streams) - or streams * 2 for the split form; 4 wavefronts, each owns
// 32 keys (a lane owns one key column); query tiles of 64 from the diagonal to the end of the
// sequence.  Scores are computed as S = Q K^T with the query index in the accumulator rows, so P
// and dS feed the products dV^T = dO^T P and dK^T = Q^T dS directly from registers.
// WHAT: 0 = dK and dV in one pass; 1 = dV only; 2 = dK only.  At head width 128 the one-pass form
// holds 64 registers of K / V fragments and 128 of accumulators: it does not fit the 256
// architectural registers, runs one wavefront per SIMD and pays accumulation-register moves.  Split
// into a dV pass (K fragments, 64 accumulator registers) and a dK pass (K and V fragments, 64
// accumulator registers), both fit with two wavefronts per SIMD; the score product is computed in
// both (40 matrix instructions per 32x32 sub-tile instead of 32), which the kernel - bound by
// latency, not by the matrix unit - more than wins back.
template <int DH, int WHAT>
__device__ __forceinline__ void attn_bwd_dkv_body(const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ d_o,
                                                  const float *__restrict__ lse, const float *__restrict__ dsum, int B,
                                                  int T, int H, int sidx, bf16_t *__restrict__ dqkv, char *smem) {
  constexpr bool DO_DV = WHAT != 2, DO_DK = WHAT != 1;
  constexpr int BKV = 128, BQ = 64;
  constexpr int QT = BQ * DH * 2;                 // one staged tile
  constexpr int STAGE = 2 * QT + 2 * BQ * 4;      // Q, dO as stored, lse, dsum; smem holds two stages
  typedef TokTile<BQ, DH> Tile;
  const int t = threadIdx.x, lane = t & 63, hh = lane >> 5, lk_ = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const CausalTile ct = causal_tile();  // the first key tile is the longest
  const int b = ct.y / H, h = ct.y % H;
  const int d = H * DH;
  const size_t ld3 = 3 * (size_t)d, N = (size_t)B * T;
  const bf16_t *qbase = qkv + (size_t)b * T * ld3 + h * DH;
  const bf16_t *kbase = qbase + d, *vbase = qbase + 2 * d;
  const bf16_t *gbase = d_o + (sidx * N + (size_t)b * T) * d + h * DH;
  const float *lrow = lse + ((size_t)b * H + h) * T;
  const float *drow = dsum + (sidx * (size_t)B * H + ct.y) * T;
  const int kv0 = ct.rank * BKV, kvw0 = kv0 + 32 * wave, kv = kvw0 + lk_;
  const int qt0 = kv0 / BQ, nqt = (T + BQ - 1) / BQ;

  Frag kf[DH / 16], vf[DO_DK ? DH / 16 : 1];
#pragma unroll
  for (int ks = 0; ks < DH / 16; ++ks) {
    if (kv < T) {
      kf[ks].q = ldg16(kbase + (size_t)kv * ld3 + 16 * ks + 8 * hh);
      if constexpr (DO_DK) vf[ks].q = ldg16(vbase + (size_t)kv * ld3 + 16 * ks + 8 * hh);
    } else {
      kf[ks].q = make_uint4(0, 0, 0, 0);
      if constexpr (DO_DK) vf[ks].q = make_uint4(0, 0, 0, 0);
    }
  }
  floatx16 dk[DO_DK ? DH / 32 : 1], dv[DO_DV ? DH / 32 : 1];
#pragma unroll
  for (int i = 0; i < DH / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      if constexpr (DO_DK) dk[i][r] = 0.f;
      if constexpr (DO_DV) dv[i][r] = 0.f;
    }
  const float sc = rsqrtf((float)DH);
  const float sc2 = sc * kLog2e;

  const BufRsrc rq = make_rsrc(qbase, (size_t)T * ld3 * 2 - (size_t)h * DH * 2);
  const BufRsrc rg = make_rsrc(gbase, (size_t)T * d * 2 - (size_t)h * DH * 2);
  Tile lq, lg;
  lq.init(0, (int)ld3, t);
  lg.init(0, d, t);
  const BufRsrc rl = make_rsrc(lrow, (size_t)T * 4), rd = make_rsrc(drow, (size_t)T * 4);
  auto issue = [&](int qt, char *base) {  // direct loads of the Q and dO tiles and of 64 lse / dsum values
    const int r0 = qt * BQ;
    lq.issue(rq, base, wave, r0, T);
    lg.issue(rg, base + QT, wave, r0, T);
    if (wave == 0) dma4(rl, lds_address(base + 2 * QT), (uint32_t)(r0 + lane) * 4u);
    if (DO_DK && wave == 1) dma4(rd, lds_address(base + 2 * QT + BQ * 4), (uint32_t)(r0 + lane) * 4u);
  };
  if (qt0 < nqt) issue(qt0, smem);

  for (int qt = qt0; qt < nqt; ++qt) {
    const int it = qt - qt0;
    const char *sq = smem + (it & 1) * STAGE, *sg = sq + QT;
    const float *sl = reinterpret_cast<const float *>(sq + 2 * QT), *sd = sl + BQ;
    const int qb0 = qt * BQ;
    wait_vmcnt<0>();
    __syncthreads();
    if (qt + 1 < nqt) issue(qt + 1, smem + ((it + 1) & 1) * STAGE);
#pragma unroll(DH > 64 ? 1 : 2)
    for (int a = 0; a < BQ / 32; ++a) {
      const int qa0 = qb0 + 32 * a;
      if (qa0 + 31 < kvw0 || qa0 >= T) continue;  // every query of the sub-tile precedes every key
      floatx16 s = kZero16, dp = kZero16;
#pragma unroll
      for (int ks = 0; ks < DH / 16; ++ks) {
        const bf16x8 qf = Tile::rowfrag(sq, 32 * a, ks, lane);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kf[ks].v, s, 0, 0, 0);
        if constexpr (DO_DK) {
          const bf16x8 gf = Tile::rowfrag(sg, 32 * a, ks, lane);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gf, vf[ks].v, dp, 0, 0, 0);
        }
      }
      const bool diag = qa0 < kvw0 + 31 || qa0 + 32 > T;
      Frag pf[2], sf[2];  // P and dS of the sub-tile, packed to bf16 as they are produced
      auto probs = [&](auto masked) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const float4 l4 = *reinterpret_cast<const float4 *>(sl + 32 * a + 8 * g + 4 * hh);
          const float lv4[4] = {l4.x, l4.y, l4.z, l4.w};
          float dv4[4] = {0.f, 0.f, 0.f, 0.f};
          if constexpr (DO_DK) {
            const float4 d4 = *reinterpret_cast<const float4 *>(sd + 32 * a + 8 * g + 4 * hh);
            dv4[0] = d4.x; dv4[1] = d4.y; dv4[2] = d4.z; dv4[3] = d4.w;
          }
          float p4[4], s4[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int r = 4 * g + e;
            float p = __builtin_amdgcn_exp2f(s[r] * sc2 - lv4[e] * kLog2e);
            if constexpr (decltype(masked)::value) {
              const int qq = qa0 + 8 * g + 4 * hh + e;
              if ((DH <= 128 || diag) && (kv > qq || qq >= T)) p = 0.f;
            }
            p4[e] = p;
            s4[e] = p * (dp[r] - dv4[e]) * sc;  // dS
          }
          if constexpr (DO_DV) {
            pf[g >> 1].u[2 * (g & 1)] = pack2(p4[0], p4[1]);
            pf[g >> 1].u[2 * (g & 1) + 1] = pack2(p4[2], p4[3]);
          }
          if constexpr (DO_DK) {
            sf[g >> 1].u[2 * (g & 1)] = pack2(s4[0], s4[1]);
            sf[g >> 1].u[2 * (g & 1) + 1] = pack2(s4[2], s4[3]);
          }
        }
      };
      if (DH > 128 || diag)
        probs(std::true_type{});
      else
        probs(std::false_type{});
#pragma unroll
      for (int bq = 0; bq < 2; ++bq) {
#pragma unroll
        for (int dt = 0; dt < DH / 32; ++dt) {
          if constexpr (DO_DV) {
            const bf16x8 gt = Tile::trfrag(sg, 32 * a + 16 * bq, dt, lane);
            dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gt, pf[bq].v, dv[dt], 0, 0, 0);
          }
          if constexpr (DO_DK) {
            const bf16x8 qtf = Tile::trfrag(sq, 32 * a + 16 * bq, dt, lane);
            dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qtf, sf[bq].v, dk[dt], 0, 0, 0);
          }
        }
      }
    }
  }
  if (kv < T) {
    bf16_t *kp = dqkv + (sidx * N + (size_t)b * T + kv) * ld3 + d + h * DH;
#pragma unroll
    for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 v;
        if constexpr (DO_DK) {
          v.x = pack2(dk[dt][4 * g], dk[dt][4 * g + 1]);
          v.y = pack2(dk[dt][4 * g + 2], dk[dt][4 * g + 3]);
          *reinterpret_cast<uint2 *>(kp + dt * 32 + 8 * g + 4 * hh) = v;
        }
        if constexpr (DO_DV) {
          v.x = pack2(dv[dt][4 * g], dv[dt][4 * g + 1]);
          v.y = pack2(dv[dt][4 * g + 2], dv[dt][4 * g + 3]);
          *reinterpret_cast<uint2 *>(kp + d + dt * 32 + 8 * g + 4 * hh) = v;
        }
      }
  }
}

// The kernels proper.  With at least two wavefronts per SIMD demanded, the register budget is the
// 256 architectural VGPRs and the compiler keeps the MFMA accumulators there; without, it places
// them in the accumulation registers and moves every score to a VGPR and back (a third of the
// vector instructions at head width 64).  Head widths above 64 do not fit that budget.
template <int DH>
__global__ __launch_bounds__(256) void attn_bwd_dq_mfma(const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ o,
                                                        const bf16_t *__restrict__ d_o,
                                                        const float *__restrict__ lse, int B, int T, int H,
                                                        bf16_t *__restrict__ dqkv, float *__restrict__ dsum) {
  attn_bwd_dq_body<DH>(qkv, o, d_o, lse, B, T, H, dqkv, dsum);
}
template <int DH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void attn_bwd_dq_mfma_v(
    const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ o, const bf16_t *__restrict__ d_o,
    const float *__restrict__ lse, int B, int T, int H, bf16_t *__restrict__ dqkv, float *__restrict__ dsum) {
  attn_bwd_dq_body<DH>(qkv, o, d_o, lse, B, T, H, dqkv, dsum);
}
template <int DH>
__global__ __launch_bounds__(256) void attn_bwd_dkv_mfma(const bf16_t *__restrict__ qkv,
                                                         const bf16_t *__restrict__ d_o,
                                                         const float *__restrict__ lse,
                                                         const float *__restrict__ dsum, int B, int T, int H,
                                                         bf16_t *__restrict__ dqkv) {
  __shared__ __attribute__((aligned(16))) char smem[2 * (2 * 64 * DH * 2 + 2 * 64 * 4)];
  attn_bwd_dkv_body<DH, 0>(qkv, d_o, lse, dsum, B, T, H, blockIdx.z, dqkv, smem);
}
template <int DH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void attn_bwd_dkv_mfma_v(
    const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ d_o, const float *__restrict__ lse,
    const float *__restrict__ dsum, int B, int T, int H, bf16_t *__restrict__ dqkv) {
  __shared__ __attribute__((aligned(16))) char smem[2 * (2 * 64 * DH * 2 + 2 * 64 * 4)];
  attn_bwd_dkv_body<DH, 0>(qkv, d_o, lse, dsum, B, T, H, blockIdx.z, dqkv, smem);
}
// The split form: grid.z = 2 * streams; even z computes dK of stream z / 2 (the longer pass, dispatched
// first), odd z its dV.
template <int DH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void attn_bwd_dkv_split_mfma(
    const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ d_o, const float *__restrict__ lse,
    const float *__restrict__ dsum, int B, int T, int H, bf16_t *__restrict__ dqkv) {
  __shared__ __attribute__((aligned(16))) char smem[2 * (2 * 64 * DH * 2 + 2 * 64 * 4)];
  if (blockIdx.z & 1)
    attn_bwd_dkv_body<DH, 1>(qkv, d_o, lse, dsum, B, T, H, blockIdx.z >> 1, dqkv, smem);
  else
    attn_bwd_dkv_body<DH, 2>(qkv, d_o, lse, dsum, B, T, H, blockIdx.z >> 1, dqkv, smem);
}

}  // namespace

hipError_t attention_forward_mfma(const void *qkv, int B, int T, int H, int dh, void *o, float *lse,
                                  hipStream_t s) {
  dim3 grid((T + 127) / 128, B * H);
  if (dh == 64)
    hipLaunchKernelGGL(attn_fwd_mfma<64>, grid, dim3(256), 0, s, (const bf16_t *)qkv, T, H, (bf16_t *)o, lse);
  else if (dh == 128)
    hipLaunchKernelGGL(attn_fwd_mfma<128>, grid, dim3(256), 0, s, (const bf16_t *)qkv, T, H, (bf16_t *)o, lse);
  else if (dh == 256)
    hipLaunchKernelGGL(attn_fwd_mfma<256>, grid, dim3(256), 0, s, (const bf16_t *)qkv, T, H, (bf16_t *)o, lse);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t attention_backward_mfma(const void *qkv, const void *o, const void *d_o, const float *lse, int ns,
                                   int B, int T, int H, int dh, void *dqkv, float *dsum, hipStream_t s) {
  dim3 grid((T + 127) / 128, B * H, ns);
  if (dh == 64) {
    hipLaunchKernelGGL(attn_bwd_dq_mfma_v<64>, grid, dim3(256), 0, s, (const bf16_t *)qkv, (const bf16_t *)o,
                       (const bf16_t *)d_o, lse, B, T, H, (bf16_t *)dqkv, dsum);
    hipLaunchKernelGGL(attn_bwd_dkv_mfma_v<64>, grid, dim3(256), 0, s, (const bf16_t *)qkv, (const bf16_t *)d_o, lse,
                       dsum, B, T, H, (bf16_t *)dqkv);
  } else if (dh == 128) {
    hipLaunchKernelGGL(attn_bwd_dq_mfma_v<128>, grid, dim3(256), 0, s, (const bf16_t *)qkv, (const bf16_t *)o,
                       (const bf16_t *)d_o, lse, B, T, H, (bf16_t *)dqkv, dsum);
    hipLaunchKernelGGL(attn_bwd_dkv_split_mfma<128>, dim3(grid.x, grid.y, 2 * ns), dim3(256), 0, s, (const bf16_t *)qkv,
                       (const bf16_t *)d_o, lse, dsum, B, T, H, (bf16_t *)dqkv);
  } else if (dh == 256) {
    hipLaunchKernelGGL(attn_bwd_dq_mfma<256>, grid, dim3(256), 0, s, (const bf16_t *)qkv, (const bf16_t *)o,
                       (const bf16_t *)d_o, lse, B, T, H, (bf16_t *)dqkv, dsum);
    hipLaunchKernelGGL(attn_bwd_dkv_mfma<256>, grid, dim3(256), 0, s, (const bf16_t *)qkv, (const bf16_t *)d_o, lse,
                       dsum, B, T, H, (bf16_t *)dqkv);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace il
