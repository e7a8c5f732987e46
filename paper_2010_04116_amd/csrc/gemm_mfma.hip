// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulate,
// with the library's fused epilogues.
//
// Tiling.  A workgroup of WGM x WGN wavefronts owns a BM x BN tile of C and walks K in steps
// of 64.  Each wavefront owns (BM/WGM) x (BN/WGN) = MI x NI MFMA tiles of 32x32, all held in
// accumulator registers.  Instantiated: 256x256 with 4 or 8 wavefronts, 128x128 with 4.
//
// Operand layouts.  An operand is either "k-contiguous" ([rows, K] row-major: activations
// in forward / dgrad, weights in dgrad) or "k-major" ([K, rows] row-major: weights in
// forward, both operands of a weight gradient).
//
// Staging.  Operand tiles go HBM -> LDS directly (buffer loads with LDS destination): no
// staging registers, no ds_write instructions, and the buffer descriptor's range check
// zero-fills rows or k beyond the operand's edge without a branch.  NSTAGE LDS buffers rotate;
// one barrier per K step.  K-contiguous tiles are read with ds_read_b128, k-major tiles with
// the LDS transposing read (ds_read_b64_tr_b16), which delivers the MFMA operand order
// straight from the [k][row] image.
//
// The grid is one-dimensional; tile ids are regrouped so that the workgroups that land on
// one XCD (id mod 8) work on neighbouring tiles and share their operands in that XCD's L2.
#include <algorithm>
#include <cstring>

#include <hip/hip_ext.h>

#include "common.h"
#include "lds_dma.h"
#include <type_traits>
#include <utility>

namespace il {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;

__device__ inline void unpack8(const u32x4 v, float (&f)[8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[2 * i] = bf16_to_f32((bf16_t)(v[i] & 0xFFFFu));
    f[2 * i + 1] = bf16_to_f32((bf16_t)(v[i] >> 16));
  }
}
__device__ inline u32x4 pack8(const float (&f)[8]) {
  u32x4 v;
#pragma unroll
  for (int i = 0; i < 4; ++i) v[i] = pack_bf16x2(f[2 * i], f[2 * i + 1]);
  return v;
}

// A value from another lane of the same 16-lane row through the data-parallel path of the vector ALU (no
// LDS traffic): CTRL 0xB1 = lane ^ 1, 0x4E = lane ^ 2 (quad permutes), 0x141 = lane 7 - i of each half row.
template <int CTRL>
__device__ inline float dpp_f32(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}

// One row's eight consecutive output columns: the epilogue operation and the store.
template <int EPI>
__device__ inline void emit8(const GemmArgs &g, float4 v0, float4 v1, int grow, int gcol, const float (&bv)[8]) {
  if (grow >= g.M || gcol >= g.N) return;
  float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
  const size_t o = (size_t)grow * g.ldc + gcol;
  if constexpr (EPI == EPI_STORE) {
    *reinterpret_cast<u32x4 *>((bf16_t *)g.C + o) = pack8(v);
  } else if constexpr (EPI == EPI_LOGITS) {
    u32x4 h;
#pragma unroll
    for (int i = 0; i < 4; ++i) h[i] = pack_f16x2(v[2 * i], v[2 * i + 1]);
    *reinterpret_cast<u32x4 *>((uint16_t *)g.C + o) = h;
  } else if constexpr (EPI == EPI_BIAS) {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] += bv[e];
    *reinterpret_cast<u32x4 *>((bf16_t *)g.C + o) = pack8(v);
  } else if constexpr (EPI == EPI_BIAS_GELU) {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] += bv[e];
    const u32x4 u = pack8(v);
    *reinterpret_cast<u32x4 *>((bf16_t *)g.C + o) = u;
    unpack8(u, v);  // the activation is taken of the stored (rounded) pre-activation
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = gelu_f(v[e]);
    *reinterpret_cast<u32x4 *>((bf16_t *)g.C2 + o) = pack8(v);
  } else if constexpr (EPI == EPI_BIAS_RES) {
    const float4 r0 = *reinterpret_cast<const float4 *>(g.res + o);
    const float4 r1 = *reinterpret_cast<const float4 *>(g.res + o + 4);
    float4 o0 = {v[0] + bv[0] + r0.x, v[1] + bv[1] + r0.y, v[2] + bv[2] + r0.z, v[3] + bv[3] + r0.w};
    float4 o1 = {v[4] + bv[4] + r1.x, v[5] + bv[5] + r1.y, v[6] + bv[6] + r1.z, v[7] + bv[7] + r1.w};
    *reinterpret_cast<float4 *>((float *)g.C + o) = o0;
    *reinterpret_cast<float4 *>((float *)g.C + o + 4) = o1;
  } else if constexpr (EPI == EPI_GELU_BWD) {
    float u[8];
    unpack8(*reinterpret_cast<const u32x4 *>((const bf16_t *)g.aux + (size_t)(grow % g.aux_wrap) * g.ldc + gcol), u);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] *= gelu_grad_f(u[e]);
    *reinterpret_cast<u32x4 *>((bf16_t *)g.C + o) = pack8(v);
  } else if constexpr (EPI == EPI_STORE_F32) {
    *reinterpret_cast<float4 *>((float *)g.C + o) = v0;
    *reinterpret_cast<float4 *>((float *)g.C + o + 4) = v1;
  } else {  // EPI_WGRAD
    float *c = (float *)g.C + o;
    float4 o0 = {g.scale * v[0], g.scale * v[1], g.scale * v[2], g.scale * v[3]};
    float4 o1 = {g.scale * v[4], g.scale * v[5], g.scale * v[6], g.scale * v[7]};
    if (g.beta) {
      const float4 c0 = *reinterpret_cast<const float4 *>(c), c1 = *reinterpret_cast<const float4 *>(c + 4);
      o0.x += c0.x; o0.y += c0.y; o0.z += c0.z; o0.w += c0.w;
      o1.x += c1.x; o1.y += c1.y; o1.z += c1.z; o1.w += c1.w;
    }
    *reinterpret_cast<float4 *>(c) = o0;
    *reinterpret_cast<float4 *>(c + 4) = o1;
  }
}

// ---- epilogue shared by the kernels ---------------------------------------------------------
// A lane holds column (lane & 31) and rows 8*(r/4) + 4*(lane>>5) + (r&3) of each 32x32 block.  Each
// wavefront passes strips of 8 (64-wide wave tile) or 16 rows through an LDS region of its own so
// that every lane ends up with 8 consecutive columns of one row: 16-byte bf16 / 32-byte fp32 stores
// and equally wide reads of bias, residual and pre-activation.  No workgroup barrier is involved:
// the strip is private to the wavefront, whose LDS operations complete in issue order.
template <int WTN>
struct EpiStrip {
  static constexpr int SP = WTN + 4, LPR = WTN / 8, RPP = 64 / LPR, GPS = RPP / 8, NSTRIP = 32 / RPP;
  static constexpr int FLOATS = RPP * SP;  // per wavefront
};
template <int WTN, int EPI, int MI, int NI>
__device__ inline void epilogue_strips(const GemmArgs &g, floatx16 (&acc)[MI][NI], float *stg, int row0, int col0,
                                       int lane) {
  typedef EpiStrip<WTN> E;
  constexpr int SP = E::SP;
  const int hh = lane >> 5, lq = lane & 31;
  const int col_l = (lane % E::LPR) * 8, row_in = lane / E::LPR;
  const int gcol = col0 + col_l;
  float bv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if constexpr (EPI == EPI_BIAS || EPI == EPI_BIAS_GELU || EPI == EPI_BIAS_RES) {
    if (gcol < g.N) unpack8(*reinterpret_cast<const u32x4 *>((const bf16_t *)g.bias + gcol), bv);
  }
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int p = 0; p < E::NSTRIP; ++p) {
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int gq = 0; gq < E::GPS; ++gq)
#pragma unroll
          for (int e = 0; e < 4; ++e)
            stg[(8 * gq + 4 * hh + e) * SP + j * 32 + lq] = acc[i][j][4 * (p * E::GPS + gq) + e];
      asm volatile("" ::: "memory");
      const float4 v0 = *reinterpret_cast<const float4 *>(stg + row_in * SP + col_l);
      const float4 v1 = *reinterpret_cast<const float4 *>(stg + row_in * SP + col_l + 4);
      asm volatile("" ::: "memory");
      const int grow = row0 + i * 32 + p * E::RPP + row_in;
      if constexpr (EPI == EPI_LOGITS) {
        // Softmax statistics of this row's 64 columns from the fp32 accumulators (before any rounding):
        // the row's eight lanes (consecutive lane ids) each hold eight columns; N is a multiple of 8, so a
        // lane's columns are all inside the matrix or all outside.
        static_assert((WTN == kStatGroup && E::LPR == 8) || EPI != EPI_LOGITS, "one statistics group per wave-tile row");
        if (g.row_stats) {
          const float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
          const bool in = gcol < g.N;
          float m = -INFINITY;
#pragma unroll
          for (int e = 0; e < 8; ++e) m = fmaxf(m, in ? v[e] : -INFINITY);
          m = fmaxf(m, dpp_f32<0xB1>(m));   // lane ^ 1
          m = fmaxf(m, dpp_f32<0x4E>(m));   // lane ^ 2
          m = fmaxf(m, dpp_f32<0x141>(m));  // the other quad of the eight lanes
          float se = 0.f;
          if (in) {
            const float m2 = m * 1.4426950408889634f;
#pragma unroll
            for (int e = 0; e < 8; ++e) se += __builtin_amdgcn_exp2f(v[e] * 1.4426950408889634f - m2);
          }
          se += dpp_f32<0xB1>(se);
          se += dpp_f32<0x4E>(se);
          se += dpp_f32<0x141>(se);
          if (grow < g.M) {
            if (lane % E::LPR == 0 && col0 < g.N) {
              float *st = g.row_stats + ((size_t)grow * ((g.N + kStatGroup - 1) / kStatGroup) + col0 / kStatGroup) * 2;
              st[0] = m;
              st[1] = se;
            }
            const int tgt = g.row_targets[grow];
            if (in && tgt >= gcol && tgt < gcol + 8) {
#pragma unroll
              for (int e = 0; e < 8; ++e)
                if (gcol + e == tgt) g.row_ztgt[grow] = v[e];
            }
          }
        }
      }
      emit8<EPI>(g, v0, v1, grow, gcol, bv);
    }
}

// ------------------------------------------------------------------------------------------
// Direct loads write 16 bytes per lane at consecutive LDS addresses in lane order, so the
// LDS image of a tile is fixed and the swizzle is applied on the global side: the thread that
// fills LDS chunk position p fetches the logical chunk that belongs there.
//   k-contiguous tile: [row][BKT] (BKT*2 bytes per row), chunk c of row r at c ^ g(r)
//   k-major tile:      [k][ROWS]  (ROWS*2 bytes per k),  chunk c of k-row k at c ^ KS(k & 3), KS = 4 for k-rows of
//                      256 bytes or more (all start at bank 0 of the 64 four-byte banks: the four k-rows that one
//                      cycle of a transposing read touches, 64 bytes each, go to the four quarters of the bank
//                      span), 2 for 128-byte k-rows (which alternate between the halves of the span by themselves)
// A k-major fragment is two ds_read_b64_tr_b16: within 16 lanes, lane i points at 4
// consecutive rows-elements of k-row kb + i/4, column group 4(i%4); the instruction hands
// lane j the four k values kb..kb+3 of row j - exactly the MFMA operand order.
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short short4v;

template <int ROWS, int BKT, bool KMAJOR, int NT>
struct DmaTile {
  static constexpr int BYTES = ROWS * BKT * 2;
  static constexpr int NLD = BYTES / (NT * 16);  // loads per thread per K step
  static_assert(BYTES % (NT * 16) == 0 && NLD >= 1, "tile must divide over the threads");
  static constexpr int RB = KMAJOR ? ROWS * 2 : BKT * 2;  // LDS bytes per row
  static constexpr int KS = ROWS >= 128 ? 4 : 2;          // k-major swizzle step, in 16-byte chunks
  uint32_t voff[NLD];
  int kadd[NLD];
  uint32_t kstride;

  __device__ static inline int g(int row) { return BKT == 64 ? ((row ^ (row >> 3)) & 7) : ((row >> 1) & 3); }

  __device__ inline void init(int row0, int rows, int ld, int t) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int p = i * NT + t;
      if constexpr (!KMAJOR) {
        constexpr int CPR = BKT / 8;
        const int row = p / CPR, chunk = (p % CPR) ^ g(row);
        kadd[i] = chunk * 8;
        voff[i] = row0 + row < rows ? ((uint32_t)(row0 + row) * ld + chunk * 8) * 2u : kOob;
        kstride = 2;
      } else {
        constexpr int CPR = ROWS / 8;
        const int krow = p / CPR, chunk = (p % CPR) ^ (KS * (krow & 3));
        kadd[i] = krow;
        voff[i] = row0 + chunk * 8 < rows ? ((uint32_t)krow * ld + row0 + chunk * 8) * 2u : kOob;
        kstride = (uint32_t)ld * 2u;
      }
    }
  }
  // lds: stage base of this operand (wave-uniform); wave: wave id (uniform)
  __device__ inline void issue(BufRsrc rs, char *lds, int wave, int k0, int kend) const {
    const uint32_t adv = (uint32_t)k0 * kstride;
    const uint32_t base = lds_address(lds) + wave * 1024;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const bool ok = k0 + kadd[i] < kend;
      dma16(rs, base + i * (NT * 16), ok ? voff[i] + adv : kOob);
    }
  }
  // K-contiguous tiles with a 64-deep K step: the swizzled address of fragment (row block i, k
  // slice ks) differs from that of (0, 0) in bits 5-6 only, by an exclusive-or with a constant
  // (32 rows toggle bit 2 of g, a k slice adds 2 to the chunk index).  One lane-dependent base per
  // operand plus a constant per read costs no registers for precomputed addresses, which the
  // multiply loop of the large tile needs for its accumulators.
  static constexpr bool XOR_FORM = !KMAJOR && BKT == 64;
  __device__ static inline uint32_t lane_base(uint32_t lds_addr, int rbase0, int lane) {
    const int row = rbase0 + (lane & 31);
    return lds_addr + row * RB + ((((lane >> 5) ^ g(row)) & 7) << 4);
  }
  __device__ static inline bf16x8 frag_x(uint32_t base, int i, int ks) {
    typedef __attribute__((address_space(3))) const bf16x8 *lds_frag;
    const uint32_t a = (base ^ (uint32_t)(((2 * ks) ^ (4 * (i & 1))) << 4)) + i * 32 * RB;
    return *reinterpret_cast<lds_frag>((uintptr_t)a);
  }
  // 32 x 16 MFMA fragment of rows [rbase, rbase+32), k slice ks of the staged K step
  __device__ static inline bf16x8 frag(const char *lds, int rbase, int ks, int lane) {
    if constexpr (!KMAJOR) {
      const int row = rbase + (lane & 31), chunk = 2 * ks + (lane >> 5);
      return *reinterpret_cast<const bf16x8 *>(lds + row * RB + ((chunk ^ g(row)) << 4));
    } else {
      const int g16 = lane >> 4, i = lane & 15;
      const int m = rbase + 16 * (g16 & 1) + 4 * (i & 3);
      const int k = 16 * ks + 8 * (g16 >> 1) + (i >> 2);
      const int col = (((m >> 3) ^ (KS * (i >> 2))) << 4) + ((m >> 2) & 1) * 8;
      union { short4v h[2]; bf16x8 v; } f;
      f.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) short4v *)(lds + k * RB + col));
      f.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) short4v *)(lds + (k + 4) * RB + col));
      return f.v;
    }
  }
};

// f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{})
template <class F, int... I>
__device__ inline void static_for_impl(F &&f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ inline void static_for(F &&f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

struct GemmBatch {
  int count;
  int tile_end[kMaxBatch];  // exclusive prefix of tile counts
  GemmArgs p[kMaxBatch];
};

// Who issues the direct loads.  A wavefront's LDS operations complete in issue order and a direct
// load is one of them, so a wavefront that loads the next tile and then reads fragments of the
// current one waits for its own loads.  With LOADERS four extra wavefronts (one per SIMD) do
// nothing but load, NSTAGE-1 tiles ahead, and the multiplying wavefronts never have a load in
// their LDS queue; without, every wavefront loads its share and then multiplies (the cheaper
// arrangement when many small workgroups share a CU and cover for each other).
// LOADERS: 0 = every wavefront loads; 1 = loader wavefronts, multiply loop as the compiler
// schedules it; 2 = loader wavefronts and the hand-pipelined multiply loop (what the library uses).
constexpr int kLoaderWaves = 4;
template <int BM, int BN, int WGM, int WGN, int BKT, int NSTAGE, bool AKM, bool BKM, int EPI, int LOADERS = 0>
__global__ __launch_bounds__(64 * (WGM * WGN + (LOADERS ? kLoaderWaves : 0))) void gemm_dma_kernel(GemmBatch batch) {
  constexpr bool SPEC = LOADERS != 0, PIPE = LOADERS == 2;
  constexpr int NC = 64 * WGM * WGN;                // multiplying threads
  constexpr int NL = SPEC ? 64 * kLoaderWaves : NC;  // threads that share the loading of one tile
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int MI = WTM / 32, NI = WTN / 32;
  constexpr int ABYTES = BM * BKT * 2, STAGE = (BM + BN) * BKT * 2;
  constexpr int EPIB = WGM * WGN * EpiStrip<WTN>::FLOATS * 4;  // epilogue staging reuses the operand buffers
  __shared__ __attribute__((aligned(1024))) char smem[NSTAGE * STAGE > EPIB ? NSTAGE * STAGE : EPIB];

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave / WGN, wn = wave % WGN;

  // which problem of the batch this workgroup belongs to (uniform)
  int prob = 0, tile0 = 0;
  for (int i = 0; i < batch.count - 1; ++i)
    if ((int)blockIdx.x >= batch.tile_end[i]) { prob = i + 1; tile0 = batch.tile_end[i]; }
  const GemmArgs &g = batch.p[prob];
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  const int total = tiles_m * tiles_n;
  int pid = blockIdx.x - tile0;
  if ((total & 7) == 0) pid = (pid & 7) * (total >> 3) + (pid >> 3);
  constexpr int GM = 8;
  const int per_group = GM * tiles_n;
  const int group = pid / per_group, first_m = group * GM;
  const int gsize = min(tiles_m - first_m, GM);
  const int tm = first_m + (pid % per_group) % gsize, tn = (pid % per_group) / gsize;
  const int m0 = tm * BM, n0 = tn * BN;

  const BufRsrc ra = make_rsrc(g.A, g.a_bytes), rb = make_rsrc(g.B, g.b_bytes);
  typedef DmaTile<BM, BKT, AKM, NL> TA;
  typedef DmaTile<BN, BKT, BKM, NL> TB;
  TA la;
  TB lb;
  la.init(m0, g.M, g.lda, t % NL);
  lb.init(n0, g.N, g.ldb, t % NL);
  const int lwave = wave % (NL / 64);             // position of this wavefront among the loaders of a tile
  const bool loader = SPEC && wave >= WGM * WGN;  // this wavefront only loads (uniform)
  constexpr int LPS = TA::NLD + TB::NLD;  // loads per thread per K step
  const int kb0 = g.k_end > 0 ? g.k_begin : 0, ke = g.k_end > 0 ? g.k_end : g.K;
  const int nk = (ke - kb0 + BKT - 1) / BKT;
  auto issue = [&](int kt) {
    char *st = smem + (kt % NSTAGE) * STAGE;
    la.issue(ra, st, lwave, kb0 + kt * BKT, ke);
    lb.issue(rb, st + ABYTES, lwave, kb0 + kt * BKT, ke);
  };

  floatx16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const uint32_t xa = TA::lane_base(lds_address(smem), wm * WTM, lane);
  const uint32_t xb = TB::lane_base(lds_address(smem) + ABYTES, wn * WTN, lane);
  // K steps kt .. kt+NSTAGE-2 are in flight while step kt is multiplied; one barrier per step:
  // it publishes step kt (every loading thread waited for its own loads of it) and retires the
  // buffer of step kt-1, which the loads issued right after it overwrite.
  if (!SPEC || loader) {
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s)
      if (s < nk) issue(s);
  }
  if (loader) {
    // the same barriers as the multiplying wavefronts, through the epilogue's, then done
    for (int kt = 0; kt < nk; ++kt) {
      if (nk - 1 - kt >= NSTAGE - 2)
        wait_vmcnt<(NSTAGE - 2) * LPS>();
      else
        wait_vmcnt<0>();
      __syncthreads();
      if (kt + NSTAGE - 1 < nk) issue(kt + NSTAGE - 1);
    }
    __syncthreads();  // (the one barrier between the last multiply and the epilogue's use of the ring)
    return;
  }

  for (int kt = 0; kt < nk; ++kt) {
    if constexpr (!SPEC) {
      if (nk - 1 - kt >= NSTAGE - 2)
        wait_vmcnt<(NSTAGE - 2) * LPS>();
      else
        wait_vmcnt<0>();
    }
    __syncthreads();
    if constexpr (!SPEC) {
      if (kt + NSTAGE - 1 < nk) issue(kt + NSTAGE - 1);
    }
    const char *sa = smem + (kt % NSTAGE) * STAGE;
    const char *sb = sa + ABYTES;
    const uint32_t soff = (uint32_t)(kt % NSTAGE) * STAGE;  // (added before the exclusive-or: no carry into bits 4-6)
    if constexpr (PIPE) {
      // Software pipeline over the (k slice, row block) slots of the step: the A fragment of the next
      // slot and, two slots before a new k slice, its B fragments are requested before the MFMAs of
      // the current slot, and the scheduler is held to that order (one group of LDS reads, then the
      // slot's MFMAs), so a read's latency passes under the previous slot's matrix work.
      constexpr int KS = BKT / 16, ARD = AKM ? 2 : 1, BRD = BKM ? 2 : 1;  // LDS instructions per fragment
      auto getA = [&](int ks, int i) {
        return TA::XOR_FORM ? TA::frag_x(xa + soff, i, ks) : TA::frag(sa, wm * WTM + i * 32, ks, lane);
      };
      auto getB = [&](int ks, int j) {
        return TB::XOR_FORM ? TB::frag_x(xb + soff, j, ks) : TB::frag(sb, wn * WTN + j * 32, ks, lane);
      };
      // D slots ahead: two where the accumulators leave room for a third A fragment, else one
      constexpr int D = (MI * NI <= 4 && MI >= 2) ? 2 : 1;
      static_assert(D <= MI || MI == 1, "a k slice's B fragments are requested while the previous slice is in use");
      bf16x8 aq[D + 1], bq[2][NI];
#pragma unroll
      for (int j = 0; j < NI; ++j) bq[0][j] = getB(0, j);
#pragma unroll
      for (int p = 0; p < D; ++p)
        if (p < KS * MI) aq[p] = getA(p / MI, p % MI);
      __builtin_amdgcn_sched_group_barrier(0x100, NI * BRD + D * ARD, 0);
      static_for<KS * MI>([&](auto slot_c) {
        constexpr int slot = decltype(slot_c)::value, ks = slot / MI, i = slot % MI;
        constexpr int ahead = slot + D;
        constexpr bool nextA = ahead < KS * MI;
        constexpr bool nextB = nextA && ahead % MI == 0;
        if constexpr (nextA) aq[ahead % (D + 1)] = getA(ahead / MI, ahead % MI);
        if constexpr (nextB) {
#pragma unroll
          for (int j = 0; j < NI; ++j) bq[(ahead / MI) & 1][j] = getB(ahead / MI, j);
        }
#pragma unroll
        for (int j = 0; j < NI; ++j)
          acc[i][j] =
              __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq[slot % (D + 1)], bq[ks & 1][j], acc[i][j], 0, 0, 0);
        constexpr int reads = (nextA ? ARD : 0) + (nextB ? NI * BRD : 0);
        if constexpr (reads > 0) __builtin_amdgcn_sched_group_barrier(0x100, reads, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, NI, 0);
      });
      continue;
    }
#pragma unroll
    for (int ks = 0; ks < BKT / 16; ++ks) {
      bf16x8 af[MI], bfr[NI];
#pragma unroll
      for (int i = 0; i < MI; ++i)
        af[i] = TA::XOR_FORM ? TA::frag_x(xa + soff, i, ks) : TA::frag(sa, wm * WTM + i * 32, ks, lane);
#pragma unroll
      for (int j = 0; j < NI; ++j)
        bfr[j] = TB::XOR_FORM ? TB::frag_x(xb + soff, j, ks) : TB::frag(sb, wn * WTN + j * 32, ks, lane);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
  }
  __syncthreads();  // every wavefront is done with the ring
  epilogue_strips<WTN, EPI>(g, acc, reinterpret_cast<float *>(smem) + wave * EpiStrip<WTN>::FLOATS, m0 + wm * WTM,
                            n0 + wn * WTN, lane);
}

// ------------------------------------------------------------------------------------------
// Persistent variant of the two-stage loader kernel for launches of several rounds: one workgroup
// per CU walks over tiles blockIdx.x, blockIdx.x + gridDim.x, ...  The K steps of successive tiles
// form one sequence through the two-stage ring, so the loader wavefronts fetch the first step of the
// next tile while the multiplying wavefronts are in the epilogue of the current one, and no workgroup
// is launched per tile.  The epilogue stages 8-row strips in LDS of its own behind the ring (the ring
// is busy) and needs no workgroup barrier: a strip is private to its wavefront, whose LDS
// operations complete in order.
template <int BM, int BN, int WGM, int WGN, int BKT, bool AKM, bool BKM, int EPI>
__global__ __launch_bounds__(64 * (WGM * WGN + kLoaderWaves)) void gemm_persist_kernel(GemmBatch batch) {
  constexpr int NSTAGE = 2;
  constexpr int NC = 64 * WGM * WGN, NL = 64 * kLoaderWaves;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int MI = WTM / 32, NI = WTN / 32;
  constexpr int ABYTES = BM * BKT * 2, STAGE = (BM + BN) * BKT * 2;
  __shared__ __attribute__((aligned(1024))) char smem[NSTAGE * STAGE + WGM * WGN * EpiStrip<WTN>::FLOATS * 4];

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave / WGN, wn = wave % WGN;
  const bool loader = wave >= WGM * WGN;
  const int lwave = wave % (NL / 64);
  const int ntiles = batch.tile_end[batch.count - 1];
  typedef DmaTile<BM, BKT, AKM, NL> TA;
  typedef DmaTile<BN, BKT, BKM, NL> TB;

  // tile id -> problem, tile origin, K range (uniform)
  struct Where { int prob, m0, n0, kb0, ke, nk; };
  auto locate = [&](int tl) {
    Where w;
    w.prob = 0;
    int tile0 = 0;
    for (int i = 0; i < batch.count - 1; ++i)
      if (tl >= batch.tile_end[i]) { w.prob = i + 1; tile0 = batch.tile_end[i]; }
    const GemmArgs &g = batch.p[w.prob];
    const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    const int total = tiles_m * tiles_n;
    int pid = tl - tile0;
    if ((total & 7) == 0) pid = (pid & 7) * (total >> 3) + (pid >> 3);
    constexpr int GM = 8;
    const int per_group = GM * tiles_n;
    const int group = pid / per_group, first_m = group * GM;
    const int gsize = min(tiles_m - first_m, GM);
    w.m0 = (first_m + (pid % per_group) % gsize) * BM;
    w.n0 = ((pid % per_group) / gsize) * BN;
    w.kb0 = g.k_end > 0 ? g.k_begin : 0;
    w.ke = g.k_end > 0 ? g.k_end : g.K;
    w.nk = (w.ke - w.kb0 + BKT - 1) / BKT;
    return w;
  };

  if (loader) {
    // Step s of the sequence goes to ring slot s & 1; it is issued right after the barrier of step
    // s - 1 (which retires slot s & 1) and awaited before the barrier of step s.
    int seq = 0;
    TA la;
    TB lb;
    BufRsrc ra, rb;
    Where w = locate(blockIdx.x);
    auto setup = [&]() {
      const GemmArgs &g = batch.p[w.prob];
      ra = make_rsrc(g.A, g.a_bytes);
      rb = make_rsrc(g.B, g.b_bytes);
      la.init(w.m0, g.M, g.lda, t % NL);
      lb.init(w.n0, g.N, g.ldb, t % NL);
    };
    auto issue = [&](int kt, int slot) {
      char *st = smem + slot * STAGE;
      la.issue(ra, st, lwave, w.kb0 + kt * BKT, w.ke);
      lb.issue(rb, st + ABYTES, lwave, w.kb0 + kt * BKT, w.ke);
    };
    setup();
    issue(0, 0);
    for (int tl = blockIdx.x; tl < ntiles; tl += gridDim.x) {
      for (int kt = 0; kt < w.nk; ++kt) {
        wait_vmcnt<0>();
        __syncthreads();
        ++seq;
        if (kt + 1 < w.nk) {
          issue(kt + 1, seq & 1);
        } else if (tl + (int)gridDim.x < ntiles) {  // first step of the next tile
          w = locate(tl + gridDim.x);
          setup();
          issue(0, seq & 1);
          break;  // (w now describes the next tile)
        }
      }
    }
    wait_vmcnt<0>();
    return;
  }

  const uint32_t xa = TA::lane_base(lds_address(smem), wm * WTM, lane);
  const uint32_t xb = TB::lane_base(lds_address(smem) + ABYTES, wn * WTN, lane);
  float *stg = reinterpret_cast<float *>(smem + NSTAGE * STAGE) + wave * EpiStrip<WTN>::FLOATS;
  int seq = 0;
  for (int tl = blockIdx.x; tl < ntiles; tl += gridDim.x) {
    const Where w = locate(tl);
    const GemmArgs &g = batch.p[w.prob];
    floatx16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    for (int kt = 0; kt < w.nk; ++kt) {
      __syncthreads();
      const uint32_t soff = (uint32_t)(seq & 1) * STAGE;
      const char *sa = smem + soff, *sb = sa + ABYTES;
      ++seq;
      constexpr int KS = BKT / 16, ARD = AKM ? 2 : 1, BRD = BKM ? 2 : 1;
      auto getA = [&](int ks, int i) {
        return TA::XOR_FORM ? TA::frag_x(xa + soff, i, ks) : TA::frag(sa, wm * WTM + i * 32, ks, lane);
      };
      auto getB = [&](int ks, int j) {
        return TB::XOR_FORM ? TB::frag_x(xb + soff, j, ks) : TB::frag(sb, wn * WTN + j * 32, ks, lane);
      };
      bf16x8 aq[2], bq[2][NI];
#pragma unroll
      for (int j = 0; j < NI; ++j) bq[0][j] = getB(0, j);
      aq[0] = getA(0, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, NI * BRD + ARD, 0);
      static_for<KS * MI>([&](auto slot_c) {
        constexpr int slot = decltype(slot_c)::value, ks = slot / MI, i = slot % MI;
        constexpr int ahead = slot + 1;
        constexpr bool nextA = ahead < KS * MI;
        constexpr bool nextB = nextA && ahead % MI == 0;
        if constexpr (nextA) aq[ahead & 1] = getA(ahead / MI, ahead % MI);
        if constexpr (nextB) {
#pragma unroll
          for (int j = 0; j < NI; ++j) bq[(ahead / MI) & 1][j] = getB(ahead / MI, j);
        }
#pragma unroll
        for (int j = 0; j < NI; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq[slot & 1], bq[ks & 1][j], acc[i][j], 0, 0, 0);
        constexpr int reads = (nextA ? ARD : 0) + (nextB ? NI * BRD : 0);
        if constexpr (reads > 0) __builtin_amdgcn_sched_group_barrier(0x100, reads, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, NI, 0);
      });
    }
    epilogue_strips<WTN, EPI>(g, acc, stg, w.m0 + wm * WTM, w.n0 + wn * WTN, lane);
  }
}

thread_local const KernelTimer *tl_timer = nullptr;  // armed by gemm_time_next()

template <int BM, int BN, int WGM, int WGN, int BKT, int NSTAGE, bool AKM, bool BKM, int EPI, int LOADERS = 0>
hipError_t launch_dma(GemmBatch &b, hipStream_t s) {
  int tiles = 0;
  for (int i = 0; i < b.count; ++i) {
    tiles += ((b.p[i].M + BM - 1) / BM) * ((b.p[i].N + BN - 1) / BN);
    b.tile_end[i] = tiles;
  }
  constexpr int nthreads = 64 * (WGM * WGN + (LOADERS ? kLoaderWaves : 0));
  if (const KernelTimer *t = tl_timer) {
    tl_timer = nullptr;
    hipExtLaunchKernelGGL((gemm_dma_kernel<BM, BN, WGM, WGN, BKT, NSTAGE, AKM, BKM, EPI, LOADERS>), dim3(tiles),
                          dim3(nthreads), 0, s, t->start, t->stop, 0, b);
  } else {
    hipLaunchKernelGGL((gemm_dma_kernel<BM, BN, WGM, WGN, BKT, NSTAGE, AKM, BKM, EPI, LOADERS>), dim3(tiles),
                       dim3(nthreads), 0, s, b);
  }
  return hipGetLastError();
}

template <int BM, int BN, int WGM, int WGN, int BKT, bool AKM, bool BKM, int EPI>
hipError_t launch_persist(GemmBatch &b, hipStream_t s) {
  int tiles = 0;
  for (int i = 0; i < b.count; ++i) {
    tiles += ((b.p[i].M + BM - 1) / BM) * ((b.p[i].N + BN - 1) / BN);
    b.tile_end[i] = tiles;
  }
  constexpr int nthreads = 64 * (WGM * WGN + kLoaderWaves);
  const int grid = std::min(tiles, 256);  // one workgroup per CU
  if (const KernelTimer *t = tl_timer) {
    tl_timer = nullptr;
    hipExtLaunchKernelGGL((gemm_persist_kernel<BM, BN, WGM, WGN, BKT, AKM, BKM, EPI>), dim3(grid), dim3(nthreads), 0, s,
                          t->start, t->stop, 0, b);
  } else {
    hipLaunchKernelGGL((gemm_persist_kernel<BM, BN, WGM, WGN, BKT, AKM, BKM, EPI>), dim3(grid), dim3(nthreads), 0, s, b);
  }
  return hipGetLastError();
}

template <bool AKM, bool BKM, int EPI>
hipError_t pick_tile(GemmBatch &b, hipStream_t s) {
  long t256 = 0, t128 = 0, t64 = 0, t256x128 = 0, t128x256 = 0;
  for (int i = 0; i < b.count; ++i) {
    t256x128 += (long)((b.p[i].M + 255) / 256) * ((b.p[i].N + 127) / 128);
    t128x256 += (long)((b.p[i].M + 127) / 128) * ((b.p[i].N + 255) / 256);
    t64 += (long)((b.p[i].M + 63) / 64) * ((b.p[i].N + 63) / 64);
    t256 += (long)((b.p[i].M + 255) / 256) * ((b.p[i].N + 255) / 256);
    t128 += (long)((b.p[i].M + 127) / 128) * ((b.p[i].N + 127) / 128);
  }
  if constexpr (EPI == EPI_LOGITS) {
    // a statistics group is the 64 columns of one wave tile: every tile but the 64x64 ones (32-wide wave tiles)
    if (b.p[0].tile == 4 || b.p[0].tile == 5) return hipErrorInvalidValue;
  }
  switch (b.p[0].tile) {
    case 1: return launch_dma<256, 256, 2, 4, 64, 2, AKM, BKM, EPI, 2>(b, s);
    case 2: return launch_dma<128, 128, 2, 2, 64, 2, AKM, BKM, EPI, 2>(b, s);
    case 3: return launch_dma<128, 128, 2, 2, 64, 4, AKM, BKM, EPI, 2>(b, s);
    case 4: if constexpr (EPI != EPI_LOGITS) return launch_dma<64, 64, 2, 2, 64, 2, AKM, BKM, EPI>(b, s); else break;
    case 5: if constexpr (EPI != EPI_LOGITS) return launch_dma<64, 64, 2, 2, 64, 4, AKM, BKM, EPI, 2>(b, s); else break;
    case 6: return launch_dma<256, 128, 4, 2, 64, 3, AKM, BKM, EPI, 2>(b, s);
    case 7: return launch_dma<128, 256, 2, 4, 64, 3, AKM, BKM, EPI, 2>(b, s);
    case 8: return launch_persist<256, 256, 2, 4, 64, AKM, BKM, EPI>(b, s);
    default: break;
  }
  // Measured on MI355X, with operands that are not already in cache (inside a training step a
  // weight was last used a step ago).  With enough 256x256 tiles to cover most of the 256 CUs the
  // large tile wins (fewest operand bytes per flop).  Below that the 128x128 tile: two workgroups per
  // CU with two stages when there are more tiles than CUs, one workgroup with four stages in flight
  // when each CU gets at most one.  When even those leave CUs idle, 64x64 tiles shorten each
  // workgroup's K loop, which is what bounds such a launch: loader wavefronts and four stages while at
  // most two workgroups land on a CU (the deeper ring covers the trip to HBM), beyond that up to five
  // plain small workgroups per CU that cover for each other.
  if (t256 >= 160) return launch_persist<256, 256, 2, 4, 64, AKM, BKM, EPI>(b, s);
  if (t128 >= 192 && t128 <= 256) return launch_dma<128, 128, 2, 2, 64, 4, AKM, BKM, EPI, 2>(b, s);
  // about one 256x128 (or 128x256) tile per CU, three stages: as good as the 128x128 tile on cached
  // operands and 15-20 % better on operands from HBM (fewer bytes per flop, deeper ring)
  if (std::min(t256x128, t128x256) >= 192 && std::min(t256x128, t128x256) <= 256)
    return t128x256 <= t256x128 ? launch_dma<128, 256, 2, 4, 64, 3, AKM, BKM, EPI, 2>(b, s)
                                : launch_dma<256, 128, 4, 2, 64, 3, AKM, BKM, EPI, 2>(b, s);
  if (t128 > 256) return launch_dma<128, 128, 2, 2, 64, 2, AKM, BKM, EPI, 2>(b, s);
  if constexpr (EPI == EPI_LOGITS) {
    return launch_dma<128, 128, 2, 2, 64, 4, AKM, BKM, EPI, 2>(b, s);  // (never the 32-wide wave tiles)
  } else {
    if (t64 <= 512) return launch_dma<64, 64, 2, 2, 64, 4, AKM, BKM, EPI, 2>(b, s);
    return launch_dma<64, 64, 2, 2, 64, 2, AKM, BKM, EPI>(b, s);
  }
}

// argument checks and buffer extents of one problem
hipError_t prepare(GemmArgs &g) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipErrorInvalidValue;
  if ((g.N & 7) || (g.ldc & 7) || ((uintptr_t)g.C & 15)) return hipErrorInvalidValue;
  if ((g.lda & 7) || (g.ldb & 7) || ((uintptr_t)g.A & 15) || ((uintptr_t)g.B & 15)) return hipErrorInvalidValue;
  if (g.a_kmajor && (g.M & 7)) return hipErrorInvalidValue;
  if (g.b_kmajor && (g.N & 7)) return hipErrorInvalidValue;
  if (!g.a_kmajor && (g.K & 7)) return hipErrorInvalidValue;
  if (!g.b_kmajor && (g.K & 7)) return hipErrorInvalidValue;
  if (g.k_end < 0 || g.k_begin < 0 || g.k_end > g.K || (g.k_end > 0 && g.k_begin >= g.k_end) || (g.k_begin & 7) ||
      (g.k_end & 7))
    return hipErrorInvalidValue;
  if (g.epi == EPI_LOGITS && g.row_stats && (!g.row_targets || !g.row_ztgt)) return hipErrorInvalidValue;
  const size_t arows = g.a_kmajor ? (size_t)g.K : (size_t)g.M;
  const size_t brows = g.b_kmajor ? (size_t)g.K : (size_t)g.N;
  const size_t ab = arows * g.lda * 2, bb = brows * g.ldb * 2;  // bytes, below 2 GiB
  if (ab >= 0x7FFFFFFFull || bb >= 0x7FFFFFFFull) return hipErrorInvalidValue;
  g.a_bytes = (uint32_t)ab;
  g.b_bytes = (uint32_t)bb;
  return hipSuccess;
}

__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ part, int splits, size_t stride,
                                                            int rows, int cols, float *out, int ldc, float scale,
                                                            int beta) {
  const int c4 = cols >> 2;
  const size_t total = (size_t)rows * c4;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const int r = (int)(i / c4), c = (int)(i % c4) * 4;
    float4 a = *reinterpret_cast<const float4 *>(part + (size_t)r * cols + c);
    for (int p = 1; p < splits; ++p) {
      const float4 b = *reinterpret_cast<const float4 *>(part + p * stride + (size_t)r * cols + c);
      a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    float *o = out + (size_t)r * ldc + c;
    a.x *= scale; a.y *= scale; a.z *= scale; a.w *= scale;
    if (beta) {
      const float4 b = *reinterpret_cast<const float4 *>(o);
      a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    *reinterpret_cast<float4 *>(o) = a;
  }
}

}  // namespace

const KernelTimer *gemm_time_next(const KernelTimer *t) {
  const KernelTimer *old = tl_timer;
  tl_timer = t;
  return old;
}

// The step uses exactly these (layout, epilogue) combinations; anything else is a
// programming error in the caller and is reported instead of silently taking another path.
hipError_t gemm_bf16_batch(const GemmArgs *list, int count, hipStream_t s) {
  if (count < 1 || count > kMaxBatch) return hipErrorInvalidValue;
  GemmBatch b;
  memset(&b, 0, sizeof(b));
  b.count = count;
  for (int i = 0; i < count; ++i) {
    b.p[i] = list[i];
    if (list[i].a_kmajor != list[0].a_kmajor || list[i].b_kmajor != list[0].b_kmajor || list[i].epi != list[0].epi)
      return hipErrorInvalidValue;
    const hipError_t e = prepare(b.p[i]);
    if (e != hipSuccess) return e;
  }
  const GemmArgs &g = b.p[0];
  const int lay = g.a_kmajor * 2 + g.b_kmajor;
  switch (lay) {
    case 1:  // activations x weights[K,N]: forward linears, head logits
      switch (g.epi) {
        case EPI_STORE: return pick_tile<false, true, EPI_STORE>(b, s);
        case EPI_LOGITS: return pick_tile<false, true, EPI_LOGITS>(b, s);
        case EPI_BIAS: return pick_tile<false, true, EPI_BIAS>(b, s);
        case EPI_BIAS_GELU: return pick_tile<false, true, EPI_BIAS_GELU>(b, s);
        case EPI_BIAS_RES: return pick_tile<false, true, EPI_BIAS_RES>(b, s);
        default: return hipErrorInvalidValue;
      }
    case 0:  // dY x W^T with W stored [N,K]: data gradients
      switch (g.epi) {
        case EPI_STORE: return pick_tile<false, false, EPI_STORE>(b, s);
        case EPI_GELU_BWD: return pick_tile<false, false, EPI_GELU_BWD>(b, s);
        case EPI_STORE_F32: return pick_tile<false, false, EPI_STORE_F32>(b, s);
        default: return hipErrorInvalidValue;
      }
    case 3:  // X^T dY: weight gradients
      if (g.epi == EPI_WGRAD) return pick_tile<true, true, EPI_WGRAD>(b, s);
      return hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
  }
}

hipError_t gemm_bf16(const GemmArgs &g, hipStream_t s) { return gemm_bf16_batch(&g, 1, s); }

hipError_t splitk_reduce(const float *part, int splits, size_t stride, int rows, int cols, float *out, int ldc,
                         float scale, int beta, hipStream_t s) {
  if ((cols & 3) || (ldc & 3)) return hipErrorInvalidValue;
  size_t blocks = ((size_t)rows * (cols >> 2) + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, s, part, splits, stride, rows, cols,
                     out, ldc, scale, beta);
  return hipGetLastError();
}

hipError_t gemm_bf16_splitk(const GemmArgs &g, int splits, float *ws, hipStream_t s) {
  if (splits < 2 || splits > kMaxBatch || !ws) return hipErrorInvalidValue;
  if (g.epi != EPI_STORE_F32 && g.epi != EPI_WGRAD) return hipErrorInvalidValue;
  GemmArgs list[kMaxBatch];
  const int steps = (g.K + 63) / 64, per = (steps + splits - 1) / splits;
  int n = 0;
  for (int i = 0; i < splits; ++i) {
    const int k0 = i * per * 64, k1 = std::min(g.K, (i + 1) * per * 64);
    if (k0 >= k1) break;
    list[n] = g;
    list[n].k_begin = k0; list[n].k_end = k1;
    list[n].C = ws + (size_t)n * g.M * g.N; list[n].ldc = g.N;
    list[n].scale = 1.f; list[n].beta = 0;
    ++n;
  }
  hipError_t e = gemm_bf16_batch(list, n, s);
  if (e != hipSuccess) return e;
  return splitk_reduce(ws, n, (size_t)g.M * g.N, g.M, g.N, (float *)g.C, g.ldc, g.epi == EPI_WGRAD ? g.scale : 1.f,
                       g.epi == EPI_WGRAD ? g.beta : 0, s);
}

}  // namespace il
