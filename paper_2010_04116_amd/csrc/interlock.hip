// libinterlock: context, routing plan, workspace layout and the C-ABI entry points.
// The step is K x (il_stage_forward, il_head_xent) followed by il_stage_backward_nwise
// for k = K..1.  Gradient streams (one per head, merged where they share their remaining
// route) live in fp32 "slots" ordered by the lowest component they reach.  Under the
// window-sum and far-head routings the streams live at any component occupy adjacent
// slots, i.e. one contiguous stack [cnt*N, d], and every backward GEMM processes all of
// them in a single launch; where the live slots are not adjacent the component's backward
// runs once per contiguous range and the later ranges accumulate.
#include "../../include/interlock.h"
#include "../../include/interlock_test.h"

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "common.h"

using namespace il;

namespace il {
hipError_t attention_forward_simt(int, const void *, int, int, int, int, void *, float *, hipStream_t);
hipError_t attention_backward_simt(int, const void *, const void *, const void *, const float *, int, int, int,
                                   int, int, void *, float *, hipStream_t);
}  // namespace il

namespace {

// ------------------------------------------------------------------ routing plan ----
struct StreamDesc {
  int lo, hi;  // lowest / highest component the stream passes through (1-based)
};
struct Run {                    // a contiguous range of live slots, processed as one stack
  int s0 = 0, cnt = 0;          // slots [s0, s0+cnt)
  float wt[kMaxStreams] = {};   // routing weight of each stream at this component
  int nweighted = 0;            // streams with non-zero weight
  int first_weighted = -1;      // index of the first of them in the stack
  float wscale = 1.f;           // weight of the last of them (used when there is exactly one)
  int acc = 0;                  // 1: parameter gradients add to what an earlier run wrote
};
struct CompPlan {
  std::vector<Run> runs;        // usually one; several only when the live slots are not adjacent
  int cnt = 0;                  // live streams in total
  int inject_slot = -1;         // slot head k's fresh gradient joins, -1: head k is not used
  int inject_acc = 0;           // 1: add to the stream already in the slot
  int passes = 0;               // heads whose gradient passes through this component
};
struct Plan {
  int K = 0, nslots = 0, maxcnt = 0;
  std::vector<StreamDesc> streams;
  std::vector<CompPlan> comp;   // index k-1
};

int route_weights(int K, int n, int route, std::vector<double> &w) {
  if (K < 1 || n < 1 || n > K) return IL_E_ARG;
  w.assign((size_t)K * K, 0.0);
  for (int k = 1; k <= K; ++k) {
    const int far = std::min(k + n - 1, K);
    switch (route) {
      case IL_ROUTE_WINDOW_SUM:
        for (int j = k; j <= far; ++j) w[(k - 1) * K + j - 1] = 1.0;
        break;
      case IL_ROUTE_FAR_HEAD: w[(k - 1) * K + far - 1] = 1.0; break;
      case IL_ROUTE_MEAN_LOCAL_FAR:
        w[(k - 1) * K + k - 1] += 0.5;
        w[(k - 1) * K + far - 1] += 0.5;
        break;
      default: return IL_E_ARG;
    }
  }
  return IL_OK;
}

int build_plan(int K, int n, int route, Plan &p) {
  std::vector<double> w;
  int rc = route_weights(K, n, route, w);
  if (rc) return rc;
  auto W = [&](int k, int j) { return w[(size_t)(k - 1) * K + j - 1]; };
  p = Plan();
  p.K = K;
  p.comp.assign(K, CompPlan());
  std::vector<int> lo(K + 1, 0), group(K + 1, -1);
  for (int j = 1; j <= K; ++j)
    for (int k = 1; k <= j; ++k)
      if (W(k, j) != 0.0) { lo[j] = k; break; }
  // group heads top-down: head j joins a stream created by a higher head when both stop at
  // the same component and carry the same weights over every component they share
  struct G { int lo, hi; };
  std::vector<G> groups;
  for (int j = K; j >= 1; --j) {
    if (!lo[j]) continue;
    int found = -1;
    for (size_t g = 0; g < groups.size() && found < 0; ++g) {
      if (groups[g].lo != lo[j]) continue;
      bool same = true;
      for (int k = lo[j]; k <= j; ++k) same = same && (W(k, j) == W(k, groups[g].hi));
      if (same) found = (int)g;
    }
    if (found < 0) { groups.push_back({lo[j], j}); found = (int)groups.size() - 1; }
    group[j] = found;
  }
  // slots: ascending (lo, hi)
  std::vector<int> order(groups.size());
  for (size_t i = 0; i < order.size(); ++i) order[i] = (int)i;
  for (size_t a = 0; a < order.size(); ++a)
    for (size_t b = a + 1; b < order.size(); ++b) {
      const G &x = groups[order[a]], &y = groups[order[b]];
      if (y.lo < x.lo || (y.lo == x.lo && y.hi < x.hi)) std::swap(order[a], order[b]);
    }
  std::vector<int> slot_of(groups.size());
  for (size_t s = 0; s < order.size(); ++s) {
    slot_of[order[s]] = (int)s;
    p.streams.push_back({groups[order[s]].lo, groups[order[s]].hi});
  }
  p.nslots = (int)groups.size();
  for (int k = 1; k <= K; ++k) {
    CompPlan &c = p.comp[k - 1];
    bool written = false;
    for (int s = 0; s < p.nslots; ++s) {
      if (!(p.streams[s].lo <= k && k <= p.streams[s].hi)) continue;
      if (c.runs.empty() || c.runs.back().s0 + c.runs.back().cnt != s || c.runs.back().cnt == kMaxStreams) {
        Run r;
        r.s0 = s;
        c.runs.push_back(r);
      }
      const float wt = (float)W(k, p.streams[s].hi);
      Run &q = c.runs.back();
      q.wt[q.cnt] = wt;
      if (wt != 0.f) {
        q.wscale = wt;
        if (q.nweighted++ == 0) q.first_weighted = q.cnt;
      }
      ++q.cnt;
      ++c.cnt;
    }
    for (Run &r : c.runs) {
      p.maxcnt = std::max(p.maxcnt, r.cnt);
      if (r.nweighted) { r.acc = written; written = true; }
    }
    if (!written) return IL_E_ARG;  // a component no loss is credited to
    for (int j = k; j <= K; ++j)
      if (lo[j] && lo[j] <= k) ++c.passes;
    if (lo[k]) {
      c.inject_slot = slot_of[group[k]];
      c.inject_acc = (groups[group[k]].hi != k);
    }
  }
  return IL_OK;
}

// ------------------------------------------------------------------ context --------
enum KClass { KC_GEMM_FWD, KC_GEMM_DGRAD, KC_GEMM_WGRAD, KC_GEMM_HEAD, KC_ATTN_FWD, KC_ATTN_BWD, KC_LN_FWD,
              KC_LN_BWD, KC_COLSUM, KC_XENT, KC_MISC, KC_COUNT };
const char *kClassNames[KC_COUNT] = {"gemm_fwd", "gemm_dgrad", "gemm_wgrad", "gemm_head", "attn_fwd", "attn_bwd",
                                     "ln_fwd",   "ln_bwd",     "colsum",     "xent",      "misc"};

struct BlockOff {  // element offsets inside the flat parameter / gradient buffers
  size_t ln1_g, ln1_b, w_qkv, b_qkv, w_o, b_o, ln2_g, ln2_b, w_fc1, b_fc1, w_fc2, b_fc2;
};
struct BlockSave {  // workspace pointers of one block's saved activations
  float *xs, *st1, *lse, *a, *st2;
  char *h1, *qkv, *o, *h2, *u, *gl;
};
struct ProfRec { int cls; bool kernel, bracket; hipEvent_t e0, e1; KernelTimer kt; };

}  // namespace

struct il_ctx {
  il_config cfg;
  Plan plan;
  int N, d, m, V, H, dh, L, K, eb, Lh;
  hipStream_t stream;
  std::vector<BlockOff> boff;      // K*L
  std::vector<size_t> hoff;        // K
  std::vector<BlockSave> save;     // K*L
  std::vector<BlockOff> hboff;     // K*Lh: the heads' own blocks
  std::vector<BlockSave> hsave;    // K*Lh
  float *hy = nullptr;             // output of a head's last block, fp32 [N,d]
  int accumulate = 0;              // micro-batching: add into grads instead of overwriting
  float grad_scale = 1.f;          // ... and scale every gradient (applied to dlogits)
  bool tail_inline = false;        // block_backward is running on the side stream already (inside a head)
  float *G; char *Gb;              // stream slots [nslots][N,d]
  char *DU, *DH, *DQKV, *YS[4]; float *dsum, *partials[6], *skws; size_t skws_floats; ColsumJobs jobs;
  // The end of a block's backward (final column sums, the four weight gradients) runs on the side
  // stream while the main stream goes on with the next block: its inputs are double-buffered.
  char *YS2[2][4]; float *partials2[2][6];
  int bparity = 0;
  hipEvent_t ev_blk_ready[2] = {nullptr, nullptr}, ev_blk_done[2] = {nullptr, nullptr};
  char blk_pending[2] = {0, 0};
  // bf16: the stream sums / first-stage column sums of a block (two launches) also run on the side
  // stream; Gb_alt is the second home of the bf16 gradient stream that makes this possible
  char *Gb_alt = nullptr;
  hipEvent_t ev_fl_ready[2] = {nullptr, nullptr}, ev_fl_done[2] = {nullptr, nullptr};
  char fl_pending[2] = {0, 0};
  bool flush_async = false;
  int flush_idx = 0;
  SumColsumJobs pending; float *pending_out[kMaxSumColsumJobs]; int pending_acc[kMaxSumColsumJobs];
  double pending_bytes = 0;
  char *xb, *Z; float *rowloss, *dxh, *hstats = nullptr, *hztgt = nullptr;
  int Nc;
  std::vector<char> fwd_done, head_done, bwd_done;
  // heads run on a side stream, concurrently with the next component's forward
  hipStream_t main_stream = nullptr, side = nullptr;
  hipEvent_t ev_fork = nullptr;
  std::vector<hipEvent_t> ev_head;   // K: head k finished (side stream)
  std::vector<char> head_pending;    // main stream has not yet waited for ev_head[k]
  // profiling
  std::vector<ProfRec> recs; size_t nrec = 0;
  double flops[KC_COUNT] = {}, bytes[KC_COUNT] = {};
};

namespace {

struct Carver {
  char *base; size_t off = 0;
  explicit Carver(void *b) : base((char *)b) {}
  void *take(size_t bytes) {
    void *p = base ? base + off : nullptr;
    off += (bytes + 255) & ~(size_t)255;
    return p;
  }
};

size_t layout_params(il_ctx *c) {
  const size_t d = c->d, m = c->m;
  size_t o = 0;
  c->boff.resize((size_t)c->K * c->L);
  for (auto &b : c->boff) {
    b.ln1_g = o; o += d; b.ln1_b = o; o += d; b.w_qkv = o; o += 3 * d * d; b.b_qkv = o; o += 3 * d;
    b.w_o = o; o += d * d; b.b_o = o; o += d; b.ln2_g = o; o += d; b.ln2_b = o; o += d;
    b.w_fc1 = o; o += d * m; b.b_fc1 = o; o += m; b.w_fc2 = o; o += m * d; b.b_fc2 = o; o += d;
  }
  auto lay = [&](BlockOff &b) {
    b.ln1_g = o; o += d; b.ln1_b = o; o += d; b.w_qkv = o; o += 3 * d * d; b.b_qkv = o; o += 3 * d;
    b.w_o = o; o += d * d; b.b_o = o; o += d; b.ln2_g = o; o += d; b.ln2_b = o; o += d;
    b.w_fc1 = o; o += d * m; b.b_fc1 = o; o += m; b.w_fc2 = o; o += m * d; b.b_fc2 = o; o += d;
  };
  c->hoff.resize(c->K);
  c->hboff.resize((size_t)c->K * c->Lh);
  for (int k = 0; k < c->K; ++k) {
    for (int l = 0; l < c->Lh; ++l) lay(c->hboff[(size_t)k * c->Lh + l]);
    c->hoff[k] = o; o += d * (size_t)c->V;
  }
  return o;
}

// bf16: (max, sum-exp) per row of the logits tile and per group of kStatGroup vocabulary columns
size_t head_stats_bytes(const il_ctx *c) {
  return c->eb == 2 ? (size_t)c->Nc * ((c->V + kStatGroup - 1) / kStatGroup) * 2 * 4 : 0;
}

size_t layout_workspace(il_ctx *c, void *base) {
  Carver cv(base);
  const size_t N = c->N, d = c->d, m = c->m, eb = c->eb, H = c->H;
  c->save.resize((size_t)c->K * c->L);
  for (auto &s : c->save) {
    s.xs = (float *)cv.take(N * d * 4); s.st1 = (float *)cv.take(N * 2 * 4);
    s.h1 = (char *)cv.take(N * d * eb); s.qkv = (char *)cv.take(N * 3 * d * eb);
    s.lse = (float *)cv.take(N * H * 4); s.o = (char *)cv.take(N * d * eb);
    s.a = (float *)cv.take(N * d * 4); s.st2 = (float *)cv.take(N * 2 * 4);
    s.h2 = (char *)cv.take(N * d * eb); s.u = (char *)cv.take(N * m * eb); s.gl = (char *)cv.take(N * m * eb);
  }
  c->hsave.resize((size_t)c->K * c->Lh);
  for (auto &s : c->hsave) {
    s.xs = (float *)cv.take(N * d * 4); s.st1 = (float *)cv.take(N * 2 * 4);
    s.h1 = (char *)cv.take(N * d * eb); s.qkv = (char *)cv.take(N * 3 * d * eb);
    s.lse = (float *)cv.take(N * H * 4); s.o = (char *)cv.take(N * d * eb);
    s.a = (float *)cv.take(N * d * 4); s.st2 = (float *)cv.take(N * 2 * 4);
    s.h2 = (char *)cv.take(N * d * eb); s.u = (char *)cv.take(N * m * eb); s.gl = (char *)cv.take(N * m * eb);
  }
  if (c->Lh) c->hy = (float *)cv.take(N * d * 4);
  // (one more stream slot carries a head's gradient through its own blocks)
  const size_t ns = c->plan.nslots + (c->Lh ? 1 : 0), S = (size_t)std::max(c->plan.maxcnt, 1) * N;
  c->G = (float *)cv.take(ns * N * d * 4);
  c->Gb = (c->eb == 4) ? (char *)c->G : (char *)cv.take(ns * N * d * eb);
  c->Gb_alt = (c->eb == 4) ? nullptr : (char *)cv.take(ns * N * d * eb);
  c->DU = (char *)cv.take(S * m * eb);
  c->DH = (char *)cv.take(S * d * eb);
  c->DQKV = (char *)cv.take(S * 3 * d * eb);
  c->dsum = (float *)cv.take(S * H * 4);
  for (int p = 0; p < 2; ++p) {
    c->YS2[p][0] = (char *)cv.take(N * d * eb);      // summed dY of FC2
    c->YS2[p][1] = (char *)cv.take(N * m * eb);      // FC1
    c->YS2[p][2] = (char *)cv.take(N * d * eb);      // attention output projection
    c->YS2[p][3] = (char *)cv.take(N * 3 * d * eb);  // QKV
  }
  for (int i = 0; i < 4; ++i) c->YS[i] = c->YS2[0][i];
  c->skws_floats = (size_t)kMaxBatch * c->Nc * d;
  c->skws = (float *)cv.take(c->skws_floats * 4);
  size_t pcols = std::max((size_t)3 * d, m);
  size_t pbytes = std::max((size_t)ln_backward_max_blocks() * 2 * d, (size_t)colsum_max_blocks() * pcols) * 4;
  for (int p = 0; p < 2; ++p)
    for (int i = 0; i < 6; ++i) c->partials2[p][i] = (float *)cv.take(pbytes);
  for (int i = 0; i < 6; ++i) c->partials[i] = c->partials2[0][i];
  c->jobs.count = 0;
  c->xb = (char *)cv.take(N * d * eb);
  c->Z = (char *)cv.take((size_t)c->Nc * c->V * eb);
  c->rowloss = (float *)cv.take(N * 4);
  c->hstats = (float *)cv.take(head_stats_bytes(c));
  c->hztgt = (float *)cv.take(eb == 2 ? (size_t)c->Nc * 4 : 0);
  c->dxh = (float *)cv.take((size_t)c->K * N * d * 4);
  return cv.off;
}

// --- launch bookkeeping -----------------------------------------------------------------
struct Scope {  // brackets a group of launches with events when profiling is on
  il_ctx *c; int cls; ProfRec *r = nullptr;
  Scope(il_ctx *ctx, int cls_, double flops, double bytes) : c(ctx), cls(cls_) {
    if (!c->cfg.profile) return;
    c->flops[cls] += flops; c->bytes[cls] += bytes;
    // mode 2: the step runs as it does unprofiled (two streams); only the bf16 GEMM dispatches carry timers
    const bool in_step = c->cfg.profile == 2;
    if (in_step && !(c->cfg.dtype == IL_BF16 && cls <= KC_GEMM_HEAD)) return;
    if (c->nrec == c->recs.size()) {
      ProfRec n{};
      if (hipEventCreate(&n.e0) != hipSuccess || hipEventCreate(&n.e1) != hipSuccess ||
          hipEventCreate(&n.kt.start) != hipSuccess || hipEventCreate(&n.kt.stop) != hipSuccess)
        return;
      c->recs.push_back(n);
    }
    r = &c->recs[c->nrec++];
    r->cls = cls;
    // bf16 GEMM scopes also time their MFMA kernel launch by itself (events on the dispatch)
    r->kernel = c->cfg.dtype == IL_BF16 && cls <= KC_GEMM_HEAD;
    r->bracket = !in_step;
    if (r->kernel) gemm_time_next(&r->kt);
    if (r->bracket) hipEventRecord(r->e0, c->stream);
  }
  ~Scope() {
    if (!r) return;
    if (gemm_time_next(nullptr)) r->kernel = false;  // no MFMA GEMM was launched in this scope
    if (r->bracket) hipEventRecord(r->e1, c->stream);
  }
};

#define IL_TRY(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return IL_E_HIP; } while (0)

hipError_t gemm(il_ctx *c, const GemmArgs &g) {
  return c->cfg.dtype == IL_F32 ? gemm_f32(g, c->stream) : gemm_bf16(g, c->stream);
}

inline const char *P(il_ctx *c, size_t off) { return (const char *)c->cfg.params + off * c->eb; }
inline float *Gr(il_ctx *c, size_t off) { return (float *)c->cfg.grads + off; }

// Algorithmic bytes of one GEMM: both operands once, the output once (and the operands the
// epilogue adds: residual, pre-activation, or the accumulated-into output).
double gemm_bytes(il_ctx *c, const GemmArgs &g) {
  const double eb = c->eb, mn = (double)g.M * g.N;
  double b = ((double)g.M * g.K + (double)g.K * g.N) * eb;
  switch (g.epi) {
    case EPI_BIAS_GELU: b += 2 * mn * eb; break;
    case EPI_BIAS_RES: b += 2 * mn * 4; break;
    case EPI_GELU_BWD: b += 2 * mn * eb; break;
    case EPI_STORE_F32: b += mn * 4; break;
    case EPI_WGRAD: b += mn * 4 * (g.beta ? 2 : 1); break;
    default: b += mn * eb; break;
  }
  return b;
}

GemmArgs base_args() {
  GemmArgs g;
  memset(&g, 0, sizeof(g));
  g.scale = 1.f;
  return g;
}

// y[M,N] = x[M,K] W[K,N] (+ epilogue)
int linear_fwd(il_ctx *c, const void *x, size_t w_off, size_t b_off, int M, int Kd, int Nn, int epi, void *out,
               void *out2, const float *res) {
  GemmArgs g = base_args();
  g.A = x; g.lda = Kd; g.a_kmajor = 0;
  g.B = P(c, w_off); g.ldb = Nn; g.b_kmajor = 1;
  g.M = M; g.N = Nn; g.K = Kd; g.epi = epi; g.C = out; g.C2 = out2; g.ldc = Nn;
  g.bias = P(c, b_off); g.res = res;
  Scope sc(c, KC_GEMM_FWD, 2.0 * M * Nn * Kd, gemm_bytes(c, g));
  IL_TRY(gemm(c, g));
  return IL_OK;
}

// dx[M,Kin] = dy[M,Nout] W[Kin,Nout]^T
int linear_dgrad(il_ctx *c, const void *dy, size_t w_off, int M, int Kin, int Nout, int epi, void *out,
                 const void *aux, int aux_wrap) {
  GemmArgs g = base_args();
  g.A = dy; g.lda = Nout; g.a_kmajor = 0;
  g.B = P(c, w_off); g.ldb = Nout; g.b_kmajor = 0;
  g.M = M; g.N = Kin; g.K = Nout; g.epi = epi; g.C = out; g.ldc = Kin; g.aux = aux; g.aux_wrap = aux_wrap;
  Scope sc(c, KC_GEMM_DGRAD, 2.0 * M * Kin * Nout, gemm_bytes(c, g));
  IL_TRY(gemm(c, g));
  return IL_OK;
}

// The context's second stream (non-blocking, default priority) and the events that tie it to the
// caller's stream; created on first use.
int ensure_side(il_ctx *c) {
  if (c->side) return IL_OK;
  IL_TRY(hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking));
  IL_TRY(hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming));
  c->ev_head.assign(c->K + 1, nullptr);
  for (int j = 1; j <= c->K; ++j) IL_TRY(hipEventCreateWithFlags(&c->ev_head[j], hipEventDisableTiming));
  for (int p = 0; p < 2; ++p) {
    IL_TRY(hipEventCreateWithFlags(&c->ev_blk_ready[p], hipEventDisableTiming));
    IL_TRY(hipEventCreateWithFlags(&c->ev_blk_done[p], hipEventDisableTiming));
    IL_TRY(hipEventCreateWithFlags(&c->ev_fl_ready[p], hipEventDisableTiming));
    IL_TRY(hipEventCreateWithFlags(&c->ev_fl_done[p], hipEventDisableTiming));
  }
  return IL_OK;
}

// The caller's stream waits for every block tail still running on the side stream.
int join_block_tails(il_ctx *c) {
  for (int p = 0; p < 2; ++p)
    if (c->blk_pending[p]) {
      IL_TRY(hipStreamWaitEvent(c->main_stream, c->ev_blk_done[p], 0));
      c->blk_pending[p] = 0;
    }
  c->fl_pending[0] = c->fl_pending[1] = 0;  // (the side stream is in order: the tails came after them)
  return IL_OK;
}

// Launch the queued stream-sum / column-sum reductions (at most two, one launch) and register their
// second stages.  Must run before a queued operand is overwritten (LayerNorm backward rewrites the
// gradient stream) and before the block's final column reduction.
int flush_colsums(il_ctx *c) {
  if (c->pending.count == 0) return IL_OK;
  int nblk = 0;
  if (c->flush_async) {
    const int which = c->flush_idx++ & 1;  // first or second launch of this block
    // On the side stream, after what the caller's stream has produced so far.  The caller's stream
    // waits for ev_fl_done[which] before it next overwrites an operand (block_backward).
    IL_TRY(hipEventRecord(c->ev_fl_ready[which], c->main_stream));
    IL_TRY(hipStreamWaitEvent(c->side, c->ev_fl_ready[which], 0));
    IL_TRY(sum_colsum_multi(c->cfg.dtype, c->pending, &nblk, c->side));
    IL_TRY(hipEventRecord(c->ev_fl_done[which], c->side));
    c->fl_pending[which] = 1;
  } else {
    Scope sc(c, KC_COLSUM, 0, c->pending_bytes);
    IL_TRY(sum_colsum_multi(c->cfg.dtype, c->pending, &nblk, c->stream));
  }
  for (int i = 0; i < c->pending.count; ++i)
    c->jobs.job[c->jobs.count++] = ColsumJob{c->pending.job[i].partials, nblk, c->pending.job[i].cols,
                                             c->pending_out[i], c->pending_acc[i]};
  c->pending.count = 0;
  c->pending_bytes = 0;
  return IL_OK;
}

// dW[Kin,Nout] = x[N,Kin]^T (sum_s w_s dy_s[N,Nout]);  db = column sums of the same weighted sum.
// The streams are summed first (linearity of the weight gradient), fused with the first stage of
// the bias-gradient column sum.  The GEMM itself is only described here (`out`); the four weight
// gradients of a block are launched together at the end of the block's backward so that their
// tiles share one grid.  `keep`: dy is overwritten before then, so the sum must be materialised
// even for a single stream of weight 1.  `direct`: dy IS the block's double-buffered operand
// YS[slot] - a single stream of weight 1 whose producer wrote straight into it - so nothing is
// copied and the reduction only reads.
int linear_wgrad(il_ctx *c, const Run &cp, const void *x, const void *dy, int Kin, int Nout, size_t w_off,
                 size_t b_off, int slot, bool keep, bool direct, GemmArgs *out, int *nout) {
  if (cp.nweighted == 0) return IL_OK;  // pass-through streams only: nothing is credited
  // (with the block tail on the side stream every operand is materialised: the scratch it would
  // be read from is rewritten by the next block meanwhile)
  const bool in_place =
      direct || (cp.nweighted == 1 && cp.wscale == 1.f && !keep && (c->cfg.profile == 1 || c->tail_inline));
  const char *dys = direct     ? (const char *)dy
                    : in_place ? (const char *)dy + (size_t)cp.first_weighted * c->N * Nout * c->eb
                               : c->YS[slot];
  {
    // queued: two of a block's four reductions are ready at the same point of the backward and
    // share one launch (flush_colsums)
    SumColsumJob jb;
    memset(&jb, 0, sizeof(jb));
    jb.N = c->N; jb.cols = Nout; jb.ldy = Nout; jb.partials = c->partials[slot];
    if (in_place) {
      jb.Y = dys; jb.ns = 1; jb.sw.w[0] = 1.f; jb.ysum = nullptr;
    } else {
      jb.Y = dy; jb.ns = cp.cnt; memcpy(jb.sw.w, cp.wt, sizeof(jb.sw.w)); jb.ysum = c->YS[slot];
    }
    c->pending.job[c->pending.count] = jb;
    c->pending_out[c->pending.count] = Gr(c, b_off);
    c->pending_acc[c->pending.count] = cp.acc | c->accumulate;
    c->pending_bytes += (double)(in_place ? 1 : cp.nweighted + 1) * c->N * Nout * c->eb;
    ++c->pending.count;
    if (c->pending.count == kMaxSumColsumJobs) {
      const int rc = flush_colsums(c);
      if (rc) return rc;
    }
  }
  GemmArgs g = base_args();
  g.A = x; g.lda = Kin; g.a_kmajor = 1;
  g.B = dys; g.ldb = Nout; g.b_kmajor = 1;
  g.M = Kin; g.N = Nout; g.K = c->N;
  g.epi = EPI_WGRAD; g.C = Gr(c, w_off); g.ldc = Nout; g.scale = 1.f; g.beta = cp.acc | c->accumulate;
  out[(*nout)++] = g;
  return IL_OK;
}

int launch_wgrads(il_ctx *c, const GemmArgs *list, int n) {
  if (n == 0) return IL_OK;
  double fl = 0, by = 0;
  for (int i = 0; i < n; ++i) {
    fl += 2.0 * list[i].M * list[i].N * list[i].K;
    by += gemm_bytes(c, list[i]);
  }
  Scope sc(c, KC_GEMM_WGRAD, fl, by);
  if (c->cfg.dtype == IL_F32) {
    for (int i = 0; i < n; ++i) IL_TRY(gemm_f32(list[i], c->stream));
  } else {
    IL_TRY(gemm_bf16_batch(list, n, c->stream));
  }
  return IL_OK;
}

// Split-K factor for an fp32-output GEMM (the head's dx: few output tiles, K = vocabulary).
// Two ways to fill the chip are priced with measured per-K-step times and the better one is taken:
// 128x128 tiles, two workgroups per CU (0.96 us per 64-deep step), split until about 512 tiles;
// or 256x256 tiles, one per CU (1.6 us per step, 2.6x the flops), split until about 256 tiles.
// gemm_bf16_batch then picks the matching tile from the tile counts of the split problem.
int choose_splits(il_ctx *c, size_t skws_floats, int M, int N, int K) {
  if (c->cfg.dtype != IL_BF16) return 1;
  const long t128 = (long)((M + 127) / 128) * ((N + 127) / 128);
  const long t256 = (long)((M + 255) / 256) * ((N + 255) / 256);
  const long cap = std::min<long>(kMaxBatch, (long)(skws_floats / ((size_t)M * N)));
  auto reduce_us = [&](long sp) { return sp < 2 ? 0.0 : 6.0 + (double)(sp + 1) * M * N * 4.0 / 3.0e6; };
  const double steps = K / 64.0;
  long sp128 = 1;
  if (t128 < 200) sp128 = std::max<long>(1, std::min<long>({512 / t128, cap, (long)(K / 1024)}));
  const double per128 = t128 * sp128 > 256 ? 0.96 : 0.6;  // one workgroup per CU: deeper ring, faster steps
  const double cost128 = (double)((t128 * sp128 + 511) / 512) * (steps / sp128) * per128 + reduce_us(sp128);
  long sp256 = std::max<long>(1, std::min<long>({(256 + t256 / 2) / t256, cap, (long)(K / 2048)}));
  if (t256 * sp256 < 160) return (int)sp128;  // the large tile would not be chosen
  const double cost256 = (double)((t256 * sp256 + 255) / 256) * (steps / sp256) * 1.6 + reduce_us(sp256);
  return (int)(cost256 < cost128 ? sp256 : sp128);
}

int attention_fwd(il_ctx *c, const void *qkv, void *o, float *lse) {
  Scope sc(c, KC_ATTN_FWD, 2.0 * c->cfg.batch * (double)c->cfg.seq * c->cfg.seq * c->d, 0);
  IL_TRY(attention_forward(c->cfg.dtype, qkv, c->cfg.batch, c->cfg.seq, c->H, c->dh, o, lse, c->stream));
  return IL_OK;
}

int attention_bwd(il_ctx *c, const BlockSave &s, const void *d_o, int cnt, void *dqkv) {
  Scope sc(c, KC_ATTN_BWD, 5.0 * cnt * c->cfg.batch * (double)c->cfg.seq * c->cfg.seq * c->d, 0);
  IL_TRY(attention_backward(c->cfg.dtype, s.qkv, s.o, d_o, s.lse, cnt, c->cfg.batch, c->cfg.seq, c->H, c->dh,
                            dqkv, c->dsum, c->stream));
  return IL_OK;
}

int ln_bwd(il_ctx *c, const Run &cp, const void *dy, const float *x, const float *stats, size_t g_off,
           float *G, void *Gb, int slot) {
  StreamWeights sw;
  memcpy(sw.w, cp.wt, sizeof(sw.w));
  const int rows = cp.cnt * c->N;
  int nblk = 0;
  Scope sc(c, KC_LN_BWD, 0, (double)rows * c->d * (c->eb + 8 + c->eb) + (double)c->N * c->d * 4);
  IL_TRY(ln_backward_residual(c->cfg.dtype, dy, x, stats, P(c, g_off), rows, c->N, c->d, G, Gb, sw,
                              c->partials[slot], &nblk, c->stream));
  if (cp.nweighted) c->jobs.job[c->jobs.count++] = ColsumJob{c->partials[slot], nblk, 2 * c->d, Gr(c, g_off),
                                                              cp.acc | c->accumulate};
  return IL_OK;
}

int block_forward(il_ctx *c, const BlockOff &b, const BlockSave &s, const float *x, float *xcopy, float *x_out) {
  const int N = c->N, d = c->d, m = c->m, dt = c->cfg.dtype;
  {
    Scope sc(c, KC_LN_FWD, 0, (double)N * d * (4 + c->eb));
    IL_TRY(ln_forward(dt, x, P(c, b.ln1_g), P(c, b.ln1_b), c->cfg.ln_eps, N, d, s.h1, s.st1, xcopy, c->stream));
  }
  int rc;
  if ((rc = linear_fwd(c, s.h1, b.w_qkv, b.b_qkv, N, d, 3 * d, EPI_BIAS, s.qkv, nullptr, nullptr))) return rc;
  if ((rc = attention_fwd(c, s.qkv, s.o, s.lse))) return rc;
  if ((rc = linear_fwd(c, s.o, b.w_o, b.b_o, N, d, d, EPI_BIAS_RES, s.a, nullptr, x))) return rc;
  {
    Scope sc(c, KC_LN_FWD, 0, (double)N * d * (4 + c->eb));
    IL_TRY(ln_forward(dt, s.a, P(c, b.ln2_g), P(c, b.ln2_b), c->cfg.ln_eps, N, d, s.h2, s.st2, nullptr,
                      c->stream));
  }
  if ((rc = linear_fwd(c, s.h2, b.w_fc1, b.b_fc1, N, d, m, EPI_BIAS_GELU, s.u, s.gl, nullptr))) return rc;
  if ((rc = linear_fwd(c, s.gl, b.w_fc2, b.b_fc2, N, m, d, EPI_BIAS_RES, x_out, nullptr, s.a))) return rc;
  return IL_OK;
}

int block_backward(il_ctx *c, const Run &cp, const BlockOff &b, const BlockSave &s) {
  const int N = c->N, d = c->d, m = c->m;
  const int S = cp.cnt * N;
  float *G = c->G + (size_t)cp.s0 * N * d;
  char *Gb = c->Gb + (size_t)cp.s0 * N * d * c->eb;
  int rc, nw = 0;
  GemmArgs wg[4];
  c->jobs.count = 0;
  c->pending.count = 0;
  c->pending_bytes = 0;
  const bool async_tail = c->cfg.profile != 1 && !c->tail_inline;
  const int par = c->bparity;
  if (async_tail) {
    if ((rc = ensure_side(c))) return rc;
    c->bparity ^= 1;
    if (c->blk_pending[par]) {  // the tail that last used this half of the buffers
      IL_TRY(hipStreamWaitEvent(c->stream, c->ev_blk_done[par], 0));
      c->blk_pending[par] = 0;
    }
    for (int i = 0; i < 4; ++i) c->YS[i] = c->YS2[par][i];
    for (int i = 0; i < 6; ++i) c->partials[i] = c->partials2[par][i];
  }
  // bf16: the two stream-sum launches go to the side stream as well.  LayerNorm 2's backward then
  // writes the bf16 stream to its second home (the first is still being read there) and LayerNorm 1's
  // writes it back; each waits for the side-stream launch that last read what it overwrites (Gb_alt
  // and DQKV: the previous block's second launch; Gb and DU: this block's first).
  c->flush_async = async_tail && c->eb == 2;
  c->flush_idx = 0;
  char *Gb2 = c->flush_async ? c->Gb_alt + (size_t)cp.s0 * N * d * c->eb : Gb;
  auto wait_flush = [&](int which) -> int {
    if (c->flush_async && c->fl_pending[which]) {
      IL_TRY(hipStreamWaitEvent(c->main_stream, c->ev_fl_done[which], 0));
      c->fl_pending[which] = 0;
    }
    return IL_OK;
  };
  // A single stream of weight 1 (all of n = 1 and n = K, the ends of the stack otherwise): the two wide
  // data gradients - into the MLP's hidden layer and into Q|K|V - are produced straight into this
  // block's half of the double-buffered weight-gradient operands, so the stream-sum pass has nothing
  // to copy there.  (The two model-width operands are the gradient stream itself, which the
  // LayerNorm backward rewrites; they are still copied.)
  const bool direct = async_tail && cp.cnt == 1 && cp.nweighted == 1 && cp.wscale == 1.f;
  char *DU = direct ? c->YS[1] : c->DU, *DQKV = direct ? c->YS[3] : c->DQKV;
  // MLP
  if ((rc = linear_dgrad(c, Gb, b.w_fc2, S, m, d, EPI_GELU_BWD, DU, s.u, N))) return rc;
  if ((rc = linear_wgrad(c, cp, s.gl, Gb, m, d, b.w_fc2, b.b_fc2, 0, true, false, wg, &nw))) return rc;
  if ((rc = linear_wgrad(c, cp, s.h2, DU, d, m, b.w_fc1, b.b_fc1, 1, false, direct, wg, &nw))) return rc;
  if ((rc = linear_dgrad(c, DU, b.w_fc1, S, d, m, EPI_STORE, c->DH, nullptr, 0))) return rc;
  if ((rc = flush_colsums(c))) return rc;  // the stream is about to change
  if ((rc = wait_flush(1))) return rc;
  if ((rc = ln_bwd(c, cp, c->DH, s.a, s.st2, b.ln2_g, G, Gb2, 4))) return rc;
  // attention
  if ((rc = linear_wgrad(c, cp, s.o, Gb2, d, d, b.w_o, b.b_o, 2, true, false, wg, &nw))) return rc;
  if ((rc = linear_dgrad(c, Gb2, b.w_o, S, d, d, EPI_STORE, c->DH, nullptr, 0))) return rc;
  if ((rc = attention_bwd(c, s, c->DH, cp.cnt, DQKV))) return rc;
  if ((rc = linear_wgrad(c, cp, s.h1, DQKV, d, 3 * d, b.w_qkv, b.b_qkv, 3, false, direct, wg, &nw))) return rc;
  if ((rc = linear_dgrad(c, DQKV, b.w_qkv, S, d, 3 * d, EPI_STORE, c->DH, nullptr, 0))) return rc;
  if ((rc = flush_colsums(c))) return rc;
  if ((rc = wait_flush(0))) return rc;
  if ((rc = ln_bwd(c, cp, c->DH, s.xs, s.st1, b.ln1_g, G, Gb, 5))) return rc;
  c->flush_async = false;
  // The block's tail - second stage of the six column reductions (four bias gradients, two LayerNorm
  // gain/bias pairs) and the four weight gradients in one launch - depends on nothing later and nothing
  // later depends on it: it runs on the side stream, concurrently with the next block's backward.
  struct StreamSwap {
    il_ctx *c; bool on;
    ~StreamSwap() { if (on) c->stream = c->main_stream; }
  } swap{c, false};
  if (async_tail) {
    IL_TRY(hipEventRecord(c->ev_blk_ready[par], c->main_stream));
    IL_TRY(hipStreamWaitEvent(c->side, c->ev_blk_ready[par], 0));
    c->stream = c->side;
    swap.on = true;
  }
  {
    Scope sc(c, KC_COLSUM, 0, 0);
    IL_TRY(colsum_final_multi(c->jobs, c->stream));
    c->jobs.count = 0;
  }
  if ((rc = launch_wgrads(c, wg, nw))) return rc;
  if (async_tail) {
    IL_TRY(hipEventRecord(c->ev_blk_done[par], c->side));
    c->blk_pending[par] = 1;
  }
  return IL_OK;
}

int validate(const il_config *cfg) {
  if (cfg->K < 1 || cfg->blocks_per_component < 1 || cfg->d_model < 1 || cfg->n_heads < 1 || cfg->d_mlp < 1 ||
      cfg->vocab < 2 || cfg->batch < 1 || cfg->seq < 1)
    return IL_E_ARG;
  if (cfg->n < 1 || cfg->n > cfg->K) return IL_E_ARG;
  if (cfg->dtype != IL_F32 && cfg->dtype != IL_BF16) return IL_E_ARG;
  if (cfg->route < 0 || cfg->route > IL_ROUTE_MEAN_LOCAL_FAR) return IL_E_ARG;
  if (!(cfg->ln_eps > 0.f)) return IL_E_ARG;
  if (cfg->profile < 0 || cfg->profile > 2) return IL_E_ARG;
  if (cfg->head_chunk < 0 || cfg->head_blocks < 0 || cfg->head_blocks > 64 || cfg->reserved != 0) return IL_E_ARG;
  if (cfg->d_model % cfg->n_heads) return IL_E_SHAPE;
  const int dh = cfg->d_model / cfg->n_heads;
  if (dh != 16 && dh != 32 && dh != 64 && dh != 128 && !(dh == 256 && cfg->dtype == IL_BF16)) return IL_E_SHAPE;
  if (cfg->d_model > 2048) return IL_E_SHAPE;
  const long long N = (long long)cfg->batch * cfg->seq;
  if (N > (1 << 24) || (long long)cfg->vocab > (1 << 24)) return IL_E_SHAPE;
  if ((long long)cfg->batch * cfg->n_heads > 65535) return IL_E_SHAPE;  // the attention grids' y extent
  if (cfg->dtype == IL_BF16) {
    if (cfg->d_model % 8 || cfg->d_mlp % 8 || cfg->vocab % 8 || N % 64) return IL_E_SHAPE;
    if (cfg->head_chunk % 64) return IL_E_SHAPE;
  }
  return IL_OK;
}

}  // namespace

extern "C" {

const char *il_status_string(int status) {
  switch (status) {
    case IL_OK: return "IL_OK";
    case IL_E_ARG: return "IL_E_ARG: invalid argument";
    case IL_E_SHAPE: return "IL_E_SHAPE: size not supported by the kernels";
    case IL_E_STATE: return "IL_E_STATE: call order violated";
    case IL_E_WORKSPACE: return "IL_E_WORKSPACE: buffer missing or too small";
    case IL_E_HIP: return "IL_E_HIP: HIP runtime error";
    default: return "unknown status";
  }
}

int il_routing_plan(int32_t K, int32_t n, int32_t route, int32_t *live, int32_t *passes) {
  Plan p;
  int rc = build_plan(K, n, route, p);
  if (rc) return rc;
  for (int k = 0; k < K; ++k) {
    if (live) live[k] = p.comp[k].cnt;
    if (passes) passes[k] = p.comp[k].passes;
  }
  return IL_OK;
}

int il_init(il_config *cfg, il_ctx **out) {
  if (!cfg || !out) return IL_E_ARG;
  *out = nullptr;
  int rc = validate(cfg);
  if (rc) return rc;
  il_ctx *c = new (std::nothrow) il_ctx();
  if (!c) return IL_E_ARG;
  c->cfg = *cfg;
  c->K = cfg->K; c->L = cfg->blocks_per_component; c->d = cfg->d_model; c->m = cfg->d_mlp; c->V = cfg->vocab;
  c->H = cfg->n_heads; c->dh = c->d / c->H; c->N = cfg->batch * cfg->seq;
  c->eb = cfg->dtype == IL_F32 ? 4 : 2;
  c->Lh = cfg->head_blocks;
  c->stream = (hipStream_t)cfg->stream;
  c->main_stream = c->stream;
  rc = build_plan(c->K, cfg->n, cfg->route, c->plan);
  if (rc) { delete c; return rc; }
  {
    // every GEMM operand is addressed through a 32-bit buffer descriptor: below 2 GiB each
    const unsigned long long lim = 0x7FFFFFFFull, eb = c->eb, N = c->N, d = c->d, m = c->m, V = c->V;
    const unsigned long long S = (unsigned long long)std::max(c->plan.maxcnt, 1) * N;
    if (S * std::max(3 * d, m) * eb >= lim || d * V * eb >= lim || d * m * eb >= lim || 3 * d * d * eb >= lim) {
      delete c;
      return IL_E_SHAPE;
    }
  }
  int nc = cfg->head_chunk;
  if (nc == 0) {
    // default: half the rows, at most 2048, so that logits / probabilities never exist for all tokens
    // at once; halved until the tile is addressable (below 2 GiB)
    nc = std::min(c->N / 2, 2048);
    while (nc > 64 && (unsigned long long)nc * c->V * c->eb >= 0x7FFFFFFFull) nc /= 2;
    if (cfg->dtype == IL_BF16) nc = std::max((nc / 64) * 64, 64);
    if (nc < 1) nc = c->N;
  }
  c->Nc = std::min(nc, c->N);
  if ((unsigned long long)c->Nc * c->V * c->eb >= 0x7FFFFFFFull) {  // the logits tile is a GEMM operand too
    delete c;
    return IL_E_SHAPE;
  }
  const size_t pbytes = layout_params(c) * c->eb;
  const size_t gbytes = pbytes / c->eb * 4;
  const size_t wbytes = layout_workspace(c, cfg->workspace);
  if (!cfg->workspace) {
    cfg->params_bytes = pbytes; cfg->grads_bytes = gbytes; cfg->workspace_bytes = wbytes;
    delete c;
    return IL_E_WORKSPACE;
  }
  if (!cfg->params || !cfg->grads || cfg->params_bytes < pbytes || cfg->grads_bytes < gbytes ||
      cfg->workspace_bytes < wbytes || ((uintptr_t)cfg->workspace & 255) || ((uintptr_t)cfg->params & 15) ||
      ((uintptr_t)cfg->grads & 15)) {
    delete c;
    return IL_E_WORKSPACE;
  }
  c->fwd_done.assign(c->K + 1, 0); c->head_done.assign(c->K + 1, 0); c->bwd_done.assign(c->K + 2, 0);
  c->head_pending.assign(c->K + 1, 0);
  *out = c;
  return IL_OK;
}

int il_stage_forward(il_ctx *c, int32_t k, const float *x_in, float *x_out) {
  if (!c || !x_in || !x_out || x_in == x_out) return IL_E_ARG;
  if (k < 1 || k > c->K) return IL_E_ARG;
  if (k == 1) {
    std::fill(c->fwd_done.begin(), c->fwd_done.end(), 0);
    std::fill(c->head_done.begin(), c->head_done.end(), 0);
    std::fill(c->bwd_done.begin(), c->bwd_done.end(), 0);
    // an abandoned step may have left heads running on the side stream: they share the scratch
    // that this step's heads will use and read buffers the caller is about to overwrite
    for (int j = 1; j <= c->K; ++j)
      if (c->head_pending[j]) {
        if (hipStreamWaitEvent(c->stream, c->ev_head[j], 0) != hipSuccess) return IL_E_HIP;
        c->head_pending[j] = 0;
      }
    { const int rc = join_block_tails(c); if (rc) return rc; }  // ... or weight gradients of its backward
  } else if (!c->fwd_done[k - 1]) {
    return IL_E_STATE;
  }
  for (int l = 0; l < c->L; ++l) {
    const size_t bi = (size_t)(k - 1) * c->L + l;
    const BlockSave &s = c->save[bi];
    const float *xin = l == 0 ? x_in : s.xs;
    float *xout = l == c->L - 1 ? x_out : c->save[bi + 1].xs;
    int rc = block_forward(c, c->boff[bi], s, xin, l == 0 ? s.xs : nullptr, xout);
    if (rc) return rc;
  }
  c->fwd_done[k] = 1;
  c->head_done[k] = 0;
  return IL_OK;
}

// The head's scratch: the bf16 / fp32 copy of its input, one logits tile, per-row losses and the
// split-K partial products of dx.  il_head_xent takes it from the caller's workspace,
// il_head_xent_static from the library's static device array.
struct HeadScratch {
  char *xb, *Z; float *rowloss, *skws; size_t skws_floats;
  float *stats, *ztgt;  // bf16: per-row softmax statistics of the tile ([Nc][ceil(V/64)][2]) and target logits ([Nc])
};

static int head_xent_impl(il_ctx *c, int32_t k, const float *x_k, const int32_t *targets, float *loss_out,
                          const HeadScratch &hs, bool in_line) {
  if (!c || !x_k || !targets || !loss_out) return IL_E_ARG;
  if (k < 1 || k > c->K) return IL_E_ARG;
  if (!c->fwd_done[k]) return IL_E_STATE;
  // a head with blocks of its own shares the backward scratch: it may not start once the step's
  // backward has (the backward could not order itself against it)
  if (c->Lh > 0 && c->bwd_done[c->K]) return IL_E_STATE;
  const int N = c->N, d = c->d, V = c->V, dt = c->cfg.dtype;
  const size_t eb = c->eb;
  // Head k only needs x_k; it runs on a side stream so that the next component's forward (and,
  // later, other heads' consumers) overlap with it.  il_stage_backward_nwise(k) joins.
  struct StreamSwap {
    il_ctx *c; bool on;
    ~StreamSwap() { if (on) c->stream = c->main_stream; }
  } swap{c, false};
  if (c->cfg.profile != 1 && !in_line) {
    { const int rc = ensure_side(c); if (rc) return rc; }
    IL_TRY(hipEventRecord(c->ev_fork, c->main_stream));
    IL_TRY(hipStreamWaitEvent(c->side, c->ev_fork, 0));
    c->stream = c->side;
    swap.on = true;
  }
  // the head's own blocks (App. B: the auxiliary network is Transformer blocks and an output matrix)
  const float *y = x_k;
  for (int l = 0; l < c->Lh; ++l) {
    const size_t bi = (size_t)(k - 1) * c->Lh + l;
    const BlockSave &s = c->hsave[bi];
    float *yout = l == c->Lh - 1 ? c->hy : c->hsave[bi + 1].xs;
    int rc = block_forward(c, c->hboff[bi], s, y, l == 0 ? s.xs : nullptr, yout);
    if (rc) return rc;
    y = yout;
  }
  {
    Scope sc(c, KC_MISC, 0, (double)N * d * (4 + eb));
    IL_TRY(convert_f32(dt, y, hs.xb, (size_t)N * d, c->stream));
  }
  float *dx = c->dxh + (size_t)(k - 1) * N * d;
  for (int r0 = 0, chunk = 0; r0 < N; r0 += c->Nc, ++chunk) {
    const int rows = std::min(c->Nc, N - r0);
    const char *xc = hs.xb + (size_t)r0 * d * eb;
    GemmArgs g = base_args();  // logits tile z = x W_h
    g.A = xc; g.lda = d; g.a_kmajor = 0;
    g.B = P(c, c->hoff[k - 1]); g.ldb = V; g.b_kmajor = 1;
    // bf16 mode: the tile holds the logits as IEEE half (three more mantissa bits for the softmax's
    // exponentials) and the GEMM's epilogue leaves the softmax statistics of every 64-column group,
    // taken from its fp32 accumulators, and the target logits beside it
    const bool fused = dt == IL_BF16;
    g.M = rows; g.N = V; g.K = d; g.epi = fused ? EPI_LOGITS : EPI_STORE; g.C = hs.Z; g.ldc = V;
    if (fused) { g.row_stats = hs.stats; g.row_targets = targets + r0; g.row_ztgt = hs.ztgt; }
    {
      Scope sc(c, KC_GEMM_HEAD, 2.0 * rows * V * d, gemm_bytes(c, g));
      IL_TRY(gemm(c, g));
    }
    {
      Scope sc(c, KC_XENT, 0, 2.0 * rows * V * eb);
      if (fused)
        IL_TRY(xent_rows_from_stats(hs.Z, hs.stats, hs.ztgt, targets + r0, rows, V, c->grad_scale / N,
                                    hs.rowloss + r0, c->stream));
      else
        IL_TRY(xent_rows(dt, hs.Z, targets + r0, rows, V, c->grad_scale / N, hs.rowloss + r0, c->stream));
    }
    g = base_args();  // dx = dz W_h^T
    g.A = hs.Z; g.lda = V; g.a_kmajor = 0;
    g.B = P(c, c->hoff[k - 1]); g.ldb = V; g.b_kmajor = 0;
    g.M = rows; g.N = d; g.K = V; g.epi = EPI_STORE_F32; g.C = dx + (size_t)r0 * d; g.ldc = d;
    {
      Scope sc(c, KC_GEMM_HEAD, 2.0 * rows * V * d, gemm_bytes(c, g));
      const int sp = choose_splits(c, hs.skws_floats, rows, d, V);
      if (sp > 1) IL_TRY(gemm_bf16_splitk(g, sp, hs.skws, c->stream));
      else IL_TRY(gemm(c, g));
    }
    g = base_args();  // dW_h (+)= x^T dz
    g.A = xc; g.lda = d; g.a_kmajor = 1;
    g.B = hs.Z; g.ldb = V; g.b_kmajor = 1;
    g.M = d; g.N = V; g.K = rows; g.epi = EPI_WGRAD; g.C = Gr(c, c->hoff[k - 1]); g.ldc = V;
    g.beta = chunk > 0 || c->accumulate;
    {
      Scope sc(c, KC_GEMM_HEAD, 2.0 * rows * V * d, gemm_bytes(c, g));
      IL_TRY(gemm(c, g));
    }
  }
  {
    Scope sc(c, KC_MISC, 0, (double)N * 4);
    IL_TRY(sum_scalar(hs.rowloss, N, 1.f / N, loss_out, c->stream));
  }
  if (c->Lh) {
    // dL_k/dy goes back through the head's blocks as a single stream of weight 1 in a slot of its own;
    // what arrives at x_k replaces it as the head's gradient stream.
    const size_t nd = (size_t)N * d;
    const int slot = c->plan.nslots;
    float *Gh = c->G + (size_t)slot * nd;
    {
      Scope sc(c, KC_MISC, 0, (double)nd * (8 + eb));
      IL_TRY(stream_inject(dt, dx, Gh, c->Gb + (size_t)slot * nd * eb, nd, 0, c->stream));
    }
    Run r;
    r.s0 = slot; r.cnt = 1; r.wt[0] = 1.f; r.nweighted = 1; r.first_weighted = 0; r.wscale = 1.f; r.acc = 0;
    struct Inline { il_ctx *c; bool old; ~Inline() { c->tail_inline = old; } } guard{c, c->tail_inline};
    c->tail_inline = true;  // already off the caller's stream: the block tails run in line
    for (int l = c->Lh - 1; l >= 0; --l) {
      const size_t bi = (size_t)(k - 1) * c->Lh + l;
      int rc = block_backward(c, r, c->hboff[bi], c->hsave[bi]);
      if (rc) return rc;
    }
    StreamWeights one;
    memset(&one, 0, sizeof(one));
    one.w[0] = 1.f;
    Scope sc(c, KC_MISC, 0, (double)nd * 8);
    IL_TRY(stream_combine(Gh, nd, 1, one, dx, nd, 0, c->stream));
  }
  if (swap.on) {
    IL_TRY(hipEventRecord(c->ev_head[k], c->side));
    c->head_pending[k] = 1;
    // The last head joins the side stream back (it is in order, so this covers every earlier head):
    // component K's backward needs this head at once anyway, and a caller that stops after the
    // heads finds every loss final on its own stream.
    if (k == c->K) {
      IL_TRY(hipStreamWaitEvent(c->main_stream, c->ev_head[k], 0));
      std::fill(c->head_pending.begin(), c->head_pending.end(), 0);
    }
  }
  c->head_done[k] = 1;
  return IL_OK;
}

int il_head_xent(il_ctx *c, int32_t k, const float *x_k, const int32_t *targets, float *loss_out) {
  if (!c) return IL_E_ARG;
  const HeadScratch hs{c->xb, c->Z, c->rowloss, c->skws, c->skws_floats, c->hstats, c->hztgt};
  return head_xent_impl(c, k, x_k, targets, loss_out, hs, false);
}

// ---- the head without a workspace of its own -------------------------------------------------
// The library's static scratch: every GPU the library runs on holds its own copy of this array at
// its own address until the process ends.  Host code never passes the array's name to a kernel (on
// the host it is a stand-in, not a device address): the address is looked up once per device.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

// The current device's copy of `scratch` (looked up on the first call on that device).
int static_scratch(char **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return IL_E_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return IL_E_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = (char *)g_scratch_ptr[dev];
  return IL_OK;
}
}  // namespace

int il_head_xent_static(il_ctx *c, int32_t k, const float *x_k, const int32_t *targets, float *loss_out) {
  if (!c) return IL_E_ARG;
  if (c->Lh > 0) return IL_E_SHAPE;  // heads with blocks of their own need the workspace's saved activations
  // the four pieces the head's kernels use, carved from the static array (256-byte aligned pieces)
  Carver cv(nullptr);
  const size_t o_xb = cv.off; cv.take((size_t)c->N * c->d * c->eb);
  const size_t o_z = cv.off; cv.take((size_t)c->Nc * c->V * c->eb);
  const size_t o_rl = cv.off; cv.take((size_t)c->N * 4);
  const size_t o_sk = cv.off; cv.take(c->skws_floats * 4);
  const size_t o_hs = cv.off; cv.take(head_stats_bytes(c));
  const size_t o_zt = cv.off; cv.take(c->eb == 2 ? (size_t)c->Nc * 4 : 0);
  if (cv.off > kStaticScratchBytes) return IL_E_WORKSPACE;
  char *base = nullptr;
  { const int rc = static_scratch(&base); if (rc) return rc; }
  const HeadScratch hs{base + o_xb, base + o_z, (float *)(base + o_rl), (float *)(base + o_sk), c->skws_floats,
                       (float *)(base + o_hs), (float *)(base + o_zt)};
  return head_xent_impl(c, k, x_k, targets, loss_out, hs, true);
}

int il_stage_backward_nwise(il_ctx *c, int32_t k, float *dx0_out) {
  if (!c) return IL_E_ARG;
  if (k < 1 || k > c->K) return IL_E_ARG;
  for (int j = 1; j <= c->K; ++j)
    if (!c->fwd_done[j]) return IL_E_STATE;
  if (c->bwd_done[k] || (k < c->K && !c->bwd_done[k + 1])) return IL_E_STATE;
  const CompPlan &cp = c->plan.comp[k - 1];
  if (cp.inject_slot >= 0 && !c->head_done[k]) return IL_E_STATE;
  // join the side stream: head k before its gradient is injected; every head before the step ends.
  // Heads with blocks of their own run a block backward there, over the scratch this call is about to
  // use: then every head still pending is joined, whatever the order the heads were enqueued in.
  const bool all_heads = k == 1 || c->Lh > 0;
  for (int j = (all_heads ? 1 : k); j <= (all_heads ? c->K : k); ++j)
    if (c->head_pending[j]) {
      IL_TRY(hipStreamWaitEvent(c->stream, c->ev_head[j], 0));
      c->head_pending[j] = 0;
    }
  const size_t nd = (size_t)c->N * c->d;
  if (cp.inject_slot >= 0) {
    Scope sc(c, KC_MISC, 0, (double)nd * (8 + c->eb));
    IL_TRY(stream_inject(c->cfg.dtype, c->dxh + (size_t)(k - 1) * nd, c->G + cp.inject_slot * nd,
                         c->Gb + cp.inject_slot * nd * c->eb, nd, cp.inject_acc, c->stream));
  }
  for (int l = c->L - 1; l >= 0; --l) {
    const size_t bi = (size_t)(k - 1) * c->L + l;
    for (const Run &r : cp.runs) {
      int rc = block_backward(c, r, c->boff[bi], c->save[bi]);
      if (rc) return rc;
    }
  }
  if (k == 1 && dx0_out) {
    Scope sc(c, KC_MISC, 0, (double)nd * 4 * (cp.cnt + 1));
    for (size_t i = 0; i < cp.runs.size(); ++i) {
      const Run &r = cp.runs[i];
      StreamWeights sw;
      memcpy(sw.w, r.wt, sizeof(sw.w));
      IL_TRY(stream_combine(c->G + r.s0 * nd, nd, r.cnt, sw, dx0_out, nd, i > 0, c->stream));
    }
  }
  c->bwd_done[k] = 1;
  // the step's last backward call joins the block tails still running on the side stream
  if (k == 1) { const int rc = join_block_tails(c); if (rc) return rc; }
  return IL_OK;
}

int il_profile_read(il_ctx *c, int32_t cap, const char **names, int64_t *launches, double *ms, double *flops,
                    double *bytes, double *kernel_ms) {
  if (!c || cap < 0) return IL_E_ARG;
  if (hipStreamSynchronize(c->stream) != hipSuccess) return IL_E_HIP;
  if (c->side && hipStreamSynchronize(c->side) != hipSuccess) return IL_E_HIP;
  double t[KC_COUNT] = {}, tk[KC_COUNT] = {};
  int64_t n[KC_COUNT] = {};
  for (size_t i = 0; i < c->nrec; ++i) {
    float e = 0.f;
    if (c->recs[i].bracket) {
      if (hipEventElapsedTime(&e, c->recs[i].e0, c->recs[i].e1) != hipSuccess) return IL_E_HIP;
      t[c->recs[i].cls] += e;
    }
    n[c->recs[i].cls] += 1;
    if (c->recs[i].kernel) {
      if (hipEventElapsedTime(&e, c->recs[i].kt.start, c->recs[i].kt.stop) != hipSuccess) return IL_E_HIP;
      tk[c->recs[i].cls] += e;
    }
  }
  const int cnt = std::min<int>(cap, KC_COUNT);
  for (int i = 0; i < cnt; ++i) {
    if (names) names[i] = kClassNames[i];
    if (launches) launches[i] = n[i];
    if (ms) ms[i] = t[i];
    if (kernel_ms) kernel_ms[i] = tk[i];
    if (flops) flops[i] = c->flops[i];
    if (bytes) bytes[i] = c->bytes[i];
  }
  c->nrec = 0;
  memset(c->flops, 0, sizeof(c->flops));
  memset(c->bytes, 0, sizeof(c->bytes));
  return cnt;
}

int il_test_gemm(int32_t dtype, const void *A, const void *B, int32_t M, int32_t N, int32_t K, int32_t lda,
                 int32_t ldb, int32_t a_kmajor, int32_t b_kmajor, int32_t epi, void *C, void *C2, int32_t ldc,
                 const void *bias, const float *res, const void *aux, int32_t aux_wrap, float scale,
                 int32_t beta, int32_t tile, void *stream) {
  if (!A || !B || !C || M < 1 || N < 1 || K < 1) return IL_E_ARG;
  if (dtype != IL_F32 && dtype != IL_BF16) return IL_E_ARG;
  if (epi < EPI_STORE || epi > EPI_LOGITS || tile < 0 || tile > 8) return IL_E_ARG;
  if (epi == EPI_LOGITS && (dtype != IL_BF16 || (C2 && !aux))) return IL_E_ARG;
  if ((epi == EPI_BIAS || epi == EPI_BIAS_GELU || epi == EPI_BIAS_RES) && !bias) return IL_E_ARG;
  if ((epi == EPI_BIAS_RES && !res) || (epi == EPI_BIAS_GELU && !C2)) return IL_E_ARG;
  if (epi == EPI_GELU_BWD && (!aux || aux_wrap < 1)) return IL_E_ARG;
  GemmArgs g = base_args();
  g.A = A; g.B = B; g.M = M; g.N = N; g.K = K; g.lda = lda; g.ldb = ldb;
  g.a_kmajor = a_kmajor != 0; g.b_kmajor = b_kmajor != 0; g.epi = epi; g.C = C; g.C2 = C2; g.ldc = ldc;
  g.bias = bias; g.res = res; g.aux = aux; g.aux_wrap = aux_wrap; g.scale = scale; g.beta = beta; g.tile = tile;
  if (epi == EPI_LOGITS && C2) {  // statistics and target logits share the second output buffer
    g.row_stats = (float *)C2;
    g.row_targets = (const int32_t *)aux;
    g.row_ztgt = (float *)C2 + (size_t)M * ((N + kStatGroup - 1) / kStatGroup) * 2;
    g.C2 = nullptr;
    g.aux = nullptr;
  }
  const hipError_t e = dtype == IL_F32 ? gemm_f32(g, (hipStream_t)stream) : gemm_bf16(g, (hipStream_t)stream);
  return e == hipSuccess ? IL_OK : (e == hipErrorInvalidValue ? IL_E_SHAPE : IL_E_HIP);
}

int il_set_accumulation(il_ctx *c, int32_t accumulate, float grad_scale) {
  if (!c || !(grad_scale > 0.f) || !std::isfinite(grad_scale)) return IL_E_ARG;
  c->accumulate = accumulate ? 1 : 0;
  c->grad_scale = grad_scale;
  return IL_OK;
}

int il_free(il_ctx *c) {
  if (!c) return IL_E_ARG;
  if (c->side) hipStreamSynchronize(c->side);  // nothing of this context is left running on it
  for (auto &r : c->recs) {
    hipEventDestroy(r.e0); hipEventDestroy(r.e1);
    hipEventDestroy(r.kt.start); hipEventDestroy(r.kt.stop);
  }
  for (hipEvent_t e : c->ev_head) if (e) hipEventDestroy(e);
  if (c->ev_fork) hipEventDestroy(c->ev_fork);
  for (int p = 0; p < 2; ++p) {
    if (c->ev_blk_ready[p]) hipEventDestroy(c->ev_blk_ready[p]);
    if (c->ev_blk_done[p]) hipEventDestroy(c->ev_blk_done[p]);
    if (c->ev_fl_ready[p]) hipEventDestroy(c->ev_fl_ready[p]);
    if (c->ev_fl_done[p]) hipEventDestroy(c->ev_fl_done[p]);
  }
  if (c->side) hipStreamDestroy(c->side);
  delete c;
  return IL_OK;
}

}  // extern "C"
