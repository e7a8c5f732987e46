/*
 * interlock.h - C ABI of the single-GPU n-wise interlocking-backpropagation step
 * for MI355X (gfx950).
 *
 * The library runs one training step over a stack of K Transformer components
 * ("modules" in the paper, Sec. 3), each followed by its own auxiliary
 * classification head: the forward pass, the K softmax cross-entropy losses, and
 * the n-wise truncated backward in which the gradient of head j's loss travels
 * through component j and across n-1 component boundaries and then stops (Fig. 1
 * caption; Sec. 3, paragraph introducing n-wise interlocking backpropagation).
 *
 * All pointers named "device" are HIP device pointers owned by the caller.  The
 * library allocates no device memory: parameters, gradients, the workspace and the
 * stream come from the caller.  All work is enqueued asynchronously, ordered with
 * il_config.stream: the caller synchronises that stream before reading results.  (The
 * context owns one further non-blocking stream and a few events.  il_head_xent runs on it,
 * concurrently with the next component's forward; il_head_xent(K), the step's last head,
 * and il_stage_backward_nwise join it back into il_config.stream.  The tail of every
 * block's backward - bias and LayerNorm gradient reductions, weight gradients - runs on it
 * too, concurrently with the next block; il_stage_backward_nwise(1), the step's last call,
 * joins it back.  So the caller never sees that stream: losses and head gradients are
 * final on il_config.stream once il_head_xent(K) has been enqueued, component gradients
 * once il_stage_backward_nwise(1) has been; until then the x_k and targets buffers handed
 * to il_head_xent must not be overwritten.)
 * Every function returns an il_status; nothing is printed and nothing aborts.
 *
 * Components and heads are numbered 1..K as in the paper.
 */
#ifndef INTERLOCK_H
#define INTERLOCK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct il_ctx il_ctx; /* opaque, host memory only */

typedef enum {
  IL_OK = 0,
  IL_E_ARG = -1,       /* NULL pointer, k outside [1,K], n outside [1,K], unknown enum */
  IL_E_SHAPE = -2,     /* a size the kernels cannot handle (see il_init)               */
  IL_E_STATE = -3,     /* call-order contract violated                                 */
  IL_E_WORKSPACE = -4, /* workspace / params / grads buffer missing or too small       */
  IL_E_HIP = -5        /* a HIP runtime call or kernel launch failed                   */
} il_status;

typedef enum {
  IL_F32 = 0, /* parameters, GEMM operands and saved activations in fp32 */
  IL_BF16 = 1 /* ... in bfloat16 (round to nearest even); accumulators, LayerNorm
                 statistics, softmax, the residual stream, losses and gradients of
                 parameters stay fp32 */
} il_dtype;

/*
 * Which losses are credited to component k (a K x K weight table w[k][j]):
 *  WINDOW_SUM     every head whose n-window covers k: j in [k, min(k+n-1,K)], weight 1.
 *                 n=1 is local learning, n=K is backprop of the summed loss.
 *  FAR_HEAD       only j = min(k+n-1,K), weight 1 (Sec. 3: module k is updated with the
 *                 gradient of the loss n-1 modules above it).
 *  MEAN_LOCAL_FAR 1/2 on j=k and 1/2 on j=min(k+n-1,K) (Sec. 3, the variant used for the
 *                 Transformer experiments; App. B).
 * Head parameters always receive the gradient of their own loss with weight 1.
 */
typedef enum { IL_ROUTE_WINDOW_SUM = 0, IL_ROUTE_FAR_HEAD = 1, IL_ROUTE_MEAN_LOCAL_FAR = 2 } il_route;

/*
 * Problem statement.  Each component is `blocks_per_component` pre-LN Transformer
 * blocks:  a = x + O(Attn(QKV(LN1 x))),  x' = a + FC2(GELU(FC1(LN2 a)))  with causal
 * attention, tanh-GELU, biased-variance LayerNorm with ln_eps inside the root.
 * Head k is `head_blocks` further blocks of the same form (its own parameters, trained by L_k
 * alone) followed by a bias-free linear map d_model -> vocab; loss k is the mean over the
 * batch*seq positions of the natural-log cross-entropy against `targets`.
 *
 * Flat parameter layout (element type = dtype; every matrix row-major, y = x W + b,
 * W is [in, out]):
 *   for component 1..K, for block 1..L:
 *     ln1_g[d] ln1_b[d] w_qkv[d,3d] b_qkv[3d] w_o[d,d] b_o[d]
 *     ln2_g[d] ln2_b[d] w_fc1[d,m] b_fc1[m] w_fc2[m,d] b_fc2[d]
 *   then heads 1..K: head_blocks blocks (the same twelve tensors each), w_head[d,V]
 * w_qkv's columns are Q | K | V, each split into n_heads groups of d/n_heads columns.
 * `grads` has the same element order in fp32.  Every gradient element is overwritten
 * exactly once per step (no zeroing needed, nothing accumulates across steps).
 */
typedef struct il_config {
  int32_t K;                    /* components (= heads)                              */
  int32_t blocks_per_component; /* L                                                 */
  int32_t d_model, n_heads, d_mlp, vocab;
  int32_t batch, seq;           /* N = batch*seq token rows, row index = b*seq + t   */
  int32_t n;                    /* window, 1..K                                      */
  int32_t dtype;                /* il_dtype                                          */
  int32_t route;                /* il_route                                          */
  float ln_eps;                 /* e.g. 1e-5                                         */
  int32_t head_chunk;           /* token rows per head chunk (0 = library default: half the
                                   rows, at most 2048, halved until the tile is below 2 GiB);
                                   only a [head_chunk, vocab] logits tile ever exists      */
  int32_t profile;              /* 0: off.  1: HIP event times per kernel class (read with
                                   il_profile_read, interlock_test.h); everything then runs on
                                   il_config.stream alone.  2: the step runs exactly as with 0
                                   (both streams); only the bf16 GEMM dispatches carry timers */
  int32_t head_blocks;          /* Transformer blocks inside every auxiliary head, in front
                                   of its d_model -> vocab map (0 = the bare linear head;
                                   the paper's Transformer runs use 2, App. B)          */
  int32_t reserved;             /* must be 0                                          */
  void *params;                 /* device, flat layout above                         */
  size_t params_bytes;
  void *grads;                  /* device, fp32, same order                          */
  size_t grads_bytes;
  void *workspace;              /* device: saved activations, gradient streams, scratch */
  size_t workspace_bytes;
  void *stream;                 /* hipStream_t (NULL = the default stream)           */
} il_config;

/*
 * Validate cfg and create a context (host memory only).
 * Size query: call with cfg->workspace == NULL; the three *_bytes fields are filled
 * with the required sizes, *out is left NULL and IL_E_WORKSPACE is returned.
 * Limits (IL_E_SHAPE otherwise): d_model a multiple of n_heads with head width
 * d_model / n_heads in {16, 32, 64, 128}, or 256 in bf16 mode; d_model <= 2048; batch*seq <= 2^24; vocab <= 2^24;
 * batch*n_heads <= 65535;
 * in bf16 mode d_model, d_mlp and vocab multiples of 8, batch*seq and head_chunk multiples of
 * 64.  At most 16 merged gradient streams may be live at one component.  Every GEMM operand stays
 * below 2 GiB: streams * batch*seq * max(3 d_model, d_mlp), d_model * vocab, head_chunk * vocab
 * elements of `dtype`.
 * The workspace must be 256-byte aligned.
 */
int il_init(il_config *cfg, il_ctx **out);

/*
 * Component forward x_k = f_k(x_{k-1}) (Sec. 3: the model is a composition of modules).
 * x_in, x_out: device fp32 [N, d_model] (the residual stream is fp32 in both dtypes);
 * they may not alias.  Saves what the backward needs in the workspace (x_in is copied,
 * so the caller may reuse it).  k = 1 starts a new step and resets the routing state.
 * Order: k-1 must have been run in this step (IL_E_STATE otherwise).
 */
int il_stage_forward(il_ctx *ctx, int32_t k, const float *x_in, float *x_out);

/*
 * Auxiliary head k and its local loss L_k = xent(h_k(x_k), y) (Sec. 3, the equation
 * defining the local loss).  x_k: device fp32 [N, d_model]; targets: device int32 [N],
 * each in [0, vocab) - a target outside that range marks an ignored position: it adds nothing to the
 * loss or to any gradient, and the mean still divides by N; loss_out: device fp32 scalar (mean over N,
 * natural log).
 * Writes dL_k/dW_head,k (and the gradients of the head's own blocks) into grads and keeps
 * dL_k/dx_k - propagated back through those blocks - in the workspace as the
 * gradient stream of head k (age 0) for il_stage_backward_nwise.  Logits and
 * probabilities exist only one [head_chunk, vocab] tile at a time.
 * Order: after il_stage_forward(k) of the same step, in any order among the heads; with
 * head_blocks > 0 also before the step's first il_stage_backward_nwise (IL_E_STATE otherwise: the
 * head's own blocks are differentiated in the scratch the backward uses).
 */
int il_head_xent(il_ctx *ctx, int32_t k, const float *x_k, const int32_t *targets, float *loss_out);

/*
 * il_head_xent for callers that cannot allocate or hand over scratch memory for the head (code under
 * HIP graph capture, tight serving or evaluation loops, harnesses that forbid hipMalloc): the same
 * computation and results as il_head_xent(ctx, k, ...), but the head's scratch - the copy of x_k in
 * the GEMM element type, the one logits tile with its row statistics, the per-row losses and the
 * split-K partial products of dL_k/dx_k - lives in a static device array of the library (64 MiB = 67108864 bytes, held
 * by every GPU the library runs on until the process ends) instead of the context's workspace, and the
 * head runs in line on il_config.stream (the library's internal stream and its events are neither
 * created nor used).  The call allocates nothing: no hipMalloc / hipFree, no stream or event creation.
 * Inputs and outputs are as for il_head_xent (x_k, targets, loss_out; head gradients into `grads`,
 * dL_k/dx_k into the context's gradient stream).
 * IL_E_WORKSPACE when batch*seq*d_model + head_chunk*vocab elements of `dtype` + batch*seq*4 bytes +
 * the split-K partials (8 * head_chunk * d_model floats) + in bf16 the tile's softmax statistics
 * (head_chunk * (ceil(vocab/64) * 8 + 4) bytes) exceed the static array; IL_E_SHAPE when
 * head_blocks > 0 (such heads keep activations in the workspace; use il_head_xent); IL_E_HIP when the
 * array's address on the current device cannot be resolved.  Nothing in the array has to start at
 * zero: every piece is written before it is read within the call.  All calls on one GPU share the one
 * array and the array keeps the last call's contents, so calls that overlap in time on one GPU (other
 * streams, other contexts, other host threads) race: serialise them.
 */
int il_head_xent_static(il_ctx *ctx, int32_t k, const float *x_k, const int32_t *targets, float *loss_out);

/*
 * n-wise truncated backward through component k (Fig. 1; Sec. 3: each module runs up
 * to n backward passes).  Every gradient stream live at x_k - the heads whose credited
 * range reaches down to k - is carried through the component's backward; the
 * component's parameter gradient receives sum_j w[k][j] * dL_j/dtheta_k; streams whose
 * lowest credited component is k stop here (stop-gradient at the window edge).
 * Call for k = K, K-1, ..., 1, after il_head_xent(j) for every head j >= k that is live
 * at k.  The gradients of all components are final on il_config.stream after the call for
 * k = 1 (see the note on the internal stream above).  dx0_out: for k == 1, optional device fp32 [N, d_model] receiving
 * sum_j w[1][j] * dL_j/dx_0 (for the caller's embedding gradient); NULL to skip; ignored
 * for k > 1.
 */
int il_stage_backward_nwise(il_ctx *ctx, int32_t k, float *dx0_out);

/*
 * Micro-batching (Sec. 3.1: n-wise training combined with GPipe-style micro-batches).  With
 * accumulate != 0 every parameter gradient written by the following steps is ADDED to what
 * `grads` holds instead of overwriting it, and every gradient is multiplied by grad_scale
 * (1/M for the mean over M equal micro-batches; losses are reported unscaled).  The first
 * micro-batch of a mini-batch runs with accumulate = 0.  dx0_out is always overwritten (it
 * belongs to the micro-batch's own tokens).  Call between steps.  IL_E_ARG for a NULL context or
 * a grad_scale that is not positive and finite.
 */
int il_set_accumulation(il_ctx *ctx, int32_t accumulate, float grad_scale);

/* Release the context (host memory and HIP events only; no device buffer is freed). */
int il_free(il_ctx *ctx);

/* ---- host-side introspection (no GPU work) ------------------------------------ */

/*
 * The routing plan for (K, n, route): for component k = 1..K, live[k-1] receives the
 * number of gradient streams carried through component k's backward after merging
 * streams that share their remaining route, and passes[k-1] the number of heads
 * whose gradient passes through it (the paper's backward passes per module, Sec. 3).
 * Either array may be NULL.  Returns IL_E_ARG for n outside [1,K] or unknown route.
 */
int il_routing_plan(int32_t K, int32_t n, int32_t route, int32_t *live, int32_t *passes);

/* ---- input embedding of the first module (App. B: the embedding matrix in front of the blocks) ---- */

/*
 * x0[b*seq + t, :] = wte[tokens[b*seq + t], :] + wpe[t, :], fp32 [batch*seq, d_model]: the x_in of
 * il_stage_forward(1).  wte [vocab, d_model] and wpe [seq, d_model] are row-major in `dtype`
 * (il_dtype); tokens is int32 [batch*seq]; all device pointers owned by the caller; enqueued on
 * `stream`.  A token outside [0, vocab) embeds as the zero vector (nothing out of bounds is read).
 * IL_E_ARG: NULL pointer, non-positive size, unknown dtype; IL_E_SHAPE: batch*seq or vocab above
 * 2^24, or x0 not 16-byte aligned when d_model is a multiple of 4.
 */
int il_embed_forward(int32_t dtype, const void *wte, const void *wpe, const int32_t *tokens, int32_t batch,
                     int32_t seq, int32_t d_model, int32_t vocab, float *x0, void *stream);

/*
 * Gradient of the embedding, from dx0 fp32 [batch*seq, d_model] (the dx0_out of
 * il_stage_backward_nwise(1)):
 *   dwte[v, :] = sum over the positions i with tokens[i] == v of dx0[i, :]   (zero for unused rows),
 *   dwpe[t, :] = sum_b dx0[b*seq + t, :],
 * both fp32, every element written exactly once per call (no zeroing needed), no atomics, fixed
 * summation order (ascending position), so the result is bit-reproducible.  Tokens outside
 * [0, vocab) receive no gradient.  Same error codes as il_embed_forward.
 */
int il_embed_backward(const float *dx0, const int32_t *tokens, int32_t batch, int32_t seq, int32_t d_model,
                      int32_t vocab, float *dwte, float *dwpe, void *stream);

/* ---- optimiser step (App. B, training configuration of the Transformer runs) ------ */

/*
 * Learning rate d_model^-0.5 * min(step^-0.5, step * warmup_steps^-1.5), steps counted from 1
 * (host function, no GPU work).  Returns 0 for step < 1, d_model < 1 or warmup_steps < 1.
 */
double il_lr_schedule(int64_t step, int32_t d_model, int32_t warmup_steps);

/*
 * One Adam update with bias correction over `count` parameters (the paper's setting is
 * beta1 = 0.9, beta2 = 0.98, eps = 1e-9):
 *   m <- beta1 m + (1-beta1) g,  v <- beta2 v + (1-beta2) g^2,
 *   w <- w - lr * (m / (1-beta1^step)) / (sqrt(v / (1-beta2^step)) + eps).
 * No weight decay, no clipping.  All pointers are device pointers owned by the caller; the
 * work is enqueued on `stream` (hipStream_t, NULL = default stream).
 *   dtype IL_F32 : params is the fp32 weight buffer, updated in place; master must be NULL.
 *   dtype IL_BF16: master is the fp32 copy of the weights (updated in place) and params
 *                  receives its bfloat16 image (round to nearest even).
 * grads, m, v: fp32 [count] in the flat parameter order described above; m and v start at zero
 * and are updated in place; step >= 1 is the number of this update.  fp32 buffers must be 16-byte
 * aligned (bf16 params 8-byte): IL_E_SHAPE otherwise.  IL_E_ARG for NULL pointers, step < 1,
 * betas outside [0,1), negative eps or lr, or a master that does not match dtype.
 */
int il_adam_step(int32_t dtype, void *params, float *master, const float *grads, float *m, float *v,
                 size_t count, int64_t step, float lr, float beta1, float beta2, float eps, void *stream);

/* ---- timing model of the paper (Sec. 3.1, App. C; host arithmetic) ------------------- */

/*
 * Time per mini-batch on A accelerators in sequence with M micro-batches and window N (clamped to
 * A), slot cost c(M) = c0 + c1/M:
 *   M = 1:                      2 N M c(M)
 *   M = 2, or A >= 2N - 1:      (N + 1) M c(M)
 *   otherwise (M > 2):          (2 + A - N) M c(M) + 2 (2N - A - 1) c(M)
 * N = A is end-to-end training (GPipe for M >= 2), N = 1 local learning.  NaN for non-positive
 * arguments.
 */
double il_time_per_batch(int32_t A, int32_t M, int32_t N, double c0, double c1);

/* The power of two M <= max_m that minimises il_time_per_batch (the smallest on ties); negative
 * il_status for non-positive arguments. */
int32_t il_optimal_microbatches(int32_t A, int32_t N, double c0, double c1, int32_t max_m);

/* Static string for a status code. */
const char *il_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* INTERLOCK_H */
