"""CPU oracle for one n-wise interlocking-backpropagation step.  TEST INFRASTRUCTURE.

This file is the plain, slow, float64 statement of what the GPU library must
compute.  It is imported only by the tests, by the smoke check and by the
benchmark's CPU-baseline leg; the product path never calls it, and it shares no
code with the HIP sources (it imports numpy and nothing else).

What it computes (paper Sec. 3, "Interlocking Backpropagation"):

* the network is a composition of K modules ("components") x_k = f_k(x_{k-1}),
  each a group of L pre-LN Transformer blocks (Sec. 3, first paragraph;
  Sec. 4.3 / App. B for the GPT-2-like block);
* every component k has an auxiliary network h_k and a local loss
  L_k = xent(h_k(x_k), y) (Sec. 3, the equation defining the local loss);
* under n-wise training the gradient of L_j flows through component j and
  across n-1 component boundaries and then stops (Fig. 1 caption), so the
  gradient credited to component k is, under the default "window sum" routing,
      g(theta_k) = sum_{j=k}^{min(k+n-1,K)} dL_j/dtheta_k,
  and head parameters phi_j only ever see their own loss.  n=1 is local
  learning and n=K is global optimisation (Sec. 3, paragraph introducing
  n-wise).  The paper's own two routings (far head only; mean of local and far
  head) are the same computation with a different K x K weight table.

Every dL_j/dtheta_k here is the ordinary exact derivative; truncation only
selects which of them are kept.  Two independent routes to the result:

  nwise_definition : K full backward sweeps, one per loss, then the weight table.
  nwise_streams    : the algorithm as told in the paper - one forward, every head
                     emits dL_j/dx_j, the live gradient streams are carried
                     separately down through the components and dropped at the
                     window edge ("N backward passes per module", Sec. 3).

Readings where the paper is silent: LayerNorm uses the biased variance and
eps inside the square root; GELU is the tanh form; attention is causal with
scale 1/sqrt(dh); biases on all four linear maps; no dropout; the head is one
bias-free linear map d -> V; the loss is the mean over all B*T positions of the
natural-log cross-entropy.  Parity pins: see tests/test_oracle_*.py.
"""
import numpy as np

F64 = np.float64

# --------------------------------------------------------------------------
# primitives
# --------------------------------------------------------------------------


def layernorm_forward(x, gamma, beta, eps):
    """y = (x - mean) / sqrt(var + eps) * gamma + beta, statistics over the last axis."""
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = xc * rstd
    return xhat * gamma + beta, (xhat, rstd, gamma)


def layernorm_backward(dy, cache):
    """Returns (dx, dgamma, dbeta) for y = xhat*gamma + beta."""
    xhat, rstd, gamma = cache
    dxhat = dy * gamma
    m1 = dxhat.mean(axis=-1, keepdims=True)
    m2 = (dxhat * xhat).mean(axis=-1, keepdims=True)
    dx = rstd * (dxhat - m1 - xhat * m2)
    return dx, (dy * xhat).sum(axis=0), dy.sum(axis=0)


_GELU_C = np.sqrt(2.0 / np.pi)


def gelu(u):
    """0.5 u (1 + tanh(sqrt(2/pi) (u + 0.044715 u^3)))."""
    return 0.5 * u * (1.0 + np.tanh(_GELU_C * (u + 0.044715 * u ** 3)))


def gelu_grad(u):
    t = np.tanh(_GELU_C * (u + 0.044715 * u ** 3))
    return 0.5 * (1.0 + t) + 0.5 * u * (1.0 - t * t) * _GELU_C * (1.0 + 3 * 0.044715 * u * u)


def attention_forward(qkv, B, T, H):
    """Causal multi-head attention.  qkv is [B*T, 3d] with columns Q|K|V, each
    split into H heads of dh contiguous columns.  Returns o [B*T, d] and a cache."""
    N, d3 = qkv.shape
    d = d3 // 3
    dh = d // H
    q, k, v = (qkv[:, i * d:(i + 1) * d].reshape(B, T, H, dh).transpose(0, 2, 1, 3) for i in range(3))
    s = (q @ k.transpose(0, 1, 3, 2)) / np.sqrt(dh)                     # [B,H,T,T]
    future = np.triu(np.ones((T, T), dtype=bool), 1)
    s = np.where(future, -np.inf, s)
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=-1, keepdims=True)
    o = (p @ v).transpose(0, 2, 1, 3).reshape(N, d)
    return o, (q, k, v, p)


def attention_backward(do, cache):
    q, k, v, p = cache
    B, H, T, dh = q.shape
    N, d = B * T, H * dh
    do = do.reshape(B, T, H, dh).transpose(0, 2, 1, 3)
    dv = p.transpose(0, 1, 3, 2) @ do
    dp = do @ v.transpose(0, 1, 3, 2)
    ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
    ds = ds / np.sqrt(dh)
    dq = ds @ k
    dk = ds.transpose(0, 1, 3, 2) @ q
    flat = lambda a: a.transpose(0, 2, 1, 3).reshape(N, d)
    return np.concatenate([flat(dq), flat(dk), flat(dv)], axis=1)


# --------------------------------------------------------------------------
# one Transformer block, one component
# --------------------------------------------------------------------------


def block_forward(x, p, B, T, H, eps):
    """a = x + O(Attn(QKV(LN1 x)));  x' = a + FC2(GELU(FC1(LN2 a)))."""
    h1, c1 = layernorm_forward(x, p["ln1_g"], p["ln1_b"], eps)
    qkv = h1 @ p["w_qkv"] + p["b_qkv"]
    o, ca = attention_forward(qkv, B, T, H)
    a = x + o @ p["w_o"] + p["b_o"]
    h2, c2 = layernorm_forward(a, p["ln2_g"], p["ln2_b"], eps)
    u = h2 @ p["w_fc1"] + p["b_fc1"]
    g = gelu(u)
    y = a + g @ p["w_fc2"] + p["b_fc2"]
    return y, dict(c1=c1, h1=h1, ca=ca, o=o, c2=c2, h2=h2, u=u, g=g)


def block_backward(dy, p, c):
    """Exact reverse of block_forward.  Returns (dx, parameter-gradient dict)."""
    gr = {}
    dg = dy @ p["w_fc2"].T
    gr["w_fc2"] = c["g"].T @ dy
    gr["b_fc2"] = dy.sum(axis=0)
    du = dg * gelu_grad(c["u"])
    gr["w_fc1"] = c["h2"].T @ du
    gr["b_fc1"] = du.sum(axis=0)
    dh2 = du @ p["w_fc1"].T
    dln, gr["ln2_g"], gr["ln2_b"] = layernorm_backward(dh2, c["c2"])
    da = dy + dln
    do = da @ p["w_o"].T
    gr["w_o"] = c["o"].T @ da
    gr["b_o"] = da.sum(axis=0)
    dqkv = attention_backward(do, c["ca"])
    gr["w_qkv"] = c["h1"].T @ dqkv
    gr["b_qkv"] = dqkv.sum(axis=0)
    dh1 = dqkv @ p["w_qkv"].T
    dln, gr["ln1_g"], gr["ln1_b"] = layernorm_backward(dh1, c["c1"])
    return da + dln, gr


def component_forward(x, blocks, B, T, H, eps):
    caches = []
    for p in blocks:
        x, c = block_forward(x, p, B, T, H, eps)
        caches.append(c)
    return x, caches


def component_backward(dy, blocks, caches):
    grads = [None] * len(blocks)
    for l in range(len(blocks) - 1, -1, -1):
        dy, grads[l] = block_backward(dy, blocks[l], caches[l])
    return dy, grads


def head_xent(x, w_head, targets):
    """Auxiliary head h(x) = x W and the mean cross-entropy against `targets`.
    Returns (loss, dL/dx, dL/dW)."""
    N = x.shape[0]
    z = x @ w_head
    zmax = z.max(axis=-1, keepdims=True)
    lse = np.log(np.exp(z - zmax).sum(axis=-1)) + zmax[:, 0]
    rows = np.arange(N)
    loss = (lse - z[rows, targets]).mean()
    dz = np.exp(z - lse[:, None])
    dz[rows, targets] -= 1.0
    dz /= N
    return loss, dz @ w_head.T, x.T @ dz


def aux_head(x, head_blocks, w_head, targets, B, T, H, eps):
    """Auxiliary network of one module and its local loss (Sec. 3, the local-loss equation).  The
    paper's Transformer runs use Transformer blocks followed by the output embedding matrix (App. B,
    module table); with no blocks this is the bare linear head.  Returns
    (loss, dL/dx, dL/dW_head, [dL/d(block parameters)])."""
    y, caches = component_forward(x, head_blocks, B, T, H, eps)
    loss, dy, dw = head_xent(y, w_head, targets)
    dx, gblocks = component_backward(dy, head_blocks, caches)
    return loss, dx, dw, gblocks


# --------------------------------------------------------------------------
# routing
# --------------------------------------------------------------------------

ROUTES = ("window_sum", "far_head", "mean_local_far")


def routing_weights(K, n, route="window_sum"):
    """w[k-1, j-1] = weight with which dL_j/dtheta_k enters component k's gradient.

    window_sum     : 1 for k <= j <= min(k+n-1, K)  (every head whose window covers k)
    far_head       : 1 for j = min(k+n-1, K) only   (Sec. 3: module k is updated from
                     the loss n-1 modules above it)
    mean_local_far : 1/2 on j = k and 1/2 on j = min(k+n-1, K) (the variant used for
                     the Transformer runs; the two coincide when n = 1 or k = K)
    A zero entry means the gradient of L_j is not credited to component k."""
    if not 1 <= n <= K:
        raise ValueError("n must be in [1, K]")
    w = np.zeros((K, K), dtype=F64)
    for k in range(1, K + 1):
        far = min(k + n - 1, K)
        if route == "window_sum":
            w[k - 1, k - 1:far] = 1.0
        elif route == "far_head":
            w[k - 1, far - 1] = 1.0
        elif route == "mean_local_far":
            w[k - 1, k - 1] += 0.5
            w[k - 1, far - 1] += 0.5
        else:
            raise ValueError(route)
    return w


def stream_plan(K, n, route="window_sum"):
    """For each component k (1-based) the heads whose gradient stream passes
    through it: head j is live at k when lo(j) <= k <= j, where lo(j) is the lowest
    component that credits L_j (its stream stops below lo(j)).  Under window_sum
    lo(j) = max(1, j-n+1) and len(plan[k]) = min(n, K-k+1)."""
    w = routing_weights(K, n, route)
    plan = {}
    for k in range(1, K + 1):
        live = []
        for j in range(k, K + 1):
            users = np.nonzero(w[:, j - 1])[0]
            if users.size and users.min() + 1 <= k:
                live.append(j)
        plan[k] = live
    return plan


def _zeros_like_grads(blocks):
    return [{name: np.zeros_like(a, dtype=F64) for name, a in p.items()} for p in blocks]


def _axpy(acc, scale, grads):
    for ga, g in zip(acc, grads):
        for name in ga:
            ga[name] += scale * g[name]


def _to_f64(params):
    comps = [[{k: np.asarray(v, dtype=F64) for k, v in p.items()} for p in blocks]
             for blocks in params["components"]]
    heads = [np.asarray(h, dtype=F64) for h in params["heads"]]
    return comps, heads


def _head_blocks_f64(params):
    hb = params.get("head_blocks") or [[] for _ in params["heads"]]
    return [[{k: np.asarray(v, dtype=F64) for k, v in p.items()} for p in blocks] for blocks in hb]


def forward_all(params, x0, targets, B, T, H, eps=1e-5):
    """Forward through all K components and heads.  Returns per-component
    caches, activations x_1..x_K, the K losses, dL_j/dx_j, dL_j/dW_head,j and the
    gradients of the heads' own blocks."""
    comps, heads = _to_f64(params)
    hblocks = _head_blocks_f64(params)
    x = np.asarray(x0, dtype=F64)
    tg = np.asarray(targets).reshape(-1)
    xs, caches, losses, dxs, dheads = [], [], [], [], []
    dhblocks = []                         # gradients of the heads' own blocks (L_k only, weight 1)
    for blocks, wh, hb in zip(comps, heads, hblocks):
        x, c = component_forward(x, blocks, B, T, H, eps)
        loss, dx, dw, ghb = aux_head(x, hb, wh, tg, B, T, H, eps)
        xs.append(x); caches.append(c); losses.append(loss); dxs.append(dx); dheads.append(dw)
        dhblocks.append(ghb)
    return comps, heads, xs, caches, np.array(losses), dxs, dheads, dhblocks


def nwise_definition(params, x0, targets, B, T, H, n, route="window_sum", eps=1e-5,
                     return_table=False):
    """Definition path: for every head j run an ordinary, untruncated backward of
    L_j alone down to component 1, keep dL_j/dtheta_k for all k <= j, then combine
    with the routing weights.  Returns dict(losses, comp_grads, head_grads, dx0)."""
    comps, heads, xs, caches, losses, dxs, dheads, dhblocks = forward_all(params, x0, targets, B, T, H, eps)
    K = len(comps)
    w = routing_weights(K, n, route)
    acc = [_zeros_like_grads(b) for b in comps]
    dx0 = np.zeros_like(xs[0])
    table = {}
    for j in range(1, K + 1):
        g = dxs[j - 1]
        for k in range(j, 0, -1):
            g, gr = component_backward(g, comps[k - 1], caches[k - 1])
            table[(k, j)] = gr
            _axpy(acc[k - 1], w[k - 1, j - 1], gr)
        dx0 += w[0, j - 1] * g
    out = dict(losses=losses, comp_grads=acc, head_grads=dheads, dx0=dx0,
               head_block_grads=dhblocks, x=xs)
    if return_table:
        out["table"] = table
    return out


def nwise_streams(params, x0, targets, B, T, H, n, route="window_sum", eps=1e-5):
    """Stream path: one forward; walk k = K..1 carrying each live gradient stream
    separately through component k's backward, credit its parameter gradient with
    the routing weight, and drop the stream once it has passed its lowest
    crediting component (stop-gradient at the window edge)."""
    comps, heads, xs, caches, losses, dxs, dheads, dhblocks = forward_all(params, x0, targets, B, T, H, eps)
    K = len(comps)
    w = routing_weights(K, n, route)
    plan = stream_plan(K, n, route)
    acc = [_zeros_like_grads(b) for b in comps]
    dx0 = np.zeros_like(xs[0])
    live = {}                                   # head j -> gradient at the current depth
    passes = []
    for k in range(K, 0, -1):
        if k in plan[k]:
            live[k] = dxs[k - 1]                # head k's stream starts here, age 0
        for j in list(live):
            if j not in plan[k]:
                del live[j]                     # window edge: the stream stops
        passes.append(len(live))
        for j in sorted(live):
            live[j], gr = component_backward(live[j], comps[k - 1], caches[k - 1])
            _axpy(acc[k - 1], w[k - 1, j - 1], gr)
    for j, g in live.items():
        dx0 += w[0, j - 1] * g
    return dict(losses=losses, comp_grads=acc, head_grads=dheads, dx0=dx0,
                head_block_grads=dhblocks, backward_passes=passes[::-1], x=xs)
