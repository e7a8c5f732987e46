"""Pins for the oracle's primitives: closed forms, invariants, brute force on
tiny inputs and central finite differences.  CPU only."""
import math
import os

import numpy as np
import pytest

from oracle import interlock as O

RNG = np.random.default_rng(7)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def fd(f, x, eps=1e-6):
    """Central finite-difference gradient of scalar f at x (dense, small x)."""
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + eps; fp = f()
        x[i] = old - eps; fm = f()
        x[i] = old
        g[i] = (fp - fm) / (2 * eps)
    return g


def rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


# ---------------- LayerNorm ----------------

def test_layernorm_unit_gain_statistics():
    x = RNG.standard_normal((5, 16)) * 3 + 1
    eps = 1e-5
    y, _ = O.layernorm_forward(x, np.ones(16), np.zeros(16), eps)
    var = x.var(axis=-1)
    np.testing.assert_allclose(y.mean(-1), 0, atol=1e-14)
    np.testing.assert_allclose(y.var(-1), var / (var + eps), rtol=1e-12)


def test_layernorm_backward_orthogonality_and_fd():
    x = RNG.standard_normal((4, 12))
    g = RNG.standard_normal(12) + 1
    b = RNG.standard_normal(12)
    dy = RNG.standard_normal((4, 12))
    y, c = O.layernorm_forward(x, g, b, 1e-5)
    dx, dg, db = O.layernorm_backward(dy, c)
    xhat = c[0]
    np.testing.assert_allclose(dx.sum(-1), 0, atol=1e-13)          # orthogonal to 1
    # ... and to xhat up to the eps term: sum(dx*xhat) = rstd*sum(dy*g*xhat)*(1 - mean(xhat^2))
    resid = c[1][:, 0] * (dy * g * xhat).sum(-1) * (1 - (xhat * xhat).mean(-1))
    np.testing.assert_allclose((dx * xhat).sum(-1), resid, atol=1e-13)
    assert np.all(np.abs(resid) < 1e-3)
    f = lambda: (O.layernorm_forward(x, g, b, 1e-5)[0] * dy).sum()
    assert rel(dx, fd(f, x)) < 1e-7
    assert rel(dg, fd(f, g)) < 1e-7
    assert rel(db, fd(f, b)) < 1e-7


# ---------------- GELU ----------------

def test_gelu_values_and_derivative():
    assert O.gelu(np.array(0.0)) == 0.0
    np.testing.assert_allclose(O.gelu(np.array([12.0, -12.0])), [12.0, 0.0], atol=1e-12)
    # value at 1 of the tanh form, worked by hand with math.tanh
    ref = 0.5 * (1 + math.tanh(math.sqrt(2 / math.pi) * 1.044715))
    assert abs(O.gelu(np.array(1.0)) - ref) < 1e-15
    u = np.linspace(-4, 4, 41)
    num = (O.gelu(u + 1e-6) - O.gelu(u - 1e-6)) / 2e-6
    np.testing.assert_allclose(O.gelu_grad(u), num, atol=1e-8)


# ---------------- attention ----------------

def brute_attention(qkv, B, T, H):
    N, d3 = qkv.shape
    d = d3 // 3
    dh = d // H
    out = np.zeros((N, d))
    for b in range(B):
        for h in range(H):
            for t in range(T):
                q = qkv[b * T + t, h * dh:(h + 1) * dh]
                sc = []
                for u in range(t + 1):
                    kk = qkv[b * T + u, d + h * dh:d + (h + 1) * dh]
                    sc.append(float(q @ kk) / math.sqrt(dh))
                mx = max(sc)
                e = [math.exp(s - mx) for s in sc]
                z = sum(e)
                for u in range(t + 1):
                    vv = qkv[b * T + u, 2 * d + h * dh:2 * d + (h + 1) * dh]
                    out[b * T + t, h * dh:(h + 1) * dh] += e[u] / z * vv
    return out


def test_attention_matches_triple_loop():
    B, T, H, dh = 2, 5, 3, 4
    qkv = RNG.standard_normal((B * T, 3 * H * dh))
    o, c = O.attention_forward(qkv, B, T, H)
    np.testing.assert_allclose(o, brute_attention(qkv, B, T, H), atol=1e-13)
    np.testing.assert_allclose(c[3].sum(-1), 1.0, atol=1e-14)       # rows of P
    assert np.all(np.triu(c[3][0, 0], 1) == 0)                      # causal


def test_attention_T1_is_identity_on_V():
    qkv = RNG.standard_normal((3, 3 * 8))
    o, _ = O.attention_forward(qkv, 3, 1, 2)
    np.testing.assert_allclose(o, qkv[:, 16:], atol=1e-15)


def test_attention_causality_and_fd():
    B, T, H, dh = 1, 6, 2, 3
    d = H * dh
    qkv = RNG.standard_normal((B * T, 3 * d))
    o1, c = O.attention_forward(qkv, B, T, H)
    q2 = qkv.copy(); q2[4:] += 1.0                                  # edit positions >= 4
    o2, _ = O.attention_forward(q2, B, T, H)
    np.testing.assert_array_equal(o1[:4], o2[:4])
    do = RNG.standard_normal((B * T, d))
    dqkv = O.attention_backward(do, c)
    f = lambda: (O.attention_forward(qkv, B, T, H)[0] * do).sum()
    assert rel(dqkv, fd(f, qkv)) < 1e-7
    # gradient of position-t output w.r.t. later positions is zero
    do0 = np.zeros_like(do); do0[2] = 1.0
    dq0 = O.attention_backward(do0, c)
    assert np.all(dq0[3:] == 0)


# ---------------- cross-entropy head ----------------

def test_xent_zero_weight_closed_form():
    with open(os.path.join(GOLDEN, "ln_vocab.txt")) as fh:
        rows = [l.split() for l in fh if l.strip() and not l.startswith("#")]
    for V_s, lnV_s in rows:
        V, lnV = int(V_s), float(lnV_s)
        N, d = 6, 4
        x = RNG.standard_normal((N, d))
        y = RNG.integers(0, V, N)
        loss, dx, dw = O.head_xent(x, np.zeros((d, V)), y)
        assert abs(loss - lnV) < 5e-7                               # file holds 6 decimals
        assert abs(loss - math.log(V)) < 1e-12
        # dz = (1/V - onehot)/N  =>  dW = x^T dz
        dz = np.full((N, V), 1.0 / V); dz[np.arange(N), y] -= 1; dz /= N
        np.testing.assert_allclose(dw, x.T @ dz, atol=1e-15)
        np.testing.assert_allclose(dx, 0, atol=1e-15)


def test_xent_properties_and_fd():
    N, d, V = 5, 6, 9
    x = RNG.standard_normal((N, d)); w = RNG.standard_normal((d, V)) * 0.5
    y = RNG.integers(0, V, N)
    loss, dx, dw = O.head_xent(x, w, y)
    assert loss >= 0
    np.testing.assert_allclose(dw.sum(axis=1), 0, atol=1e-14)       # sum_v dz = 0
    # brute force with math.log / math.exp
    tot = 0.0
    for i in range(N):
        z = [float(x[i] @ w[:, v]) for v in range(V)]
        tot += math.log(sum(math.exp(t) for t in z)) - z[y[i]]
    assert abs(loss - tot / N) < 1e-13
    # shift invariance: adding a constant to every logit (an extra input column of
    # ones against a constant weight row) leaves the loss unchanged
    x1 = np.concatenate([x, np.ones((N, 1))], 1)
    w1 = np.concatenate([w, np.full((1, V), 3.7)], 0)
    assert abs(O.head_xent(x1, w1, y)[0] - loss) < 1e-13
    f = lambda: O.head_xent(x, w, y)[0]
    assert rel(dx, fd(f, x)) < 1e-7
    assert rel(dw, fd(f, w)) < 1e-7


# ---------------- block: finite differences on every tensor ----------------

def tiny_block(d, m):
    p = {"ln1_g": 1 + 0.1 * RNG.standard_normal(d), "ln1_b": 0.1 * RNG.standard_normal(d),
         "w_qkv": 0.3 * RNG.standard_normal((d, 3 * d)), "b_qkv": 0.1 * RNG.standard_normal(3 * d),
         "w_o": 0.3 * RNG.standard_normal((d, d)), "b_o": 0.1 * RNG.standard_normal(d),
         "ln2_g": 1 + 0.1 * RNG.standard_normal(d), "ln2_b": 0.1 * RNG.standard_normal(d),
         "w_fc1": 0.3 * RNG.standard_normal((d, m)), "b_fc1": 0.1 * RNG.standard_normal(m),
         "w_fc2": 0.3 * RNG.standard_normal((m, d)), "b_fc2": 0.1 * RNG.standard_normal(d)}
    return p


def test_block_backward_fd_all_tensors():
    B, T, H, d, m = 2, 4, 2, 6, 10
    p = tiny_block(d, m)
    x = RNG.standard_normal((B * T, d))
    dy = RNG.standard_normal((B * T, d))
    y, c = O.block_forward(x, p, B, T, H, 1e-5)
    dx, gr = O.block_backward(dy, p, c)
    f = lambda: (O.block_forward(x, p, B, T, H, 1e-5)[0] * dy).sum()
    assert rel(dx, fd(f, x)) < 1e-6
    for name in p:
        assert rel(gr[name], fd(f, p[name])) < 1e-6, name


def test_backward_is_linear_in_upstream_gradient():
    B, T, H, d, m = 2, 4, 2, 6, 10
    p = tiny_block(d, m)
    x = RNG.standard_normal((B * T, d))
    _, c = O.block_forward(x, p, B, T, H, 1e-5)
    g1 = RNG.standard_normal((B * T, d)); g2 = RNG.standard_normal((B * T, d))
    a, ga = O.block_backward(g1, p, c); b, gb = O.block_backward(g2, p, c)
    s, gs = O.block_backward(g1 + g2, p, c)
    np.testing.assert_allclose(s, a + b, atol=1e-12)
    for name in p:
        np.testing.assert_allclose(gs[name], ga[name] + gb[name], atol=1e-12)
