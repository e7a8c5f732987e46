"""Pins for auxiliary heads that contain Transformer blocks in front of their output matrix (the
paper's Transformer runs, App. B): an independent float64 autograd model with stop-gradient,
finite differences of the head's own parameters, and the reduction to the bare linear head."""
import numpy as np
import pytest
import torch

from oracle import interlock as O
from paper_2010_04116_amd import synth
from test_oracle_routing import make, rel, torch_block

W = synth.Workload("pinh", "f32", K=3, L=1, d=8, H=2, m=16, V=11, B=2, T=5, n=2, Lh=2)


def make_h(w, seed=3, scale=8.0):
    p, x0, tgt = make(w, seed, scale)
    for blocks in p["head_blocks"]:
        for b in blocks:
            for k in b:
                if k.startswith("w_"):
                    b[k] = b[k] * scale
    return p, x0, tgt


def torch_nwise_h(p, x0, tgt, w, route_w):
    """As test_oracle_routing.torch_nwise, with head j = blocks_j followed by W_j.  The gradient
    that reaches the trunk from L_j flows back through head j's blocks (their values, detached as
    parameters); the head's own parameters see L_j with the trunk detached, weight 1."""
    T_ = lambda v: torch.tensor(v, dtype=torch.float64, requires_grad=True)
    tp = [[{k: T_(v) for k, v in b.items()} for b in blocks] for blocks in p["components"]]
    hb = [[{k: T_(v) for k, v in b.items()} for b in blocks] for blocks in p["head_blocks"]]
    th = [T_(h) for h in p["heads"]]
    x0t = T_(x0)
    y = torch.tensor(tgt.reshape(-1), dtype=torch.long)
    det = lambda blocks: [{k: v.detach() for k, v in b.items()} for b in blocks]
    xent = torch.nn.functional.cross_entropy
    def head(x, j, live):
        for b in (hb[j] if live else det(hb[j])):
            x = torch_block(x, b, w.B, w.T, w.H)
        return xent(x @ (th[j] if live else th[j].detach()), y)
    total, losses, K = 0.0, [], len(tp)
    for j in range(K):
        x = x0t.detach()
        for k in range(j + 1):
            for b in det(tp[k]):
                x = torch_block(x, b, w.B, w.T, w.H)
        losses.append(head(x.detach(), j, True))
        total = total + losses[-1]
        for k in range(j + 1):
            if route_w[k, j] == 0:
                continue
            xx = x0t if k == 0 else x0t.detach()
            for kk in range(j + 1):
                for b in (tp[kk] if kk == k else det(tp[kk])):
                    xx = torch_block(xx, b, w.B, w.T, w.H)
            total = total + route_w[k, j] * head(xx, j, False)
    total.backward()
    return tp, hb, th, x0t, [float(l.detach()) for l in losses]


@pytest.mark.parametrize("route", O.ROUTES)
@pytest.mark.parametrize("n", [1, 2, 3])
def test_streams_match_autograd_with_block_heads(n, route):
    p, x0, tgt = make_h(W)
    got = O.nwise_streams(p, x0, tgt, W.B, W.T, W.H, n=n, route=route)
    tp, hb, th, x0t, losses = torch_nwise_h(p, x0, tgt, W, O.routing_weights(W.K, n, route))
    np.testing.assert_allclose(got["losses"], losses, rtol=1e-12)
    for k in range(W.K):
        for name in synth.BLOCK_TENSORS:
            ref = tp[k][0][name].grad
            ref = np.zeros_like(got["comp_grads"][k][0][name]) if ref is None else ref.numpy()
            assert np.allclose(got["comp_grads"][k][0][name], ref, rtol=1e-9, atol=1e-13), (k, name)
            for l in range(W.Lh):
                assert np.allclose(got["head_block_grads"][k][l][name], hb[k][l][name].grad.numpy(),
                                   rtol=1e-9, atol=1e-13), ("head", k, l, name)
        assert rel(got["head_grads"][k], th[k].grad.numpy()) < 1e-11
    assert rel(got["dx0"], x0t.grad.numpy()) < 1e-10


def test_finite_differences_of_the_heads_own_blocks():
    p, x0, tgt = make_h(W)
    p = {"components": [[{k: v.astype(np.float64) for k, v in b.items()} for b in bl] for bl in p["components"]],
         "heads": [h.astype(np.float64) for h in p["heads"]],
         "head_blocks": [[{k: v.astype(np.float64) for k, v in b.items()} for b in bl] for bl in p["head_blocks"]]}
    out = O.nwise_definition(p, x0, tgt, W.B, W.T, W.H, n=2)
    rng = np.random.default_rng(0)
    eps = 1e-6
    losses = lambda: O.forward_all(p, x0, tgt, W.B, W.T, W.H)[4]
    for j in range(W.K):
        for l in range(W.Lh):
            for name in synth.BLOCK_TENSORS:
                a = p["head_blocks"][j][l][name]
                i = tuple(rng.integers(0, s) for s in a.shape)
                old = a[i]
                a[i] = old + eps; lp = losses()
                a[i] = old - eps; lm = losses()
                a[i] = old
                num = (lp - lm) / (2 * eps)
                want = out["head_block_grads"][j][l][name][i]
                assert abs(num[j] - want) < 1e-7 * max(1.0, abs(want)) + 1e-9, (j, l, name)
                others = np.delete(num, j)
                assert np.all(np.abs(others) < 1e-9)          # head j's blocks touch no other loss


def test_no_blocks_is_the_linear_head():
    p, x0, tgt = make(W.with_(Lh=0))
    a = O.nwise_streams(p, x0, tgt, W.B, W.T, W.H, n=2)
    q = dict(p); q.pop("head_blocks")
    b = O.nwise_streams(q, x0, tgt, W.B, W.T, W.H, n=2)
    assert np.array_equal(a["losses"], b["losses"]) and np.array_equal(a["dx0"], b["dx0"])
    assert a["head_block_grads"] == [[], [], []]


def test_stream_path_equals_definition_path_with_block_heads():
    p, x0, tgt = make_h(W)
    for n in (1, 2, 3):
        a = O.nwise_streams(p, x0, tgt, W.B, W.T, W.H, n=n)
        b = O.nwise_definition(p, x0, tgt, W.B, W.T, W.H, n=n)
        assert rel(a["dx0"], b["dx0"]) < 1e-12
        for k in range(W.K):
            for name in synth.BLOCK_TENSORS:
                assert rel(a["comp_grads"][k][0][name], b["comp_grads"][k][0][name]) < 1e-11
