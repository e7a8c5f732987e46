"""Pins of the embedding oracle: brute force, the adjoint identity, an independent autograd model."""
import numpy as np
import torch

from oracle import embed as E


def _case(seed, B=3, T=5, d=4, V=7):
    rng = np.random.default_rng(seed)
    return (rng.normal(size=(V, d)), rng.normal(size=(T, d)), rng.integers(0, V, size=(B, T)),
            rng.normal(size=(B * T, d)))


def test_forward_and_backward_by_brute_force():
    wte, wpe, tok, dx0 = _case(0)
    B, T = tok.shape
    x0 = E.embed_forward(wte, wpe, tok)
    dwte, dwpe = E.embed_backward(dx0, tok, wte.shape[0])
    want_dwte, want_dwpe = np.zeros_like(wte), np.zeros_like(wpe)
    for b in range(B):
        for t in range(T):
            for c in range(wte.shape[1]):
                assert x0[b * T + t, c] == wte[tok[b, t], c] + wpe[t, c]
                want_dwte[tok[b, t], c] += dx0[b * T + t, c]
                want_dwpe[t, c] += dx0[b * T + t, c]
    np.testing.assert_allclose(dwte, want_dwte, rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(dwpe, want_dwpe, rtol=1e-14, atol=1e-15)


def test_repeated_and_absent_tokens():
    wte, wpe, tok, dx0 = _case(1, B=2, T=4, V=6)
    tok[:] = 2                                   # every position hits the same row
    dwte, _ = E.embed_backward(dx0, tok, 6)
    np.testing.assert_allclose(dwte[2], dx0.sum(axis=0), rtol=1e-14)
    assert not dwte[[0, 1, 3, 4, 5]].any()       # rows never looked up get exactly zero


def test_backward_is_the_adjoint_of_forward():
    """<dx0, forward(wte, wpe)> = <dwte, wte> + <dwpe, wpe> for a map that is linear in (wte, wpe)."""
    wte, wpe, tok, dx0 = _case(2, B=4, T=6, d=5, V=9)
    dwte, dwpe = E.embed_backward(dx0, tok, 9)
    lhs = float((dx0 * E.embed_forward(wte, wpe, tok)).sum())
    assert abs(lhs - float((dwte * wte).sum() + (dwpe * wpe).sum())) <= 1e-12 * abs(lhs)


def test_against_autograd_embedding():
    wte, wpe, tok, dx0 = _case(3, B=3, T=8, d=6, V=11)
    a = torch.tensor(wte, requires_grad=True)
    p = torch.tensor(wpe, requires_grad=True)
    x = torch.nn.functional.embedding(torch.tensor(tok), a) + p[None]
    np.testing.assert_allclose(x.detach().numpy().reshape(-1, 6), E.embed_forward(wte, wpe, tok), rtol=1e-15)
    x.backward(torch.tensor(dx0).reshape(3, 8, 6))
    dwte, dwpe = E.embed_backward(dx0, tok, 11)
    np.testing.assert_allclose(a.grad.numpy(), dwte, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(p.grad.numpy(), dwpe, rtol=1e-13, atol=1e-15)


def test_matches_the_input_generator_of_the_step():
    """synth.make_x0 (the harness's embedding in the step tests) is this forward on the same tables,
    up to its float32 arithmetic."""
    from paper_2010_04116_amd import synth
    w = synth.WORKLOADS["tiny"]
    inp, _ = synth.make_tokens(w)
    wte, wpe = synth.make_embeddings(w)
    np.testing.assert_allclose(synth.make_x0(w, inp), E.embed_forward(wte, wpe, inp), rtol=1e-6, atol=1e-9)
