"""GPU parity of il_embed_forward / il_embed_backward against the float64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import embed as E
from paper_2010_04116_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run(dtype, B, T, d, V, seed, tokens=None):
    rng = np.random.default_rng(seed)
    wte = (rng.normal(size=(V, d)) * 0.02).astype(np.float32)
    wpe = (rng.normal(size=(T, d)) * 0.02).astype(np.float32)
    if dtype == "bf16":
        wte, wpe = synth.round_to_bf16(wte), synth.round_to_bf16(wpe)
    tok = rng.integers(0, V, size=(B, T)).astype(np.int32) if tokens is None else tokens.astype(np.int32)
    dx0 = rng.normal(size=(B * T, d)).astype(np.float32)
    tt = torch.bfloat16 if dtype == "bf16" else torch.float32
    d_wte = torch.from_numpy(wte).to(tt).to(DEV)
    d_wpe = torch.from_numpy(wpe).to(tt).to(DEV)
    d_tok = torch.from_numpy(tok.reshape(-1)).to(DEV)
    x0 = torch.full((B * T, d), float("nan"), device=DEV)
    dwte = torch.full((V, d), float("nan"), device=DEV)          # the call must overwrite every element
    dwpe = torch.full((T, d), float("nan"), device=DEV)
    print("case embed", dtype, B, T, d, V, flush=True)
    binding.il_embed_forward(dtype, d_wte, d_wpe, d_tok, B, T, d, V, x0)
    binding.il_embed_backward(torch.from_numpy(dx0).to(DEV), d_tok, B, T, d, V, dwte, dwpe)
    torch.cuda.synchronize()
    got = dict(x0=x0.cpu().numpy(), dwte=dwte.cpu().numpy(), dwpe=dwpe.cpu().numpy())
    valid = (tok >= 0) & (tok < V)
    safe = np.where(valid, tok, 0)
    ref_x0 = E.embed_forward(wte, wpe, safe)
    ref_x0 = np.where(valid.reshape(-1, 1), ref_x0, ref_x0 - wte.astype(np.float64)[safe.reshape(-1)])
    ref_dwte, ref_dwpe = E.embed_backward(np.where(valid.reshape(-1, 1), dx0, 0.0), safe, V)
    ref_dwpe = E.embed_backward(dx0, safe, V)[1]
    return got, dict(x0=ref_x0, dwte=ref_dwte, dwpe=ref_dwpe), tok, dx0


def check(got, ref, tok, dx0, V):
    # forward: one correctly rounded fp32 add per element -> the rounded exact sum, bit for bit
    assert np.array_equal(got["x0"], ref["x0"].astype(np.float32))
    # index work, bit-exact: rows never hit are exactly zero, rows hit once are a copy of that dx0 row
    flat = tok.reshape(-1)
    counts = np.bincount(flat[(flat >= 0) & (flat < V)], minlength=V)
    assert not got["dwte"][counts == 0].any()
    once = np.flatnonzero(counts == 1)
    pos = {int(v): i for i, v in enumerate(flat)}                # (last position of each token; unique for `once`)
    for v in once[:200]:
        assert np.array_equal(got["dwte"][v], dx0[pos[int(v)]])
    # sums of a few fp32 terms in a fixed order: 1e-6 of the result's norm per tensor
    for name in ("dwte", "dwpe"):
        err = np.linalg.norm(got[name] - ref[name]) / max(np.linalg.norm(ref[name]), 1e-300)
        assert err <= 1e-6, (name, err)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,T,d,V", [(2, 32, 64, 256), (3, 13, 50, 77), (1, 1, 4, 1), (8, 256, 512, 8192)])
def test_parity(dtype, B, T, d, V):
    got, ref, tok, dx0 = run(dtype, B, T, d, V, seed=B * 1000 + T)
    check(got, ref, tok, dx0, V)


def test_every_position_hits_a_handful_of_rows():
    """5000 positions over 5 vocabulary rows: one workgroup takes them all, in several list passes."""
    got, ref, tok, dx0 = run("f32", 5, 1000, 24, 5, seed=3)
    check(got, ref, tok, dx0, 5)
    # ascending-position fp32 summation, reproduced on the host
    want = np.zeros((5, 24), dtype=np.float32)
    for i, v in enumerate(tok.reshape(-1)):
        want[v] += dx0[i]
    assert np.array_equal(got["dwte"], want)


def test_tokens_out_of_range_are_inert():
    tok = np.array([[0, 5, -1, 7, 99, 3]], dtype=np.int32)
    got, ref, tok, dx0 = run("f32", 1, 6, 8, 8, seed=4, tokens=tok)
    check(got, ref, tok, dx0, 8)


def test_bit_reproducible():
    a = run("bf16", 4, 128, 256, 300, seed=5)[0]
    b = run("bf16", 4, 128, 256, 300, seed=5)[0]
    for k in a:
        assert np.array_equal(a[k], b[k])


def test_misuse():
    x = torch.zeros(64, device=DEV)
    t = torch.zeros(8, dtype=torch.int32, device=DEV)
    with pytest.raises(binding.InterlockError) as e:
        binding.il_embed_forward("f32", x, x, t, 0, 8, 8, 8, x)
    assert e.value.status == binding.IL_E_ARG
    with pytest.raises(binding.InterlockError) as e:
        binding.il_embed_backward(x, None, 1, 8, 8, 8, x, x)
    assert e.value.status == binding.IL_E_ARG
    with pytest.raises(binding.InterlockError) as e:
        binding.il_embed_forward("f32", x, x, t, 1, 8, 8, 8, x[1:])       # misaligned output
    assert e.value.status == binding.IL_E_SHAPE
