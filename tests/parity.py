"""Shared helpers of the GPU parity tests: run the HIP path and the oracle on the same
seeded inputs and compare element by element.

Tolerances (the benchmark spec): fp32 - relative error <= 1e-4 on every loss and on every
gradient tensor; bf16 - <= 1e-3 on losses, <= 2e-2 on gradient tensors.  A loss is compared
as |a-b|/|b|; a gradient tensor as ||a-b||_2/||b||_2 over the whole tensor."""
import numpy as np

from oracle import interlock as O
from paper_2010_04116_amd import binding, synth

TOL = {"f32": dict(loss=1e-4, grad=1e-4), "bf16": dict(loss=1e-3, grad=2e-2)}


def rel(a, b):
    nb = np.linalg.norm(b)
    return np.linalg.norm(np.asarray(a, np.float64) - b) / (nb if nb > 0 else 1.0)


def make_inputs(w, seed=0, random_bias=True, random_ln=True):
    params = synth.make_params(w, synth.PARAM_SEED + seed, random_bias=random_bias, random_ln=random_ln)
    inp, tgt = synth.make_tokens(w, synth.TOKEN_SEED + seed)
    x0 = synth.make_x0(w, inp, synth.PARAM_SEED + seed)
    return params, x0, tgt


def compare(w, got, ref, label=""):
    tol = TOL[w.dtype]
    worst = {}
    for k in range(w.K):
        e = abs(got["losses"][k] - ref["losses"][k]) / abs(ref["losses"][k])
        assert e <= tol["loss"], f"{label} loss {k + 1}: rel err {e:.3e}"
        worst["loss"] = max(worst.get("loss", 0), e)
        for l in range(w.L):
            for name in synth.BLOCK_TENSORS:
                b = ref["comp_grads"][k][l][name]
                a = got["comp_grads"][k][l][name]
                if np.linalg.norm(b) == 0:
                    assert np.linalg.norm(a) == 0, f"{label} c{k + 1} b{l + 1} {name}: expected exact zero"
                    continue
                e = rel(a, b)
                assert e <= tol["grad"], f"{label} component {k + 1} block {l + 1} {name}: rel err {e:.3e}"
                worst[name] = max(worst.get(name, 0), e)
        e = rel(got["head_grads"][k], ref["head_grads"][k])
        assert e <= tol["grad"], f"{label} head {k + 1}: rel err {e:.3e}"
        worst["w_head"] = max(worst.get("w_head", 0), e)
        for l in range(w.Lh):                                  # the head's own blocks
            for name in synth.BLOCK_TENSORS:
                e = rel(got["head_block_grads"][k][l][name], ref["head_block_grads"][k][l][name])
                assert e <= tol["grad"], f"{label} head {k + 1} block {l + 1} {name}: rel err {e:.3e}"
                worst["head_" + name] = max(worst.get("head_" + name, 0), e)
    if np.linalg.norm(ref["dx0"]) > 0:
        e = rel(got["dx0"], ref["dx0"])
        assert e <= tol["grad"], f"{label} dx0: rel err {e:.3e}"
        worst["dx0"] = e
    return worst


def run_both(w, route="window_sum", seed=0, head_chunk=0, random_bias=True, random_ln=True):
    params, x0, tgt = make_inputs(w, seed, random_bias, random_ln)
    got = binding.run_step(w, params, x0, tgt, route=route, head_chunk=head_chunk)
    ref = O.nwise_streams(params, x0, tgt, w.B, w.T, w.H, w.n, route=route)
    return got, ref
