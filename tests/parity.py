"""Shared helpers of the GPU parity tests: run the HIP path and the oracle on the same
seeded inputs and compare element by element.

Tolerances (the benchmark spec): fp32 - relative error <= 1e-4 on every loss and on every
gradient tensor; bf16 - <= 1e-3 on losses, <= 2e-2 on gradient tensors.  A loss is compared
as |a-b|/|b|; a gradient tensor as ||a-b||_2/||b||_2 over the whole tensor.

A norm over a whole tensor can hide a wrong row, a dropped ragged-edge column or one bad
tile, so every tensor is also held to three element-level bounds:
  rows / cols  for every matrix, the L2 error of each row (column) relative to that row's
               (column's) own norm, with the tensor's RMS row (column) norm as a floor so that
               rows that are legitimately tiny are measured on the tensor's scale;
  elem         max |a-b| / (scale + |b|), scale = the largest of the RMS of the tensor, of the
               element's row and of its column: no single element may be off by more than a fraction
               of the typical magnitude around it or of its own magnitude.  (A head matrix's gradient
               is near zero except in the columns of the target tokens, whose entries are sums of a
               few x_r / N that are hundreds of times the tensor's RMS: the rounding of x to bf16 is
               an error on THAT scale, which is why the column's RMS belongs to the yardstick.)
A completely wrong row scores about 1 (or more) on `rows`, a zeroed tile 1 on both, a single
garbage or dropped element 0.5 or more on `elem`; rounding noise scores a small multiple of the tensor
tolerance (the bounds are ROW_FACTOR and ELEM_FACTOR times it).  Measured worst over all cases, the
full-size runs included: bf16 tensor 8.5e-3, rows 1.4e-2, cols 4.8e-2, elem 5.3e-2; fp32 9e-7, 1e-6,
2.4e-6, 3e-6.
"""
import json
import os

import numpy as np

from oracle import interlock as O
from paper_2010_04116_amd import binding, synth

TOL = {"f32": dict(loss=1e-4, grad=1e-4), "bf16": dict(loss=1e-3, grad=2e-2)}
ROW_FACTOR = 4.0      # rows / cols bound = ROW_FACTOR * tensor tolerance  (bf16: 8e-2, fp32: 4e-4)
ELEM_FACTOR = 6.0     # elem bound = ELEM_FACTOR * tensor tolerance         (bf16: 0.12, fp32: 6e-4)

# observed margins of the run, by label: written to $IL_PARITY_MARGINS (a JSON file) when set
MARGINS = {}


def rel(a, b):
    nb = np.linalg.norm(b)
    return np.linalg.norm(np.asarray(a, np.float64) - b) / (nb if nb > 0 else 1.0)


def elementwise(a, b):
    """(tensor, rows, cols, elem) error figures of a against the reference b."""
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    diff = a - b
    nb = np.linalg.norm(b)
    out = {"tensor": np.linalg.norm(diff) / (nb if nb > 0 else 1.0)}
    rms = nb / np.sqrt(b.size) if b.size else 0.0
    scale = rms if rms > 0 else 1.0
    if b.ndim == 2 and min(b.shape) > 1:
        b2 = b * b
        for name, axis in (("rows", 1), ("cols", 0)):
            nref = np.sqrt(b2.sum(axis=axis))
            floor = np.sqrt((nref * nref).mean())
            e = np.sqrt((diff * diff).sum(axis=axis)) / np.maximum(nref, floor if floor > 0 else 1.0)
            out[name] = float(e.max())
        rrms = np.sqrt(b2.mean(axis=1, keepdims=True))
        crms = np.sqrt(b2.mean(axis=0, keepdims=True))
        scale = np.maximum(np.maximum(rrms, crms), scale)
    out["elem"] = float((np.abs(diff) / (scale + np.abs(b))).max())
    return out


def check_tensor(a, b, tol, what, worst, key, elem_factor=None):
    """Holds a to the bounds; violations are collected in worst["violations"] (see assert_clean), so
    that one run reports every tensor out of bounds, not only the first."""
    bad = worst.setdefault("violations", [])
    if np.linalg.norm(b) == 0:
        if np.linalg.norm(a) != 0:
            bad.append(f"{what}: expected exact zero")
        return
    if not np.all(np.isfinite(a)):
        bad.append(f"{what}: non-finite values")
        return
    e = elementwise(a, b)
    if e["tensor"] > tol:
        bad.append(f"{what}: rel err {e['tensor']:.3e}")
    for k in ("rows", "cols"):
        if k in e and e[k] > ROW_FACTOR * tol:
            bad.append(f"{what}: worst {k[:-1]} rel err {e[k]:.3e}")
    if e["elem"] > (elem_factor or ELEM_FACTOR) * tol:
        bad.append(f"{what}: max |a-b| / (scale + |b|) = {e['elem']:.3e}")
    for k, v in e.items():
        kk = f"{key}.{k}"
        worst[kk] = max(worst.get(kk, 0.0), float(v))


def assert_clean(worst, label=""):
    bad = worst.pop("violations", [])
    assert not bad, f"{label}: {len(bad)} bound(s) exceeded:\n  " + "\n  ".join(bad[:40])


def make_inputs(w, seed=0, random_bias=True, random_ln=True):
    params = synth.make_params(w, synth.PARAM_SEED + seed, random_bias=random_bias, random_ln=random_ln)
    inp, tgt = synth.make_tokens(w, synth.TOKEN_SEED + seed)
    x0 = synth.make_x0(w, inp, synth.PARAM_SEED + seed)
    return params, x0, tgt


def compare(w, got, ref, label="", scale=1.0, head_elem_factor=None):
    """Every loss, every component / head / head-block gradient tensor and dL/dx_0 of `got`
    (the HIP path) against `ref` (the oracle).  `scale` multiplies the HIP path's gradients first
    (the ignored-target test compares half a batch with the oracle's whole one);
    `head_elem_factor` replaces ELEM_FACTOR for the head matrices' gradients (replicated-batch runs)."""
    tol = TOL[w.dtype]
    worst = {}
    for k in range(w.K):
        e = abs(got["losses"][k] - ref["losses"][k]) / abs(ref["losses"][k])
        if not e <= tol["loss"]:
            worst.setdefault("violations", []).append(f"{label} loss {k + 1}: rel err {e:.3e}")
        worst["loss"] = max(worst.get("loss", 0), float(e))
        for l in range(w.L):
            for name in synth.BLOCK_TENSORS:
                check_tensor(got["comp_grads"][k][l][name] * scale, ref["comp_grads"][k][l][name], tol["grad"],
                             f"{label} component {k + 1} block {l + 1} {name}", worst, name)
        check_tensor(got["head_grads"][k] * scale, ref["head_grads"][k], tol["grad"], f"{label} head {k + 1}",
                     worst, "w_head", head_elem_factor)
        for l in range(w.Lh):                                  # the head's own blocks
            for name in synth.BLOCK_TENSORS:
                check_tensor(got["head_block_grads"][k][l][name] * scale, ref["head_block_grads"][k][l][name],
                             tol["grad"], f"{label} head {k + 1} block {l + 1} {name}", worst, "head_" + name)
    if np.linalg.norm(ref["dx0"]) > 0:
        check_tensor(got["dx0"] * scale, ref["dx0"], tol["grad"], f"{label} dx0", worst, "dx0")
    bad = worst.get("violations", [])
    record(label, w, {k: v for k, v in worst.items() if k != "violations"})
    assert_clean(worst, label)
    return worst


def record(label, w, worst):
    MARGINS[label or w.name] = dict(dtype=w.dtype, **{k: float(v) for k, v in worst.items()})
    path = os.environ.get("IL_PARITY_MARGINS")
    if path:
        with open(path, "w") as f:
            json.dump(MARGINS, f, indent=1, sort_keys=True)


def summary(worst):
    """One short line: the largest figure of each kind over all tensors."""
    out = {}
    for k, v in worst.items():
        kind = k.rsplit(".", 1)[-1] if "." in k else k
        out[kind] = max(out.get(kind, 0.0), v)
    return " ".join(f"{k}={v:.2e}" for k, v in sorted(out.items()))


def run_both(w, route="window_sum", seed=0, head_chunk=0, random_bias=True, random_ln=True):
    params, x0, tgt = make_inputs(w, seed, random_bias, random_ln)
    got = binding.run_step(w, params, x0, tgt, route=route, head_chunk=head_chunk)
    ref = O.nwise_streams(params, x0, tgt, w.B, w.T, w.H, w.n, route=route)
    return got, ref
