"""Seeded synthetic inputs for the n-wise interlocking-backprop step.

This module only *draws* inputs (token ids, parameter tensors, the embedded
input x_0) and names the workloads; it holds none of the method's arithmetic
(no LayerNorm, attention, loss or routing).  Both the CPU oracle's tests and the
GPU harness take their inputs from here so that they see identical bits.

Workload shapes stand in for the paper's LM1B Transformer experiment (Sec. 4.3,
App. B "Transformer" paragraph: decoder-only GPT-2-like blocks grouped into
modules of equal depth, fixed-length token windows) at sizes that fit one GPU.
Tokens are i.i.d. uniform over the vocabulary, weights N(0, 0.02^2), LayerNorm
gain 1 / bias 0, linear biases 0 unless `random_bias` is set.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    """One problem instance: K components of L pre-LN blocks, one head each."""
    name: str
    dtype: str      # "f32" or "bf16": storage type of parameters / GEMM operands
    K: int          # components (the paper's modules)
    L: int          # Transformer blocks per component
    d: int          # model width
    H: int          # attention heads
    m: int          # MLP width
    V: int          # vocabulary (head output width)
    B: int          # batch (sequences)
    T: int          # sequence length
    n: int          # n-wise window
    Lh: int = 0     # Transformer blocks inside each auxiliary head, in front of its d -> V map

    @property
    def N(self) -> int:
        return self.B * self.T

    @property
    def dh(self) -> int:
        return self.d // self.H

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", "f32", K=4, L=1, d=64, H=4, m=256, V=256, B=2, T=32, n=2),
    "small": Workload("small", "bf16", K=4, L=2, d=512, H=8, m=2048, V=8192, B=8, T=256, n=2),
    "medium": Workload("medium", "bf16", K=4, L=6, d=1024, H=16, m=4096, V=32768, B=8, T=512, n=2),
    "many_head": Workload("many_head", "bf16", K=8, L=3, d=1024, H=16, m=4096, V=32768, B=8, T=512, n=3),
    "large": Workload("large", "bf16", K=6, L=6, d=2048, H=16, m=8192, V=50304, B=4, T=1024, n=2),
    # the shape of the paper's own Transformer modules (Sec. 4.3, App. B: 6 blocks per module, d = 1024,
    # 4 attention heads -> head width 256, sequences of 128, auxiliary heads of 2 blocks + output matrix),
    # one accelerator's worth of batch
    "paper": Workload("paper", "bf16", K=4, L=6, d=1024, H=4, m=4096, V=32768, B=32, T=128, n=2, Lh=2),
}
PARAM_SEED = 20100411
TOKEN_SEED = 20100511

# Parameter tensors of one block, in the order of the flat device layout.
BLOCK_TENSORS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                 "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


def block_shapes(w: Workload) -> Dict[str, Tuple[int, ...]]:
    d, m = w.d, w.m
    return {"ln1_g": (d,), "ln1_b": (d,), "w_qkv": (d, 3 * d), "b_qkv": (3 * d,),
            "w_o": (d, d), "b_o": (d,), "ln2_g": (d,), "ln2_b": (d,),
            "w_fc1": (d, m), "b_fc1": (m,), "w_fc2": (m, d), "b_fc2": (d,)}


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float32 -> nearest bfloat16 (ties to even), returned as float32 values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = u >> np.uint32(16)
    r &= np.uint32(1)
    r += np.uint32(0x7FFF)
    r += u                      # finite inputs cannot carry out of 32 bits (|a| < 2^128 - 2^112)
    r &= np.uint32(0xFFFF0000)
    return r.view(np.float32).reshape(a.shape)


def _rng(seed: int, *path: int) -> np.random.Generator:
    return np.random.default_rng([seed, *path])


def _store(w: Workload, a: np.ndarray) -> np.ndarray:
    return round_to_bf16(a) if w.dtype == "bf16" else a.astype(np.float32)


def make_block_params(w: Workload, k: int, l: int, seed: int = PARAM_SEED,
                      random_bias: bool = False, random_ln: bool = False) -> Dict[str, np.ndarray]:
    """Parameters of block l (1-based) of component k (1-based); float32 arrays
    whose values are representable in the workload's storage dtype."""
    out = {}
    for ti, (name, shp) in enumerate(block_shapes(w).items()):
        g = _rng(seed, k, l, ti)
        if name.startswith("w_"):
            a = g.standard_normal(shp, dtype=np.float32) * np.float32(0.02)
        elif name.endswith("_g"):
            a = np.ones(shp, np.float32)
            if random_ln:
                a = a + g.standard_normal(shp, dtype=np.float32) * np.float32(0.1)
        elif name.startswith("ln"):
            a = np.zeros(shp, np.float32)
            if random_ln:
                a = g.standard_normal(shp, dtype=np.float32) * np.float32(0.1)
        else:
            a = np.zeros(shp, np.float32)
            if random_bias:
                a = g.standard_normal(shp, dtype=np.float32) * np.float32(0.02)
        out[name] = _store(w, a)
    return out


def make_head_params(w: Workload, k: int, seed: int = PARAM_SEED) -> np.ndarray:
    """Head k's weight, shape [d, V]; an independent draw per head (not tied)."""
    g = _rng(seed, 1000 + k)
    return _store(w, g.standard_normal((w.d, w.V), dtype=np.float32) * np.float32(0.02))


def make_params(w: Workload, seed: int = PARAM_SEED, random_bias: bool = False,
                random_ln: bool = False) -> dict:
    """{'components': [[block dict]*L]*K, 'heads': [w_head]*K, 'head_blocks': [[block dict]*Lh]*K}.
    Every tensor has a generator of its own (seed, component, block, tensor), so the draws do not
    depend on the order they are made in: large workloads draw their blocks on a few threads."""
    blk = lambda k, l: make_block_params(w, k, l, seed, random_bias, random_ln)
    jobs = [(k, l) for k in range(1, w.K + 1) for l in range(1, w.L + 1)]
    # the blocks of head k are drawn like those of a component numbered 1000 + k
    hjobs = [(1000 + k, l) for k in range(1, w.K + 1) for l in range(1, w.Lh + 1)]
    if (len(jobs) + len(hjobs)) * w.d * (4 * w.d + 2 * w.m) > 1 << 27:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=8) as ex:
            out = list(ex.map(lambda kl: blk(*kl), jobs + hjobs))
            heads = list(ex.map(lambda k: make_head_params(w, k, seed), range(1, w.K + 1)))
    else:
        out = [blk(k, l) for k, l in jobs + hjobs]
        heads = [make_head_params(w, k, seed) for k in range(1, w.K + 1)]
    comps = [out[(k - 1) * w.L:k * w.L] for k in range(1, w.K + 1)]
    hout = out[len(jobs):]
    hblocks = [hout[(k - 1) * w.Lh:k * w.Lh] for k in range(1, w.K + 1)]
    return {"components": comps, "heads": heads, "head_blocks": hblocks}


def make_tokens(w: Workload, seed: int = TOKEN_SEED) -> Tuple[np.ndarray, np.ndarray]:
    """(inputs [B,T], targets [B,T]) int32: next-token pairs from B rows of T+1
    uniform tokens."""
    tok = _rng(seed).integers(0, w.V, size=(w.B, w.T + 1), dtype=np.int64)
    return tok[:, :-1].astype(np.int32), tok[:, 1:].astype(np.int32)


def make_embeddings(w: Workload, seed: int = PARAM_SEED):
    """The seeded token and position tables (wte [V, d], wpe [T, d], N(0, 0.02^2), float32 values
    representable in the storage dtype) that make_x0 draws internally."""
    g = _rng(seed, 2000)
    wte = g.standard_normal((w.V, w.d), dtype=np.float32) * np.float32(0.02)
    wpe = g.standard_normal((w.T, w.d), dtype=np.float32) * np.float32(0.02)
    return _store(w, wte), _store(w, wpe)


def make_x0(w: Workload, inputs: np.ndarray, seed: int = PARAM_SEED) -> np.ndarray:
    """x_0[b,t] = wte[token] + wpe[t], float32 [B*T, d], values representable in
    the storage dtype.  The embedding tables are drawn here and not returned:
    the five library calls start at component activations."""
    g = _rng(seed, 2000)
    wte = g.standard_normal((w.V, w.d), dtype=np.float32) * np.float32(0.02)
    wpe = g.standard_normal((w.T, w.d), dtype=np.float32) * np.float32(0.02)
    x0 = wte[inputs.reshape(-1)] + np.tile(wpe, (w.B, 1))
    return _store(w, x0.astype(np.float32))


def make_activation(w: Workload, seed: int, scale: float = 1.0, rows: int | None = None,
                    cols: int | None = None) -> np.ndarray:
    """A seeded N(0, scale^2) [rows, cols] float32 array (default [N, d]) for
    per-component tests that start from a given activation or upstream gradient."""
    g = _rng(seed, 3000)
    a = g.standard_normal((rows or w.N, cols or w.d), dtype=np.float32) * np.float32(scale)
    return _store(w, a)
