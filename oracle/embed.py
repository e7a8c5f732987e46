"""Float64 oracle of the input embedding that the paper places inside the first module (App. B, the
module table: an embedding matrix in front of the Transformer blocks; Sec. 4.3, GPT-2-like model) and of
its gradient.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path imports this module; only tests/,
__graft_entry__.smoke() and bench.py's cpu_baseline leg may.  It shares no code with the HIP path.

Plain definitions, written out:
    x0[b*T + t, :] = wte[tokens[b, t], :] + wpe[t, :]
    dwte[v, :]     = sum over the positions i with tokens[i] == v of dx0[i, :]     (zero if none)
    dwpe[t, :]     = sum_b dx0[b*T + t, :]
Readings where the paper is silent: learned absolute positions added to the token embedding (the
GPT-2 convention the paper says it follows), no scaling by sqrt(d), no dropout.
"""
import numpy as np


def embed_forward(wte, wpe, tokens):
    """tokens: int [B, T] -> x0 float64 [B*T, d]."""
    wte = np.asarray(wte, dtype=np.float64)
    wpe = np.asarray(wpe, dtype=np.float64)
    tokens = np.asarray(tokens)
    B, T = tokens.shape
    return (wte[tokens] + wpe[None, :T, :]).reshape(B * T, wte.shape[1])


def embed_backward(dx0, tokens, vocab):
    """dx0: [B*T, d], tokens: int [B, T] -> (dwte [vocab, d], dwpe [T, d]) float64."""
    dx0 = np.asarray(dx0, dtype=np.float64)
    tokens = np.asarray(tokens)
    B, T = tokens.shape
    d = dx0.shape[1]
    dwte = np.zeros((vocab, d))
    np.add.at(dwte, tokens.reshape(-1), dx0)          # repeated tokens accumulate, in position order
    dwpe = dx0.reshape(B, T, d).sum(axis=0)
    return dwte, dwpe
