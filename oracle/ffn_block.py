"""Plain fp64 oracle of the feed-forward block of a decoder layer, one token per sequence.

TEST INFRASTRUCTURE ONLY (see oracle/decode_block.py): nothing of the product imports this module, and it shares no
code with the HIP kernel of the block.

What it computes (paper Sec. 2.1, the FFN equation: three linear layers with a non-linear activation in between,
FFN(Z) = W3 (sigma(W1 Z) * W2 Z) with * the element-wise product), for every batch row z_b on its own:

    h = W1 z_b            [d_ff]        W1, W2: [d_ff, d_model]  (row f holds the weights of hidden unit f: the paper
    u = W2 z_b            [d_ff]                                  writes the product with the matrix on the left)
    g = sigma(h) * u      [d_ff]
    out_b = g W3          [d_model]     W3: [d_ff, d_model]      (row f holds what hidden unit f adds to the output)

Readings (the paper leaves them open): sigma is "a non-linear activation (e.g., GELU)"; the Llama-family layers whose
shapes the paper measures use SiLU, sigma(a) = a / (1 + exp(-a)), which is the default here, and GELU in its exact
form a * Phi(a) (Phi the standard normal distribution function) is the other choice.  No bias terms.  Inputs are taken
as they are (fp16 values converted exactly); nothing is rounded on the way; the result is fp64.
"""
from __future__ import annotations

import math

import numpy as np

ACT_SILU = 0
ACT_GELU = 1


def activation(a, act: int):
    a = np.asarray(a, dtype=np.float64)
    if act == ACT_SILU:
        return a / (1.0 + np.exp(-a))
    if act == ACT_GELU:
        erf = np.vectorize(math.erf, otypes=[np.float64])
        return 0.5 * a * (1.0 + erf(a / math.sqrt(2.0)))
    raise ValueError("unknown activation %r" % (act,))


def ffn_block(z, w1, w2, w3, act: int = ACT_SILU):
    """z [B, d_model]; w1, w2, w3 [d_ff, d_model].  Returns {"out": [B, d_model], "h", "u", "g": [B, d_ff]} in fp64."""
    z = np.asarray(z).astype(np.float64)
    w1 = np.asarray(w1).astype(np.float64)
    w2 = np.asarray(w2).astype(np.float64)
    w3 = np.asarray(w3).astype(np.float64)
    B, D = z.shape
    F = w1.shape[0]
    assert w1.shape == (F, D) and w2.shape == (F, D) and w3.shape == (F, D)
    h = np.empty((B, F))
    u = np.empty((B, F))
    g = np.empty((B, F))
    out = np.empty((B, D))
    for b in range(B):
        h[b] = w1 @ z[b]
        u[b] = w2 @ z[b]
        g[b] = activation(h[b], act) * u[b]
        out[b] = g[b] @ w3
    return {"out": out, "h": h, "u": u, "g": g}
