"""Plain fp64 oracle of one decode step of a transformer attention block.

TEST INFRASTRUCTURE ONLY.  Imported by tests, the smoke check and the bench's
cpu_baseline leg; never by the product path, and it imports nothing from it.

What it computes (paper Eq. 1, restricted to one new token per sequence, with
the decode semantics of Sec. 2.1: the cached keys/values are reused and the new
token's key/value are appended):

  for every batch row b:
    [q | k_new | v_new] = x_b . W_qkv          columns ordered Q heads, K heads, V heads
    q, k_new            <- RoPE(pos)           half-split pairing, theta_i = base^(-2i/d)
    K_g = cache_k[b,g,0:pos] ++ k_new[g]       pos+1 rows
    V_g = cache_v[b,g,0:pos] ++ v_new[g]
    a_i = softmax(K_g q_i / sqrt(d))^T V_g     g = i // (n_q / n_kv)
    out_b = concat_i(a_i) . W_o

Everything is evaluated in float64 from the exact values of the fp16 inputs;
nothing is blocked, fused or reordered.  The paper does not define RoPE, the
column order of W_qkv, the GQA head map, or whether the new token is part of
the attended set; the readings used here are listed in the design notes of the
repository and are stated next to each function.

Parity pins (tests/test_oracle_*.py): literal-loop brute force on tiny shapes,
RoPE identity/norm/relative-position/one-hot closed forms, uniform-softmax
closed form for x = 0, empty-cache case reducing to two matrix products,
hand-computed two-key example fixing the 1/sqrt(d) scale, convexity and
permutation invariance, GQA-vs-replicated-MHA, batch-row independence.
rms_norm / decode_layer (tests/test_oracle_layer.py): constant-row closed form, unit mean square,
scale invariance at eps = 0, a library routine (torch rms_norm in fp64), W_o = 0 leaves x, an input
of unit mean square with gamma = 1 reduces to x + decode_block(x).
"""
from __future__ import annotations

import numpy as np


def rope_angles(pos: int, head_dim: int, base: float) -> np.ndarray:
    """Angles pos * base^(-2i/d), i in [0, d/2) (fp64).  The paper is silent on
    RoPE; this is the usual definition with the frequency index over pairs."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    return float(pos) * np.power(float(base), -2.0 * i / float(head_dim))


def rope(v: np.ndarray, pos: int, base: float) -> np.ndarray:
    """Rotate the last axis of `v` (length d) at position `pos`.

    Pair i is (v[i], v[i + d/2]) ("half-split" pairing):
        out[i]       = v[i] cos(a_i) - v[i + d/2] sin(a_i)
        out[i + d/2] = v[i + d/2] cos(a_i) + v[i] sin(a_i)
    """
    v = np.asarray(v, dtype=np.float64)
    d = v.shape[-1]
    h = d // 2
    ang = rope_angles(pos, d, base)
    c, s = np.cos(ang), np.sin(ang)
    lo, hi = v[..., :h], v[..., h:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def softmax(s: np.ndarray) -> np.ndarray:
    """Softmax over the last axis with the maximum subtracted first."""
    s = np.asarray(s, dtype=np.float64)
    e = np.exp(s - np.max(s, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def decode_block(x, w_qkv, w_o, k_cache, v_cache, pos, n_q_heads, n_kv_heads,
                 head_dim, rope_base):
    """One decode step of the attention block.

    x        [B, D]                       fp16 (or any real dtype)
    w_qkv    [D, (n_q + 2 n_kv) d]        y = x . W  (paper Alg. 3: H x W^QKV)
    w_o      [n_q d, D]
    k_cache  [B, n_kv, max_seq, d]        rows 0..pos-1 are the cached, already rotated keys
    v_cache  [B, n_kv, max_seq, d]
    pos      tokens already cached == index of the new token

    Rows >= pos of the caches are never read.  Returns a dict of fp64 arrays:
      out    [B, D]         block output (not rounded)
      q_rot  [B, n_q, d]    rotated queries
      k_rot  [B, n_kv, d]   rotated new key  (what row `pos` of k_cache must hold, before fp16 rounding)
      v_new  [B, n_kv, d]   new value        (same for v_cache)
      attn   [B, n_q, d]    per-head attention output a_i
    """
    x = np.asarray(x)
    B, D = x.shape
    nq, nkv, d = int(n_q_heads), int(n_kv_heads), int(head_dim)
    G = nq // nkv
    assert nq % nkv == 0 and d % 2 == 0
    assert w_qkv.shape == (D, (nq + 2 * nkv) * d)
    assert w_o.shape == (nq * d, D)
    assert 0 <= pos < k_cache.shape[2]

    y = x.astype(np.float64) @ np.asarray(w_qkv).astype(np.float64)
    q = y[:, : nq * d].reshape(B, nq, d)
    k_new = y[:, nq * d: (nq + nkv) * d].reshape(B, nkv, d)
    v_new = y[:, (nq + nkv) * d:].reshape(B, nkv, d).copy()

    q_rot = rope(q, pos, rope_base)
    k_rot = rope(k_new, pos, rope_base)

    attn = np.empty((B, nq, d), dtype=np.float64)
    inv_sqrt_d = 1.0 / np.sqrt(float(d))
    for b in range(B):
        for g in range(nkv):
            K = np.concatenate([np.asarray(k_cache[b, g, :pos]).astype(np.float64),
                                k_rot[b, g][None, :]], axis=0)          # [pos+1, d]
            V = np.concatenate([np.asarray(v_cache[b, g, :pos]).astype(np.float64),
                                v_new[b, g][None, :]], axis=0)
            for i in range(g * G, (g + 1) * G):
                w = softmax((K @ q_rot[b, i]) * inv_sqrt_d)            # [pos+1]
                attn[b, i] = w @ V
    out = attn.reshape(B, nq * d) @ np.asarray(w_o).astype(np.float64)
    return {"out": out, "q_rot": q_rot, "k_rot": k_rot, "v_new": v_new, "attn": attn}


def rms_norm(x, gamma, eps):
    """RMSNorm of every row of x [B, D]:  x / sqrt(mean(x^2) + eps) * gamma, in fp64, nothing rounded.

    The paper does not define it (it leaves RMSNorm to other libraries, end of Sec. 3); this is the
    pre-normalisation of the Llama-family layers whose shapes the paper measures.
    """
    x = np.asarray(x).astype(np.float64)
    g = np.asarray(gamma).astype(np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + float(eps)) * g


def decode_layer(x, gamma, eps, w_qkv, w_o, k_cache, v_cache, pos, n_q_heads, n_kv_heads,
                 head_dim, rope_base):
    """The attention half of a pre-norm decoder layer:  out = x + block(rms_norm(x)).

    Same arguments and result as decode_block, plus gamma [D] and eps; `out` includes the residual.
    The normalised activations enter the block unrounded.
    """
    r = decode_block(rms_norm(x, gamma, eps), w_qkv, w_o, k_cache, v_cache, pos, n_q_heads, n_kv_heads,
                     head_dim, rope_base)
    r["out"] = r["out"] + np.asarray(x).astype(np.float64)
    return r


def decode_rows(x, gamma, eps, w_qkv, w_o, k_cache, v_cache, row_pos, n_q_heads, n_kv_heads,
                head_dim, rope_base, layer_fn=None, block_fn=None):
    """A batch whose rows have positions of their own (row b has row_pos[b] cached tokens).

    The rows of a batch do not interact anywhere in Eq. 1, so this is, by definition, the one-row computation
    applied to every row with that row's position: decode_layer when gamma is given (its `out` then includes
    the residual), else decode_block.  layer_fn / block_fn let a caller substitute another implementation of
    those two functions with the same contract (the C oracle).
    """
    layer_fn = layer_fn or decode_layer
    block_fn = block_fn or decode_block
    x = np.asarray(x)
    res = None
    for b in range(x.shape[0]):
        tail = (w_qkv, w_o, k_cache[b:b + 1], v_cache[b:b + 1], int(row_pos[b]), n_q_heads, n_kv_heads,
                head_dim, rope_base)
        r = layer_fn(x[b:b + 1], gamma, eps, *tail) if gamma is not None else block_fn(x[b:b + 1], *tail)
        if res is None:
            res = {k: [v] for k, v in r.items()}
        else:
            for k, v in r.items():
                res[k].append(v)
    return {k: np.concatenate(v, axis=0) for k, v in res.items()}


def attention_weights(q_rot_i, K):
    """Softmax weights of one query head over the rows of K (Eq. 1), exposed so
    that tests can check that they are non-negative and sum to one."""
    d = K.shape[-1]
    return softmax((np.asarray(K, np.float64) @ np.asarray(q_rot_i, np.float64)) / np.sqrt(float(d)))


# ---------------------------------------------------------------------------
# Split-KV partials and their merge (paper Alg. 3, steps 4-7)
# ---------------------------------------------------------------------------

def partial_attention(q, K, V):
    """FlashDecoding-style partial over one slice of the keys (Alg. 3 step 4):
    local max m, local sum l of exp(s - m), unnormalised acc = sum exp(s-m) v.
    An empty slice gives (-inf, 0, 0)."""
    d = q.shape[-1]
    if K.shape[0] == 0:
        return -np.inf, 0.0, np.zeros(V.shape[-1], dtype=np.float64)
    s = (np.asarray(K, np.float64) @ np.asarray(q, np.float64)) / np.sqrt(float(d))
    m = float(np.max(s))
    p = np.exp(s - m)
    return m, float(np.sum(p)), p @ np.asarray(V, np.float64)


def merge_partials(parts):
    """Combine per-slice (m, l, acc) into the softmax-weighted value (Alg. 3
    steps 5-7).  As printed, the algorithm sums the local sums next to taking
    the global max; local sums taken against different local maxima can only be
    added after rescaling, so the reading used is
        M = max m_i,  Lsum = sum l_i e^{m_i - M},  A = sum acc_i e^{m_i - M} / Lsum.
    Empty slices (m = -inf) contribute nothing."""
    M = max(m for m, _, _ in parts)
    Lsum = 0.0
    A = None
    for m, l, acc in parts:
        w = 0.0 if m == -np.inf else float(np.exp(m - M))
        Lsum += l * w
        A = acc * w if A is None else A + acc * w
    return A / Lsum
