"""Plain fp64 oracle of one decode step of a Multi-Head Latent Attention block with weight absorption.

TEST INFRASTRUCTURE ONLY (see oracle/decode_block.py): it shares nothing with the HIP kernel of this block and was
written and pinned before it.

What it computes (paper Appendix B, "weight absorption" form: the three equations
Q = Hidden W_Q W_Up, K = Hidden W_K, V = K[:kv_lora_rank];  Z = Concat_i softmax(Q_i K^T / sqrt(d_k)) V;
Output = Z W_Down ... W_O, and Alg. 4), for one new token per sequence with the decode semantics of Sec. 2.1:

  for every batch row b, with l = kv_lora_rank, r = rope_dim, n = nope_dim, v = v_head_dim:
    q_i            = x_b . W_Q[:, head i]            [n + r]   -> (q_nope_i [n], q_rope_i [r])
    kv_new         = x_b . W_KV                      [l + r]   -> (c_new [l], k_rope_new [r])
    q_rope_i, k_rope_new <- RoPE(pos)                           half-split pairing, as in the other oracle
    q_lat_i        = q_nope_i . W_Up[i]              [l]        W_Up[i] is [n, l]   (the absorbed key up-projection)
    K              = cache[b, 0:pos] ++ (c_new | k_rope_new)    [pos+1, l + r]: one latent "head" shared by all heads (MQA)
    V              = K[:, :l]
    s_i            = ((q_lat_i | q_rope_i) . K^T) / sqrt(n + r)
    z_i            = softmax(s_i) . V                [l]
    a_i            = z_i . W_Down[i]                 [v]        W_Down[i] is [l, v]  (the value up-projection)
    out_b          = concat_i(a_i) . W_O             [D]

Readings (the paper leaves these open; each is also listed in the design notes):
  * the rotary part: the paper's Alg. 4 drops rope_dim "for simplicity" while its figure and its formula
    V = K[:kv_lora_rank] keep it; here q and the cached row carry r extra, rotated, dimensions that enter the
    scores only, which is what makes V the first l entries of K;
  * d_k in the softmax scale is the query/key head dimension of the un-absorbed form, n + r, so that the absorbed
    and the un-absorbed computation give the same result (pinned in tests/test_oracle_mla.py);
  * no normalisation of the latent vector is applied (the model the paper names has one; the paper's equations do
    not), and W_Q is a single matrix (the "Lite" variant has no low-rank query projection);
  * the new token is part of the attended set and its (c_new | k_rope_new) row is what a cache append stores.
"""
from __future__ import annotations

import numpy as np

from .decode_block import rope, softmax


def mla_decode_block(x, w_q, w_kv, w_up, w_down, w_o, kv_cache, pos, n_heads, nope_dim, rope_dim, kv_lora_rank,
                     v_head_dim, rope_base):
    """One decode step of the weight-absorbed MLA block.

    x         [B, D]
    w_q       [D, n_heads * (nope_dim + rope_dim)]   per head: nope part, then rope part
    w_kv      [D, kv_lora_rank + rope_dim]           latent part, then the shared rotary key
    w_up      [n_heads, nope_dim, kv_lora_rank]
    w_down    [n_heads, kv_lora_rank, v_head_dim]
    w_o       [n_heads * v_head_dim, D]
    kv_cache  [B, max_seq, kv_lora_rank + rope_dim]  rows 0..pos-1: cached (latent | rotated rotary key)
    Returns fp64 arrays: out [B, D], q_lat [B, n_heads, l], q_rope [B, n_heads, r] (rotated),
    kv_new [B, l + r] (the row to append), z [B, n_heads, l], a [B, n_heads, v].
    """
    x = np.asarray(x).astype(np.float64)
    B, D = x.shape
    nh, n, r, l, v = int(n_heads), int(nope_dim), int(rope_dim), int(kv_lora_rank), int(v_head_dim)
    assert r % 2 == 0
    assert w_q.shape == (D, nh * (n + r)) and w_kv.shape == (D, l + r)
    assert w_up.shape == (nh, n, l) and w_down.shape == (nh, l, v) and w_o.shape == (nh * v, D)
    assert kv_cache.shape[0] == B and kv_cache.shape[2] == l + r and 0 <= pos < kv_cache.shape[1]
    f = lambda a: np.asarray(a).astype(np.float64)          # noqa: E731

    q = (x @ f(w_q)).reshape(B, nh, n + r)
    kv_new = x @ f(w_kv)                                    # [B, l + r]
    q_rope = rope(q[:, :, n:], pos, rope_base)
    kv_new = np.concatenate([kv_new[:, :l], rope(kv_new[:, l:], pos, rope_base)], axis=-1)
    q_lat = np.einsum("bin,inl->bil", q[:, :, :n], f(w_up))

    scale = 1.0 / np.sqrt(float(n + r))
    z = np.empty((B, nh, l), dtype=np.float64)
    for b in range(B):
        K = np.concatenate([f(kv_cache[b, :pos]), kv_new[b][None, :]], axis=0)     # [pos+1, l + r]
        V = K[:, :l]
        for i in range(nh):
            qi = np.concatenate([q_lat[b, i], q_rope[b, i]])
            z[b, i] = softmax((K @ qi) * scale) @ V
    a = np.einsum("bil,ilv->biv", z, f(w_down))
    out = a.reshape(B, nh * v) @ f(w_o)
    return {"out": out, "q_lat": q_lat, "q_rope": q_rope, "kv_new": kv_new, "z": z, "a": a}
