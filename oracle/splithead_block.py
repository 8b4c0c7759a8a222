"""The SplitHead dataflow (paper Appendix B, Alg. 5) executed block by block on the CPU, in fp64.

TEST INFRASTRUCTURE ONLY.  Imported by tests; never by the product path, and it imports nothing from it.

Alg. 5 is a different division of the work of the decode block of oracle/decode_block.py (Eq. 1 with the decode
semantics of Sec. 2.1), not a different function.  This module takes Alg. 5's steps in the paper's order, for every
head (cluster) and every block b of its N blocks, with the two ClusterReduce steps executed by the simulation of
Alg. 1 in oracle/cluster_collectives.py, so that a test can show that the steps as read here give the block of Eq. 1
and exchange the number of elements the paper's traffic model states.  It is what justifies checking the SplitHead
kernel against oracle/decode_block.py.

Readings (the paper does not say):
  * which dimensions of the head a block owns.  RoPE (not part of Alg. 5; required by the task's definition of the
    block) pairs dimension i with i + d/2, so a block owns h2 = d / (2N) pairs: dimensions b*h2 + j and
    d/2 + b*h2 + j, j < h2.  Any partition gives the same result; this one keeps a pair in one block.
  * where the 1/sqrt(d) of Eq. 1 goes: applied to the complete scores, after the ClusterReduce.
  * the new token is part of the attended set (row S-1 of the scores), as in the decode block.

Pins (tests/test_oracle_splithead.py): equality with decode_block for N = 1, 2, 4, 8 (N = 1 is the plain block);
the elements counted by the two ClusterReduce steps against Traffic_Reduce(S, N) + Traffic_Reduce(D, N) (Appendix B);
a planted mistake (scores not reduced) must break the equality.
"""
from __future__ import annotations

import numpy as np

from . import cluster_collectives as cc
from .decode_block import rope_angles, softmax


def block_dims(b, n_blocks, head_dim):
    """Dimensions of the head owned by block b: its RoPE pairs, low halves first."""
    h2 = head_dim // (2 * n_blocks)
    lo = np.arange(b * h2, (b + 1) * h2)
    return np.concatenate([lo, head_dim // 2 + lo])


def splithead_decode_block(x, w_qkv, w_o, k_cache, v_cache, pos, n_heads, head_dim, rope_base, n_blocks,
                           reduce_scores=True):
    """One decode step, batch row by batch row, one KV head per query head.

    Shapes as in decode_block.decode_block.  Returns {"out": [B, D] fp64, "k_rot", "v_new": [B, n_heads, d],
    "sent": elements sent by all ClusterReduce steps of one batch row and one head}.
    reduce_scores=False plants a mistake (each block keeps its partial scores) for the test of the pins."""
    x = np.asarray(x).astype(np.float64)
    w_qkv = np.asarray(w_qkv).astype(np.float64)
    w_o = np.asarray(w_o).astype(np.float64)
    B, D = x.shape
    nh, d, N = int(n_heads), int(head_dim), int(n_blocks)
    assert d % (2 * N) == 0 and w_qkv.shape == (D, 3 * nh * d) and w_o.shape == (nh * d, D)
    h2 = d // (2 * N)
    ang = rope_angles(pos, d, rope_base)
    out = np.zeros((B, D))
    k_rot = np.zeros((B, nh, d))
    v_new = np.zeros((B, nh, d))
    sent_one = None
    for row in range(B):
        for i in range(nh):                                        # one cluster per head
            S_b, A_in = [], []
            for b in range(N):
                dims = block_dims(b, N, d)
                # Alg. 5 step 1: the projection restricted to the columns this block owns
                Q_b = x[row] @ w_qkv[:, i * d + dims]
                K_b = x[row] @ w_qkv[:, nh * d + i * d + dims]
                V_b = x[row] @ w_qkv[:, 2 * nh * d + i * d + dims]
                c, s = np.cos(ang[b * h2:(b + 1) * h2]), np.sin(ang[b * h2:(b + 1) * h2])
                Q_b = np.concatenate([Q_b[:h2] * c - Q_b[h2:] * s, Q_b[h2:] * c + Q_b[:h2] * s])
                K_b = np.concatenate([K_b[:h2] * c - K_b[h2:] * s, K_b[h2:] * c + K_b[:h2] * s])
                k_rot[row, i, dims], v_new[row, i, dims] = K_b, V_b
                K_all = np.concatenate([np.asarray(k_cache[row, i, :pos][:, dims]).astype(np.float64), K_b[None, :]])
                V_all = np.concatenate([np.asarray(v_cache[row, i, :pos][:, dims]).astype(np.float64), V_b[None, :]])
                S_b.append(K_all @ Q_b)                            # Alg. 5 step 2: partial scores of every token
                A_in.append(V_all)
            sent = 0
            if reduce_scores:
                S_b, sent = cc.cluster_reduce(S_b, "sum")          # Alg. 5 step 3: every block gets the full scores
            O_b = []
            for b in range(N):
                P = softmax(S_b[b] / np.sqrt(float(d)))            # every block: softmax over all tokens
                A_b = P @ A_in[b]                                  # Alg. 5 step 4: weighted sum of the block's value columns
                O_b.append(A_b @ w_o[i * d + block_dims(b, N, d), :])      # Alg. 5 step 5: the block's rows of the head's W_o
            O, sent_o = cc.cluster_reduce(O_b, "sum")
            out[row] += O[0]                                       # Alg. 5 step 6: summed over the heads, once per head
            if sent_one is None:
                sent_one = sent + sent_o
    return {"out": out, "k_rot": k_rot, "v_new": v_new, "sent": sent_one}
