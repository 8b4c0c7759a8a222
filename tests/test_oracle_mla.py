"""Pins for the weight-absorbed MLA oracle (oracle/mla_block.py): the un-absorbed computation written out as plain
multi-head attention, literal loops on a tiny case, closed forms and invariants.  All CPU, no GPU."""
import math

import numpy as np
import pytest

from oracle import mla_block as mla

RNG = np.random.default_rng(99)


def rand_case(B, D, nh, n, r, l, v, L, std=0.3):
    S = L + 2
    g = lambda *shape: (std * RNG.standard_normal(shape)).astype(np.float16)     # noqa: E731
    x = RNG.standard_normal((B, D)).astype(np.float16)
    cache = np.full((B, S, l + r), np.nan, dtype=np.float16)
    cache[:, :L] = RNG.standard_normal((B, L, l + r)).astype(np.float16)
    return dict(x=x, w_q=g(D, nh * (n + r)), w_kv=g(D, l + r), w_up=g(nh, n, l), w_down=g(nh, l, v), w_o=g(nh * v, D),
                kv_cache=cache)


def run(c, pos, nh, n, r, l, v, base=10000.0):
    return mla.mla_decode_block(c["x"], c["w_q"], c["w_kv"], c["w_up"], c["w_down"], c["w_o"], c["kv_cache"], pos,
                                nh, n, r, l, v, base)


def rot(vec, pos, base):
    """RoPE with scalar loops (half-split pairing), independent of the oracle's vectorised one."""
    d = len(vec)
    out = list(vec)
    for i in range(d // 2):
        ang = pos * base ** (-2.0 * i / d)
        c, s = math.cos(ang), math.sin(ang)
        out[i] = vec[i] * c - vec[i + d // 2] * s
        out[i + d // 2] = vec[i + d // 2] * c + vec[i] * s
    return out


def test_absorbed_equals_unabsorbed_multi_head_attention():
    """Without absorption the same block is ordinary multi-head attention: every cached latent row is expanded
    to per-head keys k_i = (c W_Up[i]^T | k_rope) and values v_i = c W_Down[i], the query is (q_nope_i | q_rope_i),
    the scale is 1/sqrt(n + r).  Both orders of the matrix products must agree."""
    B, D, nh, n, r, l, v, L = 2, 24, 3, 8, 4, 16, 6, 7
    c = rand_case(B, D, nh, n, r, l, v, L)
    got = run(c, L, nh, n, r, l, v)
    f = lambda a: np.asarray(a).astype(np.float64)          # noqa: E731
    x = f(c["x"])
    q = (x @ f(c["w_q"])).reshape(B, nh, n + r)
    kvn = x @ f(c["w_kv"])
    for b in range(B):
        rows = [list(f(c["kv_cache"][b, t])) for t in range(L)]
        rows.append(list(kvn[b, :l]) + rot(list(kvn[b, l:]), L, 10000.0))
        rows = np.array(rows)                                # [L+1, l + r], the rotary part already rotated
        heads = []
        for i in range(nh):
            k_i = np.concatenate([rows[:, :l] @ f(c["w_up"][i]).T, rows[:, l:]], axis=1)      # [L+1, n + r]
            v_i = rows[:, :l] @ f(c["w_down"][i])                                               # [L+1, v]
            q_i = np.array(list(q[b, i, :n]) + rot(list(q[b, i, n:]), L, 10000.0))
            s = k_i @ q_i / math.sqrt(n + r)
            w = np.exp(s - s.max())
            w /= w.sum()
            heads.append(w @ v_i)
        want = np.concatenate(heads) @ f(c["w_o"])
        assert np.allclose(got["out"][b], want, rtol=1e-11, atol=1e-12)


def test_literal_loops_on_a_tiny_case():
    B, D, nh, n, r, l, v, L = 1, 5, 2, 2, 2, 3, 2, 2
    c = rand_case(B, D, nh, n, r, l, v, L)
    got = run(c, L, nh, n, r, l, v)
    x = [float(t) for t in c["x"][0]]
    wq, wkv = c["w_q"].astype(float), c["w_kv"].astype(float)
    q = [sum(x[d] * wq[d, j] for d in range(D)) for j in range(nh * (n + r))]
    kvn = [sum(x[d] * wkv[d, j] for d in range(D)) for j in range(l + r)]
    kvn = kvn[:l] + rot(kvn[l:], L, 10000.0)
    rows = [[float(t) for t in c["kv_cache"][0, t_]] for t_ in range(L)] + [kvn]
    concat = []
    for i in range(nh):
        qi = q[i * (n + r):(i + 1) * (n + r)]
        q_lat = [sum(qi[a] * float(c["w_up"][i, a, j]) for a in range(n)) for j in range(l)]
        q_rot = rot(qi[n:], L, 10000.0)
        s = [(sum(q_lat[j] * row[j] for j in range(l)) + sum(q_rot[j] * row[l + j] for j in range(r))) / math.sqrt(n + r)
             for row in rows]
        m = max(s)
        e = [math.exp(t - m) for t in s]
        z = [sum(e[t] * rows[t][j] for t in range(len(rows))) / sum(e) for j in range(l)]
        concat += [sum(z[j] * float(c["w_down"][i, j, k]) for j in range(l)) for k in range(v)]
    want = [sum(concat[j] * float(c["w_o"][j, d]) for j in range(nh * v)) for d in range(D)]
    assert np.allclose(got["out"][0], want, rtol=1e-12, atol=1e-13)
    assert np.allclose(got["kv_new"][0], kvn, rtol=1e-13, atol=1e-14)


def test_empty_cache_closed_form_and_cache_rows_beyond_pos_unread():
    # pos = 0: the only attended row is the new one, so z_i = c_new for every head and out = (c_new W_Down) W_O
    B, D, nh, n, r, l, v = 2, 12, 2, 4, 2, 6, 3
    c = rand_case(B, D, nh, n, r, l, v, 0)                   # the whole cache is NaN
    got = run(c, 0, nh, n, r, l, v)
    f = lambda a: np.asarray(a).astype(np.float64)           # noqa: E731
    c_new = (f(c["x"]) @ f(c["w_kv"]))[:, :l]
    a = np.einsum("bl,ilv->biv", c_new, f(c["w_down"])).reshape(B, nh * v)
    assert np.allclose(got["out"], a @ f(c["w_o"]), rtol=1e-12, atol=1e-13)
    assert np.isfinite(got["out"]).all()


def test_invariants():
    B, D, nh, n, r, l, v, L = 2, 16, 4, 4, 4, 8, 4, 9
    c = rand_case(B, D, nh, n, r, l, v, L)
    base = run(c, L, nh, n, r, l, v)
    # z is a convex combination of the latent rows: inside their per-coordinate range
    for b in range(B):
        rows = np.concatenate([c["kv_cache"][b, :L, :l].astype(np.float64), base["kv_new"][b:b + 1, :l]])
        assert (base["z"][b] <= rows.max(axis=0) + 1e-12).all() and (base["z"][b] >= rows.min(axis=0) - 1e-12).all()
    # cached rows may come in any order (their rotary parts are stored already rotated)
    perm = RNG.permutation(L)
    c2 = dict(c)
    c2["kv_cache"] = c["kv_cache"].copy()
    c2["kv_cache"][:, :L] = c["kv_cache"][:, perm]
    assert np.allclose(run(c2, L, nh, n, r, l, v)["out"], base["out"], rtol=1e-12, atol=1e-13)
    # batch rows are independent
    one = {k: (val[1:2] if k in ("x", "kv_cache") else val) for k, val in c.items()}
    assert np.allclose(run(one, L, nh, n, r, l, v)["out"], base["out"][1:2], rtol=1e-13, atol=1e-14)
    # x = 0: all scores are 0, uniform weights over the L cached rows and a zero new row
    c3 = dict(c)
    c3["x"] = np.zeros_like(c["x"])
    z0 = run(c3, L, nh, n, r, l, v)["z"]
    want = c["kv_cache"][:, :L, :l].astype(np.float64).sum(axis=1) / (L + 1)
    assert np.allclose(z0, np.broadcast_to(want[:, None, :], z0.shape), rtol=1e-12, atol=1e-13)
    # a planted row that matches the absorbed query of head 0 dominates: z_0 is that row
    c4 = dict(c)
    c4["kv_cache"] = c["kv_cache"].copy()
    target = np.concatenate([base["q_lat"][0, 0], base["q_rope"][0, 0]])
    c4["kv_cache"][0, 3] = (target * 60.0 / np.linalg.norm(target)).astype(np.float16)
    z4 = run(c4, L, nh, n, r, l, v)["z"][0, 0]
    assert np.allclose(z4, c4["kv_cache"][0, 3, :l].astype(np.float64), rtol=0, atol=1e-3 * np.abs(z4).max())
