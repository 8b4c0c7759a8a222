"""Pins for the CPU oracle: things the paper and the mathematics fix, none of
which re-use the oracle's own formulas.  All CPU, no GPU."""
import math
import os

import numpy as np
import pytest

from oracle import decode_block as orc
from oracle import c_oracle

RNG = np.random.default_rng(1234)


def rand_case(B, D, nq, nkv, d, L, S=None, std_w=0.3):
    S = S or (L + 2)
    x = RNG.standard_normal((B, D)).astype(np.float16)
    w_qkv = (std_w * RNG.standard_normal((D, (nq + 2 * nkv) * d))).astype(np.float16)
    w_o = (std_w * RNG.standard_normal((nq * d, D))).astype(np.float16)
    kc = np.full((B, nkv, S, d), np.nan, dtype=np.float16)
    vc = np.full((B, nkv, S, d), np.nan, dtype=np.float16)
    kc[:, :, :L] = RNG.standard_normal((B, nkv, L, d)).astype(np.float16)
    vc[:, :, :L] = RNG.standard_normal((B, nkv, L, d)).astype(np.float16)
    return x, w_qkv, w_o, kc, vc


# ---------------------------------------------------------------------------
# brute force: literal scalar loops written from Eq. 1 + the decode semantics
# ---------------------------------------------------------------------------

def brute_force(x, w_qkv, w_o, kc, vc, pos, nq, nkv, d, base):
    B, D = x.shape
    G = nq // nkv
    out = [[0.0] * D for _ in range(B)]
    for b in range(B):
        y = []
        for j in range((nq + 2 * nkv) * d):
            acc = 0.0
            for i in range(D):
                acc += float(x[b, i]) * float(w_qkv[i, j])
            y.append(acc)

        def rot(vec):
            res = list(vec)
            for i in range(d // 2):
                ang = pos * (base ** (-2.0 * i / d))
                c, s = math.cos(ang), math.sin(ang)
                res[i] = vec[i] * c - vec[i + d // 2] * s
                res[i + d // 2] = vec[i + d // 2] * c + vec[i] * s
            return res

        concat = []
        for h in range(nq):
            g = h // G
            q = rot(y[h * d:(h + 1) * d])
            k_new = rot(y[(nq + g) * d:(nq + g + 1) * d])
            v_new = y[(nq + nkv + g) * d:(nq + nkv + g + 1) * d]
            keys = [[float(kc[b, g, t, c]) for c in range(d)] for t in range(pos)] + [k_new]
            vals = [[float(vc[b, g, t, c]) for c in range(d)] for t in range(pos)] + [v_new]
            scores = [sum(q[c] * k[c] for c in range(d)) / math.sqrt(d) for k in keys]
            mx = max(scores)
            e = [math.exp(s - mx) for s in scores]
            z = sum(e)
            for c in range(d):
                concat.append(sum(e[t] / z * vals[t][c] for t in range(len(vals))))
        for j in range(D):
            out[b][j] = sum(concat[r] * float(w_o[r, j]) for r in range(nq * d))
    return np.array(out)


@pytest.mark.parametrize("B,D,nq,nkv,d,L", [(1, 8, 2, 2, 4, 3), (2, 12, 4, 2, 4, 5), (1, 6, 3, 1, 2, 0), (1, 16, 2, 2, 8, 1)])
def test_brute_force_tiny(B, D, nq, nkv, d, L):
    x, w_qkv, w_o, kc, vc = rand_case(B, D, nq, nkv, d, L)
    ref = brute_force(x, w_qkv, w_o, kc, vc, L, nq, nkv, d, 10000.0)
    got = orc.decode_block(x, w_qkv, w_o, kc, vc, L, nq, nkv, d, 10000.0)["out"]
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)
    got_c = c_oracle.decode_block(x, w_qkv, w_o, kc, vc, L, nq, nkv, d, 10000.0)["out"]
    np.testing.assert_allclose(got_c, ref, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------------------
# RoPE
# ---------------------------------------------------------------------------

def test_rope_pos0_identity_and_norm():
    v = RNG.standard_normal((3, 5, 64))
    np.testing.assert_array_equal(orc.rope(v, 0, 10000.0), v)
    for pos in (1, 17, 4096, 32767):
        r = orc.rope(v, pos, 10000.0)
        np.testing.assert_allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(v, axis=-1), rtol=1e-12)
        h = 32     # each (i, i+d/2) pair keeps its own norm
        np.testing.assert_allclose(r[..., :h] ** 2 + r[..., h:] ** 2, v[..., :h] ** 2 + v[..., h:] ** 2, rtol=1e-10, atol=1e-12)


def test_rope_relative_position():
    q, k = RNG.standard_normal(128), RNG.standard_normal(128)
    for (m, n, t) in [(5, 3, 11), (100, 0, 1000), (7, 7, 12345)]:
        a = orc.rope(q, m, 500000.0) @ orc.rope(k, n, 500000.0)
        b = orc.rope(q, m + t, 500000.0) @ orc.rope(k, n + t, 500000.0)
        assert abs(a - b) < 1e-9


@pytest.mark.parametrize("d,base,pos", [(8, 10000.0, 3), (64, 10000.0, 255), (128, 500000.0, 8192)])
def test_rope_one_hot_closed_form(d, base, pos):
    h = d // 2
    for i in (0, 1, h - 1):
        ang = pos * base ** (-2.0 * i / d)
        e = np.zeros(d); e[i] = 1.0
        r = orc.rope(e, pos, base)
        want = np.zeros(d); want[i] = math.cos(ang); want[i + h] = math.sin(ang)
        np.testing.assert_allclose(r, want, atol=1e-12)
        e = np.zeros(d); e[i + h] = 1.0
        r = orc.rope(e, pos, base)
        want = np.zeros(d); want[i] = -math.sin(ang); want[i + h] = math.cos(ang)
        np.testing.assert_allclose(r, want, atol=1e-12)
    # slowest pair of d=8, base 10000: exponent -2*3/8
    assert abs(orc.rope_angles(2, 8, 10000.0)[3] - 2 * 10000.0 ** -0.75) < 1e-15


# ---------------------------------------------------------------------------
# closed forms for the whole block
# ---------------------------------------------------------------------------

def test_two_key_example_by_hand():
    """d = 2 (one RoPE pair, theta_0 = 1), one head, identity projections, one
    cached key.  q_rot . k_rot = |x|^2 because both are rotated by the same
    angle, so the two softmax scores are (q_rot . k0)/sqrt(2) and |x|^2/sqrt(2)."""
    x = np.array([[1.0, 2.0]], dtype=np.float16)
    eye = np.eye(2)
    w_qkv = np.concatenate([eye, eye, eye], axis=1).astype(np.float16)      # q = k = v = x
    w_o = np.array([[1.0, 0.0], [0.0, 1.0]], dtype=np.float16)
    k0 = np.array([0.5, -1.0]); v0 = np.array([3.0, -2.0])
    kc = np.full((1, 1, 2, 2), np.nan, np.float16); vc = kc.copy()
    kc[0, 0, 0] = k0; vc[0, 0, 0] = v0
    pos = 1
    c, s = math.cos(1.0), math.sin(1.0)
    q_rot = (1.0 * c - 2.0 * s, 2.0 * c + 1.0 * s)
    s0 = (q_rot[0] * 0.5 + q_rot[1] * -1.0) / math.sqrt(2.0)
    s1 = (1.0 + 4.0) / math.sqrt(2.0)
    w0 = 1.0 / (1.0 + math.exp(s1 - s0)); w1 = 1.0 - w0
    want = np.array([w0 * 3.0 + w1 * 1.0, w0 * -2.0 + w1 * 2.0])
    for impl in (orc.decode_block, c_oracle.decode_block):
        r = impl(x, w_qkv, w_o, kc, vc, pos, 1, 1, 2, 10000.0)
        np.testing.assert_allclose(r["out"][0], want, rtol=1e-13)
        np.testing.assert_allclose(r["q_rot"][0, 0], q_rot, rtol=1e-13)
        np.testing.assert_allclose(r["v_new"][0, 0], [1.0, 2.0], rtol=0)


@pytest.mark.parametrize("impl", [orc.decode_block, c_oracle.decode_block])
def test_zero_input_gives_uniform_average(impl):
    B, D, nq, nkv, d, L = 2, 32, 4, 2, 8, 9
    x, w_qkv, w_o, kc, vc = rand_case(B, D, nq, nkv, d, L)
    x[:] = 0
    r = impl(x, w_qkv, w_o, kc, vc, L, nq, nkv, d, 10000.0)
    # q = k_new = v_new = 0: all L+1 scores are 0, weights are 1/(L+1), the new value row is 0
    mean_v = vc[:, :, :L].astype(np.float64).sum(axis=2) / (L + 1)                 # [B, nkv, d]
    concat = np.repeat(mean_v, nq // nkv, axis=1).reshape(B, nq * d)
    np.testing.assert_allclose(r["out"], concat @ w_o.astype(np.float64), rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("impl", [orc.decode_block, c_oracle.decode_block])
def test_empty_cache_returns_v_projection(impl):
    B, D, nq, nkv, d = 2, 24, 6, 2, 4
    x, w_qkv, w_o, kc, vc = rand_case(B, D, nq, nkv, d, 0, S=4)
    r = impl(x, w_qkv, w_o, kc, vc, 0, nq, nkv, d, 10000.0)
    y = x.astype(np.float64) @ w_qkv.astype(np.float64)
    v = y[:, (nq + nkv) * d:].reshape(B, nkv, d)
    concat = np.repeat(v, nq // nkv, axis=1).reshape(B, nq * d)
    np.testing.assert_allclose(r["out"], concat @ w_o.astype(np.float64), rtol=1e-12, atol=1e-14)
    # position 0: RoPE is the identity, so q_rot is the plain projection
    np.testing.assert_allclose(r["q_rot"].reshape(B, -1), y[:, :nq * d], rtol=1e-13, atol=1e-15)


def test_planted_dominant_key_selects_its_value():
    B, D, nq, nkv, d, L = 1, 16, 2, 2, 8, 12
    x, w_qkv, w_o, kc, vc = rand_case(B, D, nq, nkv, d, L, std_w=0.5)
    base = orc.decode_block(x, w_qkv, w_o, kc, vc, L, nq, nkv, d, 10000.0)
    for t in (0, 5, L - 1):
        kc2 = kc.copy()
        for h in range(nkv):
            qh = base["q_rot"][0, h]
            kc2[0, h, t] = (200.0 * qh / (qh @ qh) * math.sqrt(d) * 1.0).astype(np.float16)   # score ~ 200
        r = orc.decode_block(x, w_qkv, w_o, kc2, vc, L, nq, nkv, d, 10000.0)
        np.testing.assert_allclose(r["attn"][0], vc[0, :, t].astype(np.float64), atol=1e-9)


def test_convexity_permutation_and_weight_sum():
    B, D, nq, nkv, d, L = 1, 16, 4, 2, 4, 20
    x, w_qkv, w_o, kc, vc = rand_case(B, D, nq, nkv, d, L)
    r = orc.decode_block(x, w_qkv, w_o, kc, vc, L, nq, nkv, d, 10000.0)
    for i in range(nq):
        g = i // 2
        V = np.concatenate([vc[0, g, :L].astype(np.float64), r["v_new"][0, g][None]], 0)
        assert np.all(r["attn"][0, i] <= V.max(0) + 1e-12) and np.all(r["attn"][0, i] >= V.min(0) - 1e-12)
        K = np.concatenate([kc[0, g, :L].astype(np.float64), r["k_rot"][0, g][None]], 0)
        w = orc.attention_weights(r["q_rot"][0, i], K)
        assert np.all(w >= 0) and abs(w.sum() - 1.0) < 1e-14
        np.testing.assert_allclose(w @ V, r["attn"][0, i], rtol=1e-12)
    perm = RNG.permutation(L)
    kc2, vc2 = kc.copy(), vc.copy()
    kc2[:, :, :L] = kc[:, :, perm]; vc2[:, :, :L] = vc[:, :, perm]
    r2 = orc.decode_block(x, w_qkv, w_o, kc2, vc2, L, nq, nkv, d, 10000.0)
    np.testing.assert_allclose(r2["out"], r["out"], rtol=1e-11, atol=1e-13)


def test_nan_rows_beyond_pos_are_never_read():
    x, w_qkv, w_o, kc, vc = rand_case(1, 8, 2, 2, 4, 3, S=9)
    assert np.isnan(kc[0, 0, 3:]).all()
    for impl in (orc.decode_block, c_oracle.decode_block):
        assert np.isfinite(impl(x, w_qkv, w_o, kc, vc, 3, 2, 2, 4, 10000.0)["out"]).all()


def test_gqa_equals_mha_with_replicated_kv():
    B, D, nq, nkv, d, L = 2, 16, 4, 2, 4, 7
    G = nq // nkv
    x, w_qkv, w_o, kc, vc = rand_case(B, D, nq, nkv, d, L)
    wq = w_qkv[:, :nq * d]
    wk = w_qkv[:, nq * d:(nq + nkv) * d].reshape(D, nkv, d)
    wv = w_qkv[:, (nq + nkv) * d:].reshape(D, nkv, d)
    w_mha = np.concatenate([wq, np.repeat(wk, G, axis=1).reshape(D, nq * d),
                            np.repeat(wv, G, axis=1).reshape(D, nq * d)], axis=1)
    r_gqa = orc.decode_block(x, w_qkv, w_o, kc, vc, L, nq, nkv, d, 500000.0)
    r_mha = orc.decode_block(x, w_mha, w_o, np.repeat(kc, G, axis=1), np.repeat(vc, G, axis=1), L, nq, nq, d, 500000.0)
    np.testing.assert_allclose(r_gqa["out"], r_mha["out"], rtol=1e-12, atol=1e-14)


def test_batch_rows_are_independent():
    B, D, nq, nkv, d, L = 3, 16, 4, 2, 4, 6
    x, w_qkv, w_o, kc, vc = rand_case(B, D, nq, nkv, d, L)
    full = orc.decode_block(x, w_qkv, w_o, kc, vc, L, nq, nkv, d, 10000.0)["out"]
    for b in range(B):
        one = orc.decode_block(x[b:b + 1], w_qkv, w_o, kc[b:b + 1], vc[b:b + 1], L, nq, nkv, d, 10000.0)["out"]
        np.testing.assert_allclose(one[0], full[b], rtol=1e-13, atol=1e-15)


# ---------------------------------------------------------------------------
# split-KV partials (Alg. 3 steps 4-7)
# ---------------------------------------------------------------------------

def test_merge_over_any_partition_equals_unsplit():
    d, n = 16, 37
    q = RNG.standard_normal(d); K = 3.0 * RNG.standard_normal((n, d)); V = RNG.standard_normal((n, d))
    s = K @ q / math.sqrt(d)
    w = np.exp(s - s.max()); w /= w.sum()
    want = w @ V
    for trial in range(20):
        ncut = int(RNG.integers(0, 9))
        cuts = sorted(int(c) for c in RNG.integers(0, n + 1, size=ncut))      # repeated cuts give empty parts
        edges = [0] + cuts + [n]
        parts = [orc.partial_attention(q, K[a:b], V[a:b]) for a, b in zip(edges[:-1], edges[1:])]
        np.testing.assert_allclose(orc.merge_partials(parts), want, rtol=1e-12, atol=1e-14)
    # one-token parts
    parts = [orc.partial_attention(q, K[t:t + 1], V[t:t + 1]) for t in range(n)]
    np.testing.assert_allclose(orc.merge_partials(parts), want, rtol=1e-12, atol=1e-14)


def test_summing_unscaled_local_sums_is_wrong():
    """The literal reading of Alg. 3 (sum the local sums, rescale only the
    accumulators) does not give the softmax; this guards the reading chosen."""
    d = 4
    q = np.ones(d); K = np.array([[4.0] * d, [0.0] * d, [-4.0] * d]); V = np.eye(3, d)
    parts = [orc.partial_attention(q, K[a:b], V[a:b]) for a, b in ((0, 1), (1, 3))]
    M = max(p[0] for p in parts); naive_l = sum(p[1] for p in parts)
    naive = sum(p[2] * math.exp(p[0] - M) for p in parts) / naive_l
    s = K @ q / 2.0; w = np.exp(s - s.max()); w /= w.sum()
    assert np.abs(naive - w @ V).max() > 1e-3
    np.testing.assert_allclose(orc.merge_partials(parts), w @ V, rtol=1e-13)


# ---------------------------------------------------------------------------
# the C oracle against the numpy oracle on the tiny configuration
# ---------------------------------------------------------------------------

def test_c_oracle_matches_numpy_oracle_on_tiny_config():
    import cf_inputs
    shp = cf_inputs.SHAPES["tiny"]
    inp = cf_inputs.make_inputs(shp, seed=0)
    args = (inp["x"], inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], inp["pos"],
            shp.n_q_heads, shp.n_kv_heads, shp.head_dim, shp.rope_base)
    a = orc.decode_block(*args); b = c_oracle.decode_block(*args)
    for key in ("out", "q_rot", "k_rot", "v_new", "attn"):
        np.testing.assert_allclose(b[key], a[key], rtol=1e-10, atol=1e-12)
    import dataclasses
    gqa = dataclasses.replace(shp, n_kv_heads=2, rope_base=500000.0)
    inp = cf_inputs.make_inputs(gqa, seed=1, batch=3, kv_len=77)
    args = (inp["x"], inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], 77, 8, 2, 64, 500000.0)
    a = orc.decode_block(*args); b = c_oracle.decode_block(*args)
    np.testing.assert_allclose(b["out"], a["out"], rtol=1e-10, atol=1e-12)
