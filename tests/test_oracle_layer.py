"""Pins for the oracle's RMSNorm and decoder-layer functions (pre-normalisation and residual connection around
the block): closed forms, invariants and a library routine, none of which re-use the oracle's own formula.
All CPU, no GPU."""
import math

import numpy as np
import pytest

from oracle import decode_block as orc
from oracle import c_oracle

RNG = np.random.default_rng(4321)


def rand_case(B, D, nq, nkv, d, L, std_w=0.3):
    S = L + 2
    x = RNG.standard_normal((B, D)).astype(np.float16)
    gamma = (1.0 + 0.2 * RNG.standard_normal(D)).astype(np.float16)
    w_qkv = (std_w * RNG.standard_normal((D, (nq + 2 * nkv) * d))).astype(np.float16)
    w_o = (std_w * RNG.standard_normal((nq * d, D))).astype(np.float16)
    kc = np.full((B, nkv, S, d), np.nan, dtype=np.float16)
    vc = np.full((B, nkv, S, d), np.nan, dtype=np.float16)
    kc[:, :, :L] = RNG.standard_normal((B, nkv, L, d)).astype(np.float16)
    vc[:, :, :L] = RNG.standard_normal((B, nkv, L, d)).astype(np.float16)
    return x, gamma, w_qkv, w_o, kc, vc


def test_rms_norm_constant_row_closed_form():
    # x_j = c for all j: mean square c^2, so every output is gamma_j * c / sqrt(c^2 + eps)
    D, c, eps = 24, -1.5, 1e-3
    gamma = np.linspace(0.5, 2.0, D)
    got = orc.rms_norm(np.full((1, D), c), gamma, eps)
    for j in range(D):
        assert got[0, j] == pytest.approx(gamma[j] * c / math.sqrt(c * c + eps), rel=1e-14)


def test_rms_norm_hand_example():
    # x = (3, 4), eps = 0: mean square 12.5, rms = 5 / sqrt(2)
    got = orc.rms_norm(np.array([[3.0, 4.0]]), np.array([1.0, 2.0]), 0.0)
    assert got[0, 0] == pytest.approx(3.0 * math.sqrt(2.0) / 5.0, rel=1e-15)
    assert got[0, 1] == pytest.approx(2.0 * 4.0 * math.sqrt(2.0) / 5.0, rel=1e-15)


def test_rms_norm_unit_mean_square_and_scale_invariance():
    x = RNG.standard_normal((3, 40))
    one = np.ones(40)
    n = orc.rms_norm(x, one, 0.0)
    assert np.allclose(np.mean(n * n, axis=1), 1.0, rtol=1e-13)
    assert np.allclose(orc.rms_norm(7.5 * x, one, 0.0), n, rtol=1e-13)
    assert np.allclose(orc.rms_norm(-x, one, 0.0), -n, rtol=1e-13)
    # rows are independent of each other
    assert np.array_equal(orc.rms_norm(x[1:2], one, 1e-5), orc.rms_norm(x, one, 1e-5)[1:2])
    # eps matters exactly as an addition to the mean square: a zero row stays zero, no division by zero
    assert np.array_equal(orc.rms_norm(np.zeros((1, 8)), np.ones(8), 1e-6), np.zeros((1, 8)))


def test_rms_norm_equals_library_routine():
    torch = pytest.importorskip("torch")
    x = RNG.standard_normal((4, 96))
    gamma = 1.0 + 0.3 * RNG.standard_normal(96)
    want = torch.nn.functional.rms_norm(torch.from_numpy(x), (96,), torch.from_numpy(gamma), 1e-5).numpy()
    assert np.allclose(orc.rms_norm(x, gamma, 1e-5), want, rtol=1e-13, atol=0)


def test_layer_with_zero_output_projection_returns_x():
    x, gamma, w_qkv, w_o, kc, vc = rand_case(2, 32, 4, 2, 8, 5)
    r = orc.decode_layer(x, gamma, 1e-5, w_qkv, np.zeros_like(w_o), kc, vc, 5, 4, 2, 8, 10000.0)
    assert np.array_equal(r["out"], x.astype(np.float64))


def test_layer_reduces_to_block_for_normalised_input():
    # rows of +-1 have mean square exactly 1: with gamma = 1 and eps = 0 the normalisation is the identity
    B, D, nq, nkv, d, L = 2, 32, 4, 2, 8, 6
    _, _, w_qkv, w_o, kc, vc = rand_case(B, D, nq, nkv, d, L)
    x = np.where(RNG.random((B, D)) < 0.5, -1.0, 1.0).astype(np.float16)
    lay = orc.decode_layer(x, np.ones(D, dtype=np.float16), 0.0, w_qkv, w_o, kc, vc, L, nq, nkv, d, 10000.0)
    blk = orc.decode_block(x, w_qkv, w_o, kc, vc, L, nq, nkv, d, 10000.0)
    assert np.allclose(lay["out"], x.astype(np.float64) + blk["out"], rtol=1e-13, atol=1e-13)
    assert np.allclose(lay["q_rot"], blk["q_rot"], rtol=1e-13, atol=1e-13)


def test_layer_gamma_folds_into_the_weights():
    # diag(gamma) W_qkv applied to the plain normalised row is the same projection: the layer with gamma equals
    # the layer with gamma = 1 and rows of W_qkv scaled (scaling by powers of two is exact in fp16)
    B, D, nq, nkv, d, L = 1, 16, 2, 1, 8, 3
    x, _, w_qkv, w_o, kc, vc = rand_case(B, D, nq, nkv, d, L)
    gamma = np.array([0.5, 2.0] * (D // 2), dtype=np.float16)
    a = orc.decode_layer(x, gamma, 1e-5, w_qkv, w_o, kc, vc, L, nq, nkv, d, 10000.0)
    w2 = (w_qkv.astype(np.float32) * gamma.astype(np.float32)[:, None]).astype(np.float16)
    b = orc.decode_layer(x, np.ones(D, dtype=np.float16), 1e-5, w2, w_o, kc, vc, L, nq, nkv, d, 10000.0)
    assert np.allclose(a["out"], b["out"], rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("shape", [(1, 32, 4, 4, 8, 7), (3, 48, 6, 2, 8, 12), (2, 64, 4, 1, 16, 1)])
def test_c_oracle_layer_matches_numpy_oracle(shape):
    B, D, nq, nkv, d, L = shape
    x, gamma, w_qkv, w_o, kc, vc = rand_case(B, D, nq, nkv, d, L)
    a = orc.decode_layer(x, gamma, 1e-5, w_qkv, w_o, kc, vc, L, nq, nkv, d, 10000.0)
    c = c_oracle.decode_layer(x, gamma, 1e-5, w_qkv, w_o, kc, vc, L, nq, nkv, d, 10000.0)
    for key in ("out", "q_rot", "k_rot", "v_new", "attn"):
        assert np.allclose(a[key], c[key], rtol=1e-11, atol=1e-11), key


def test_rows_with_equal_positions_are_the_batched_call_and_rows_permute():
    B, D, nq, nkv, d, L = 3, 32, 4, 2, 8, 6
    x, gamma, w_qkv, w_o, kc, vc = rand_case(B, D, nq, nkv, d, L)
    whole = orc.decode_layer(x, gamma, 1e-5, w_qkv, w_o, kc, vc, L, nq, nkv, d, 10000.0)
    rows = orc.decode_rows(x, gamma, 1e-5, w_qkv, w_o, kc, vc, [L] * B, nq, nkv, d, 10000.0)
    for key in whole:
        assert np.allclose(whole[key], rows[key], rtol=1e-13, atol=1e-13), key
    # rows with positions of their own: each row is the one-row call at its position, wherever it sits in the batch
    pos = [2, 6, 0]
    mixed = orc.decode_rows(x, gamma, 1e-5, w_qkv, w_o, kc, vc, pos, nq, nkv, d, 10000.0)
    perm = [2, 0, 1]
    again = orc.decode_rows(x[perm], gamma, 1e-5, w_qkv, w_o, kc[perm], vc[perm], [pos[i] for i in perm], nq, nkv, d,
                            10000.0)
    for key in mixed:
        assert np.array_equal(mixed[key][perm], again[key]), key
    # a row at position 0 attends to its own new token only: out = x + v_new W_o (per KV group) for that row
    b = 2
    v = mixed["v_new"][b]                                   # [nkv, d]
    concat = np.concatenate([v[i // (nq // nkv)] for i in range(nq)])
    assert np.allclose(mixed["out"][b], x[b].astype(np.float64) + concat @ w_o.astype(np.float64), rtol=1e-12, atol=1e-12)
    # without gamma it is the bare block per row
    plain = orc.decode_rows(x, None, 0.0, w_qkv, w_o, kc, vc, pos, nq, nkv, d, 10000.0)
    one = orc.decode_block(x[1:2], w_qkv, w_o, kc[1:2], vc[1:2], pos[1], nq, nkv, d, 10000.0)
    assert np.array_equal(plain["out"][1:2], one["out"])
