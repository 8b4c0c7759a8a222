"""Pins of oracle/ffn_block.py (paper Sec. 2.1, FFN(Z) = W3 (sigma(W1 Z) * W2 Z)); CPU only.

Each pin is something other than the oracle's own formula: scalar loops, closed forms, library routines
(scipy's logistic and normal distribution functions, torch's silu / gelu in fp64), and invariants chosen so that a
swapped W1 / W2, a transposed operand, a dropped factor or a wrong activation fails one of them."""
import math

import numpy as np
import pytest
from scipy import special, stats

from oracle import ffn_block as orc


def _rand(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


@pytest.mark.parametrize("act", [orc.ACT_SILU, orc.ACT_GELU])
def test_literal_loops_on_a_tiny_case(act):
    B, D, F = 2, 5, 7
    z, w1, w2, w3 = _rand((B, D), 1), _rand((F, D), 2), _rand((F, D), 3), _rand((F, D), 4)
    want = np.zeros((B, D))
    for b in range(B):
        for f in range(F):
            h = sum(w1[f][k] * z[b][k] for k in range(D))
            u = sum(w2[f][k] * z[b][k] for k in range(D))
            if act == orc.ACT_SILU:
                s = h / (1.0 + math.exp(-h))
            else:
                s = 0.5 * h * (1.0 + math.erf(h / math.sqrt(2.0)))
            for d in range(D):
                want[b][d] += s * u * w3[f][d]
    got = orc.ffn_block(z, w1, w2, w3, act)["out"]
    assert np.abs(got - want).max() < 1e-12


def test_activations_against_library_routines():
    a = np.linspace(-12.0, 12.0, 481)
    assert np.abs(orc.activation(a, orc.ACT_SILU) - a * special.expit(a)).max() < 1e-14
    assert np.abs(orc.activation(a, orc.ACT_GELU) - a * stats.norm.cdf(a)).max() < 1e-14
    # fixed points and limits: sigma(0) = 0, sigma(a) -> a for large a, -> 0 for large negative a
    for act in (orc.ACT_SILU, orc.ACT_GELU):
        assert orc.activation(np.array([0.0]), act)[0] == 0.0
        assert abs(orc.activation(np.array([40.0]), act)[0] - 40.0) < 1e-12
        assert abs(orc.activation(np.array([-40.0]), act)[0]) < 1e-12
    # SiLU(1) = 1 / (1 + 1/e); GELU(1) = Phi(1)
    assert abs(orc.activation(np.array([1.0]), orc.ACT_SILU)[0] - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15
    assert abs(orc.activation(np.array([1.0]), orc.ACT_GELU)[0] - 0.8413447460685429) < 1e-15


@pytest.mark.parametrize("act,fn", [(orc.ACT_SILU, "silu"), (orc.ACT_GELU, "gelu")])
def test_against_torch_fp64(act, fn):
    torch = pytest.importorskip("torch")
    B, D, F = 3, 24, 40
    z, w1, w2, w3 = _rand((B, D), 5), _rand((F, D), 6, 0.3), _rand((F, D), 7, 0.3), _rand((F, D), 8, 0.3)
    tz, t1, t2, t3 = (torch.from_numpy(a) for a in (z, w1, w2, w3))
    lin = torch.nn.functional.linear           # y = x W^T for W stored [out_features, in_features]
    want = (getattr(torch.nn.functional, fn)(lin(tz, t1)) * lin(tz, t2)) @ t3
    got = orc.ffn_block(z, w1, w2, w3, act)["out"]
    assert np.abs(got - want.numpy()).max() < 1e-12


def test_one_hot_input_gives_the_closed_form():
    # z = e_k picks column k of W1 and W2; with W3 = identity rows (d_ff == d_model) the output is sigma(a) * b itself
    D = F = 6
    k = 4
    a, b = _rand((F,), 9), _rand((F,), 10)
    w1, w2 = _rand((F, D), 11), _rand((F, D), 12)
    w1[:, k], w2[:, k] = a, b
    z = np.zeros((1, D))
    z[0, k] = 1.0
    out = orc.ffn_block(z, w1, w2, np.eye(F), orc.ACT_SILU)["out"][0]
    assert np.abs(out - a * special.expit(a) * b).max() < 1e-14


def test_roles_of_the_three_matrices():
    B, D, F = 2, 9, 13
    z, w1, w2, w3 = _rand((B, D), 13), _rand((F, D), 14), _rand((F, D), 15), _rand((F, D), 16)
    base = orc.ffn_block(z, w1, w2, w3)["out"]
    # linear in W2 and in W3, not in W1 (the activation sits on the W1 branch only)
    assert np.abs(orc.ffn_block(z, w1, 3.0 * w2, w3)["out"] - 3.0 * base).max() < 1e-12
    assert np.abs(orc.ffn_block(z, w1, w2, -2.0 * w3)["out"] + 2.0 * base).max() < 1e-12
    assert np.abs(orc.ffn_block(z, 3.0 * w1, w2, w3)["out"] - 3.0 * base).max() > 1e-3
    # swapping W1 and W2 changes the result
    assert np.abs(orc.ffn_block(z, w2, w1, w3)["out"] - base).max() > 1e-3
    # zero input, zero gate branch, zero value branch
    assert np.all(orc.ffn_block(np.zeros((B, D)), w1, w2, w3)["out"] == 0.0)
    assert np.all(orc.ffn_block(z, np.zeros((F, D)), w2, w3)["out"] == 0.0)       # sigma(0) = 0
    assert np.all(orc.ffn_block(z, w1, np.zeros((F, D)), w3)["out"] == 0.0)
    # W2 z == 1 for every unit (rows of W2 = z / |z|^2, batch 1): out = sigma(W1 z) W3
    z1 = z[:1]
    w2c = np.tile(z1 / (z1 @ z1.T), (F, 1))
    want = (w1 @ z1[0]) * special.expit(w1 @ z1[0]) @ w3
    assert np.abs(orc.ffn_block(z1, w1, w2c, w3)["out"][0] - want).max() < 1e-12


def test_rows_are_independent_and_hidden_units_add_up():
    B, D, F = 4, 8, 12
    z, w1, w2, w3 = _rand((B, D), 17), _rand((F, D), 18), _rand((F, D), 19), _rand((F, D), 20)
    full = orc.ffn_block(z, w1, w2, w3, orc.ACT_GELU)["out"]
    for b in range(B):
        assert np.array_equal(orc.ffn_block(z[b:b + 1], w1, w2, w3, orc.ACT_GELU)["out"][0], full[b])
    # the output is a sum over hidden units: two halves of the units add up to the whole
    a = orc.ffn_block(z, w1[:5], w2[:5], w3[:5], orc.ACT_GELU)["out"]
    c = orc.ffn_block(z, w1[5:], w2[5:], w3[5:], orc.ACT_GELU)["out"]
    assert np.abs(a + c - full).max() < 1e-12
    # permuting the hidden units (rows of all three matrices together) changes nothing
    perm = np.random.default_rng(21).permutation(F)
    assert np.abs(orc.ffn_block(z, w1[perm], w2[perm], w3[perm], orc.ACT_GELU)["out"] - full).max() < 1e-12
