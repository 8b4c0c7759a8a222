"""Pins of the block-by-block execution of the SplitHead dataflow (oracle/splithead_block.py; paper Appendix B,
Alg. 5): it is the decode block of Eq. 1 for every cluster size, it exchanges what the paper's traffic model says,
and a planted mistake is caught.  This is what lets the SplitHead kernel be checked against oracle/decode_block.py."""
import numpy as np
import pytest

import cf_inputs
from oracle import cluster_collectives as cc
from oracle import decode_block as orc
from oracle import splithead_block as sh


def _case(d_model, heads, head_dim, kv_len, batch=1, seed=11):
    shape = cf_inputs.BlockShape("s", d_model, heads, heads, head_dim, 10000.0, 0)
    return shape, cf_inputs.make_inputs(shape, seed=seed, batch=batch, kv_len=kv_len)


@pytest.mark.parametrize("n_blocks", [1, 2, 4, 8])
@pytest.mark.parametrize("d_model,heads,head_dim,kv_len,batch", [(48, 3, 32, 19, 2), (64, 2, 64, 0, 1), (40, 1, 16, 5, 1)])
def test_alg5_is_the_decode_block(n_blocks, d_model, heads, head_dim, kv_len, batch):
    if head_dim % (2 * n_blocks):
        pytest.skip("head dimension does not split into that many blocks of RoPE pairs")
    shape, inp = _case(d_model, heads, head_dim, kv_len, batch)
    a = (inp["x"], inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], kv_len)
    ref = orc.decode_block(*a, heads, heads, head_dim, shape.rope_base)
    got = sh.splithead_decode_block(*a, heads, head_dim, shape.rope_base, n_blocks)
    scale = np.abs(ref["out"]).max()
    assert np.abs(got["out"] - ref["out"]).max() <= 1e-12 * scale
    assert np.abs(got["k_rot"] - ref["k_rot"]).max() <= 1e-12 * np.abs(ref["k_rot"]).max()
    assert np.abs(got["v_new"] - ref["v_new"]).max() <= 1e-12 * np.abs(ref["v_new"]).max()


@pytest.mark.parametrize("n_blocks", [2, 4, 8])
def test_exchanged_elements_match_the_traffic_model(n_blocks):
    """Appendix B: Traffic_Total = Traffic_Reduce(S, N) + Traffic_Reduce(D, N), S counting the new token."""
    shape, inp = _case(48, 2, 32, 21)
    got = sh.splithead_decode_block(inp["x"], inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], 21, 2, 32,
                                    shape.rope_base, n_blocks)
    assert got["sent"] == cc.traffic_reduce(22, n_blocks) + cc.traffic_reduce(48, n_blocks)
    # the part that depends on the cached length grows by log2(N) * N elements per token; Alg. 3's total,
    # Reduce(H, N) + Gather(3h, N), does not depend on it
    shape2, inp2 = _case(48, 2, 32, 30)
    got2 = sh.splithead_decode_block(inp2["x"], inp2["w_qkv"], inp2["w_o"], inp2["k_cache"], inp2["v_cache"], 30, 2, 32,
                                     shape2.rope_base, n_blocks)
    assert got2["sent"] - got["sent"] == 9 * int(np.log2(n_blocks)) * n_blocks


def test_block_dims_partition_the_head_and_keep_rope_pairs_together():
    for n in (1, 2, 4, 8):
        dims = [sh.block_dims(b, n, 64) for b in range(n)]
        assert sorted(np.concatenate(dims).tolist()) == list(range(64))
        for dd in dims:
            h2 = len(dd) // 2
            assert np.array_equal(dd[h2:], dd[:h2] + 32)


def test_unreduced_scores_are_caught():
    """The planted mistake: without the ClusterReduce of the scores every block normalises its own partial scores."""
    shape, inp = _case(48, 3, 32, 19)
    a = (inp["x"], inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], 19)
    ref = orc.decode_block(*a, 3, 3, 32, shape.rope_base)
    bad = sh.splithead_decode_block(*a, 3, 32, shape.rope_base, 4, reduce_scores=False)
    assert np.abs(bad["out"] - ref["out"]).max() > 1e-3 * np.abs(ref["out"]).max()
