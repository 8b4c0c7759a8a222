"""Pins for the simulation of the paper's ClusterReduce / ClusterGather
schedules (Alg. 1, Alg. 2) and the traffic model of Sec. 3.2."""
import os

import numpy as np
import pytest

from oracle import cluster_collectives as cc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "traffic_model.txt")


def golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append(tuple(int(v) for v in line.split()))
    return rows


@pytest.mark.parametrize("n", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("op", ["sum", "max"])
def test_reduce_gives_every_rank_the_full_reduction(n, op):
    rng = np.random.default_rng(n)
    bufs = [rng.standard_normal(5) for _ in range(n)]
    res, sent = cc.cluster_reduce(bufs, op)
    want = np.sum(bufs, axis=0) if op == "sum" else np.max(bufs, axis=0)
    for r in res:
        np.testing.assert_allclose(r, want, rtol=1e-12)
    assert sent == cc.traffic_reduce(5, n)


@pytest.mark.parametrize("n", [1, 2, 4, 8, 16])
def test_gather_slot_order_and_traffic(n):
    segs = [np.full(3, float(b)) for b in range(n)]
    res, sent = cc.cluster_gather(segs)
    for b in range(n):
        for j in range(n):
            assert np.all(res[b][j] == float((b - j) % n))
    assert sent == cc.traffic_gather(3, n)


def test_traffic_counts_match_printed_model():
    for n, red, gat in golden_rows():
        _, sent_r = cc.cluster_reduce([np.zeros(1)] * n)
        _, sent_g = cc.cluster_gather([np.zeros(1)] * n)
        assert sent_r == red == cc.traffic_reduce(1, n)
        assert sent_g == gat == cc.traffic_gather(1, n)


def test_bad_cluster_sizes_rejected():
    for n in (3, 6, 32):
        with pytest.raises(ValueError):
            cc.cluster_reduce([np.zeros(1)] * n)
