"""Parity of the team collectives (cf_team_reduce / cf_team_gather) with the CPU simulation of the paper's
Alg. 1 / Alg. 2 (oracle/cluster_collectives.py), through the C ABI, for every way of exchanging the data:
the paper's rounds inside one kernel, one hop or (reduce) two hops inside one kernel, and two kernels.

Bar: the gather and the max-reduce move or select values, so they are bit-exact.  The sum-reduce is fp32 and
adds in Alg. 1's order (rounds) or in rank order (the other two modes); the oracle executes Alg. 1 in fp64: each
result is a sum of N <= 16 values of magnitude <= ~4, and |err| <= N * 2^-24 * sum|x| (a few 1e-6) bounds the
rounding of any order of fp32 additions.
"""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from oracle import cluster_collectives as oc                      # noqa: E402
from paper_2508_18850_amd import (TeamCollectives, TEAM_SUM, TEAM_MAX, TEAM_ROUNDS, TEAM_TWO_KERNELS,   # noqa: E402
                                  TEAM_DIRECT, TEAM_TWO_HOPS)

MODES = [TEAM_ROUNDS, TEAM_TWO_KERNELS, TEAM_DIRECT]


def _log(msg):
    print("[team] " + msg, file=sys.stderr, flush=True)


def _data(teams, n, elems, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.standard_normal((teams, n, elems)).astype(np.float32)


CASES = [
    # teams, team size N, values per rank: tiny, ragged, one value per thread, several tiles, the largest buffer
    (1, 1, 7), (3, 2, 1), (2, 4, 513), (4, 8, 8192), (2, 16, 1000), (16, 16, 4096), (32, 8, 65536), (1, 8, 65536),
]


@pytest.mark.parametrize("mode", MODES + [TEAM_TWO_HOPS])
@pytest.mark.parametrize("teams,n,elems", CASES)
def test_reduce_matches_alg1(teams, n, elems, mode):
    _log("reduce teams=%d N=%d elems=%d mode=%d" % (teams, n, elems, mode))
    tc = TeamCollectives(256, 65536)
    host = _data(teams, n, elems, seed=elems + n)
    src = torch.from_numpy(host).cuda()
    for op, name in ((TEAM_SUM, "sum"), (TEAM_MAX, "max")):
        dst = torch.full_like(src, float("nan"))
        st = torch.cuda.current_stream().cuda_stream
        # two calls in a row: the second must not be confused by the first one's slots
        tc.reduce(teams, n, op, src.data_ptr(), dst.data_ptr(), elems, mode, st)
        tc.reduce(teams, n, op, src.data_ptr(), dst.data_ptr(), elems, mode, st)
        tc.status(st)
        got = dst.cpu().numpy()
        for k in range(teams):
            want, sent = oc.cluster_reduce([host[k, b] for b in range(n)], name)
            assert sent == oc.traffic_reduce(elems, n)
            for b in range(n):
                if name == "max":
                    assert np.array_equal(got[k, b], want[b].astype(np.float32))
                else:
                    tol = n * 2.0 ** -24 * np.abs(host[k]).sum(axis=0) + 1e-30
                    assert np.all(np.abs(got[k, b].astype(np.float64) - want[b]) <= tol)
        # adding in rank order, every rank of a team ends with the same bits (in Alg. 1's order each rank
        # adds in an order of its own)
        if mode != TEAM_ROUNDS:
            assert np.array_equal(got, np.broadcast_to(got[:, :1], got.shape))
    tc.close()


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("teams,n,elems", [(1, 1, 5), (3, 2, 1), (2, 4, 513), (4, 8, 8192), (2, 16, 1000), (16, 16, 4096),
                                           (32, 8, 8192), (1, 16, 4096)])
def test_gather_matches_alg2(teams, n, elems, mode):
    _log("gather teams=%d N=%d elems=%d mode=%d" % (teams, n, elems, mode))
    tc = TeamCollectives(256, 65536)
    host = _data(teams, n, elems, seed=7 * elems + n)
    src = torch.from_numpy(host).cuda()
    dst = torch.full((teams, n, n, elems), float("nan"), dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    tc.gather(teams, n, src.data_ptr(), dst.data_ptr(), elems, mode, st)
    tc.gather(teams, n, src.data_ptr(), dst.data_ptr(), elems, mode, st)
    tc.status(st)
    got = dst.cpu().numpy()
    for k in range(teams):
        want, sent = oc.cluster_gather([host[k, b] for b in range(n)])
        assert sent == oc.traffic_gather(elems, n)
        for b in range(n):
            assert np.array_equal(got[k, b], want[b].astype(np.float32))      # slot j = rank (b - j) mod N
    tc.close()


def test_bad_arguments_are_refused():
    tc = TeamCollectives(64, 1024)
    a = torch.zeros(64 * 1024, dtype=torch.float32, device="cuda")
    p = a.data_ptr()
    assert tc.reduce_rc(1, 3, TEAM_SUM, p, p, 16) == -1          # team size not a power of two
    assert tc.reduce_rc(1, 32, TEAM_SUM, p, p, 16) == -1         # more than 16
    assert tc.reduce_rc(1, 8, 5, p, p, 16) == -1                 # unknown operator
    assert tc.reduce_rc(1, 8, TEAM_SUM, p, p, 2048) == -1        # more values than the handle's capacity
    assert tc.reduce_rc(16, 8, TEAM_SUM, p, p, 16) == -1         # more ranks than the handle's capacity
    assert tc.reduce_rc(1, 8, TEAM_SUM, 0, p, 16) == -1          # null pointer
    assert tc.gather_rc(1, 8, p, p, 256) == -1                   # gathered buffer larger than the capacity
    assert tc.reduce_rc(1, 8, TEAM_SUM, p, p, 16, 4) == -1       # unknown mode
    assert tc.gather_rc(1, 8, p, p, 16, TEAM_TWO_HOPS) == -1     # a mode of the reduce only
    tc.close()
    big = TeamCollectives(1024, 16)
    assert big.reduce_rc(64, 8, TEAM_SUM, p, p, 16) == -2        # more workgroups than compute units: not resident
    big.close()
