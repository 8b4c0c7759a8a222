"""CPU simulation of the paper's two cluster-level collectives (Alg. 1 and Alg. 2).

TEST INFRASTRUCTURE ONLY.  The fused kernel's cross-workgroup exchange has to
deliver what these two schedules deliver (every participant ends up with the
reduction of all buffers / with every participant's segment); this module
states that contract by executing the schedules rank by rank on the CPU and
counting the elements that travel, so that the counts can be checked against
the paper's traffic model (Sec. 3.2).

Pins: results against the plain reduction / concatenation, slot order
(b - j) mod N, and the element counts size*N*log2(N) and size*N*(N-1).
"""
from __future__ import annotations

import numpy as np


def _check_n(n):
    if n < 1 or n > 16 or (n & (n - 1)) != 0:
        raise ValueError("cluster size must be a power of two, at most 16")


def cluster_reduce(bufs, op="sum"):
    """Alg. 1: all-reduce among N = 2^k ranks in log2 N rounds.

    In the round with stride t every rank b sends its whole buffer D_b to rank
    (b + t) mod N, receives the buffer of rank (b - t) mod N into a temporary
    and folds it into D_b; t doubles each round.  Returns (list of final D_b,
    number of elements sent)."""
    n = len(bufs)
    _check_n(n)
    fold = {"sum": np.add, "max": np.maximum}[op]
    d = [np.array(b, dtype=np.float64, copy=True) for b in bufs]
    sent = 0
    t = 1
    while t < n:
        incoming = [d[(b - t) % n].copy() for b in range(n)]   # all sends of a round happen together
        sent += sum(x.size for x in incoming)
        d = [fold(d[b], incoming[b]) for b in range(n)]
        t *= 2
    return d, sent


def cluster_gather(segs):
    """Alg. 2: all-gather among N = 2^k ranks in log2 N rounds.

    Every rank owns a buffer of N segments whose first segment is its own data.
    In the round with stride t rank b sends its first t segments to rank
    (b + t) mod N, which stores them as its segments t .. 2t-1.  Afterwards
    segment j of rank b is the data of rank (b - j) mod N.  Returns (list of
    [N, size] arrays, number of elements sent)."""
    n = len(segs)
    _check_n(n)
    size = np.asarray(segs[0]).size
    d = [np.full((n, size), np.nan, dtype=np.float64) for _ in range(n)]
    for b in range(n):
        d[b][0] = np.asarray(segs[b], dtype=np.float64).ravel()
    sent = 0
    t = 1
    while t < n:
        msgs = [d[(b - t) % n][:t].copy() for b in range(n)]
        for b in range(n):
            d[b][t:2 * t] = msgs[b]
            sent += msgs[b].size
        t *= 2
    return d, sent


def traffic_reduce(size, n):
    """Paper Sec. 3.2: size * log2(N) * N."""
    return size * int(np.log2(n)) * n


def traffic_gather(size, n):
    """Paper Sec. 3.2: size * (2^(log2(N/2)+1) - 1) * N, i.e. size * (N-1) * N."""
    if n == 1:
        return 0
    return size * (2 ** (int(np.log2(n // 2)) + 1) - 1) * n
