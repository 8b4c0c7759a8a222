#!/usr/bin/env python3
"""Latency of the team collectives against their two-kernel versions (the analogue of the paper's Table 1).

For every data size, `cf_team_reduce` (sum) and `cf_team_gather` are timed as two kernels that hand the data over
through global memory, and with the exchange inside one kernel: in the paper's log2(N) rounds and in one hop.  The
sizes are the paper's (32 .. 256 KB) and, below them, the sizes that the fused decode kernel really exchanges
(a workgroup posts 0.5 .. 8 KB there).  "Data size" is the buffer of one rank for the
reduce and the gathered buffer (team_size segments) for the gather, as in Alg. 1 / Alg. 2.  Times are per call, from
HIP events around back-to-back calls on one stream, for one team alone and for as many teams as fit the GPU.

Prints one JSON line per row and a markdown table on stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--team-size", type=int, default=8)
    ap.add_argument("--calls", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    args = ap.parse_args()
    import torch
    from paper_2508_18850_amd import TeamCollectives, TEAM_SUM, TEAM_ROUNDS, TEAM_TWO_KERNELS, TEAM_DIRECT, TEAM_TWO_HOPS
    assert torch.cuda.is_available(), "needs a GPU"
    n = args.team_size
    ncu = torch.cuda.get_device_properties(0).multi_processor_count
    tc = TeamCollectives(ncu, 65536)
    st = torch.cuda.current_stream().cuda_stream
    rows = []
    for op in ("reduce", "gather"):
        for kb in (1, 4, 16, 32, 64, 128, 256):
            values = kb * 1024 // 4                       # fp32 values of the data size
            elems = values if op == "reduce" else values // n
            for teams in (1, ncu // n):
                src = torch.randn((teams, n, elems), dtype=torch.float32, device="cuda")
                dst = torch.empty((teams, n, values if op == "reduce" else n * elems), dtype=torch.float32, device="cuda")
                t = {}
                for mode in (TEAM_TWO_KERNELS, TEAM_ROUNDS, TEAM_DIRECT) + ((TEAM_TWO_HOPS,) if op == "reduce" else ()):
                    def call():
                        if op == "reduce":
                            tc.reduce(teams, n, TEAM_SUM, src.data_ptr(), dst.data_ptr(), elems, mode, st)
                        else:
                            tc.gather(teams, n, src.data_ptr(), dst.data_ptr(), elems, mode, st)
                    for _ in range(args.warmup):
                        call()
                    tc.status(st)
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for _ in range(args.calls):
                        call()
                    e1.record()
                    torch.cuda.synchronize()
                    tc.status(st)
                    t[mode] = e0.elapsed_time(e1) / args.calls * 1e3
                row = {"operation": op, "data_kb": kb, "team_size": n, "teams": teams,
                       "two_kernels_us": t[TEAM_TWO_KERNELS], "rounds_us": t[TEAM_ROUNDS], "direct_us": t[TEAM_DIRECT],
                       "two_hops_us": t.get(TEAM_TWO_HOPS),
                       "speedup_rounds": t[TEAM_TWO_KERNELS] / t[TEAM_ROUNDS],
                       "speedup_direct": t[TEAM_TWO_KERNELS] / t[TEAM_DIRECT]}
                rows.append(row)
                print(json.dumps(row), flush=True)
    print("| operation | data size (KB) | teams | two kernels (us) | one kernel: rounds (us) | one hop (us) | two hops (us) "
          "| best one-kernel speedup |", file=sys.stderr)
    print("|---|---|---|---|---|---|---|---|", file=sys.stderr)
    for r in rows:
        th = r["two_hops_us"]
        best = min(v for v in (r["rounds_us"], r["direct_us"], th) if v is not None)
        print("| %s | %d | %d | %.2f | %.2f | %.2f | %s | %.2fx |"
              % (r["operation"], r["data_kb"], r["teams"], r["two_kernels_us"], r["rounds_us"], r["direct_us"],
                 "-" if th is None else "%.2f" % th, r["two_kernels_us"] / best), file=sys.stderr)
    tc.close()


if __name__ == "__main__":
    main()
