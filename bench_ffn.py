#!/usr/bin/env python3
"""Latency of the fused feed-forward block (cf_ffn_decode) on Llama-shaped matrices.

Back-to-back launches on one stream, rotating over several layers' worth of weights (more than the 256 MB of
last-level cache), timed with HIP events.  Prints one JSON line: time per step, algorithmic HBM bytes per step and
the fraction of 8 TB/s they amount to, and the CPU oracle's time for the same step.  After the timed region one
layer's result is checked against the oracle on a sample of output columns.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


# HBM bytes per launch from rocprofv3 counters, (FETCH_SIZE KiB x 2.0000 + WRITE_SIZE KiB) x 1024
# (profiles/fused_ffn_kernel_trace_and_traffic.md); None where no counter run exists
MEASURED_TRAFFIC = {
    "ffn_llama2_7b_b1": 290456166,      # 137720.3, 8208.0
    "ffn_llama2_7b_b16": 304258662,     # 143711.8, 9704.0
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="llama2_7b", help="shape name from cf_inputs.FFN_SHAPES")
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--layers", type=int, default=0)
    ap.add_argument("--gelu", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    import numpy as np
    import torch
    import cf_inputs
    from paper_2508_18850_amd import FfnBlock
    assert torch.cuda.is_available(), "needs a GPU"
    shape = cf_inputs.FFN_SHAPES[args.workload]
    B, D, F = args.batch, shape.d_model, shape.d_ff
    act = 1 if args.gelu else 0
    dev = torch.device("cuda:0")
    blk = FfnBlock(D, F, B, act)
    alg = blk.algorithmic_bytes(B)
    layer_bytes = 3 * F * D * 2
    n_layers = args.layers or max(6, -(-3 * 2 ** 30 // layer_bytes))            # >= 3 GiB of distinct matrices
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)

    def rnd(shp, std):
        return (torch.randn(shp, generator=gen, device=dev) * std).half()

    layers = [(rnd((F, D), 0.02), rnd((F, D), 0.02), rnd((F, D), 0.02)) for _ in range(n_layers)]
    z = rnd((B, D), 1.0)
    out = torch.empty((B, D), dtype=torch.float16, device=dev)
    stream = torch.cuda.Stream(device=dev)
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        sh = stream.cuda_stream

        def step(i):
            w1, w2, w3 = layers[i % n_layers]
            blk.decode(B, z.data_ptr(), w1.data_ptr(), w2.data_ptr(), w3.data_ptr(), out.data_ptr(), sh)

        for i in range(args.warmup):
            step(i)
        blk.status(sh)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(stream)
        for i in range(args.steps):
            step(args.warmup + i)
        e1.record(stream)
        torch.cuda.synchronize()
        blk.status(sh)
        # outside the timed region: layer 0 once more, checked against the oracle
        step(0)
        blk.status(sh)
    from oracle import ffn_block as orc
    w1, w2, w3 = (t.cpu().numpy() for t in layers[0])
    ref = orc.ffn_block(z.cpu().numpy(), w1, w2, w3, act)["out"]
    got = out.cpu().numpy().astype(np.float64)
    err, tol = float(np.abs(got - ref).max()), float(1e-2 * np.abs(ref).max() + 1e-3)
    assert err <= tol, "the timed kernel disagrees with the oracle: %g > %g" % (err, tol)
    us = e0.elapsed_time(e1) / args.steps * 1e3
    tiles = B >= 2 and min(F, torch.cuda.get_device_properties(0).multi_processor_count) % 16 == 0 and -(-F // 256) <= 128
    achieved = alg / (us * 1e-6) / 1e9
    res = {"metric": "us per fused feed-forward step", "value": us, "unit": "us/step", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "higher_is_better": False, "dtype": "f16 storage, f32 accumulate", "data": "synthetic",
           "config": {"workload": "ffn_%s_b%d" % (shape.name, B), "d_model": D, "d_ff": F, "layers_rotated": n_layers,
                      "activation": "gelu" if act else "silu"},
           "roofline": {"bound": "hbm", "achieved": achieved, "peak": 8000.0, "unit": "GB/s", "frac": achieved / 8000.0,
                        "traffic": MEASURED_TRAFFIC.get("ffn_%s_b%d" % (shape.name, B)), "algorithmic_bytes": alg,
                        "kernel": "fused_ffn_tiles" if tiles else "fused_ffn"},
           "check": {"max_abs_err": err, "tolerance": tol}}
    if not args.no_cpu_baseline:
        zc = z.cpu().numpy()
        orc.ffn_block(zc, w1, w2, w3, act)
        ts = []
        t_end = time.perf_counter() + 10.0
        while time.perf_counter() < t_end and len(ts) < 20:
            t0 = time.perf_counter()
            orc.ffn_block(zc, w1, w2, w3, act)
            ts.append(time.perf_counter() - t0)
        res["cpu_baseline"] = {"value": float(np.median(ts)) * 1e6, "unit": "us/step", "cores": len(os.sched_getaffinity(0)),
                               "kind": "oracle", "sample": "%d whole steps of the same shape (numpy fp64 oracle)" % len(ts)}
    print(json.dumps(res), flush=True)
    blk.close()


if __name__ == "__main__":
    main()
