#!/usr/bin/env python3
"""Latency of the fused MLA decode block (cf_mla_decode) on the DeepSeek-V2-Lite shape.

Back-to-back launches on one stream, rotating over several layers' worth of weights and caches (more than the
256 MB of last-level cache), timed with HIP events.  Prints one JSON line: time per step, algorithmic HBM bytes
per step and the fraction of 8 TB/s they amount to, and the CPU oracle's time for the same step.
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
# (profiles/fused_mla_deepseek_v2_lite_kv4096.md), DeepSeek-V2-Lite shape; None where no counter run exists
MEASURED_TRAFFIC = {
    "b16_kv4096": 243688448,            # 100782.5, 36412.0
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--kv-len", type=int, default=None)
    ap.add_argument("--layers", type=int, default=0)
    ap.add_argument("--ranges", type=int, default=0,
                    help="limit on the token ranges per batch row (cf_mla_set_splits); a non-zero value also selects the "
                         "token-range kernel at batch 1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    import numpy as np
    import torch
    import cf_inputs
    from paper_2508_18850_amd import MlaBlock
    assert torch.cuda.is_available(), "needs a GPU"
    shape = cf_inputs.MLA_SHAPES["deepseek_v2_lite"]
    B, Lk = args.batch, args.kv_len if args.kv_len is not None else shape.kv_len
    S = cf_inputs.default_max_seq(Lk)
    dev = torch.device("cuda:0")
    D, nh, n, r, l, v = shape.d_model, shape.n_heads, shape.nope_dim, shape.rope_dim, shape.kv_lora_rank, shape.v_head_dim
    blk = MlaBlock(D, nh, n, r, l, v, B, S, shape.rope_base)
    if args.ranges:
        blk.set_splits(args.ranges)
    alg = blk.algorithmic_bytes(B, Lk)
    layer_bytes = 2 * (D * (nh * (n + r) + l + r) + nh * n * l + nh * l * v + nh * v * D + B * S * (l + r))
    n_layers = args.layers or max(8, -(-2 ** 30 // layer_bytes))            # >= 1 GiB of distinct buffers
    gen = torch.Generator(device=dev)
    gen.manual_seed(5)

    def rnd(shp, std):
        return (torch.randn(shp, generator=gen, device=dev) * std).half()

    layers = []
    for _ in range(n_layers):
        layers.append((rnd((D, nh * (n + r)), D ** -0.5), rnd((D, l + r), D ** -0.5), rnd((nh, n, l), n ** -0.5),
                       rnd((nh, l, v), l ** -0.5), rnd((nh * v, D), (nh * v) ** -0.5), rnd((B, S, l + r), 1.0)))
    x = rnd((B, D), 1.0)
    out = torch.empty((B, D), dtype=torch.float16, device=dev)
    stream = torch.cuda.Stream(device=dev)
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        sh = stream.cuda_stream

        def step(i):
            wq, wkv, wup, wdn, wo, cache = layers[i % n_layers]
            blk.decode(B, x.data_ptr(), wq.data_ptr(), wkv.data_ptr(), wup.data_ptr(), wdn.data_ptr(), wo.data_ptr(),
                       cache.data_ptr(), Lk, out.data_ptr(), sh)

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
    assert torch.isfinite(out.float()).all()
    us = e0.elapsed_time(e1) / args.steps * 1e3
    achieved = alg / (us * 1e-6) / 1e9
    res = {"metric": "us per fused MLA decode-block step", "value": us, "unit": "us/step", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "higher_is_better": False, "dtype": "f16 storage, f32 accumulate", "data": "synthetic",
           "config": {"workload": "%s_b%d_kv%d" % (shape.name, B, Lk), "layers_rotated": n_layers},
           "roofline": {"bound": "hbm", "achieved": achieved, "peak": 8000.0, "unit": "GB/s", "frac": achieved / 8000.0,
                        "traffic": MEASURED_TRAFFIC.get("b%d_kv%d" % (B, Lk)) if not args.ranges else None,
                        "algorithmic_bytes": alg,
                        "kernel": "fused_mla_heads" if (B <= 1 and not args.ranges) else "fused_mla_decode"}}
    if not args.no_cpu_baseline:
        from oracle import mla_block as orc
        inp = cf_inputs.make_mla_inputs(shape, seed=1000, batch=B, kv_len=Lk, poison=False)
        a = (inp["x"], inp["w_q"], inp["w_kv"], inp["w_up"], inp["w_down"], inp["w_o"], inp["kv_cache"], Lk, nh, n, r, l,
             v, shape.rope_base)
        orc.mla_decode_block(*a)
        ts = []
        t_end = time.perf_counter() + 10.0
        while time.perf_counter() < t_end and len(ts) < 20:
            t0 = time.perf_counter()
            orc.mla_decode_block(*a)
            ts.append(time.perf_counter() - t0)
        res["cpu_baseline"] = {"value": float(np.median(ts)) * 1e6, "unit": "us/step", "cores": len(os.sched_getaffinity(0)),
                               "kind": "oracle", "sample": "%d whole steps of the same shape (numpy fp64 oracle)" % len(ts)}
    print(json.dumps(res), flush=True)
    blk.close()


if __name__ == "__main__":
    main()
