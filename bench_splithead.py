#!/usr/bin/env python3
"""SplitToken against SplitHead (paper Appendix B, Alg. 5 and the comparison of Appendix C): latency of the same
decode step of the Llama-2-7B-shaped block, batch 1, computed by the two kernels of this library, over a sweep of
cached lengths.

Back-to-back launches on one stream, rotating over several layers' worth of weights and caches (more than the
256 MB of last-level cache), timed with HIP events.  Prints one JSON line per cached length: microseconds per step of
both dataflows, their ratio, and the elements the paper's traffic model (Appendix B) says each dataflow exchanges
per head.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--team", type=int, default=8, help="workgroups per head of the SplitHead kernel (2, 4 or 8)")
    ap.add_argument("--kv-lens", type=str, default="1024,2048,4096,8192,16384")
    ap.add_argument("--workload", type=str, default="llama2_7b")
    args = ap.parse_args()
    import torch
    import cf_inputs
    from paper_2508_18850_amd import DecodeBlock, SplitHeadBlock, algorithmic_bytes
    assert torch.cuda.is_available(), "needs a GPU"
    shape = cf_inputs.SHAPES[args.workload]
    assert shape.n_q_heads == shape.n_kv_heads, "the SplitHead kernel is written for one KV head per query head"
    dev = torch.device("cuda:0")
    D, nh, d, N = shape.d_model, shape.n_q_heads, shape.head_dim, args.team
    gen = torch.Generator(device=dev)
    gen.manual_seed(5)

    def rnd(shp, std):
        return (torch.randn(shp, generator=gen, device=dev) * std).half()

    stream = torch.cuda.Stream(device=dev)
    for Lk in [int(v) for v in args.kv_lens.split(",")]:
        S = cf_inputs.default_max_seq(Lk)
        tok = DecodeBlock(D, nh, nh, d, 1, S, shape.rope_base)
        hd = SplitHeadBlock(D, nh, d, S, shape.rope_base, N)
        layer_bytes = 2 * (4 * D * nh * d + 2 * nh * S * d)
        n_layers = max(4, -(-2 ** 30 // layer_bytes))                       # >= 1 GiB of distinct buffers
        x = rnd((1, D), 1.0)
        out = torch.empty((1, D), dtype=torch.float16, device=dev)
        layers = []
        with torch.cuda.stream(stream):
            sh = stream.cuda_stream
            for _ in range(n_layers):
                w_qkv, w_o = rnd((D, 3 * nh * d), D ** -0.5), rnd((nh * d, D), (nh * d) ** -0.5)
                kc, vc = rnd((1, nh, S, d), 1.0), rnd((1, nh, S, d), 1.0)
                nq, no = tok.packed_sizes()
                wq_p = torch.empty(nq // 2, dtype=torch.float16, device=dev)
                wo_p = torch.empty(no // 2, dtype=torch.float16, device=dev)
                tok.pack_weights(w_qkv.data_ptr(), w_o.data_ptr(), wq_p.data_ptr(), wo_p.data_ptr(), sh)
                w_mem = torch.empty_like(w_qkv)
                hd.pack(w_qkv.data_ptr(), w_mem.data_ptr(), sh)
                stream.synchronize()
                layers.append((wq_p, wo_p, w_mem, w_o, kc, vc))
                del w_qkv

            def step_token(i):
                wq_p, wo_p, _, _, kc, vc = layers[i % n_layers]
                tok.decode_block_packed(1, x.data_ptr(), wq_p.data_ptr(), wo_p.data_ptr(), kc.data_ptr(), vc.data_ptr(), Lk,
                                        out.data_ptr(), sh)

            def step_head(i):
                _, _, w_mem, w_o, kc, vc = layers[i % n_layers]
                hd.decode(x.data_ptr(), w_mem.data_ptr(), w_o.data_ptr(), kc.data_ptr(), vc.data_ptr(), Lk, out.data_ptr(), sh)

            us = {}
            for name, step, blk in (("split_token", step_token, tok), ("split_head", step_head, hd)):
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
                us[name] = e0.elapsed_time(e1) / args.steps * 1e3
        alg = algorithmic_bytes(tok.cfg, 1, Lk)
        # Appendix B: Reduce(size, N) = size * log2(N) * N, Gather(size, N) = size * (N - 1) * N elements per cluster
        lg = math.log2(N)
        model_head = (Lk + 1) * lg * N + D * lg * N
        model_token = d * lg * N + 3 * (d // N) * (N - 1) * N
        print(json.dumps({
            "metric": "us per decode-block step, SplitToken vs SplitHead", "unit": "us/step", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "data": "synthetic", "dtype": "f16 storage, f32 accumulate",
            "config": {"workload": "%s_b1_kv%d" % (shape.name, Lk), "team_size": N, "layers_rotated": n_layers},
            "split_token_us": us["split_token"], "split_head_us": us["split_head"],
            "split_head_over_split_token": us["split_head"] / us["split_token"],
            "algorithmic_bytes": alg, "split_token_frac_of_8TBs": alg / (us["split_token"] * 1e-6) / 8e12,
            "split_head_frac_of_8TBs": alg / (us["split_head"] * 1e-6) / 8e12,
            "paper_model_exchanged_elements_per_head": {"split_token": model_token, "split_head": model_head}}), flush=True)
        tok.close()
        hd.close()
        del layers


if __name__ == "__main__":
    main()
