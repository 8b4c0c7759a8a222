#!/usr/bin/env python3
"""Benchmark of the fused decode block on one MI355X.

A step is one call of cf_decode_block (the whole hot path: QKV projection, RoPE,
KV append, split-KV attention, output projection) on one layer's buffers.  The
steps rotate over a stack of distinct layers whose total size exceeds the 256 MB
Infinity Cache, so weights and KV rows really come from HBM, as in a model with
many layers.  All inputs are synthetic, generated on the device before timing.

Prints ONE JSON line on stdout (details go to stderr).  With --sweep it prints one such line for every row
of the measurement table instead (the Llama-2-7B shape at six cache lengths, the Llama-3-8B shape at batch 1, 4
and 16, the Llama-2-70B shape and its stack of 80 distinct layers, and four rows in which one cf_decode_stack call
runs all layers of a pass in a single launch).  After the timed region, outside the events,
one more step on the first layer is checked against the C oracle at the tolerance of the parity tests, and the
same layers are run once more with one cf_decode_stack launch per pass ("one_launch_stack" in the line; `value` is
always the one-launch-per-layer figure).
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

METRIC = "µs per fused decode-block step and achieved HBM GB/s (% of peak), batch 1"
HBM_PEAK_GBS = 8000.0

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (see profiles/),
# keyed by workload name; None = not measured for that workload.
MEASURED_TRAFFIC = {
    # profiles/fused_decode_block_llama2_7b_kv4096_hbm_traffic.md and profiles/fused_decode_block_gqa_shapes.md:
    # (FETCH_SIZE KiB x 2.0000 + WRITE_SIZE KiB) x 1024, measured on fused_decode_block (one launch per layer)
    "llama2_7b_b1_kv4096": 207280105,      # 100167.0, 2088.0
    "llama3_8b_b1_kv8192": 126311424,      # 60241.5, 2868.0
    "llama3_8b_b4_kv8192": 236295724,      # 112006.8, 6744.0
    "llama3_8b_b16_kv8192": 682216448,     # 321221.5, 23784.0
    "llama2_70b_b1_kv32768": 456086118,    # 218940.3, 7516.0
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="llama2_7b", help="shape name from cf_inputs.SHAPES")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--kv-len", type=int, default=None)
    ap.add_argument("--max-seq", type=int, default=0, help="rows of a KV-cache head slice (0 = kv_len + 9, cf_inputs.default_max_seq)")
    ap.add_argument("--layers", type=int, default=0, help="distinct layer buffer sets to rotate over (0 = auto)")
    ap.add_argument("--workgroups", type=int, default=0)
    ap.add_argument("--k-splits", type=int, default=0)
    ap.add_argument("--kv-splits", type=int, default=0)
    ap.add_argument("--row-major", action="store_true",
                    help="time cf_decode_block on row-major weights instead of the packed layout")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three 1 GiB device-to-device copies (a kernel of known traffic) before the "
                         "timed region, for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings")
    ap.add_argument("--no-arena", action="store_true", help="one device allocation per tensor instead of one for all layers")
    ap.add_argument("--reps", type=int, default=1,
                    help="further timed regions of --steps launches after the first (reported as median / p10 / p90 in\n                    \"repetitions\"; the headline value is always the first region)")
    ap.add_argument("--layer", action="store_true",
                    help="time cf_decode_layer (RMSNorm in front of the block and the residual added, in the same kernel) "
                         "instead of the bare block; out then is a second buffer")
    ap.add_argument("--graph", action="store_true",
                    help="capture one pass over the rotating layers in a HIP graph and time replays of it instead of "
                         "stream launches (steps is rounded down to a multiple of the layer count)")
    ap.add_argument("--stack", action="store_true",
                    help="one cf_decode_stack call per pass over the rotating layers (every layer reads the hidden state "
                         "the previous one wrote; for the bare block that is ONE launch per pass): a timed step still is "
                         "one layer (steps is rounded down to a multiple of the layer count)")
    ap.add_argument("--ragged", action="store_true",
                    help="rows of different lengths (cf_decode_layer_rows): row b caches a seeded length between kv_len/4 "
                         "and kv_len, the first row kv_len; the algorithmic bytes count each row's own length")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget of the cpu_baseline leg")
    ap.add_argument("--no-check", action="store_true", help="skip the check of one step against the C oracle")
    ap.add_argument("--no-stack-line", action="store_true",
                    help="skip the extra measurement of the same layers with one launch per pass (\"one_launch_stack\")")
    ap.add_argument("--sweep", action="store_true",
                    help="one JSON line per row of the measurement table (each with --steps launches; the workload, "
                         "batch, cache length and layer count of the row replace those given here)")
    return ap.parse_args()


# rows of the measurement table: (workload, batch, cached tokens, layers to rotate over; 0 = enough for 3 GiB,
# one cf_decode_stack call per pass over the layers instead of one launch per layer)
SWEEP = [("llama2_7b", 1, 4096, 0, False), ("llama2_7b", 1, 1024, 0, False), ("llama2_7b", 1, 2048, 0, False),
         ("llama2_7b", 1, 8192, 0, False), ("llama2_7b", 1, 16384, 0, False), ("llama2_7b", 1, 32768, 0, False),
         ("llama3_8b", 1, 8192, 0, False), ("llama3_8b", 4, 8192, 0, False), ("llama3_8b", 16, 8192, 0, False),
         ("llama2_70b", 1, 32768, 0, False), ("llama2_70b", 1, 32768, 80, False),
         ("llama2_7b", 1, 4096, 32, True), ("llama3_8b", 1, 8192, 32, True), ("llama3_8b", 16, 8192, 32, True),
         ("llama2_70b", 1, 32768, 80, True)]


def cpu_baseline(shape, batch, kv_len, budget_s):
    """Time the plain C oracle on the host cores for the same workload (one layer): all cores, then one thread."""
    import numpy as np
    import cf_inputs
    from oracle import c_oracle
    inp = cf_inputs.make_inputs(shape, seed=1000, batch=batch, kv_len=kv_len, poison=False)
    args = (inp["x"], inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], kv_len,
            shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_base)

    def timed(threads, budget):
        c_oracle.set_num_threads(threads)
        t0 = time.perf_counter()
        c_oracle.decode_block(*args)                      # warm-up
        first = time.perf_counter() - t0
        reps = max(1, min(20, int(budget / max(first, 1e-3)) - 1))
        times = []
        for _ in range(reps):
            t0 = time.perf_counter()
            c_oracle.decode_block(*args)
            times.append(time.perf_counter() - t0)
        return float(np.median(times)), reps, int(c_oracle.num_threads())

    cores = len(os.sched_getaffinity(0))
    med, reps, used = timed(cores, 0.6 * budget_s)
    med1, reps1, _ = timed(1, 0.4 * budget_s)
    c_oracle.set_num_threads(cores)
    return {"value": med * 1e6, "unit": "us/step", "cores": used, "kind": "oracle",
            "sample": "%d full steps of the same workload (one layer, B=%d, L=%d), median; C oracle, fp64 accumulation"
                      % (reps, batch, kv_len),
            "single_thread": {"value": med1 * 1e6, "unit": "us/step", "cores": 1, "sample": "%d full steps, median" % reps1}}


def check_against_oracle(shape, B, L, x, w_qkv, w_o, kc, vc, out):
    """One step's output (device tensors, caches as they were before the step for rows < L) against the C oracle."""
    import numpy as np
    from oracle import c_oracle
    c_oracle.set_num_threads(len(os.sched_getaffinity(0)))
    ref = c_oracle.decode_block(x.cpu().numpy(), w_qkv.cpu().numpy(), w_o.cpu().numpy(), kc.cpu().numpy(), vc.cpu().numpy(), L,
                                shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_base)["out"]
    got = out.cpu().numpy().astype(np.float64)
    err, tol = float(np.abs(got - ref).max()), float(1e-2 * np.abs(ref).max() + 1e-3)
    return {"max_abs_err": err, "tolerance": tol, "ok": bool(err <= tol),
            "what": "one step on the first layer after the timed region, whole output, against the C oracle"}


def main():
    args = parse_args()
    if args.gpus != 1:
        log("bench.py measures one GPU only: this build has no multi-GPU path (--gpus %d refused)" % args.gpus)
        sys.exit(2)
    if not args.sweep:
        print(json.dumps(run_one(args)), flush=True)
        return
    import copy
    for (name, batch, kv_len, layers, stack) in SWEEP:
        a = copy.copy(args)
        a.workload, a.batch, a.kv_len, a.layers, a.max_seq, a.stack = name, batch, kv_len, layers, 0, stack
        a.cpu_seconds = min(args.cpu_seconds, 6.0)
        res = run_one(a)
        if layers:
            res["config"]["stack"] = "%d distinct layers; %.3f ms per pass over the stack" % (layers, res["value"] * layers / 1e3)
        print(json.dumps(res), flush=True)


def run_one(args):
    import torch
    import cf_inputs
    from paper_2508_18850_amd import DecodeBlock, algorithmic_bytes

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    shape = cf_inputs.SHAPES[args.workload]
    B = args.batch or shape.batch
    L = args.kv_len if args.kv_len is not None else shape.kv_len
    S = args.max_seq or cf_inputs.default_max_seq(L)
    assert S > L, "--max-seq must leave room for the new token"
    dev = torch.device("cuda:0")
    D, nq, nkv, d = shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim

    blk = DecodeBlock(D, nq, nkv, d, B, S, shape.rope_base)
    if args.workgroups or args.k_splits or args.kv_splits:
        blk.set_tuning(args.workgroups, args.k_splits, args.kv_splits, 0)
    alg_bytes = algorithmic_bytes(blk.cfg, B, L)
    row_pos = None
    if args.ragged:
        import numpy as np
        rng = np.random.Generator(np.random.PCG64(7))
        row_pos = [L] + [int(v) for v in rng.integers(L // 4, L + 1, size=B - 1)]
        # every row reads its own number of cached K/V rows: replace B * L rows by the sum of the lengths
        alg_bytes = algorithmic_bytes(blk.cfg, B, 0) + sum(row_pos) * 2 * nkv * d * 2
    layer_bytes = 2 * (D * shape.n_qkv + nq * d * D + 2 * B * nkv * S * d)
    n_layers = args.layers or max(8, -(-3 * 2 ** 30 // layer_bytes))       # >= 3 GiB of distinct buffers
    log("workload %s B=%d L=%d: %.1f MiB algorithmic bytes/step, %d layers (%.2f GiB resident)"
        % (shape.name, B, L, alg_bytes / 2 ** 20, n_layers, n_layers * layer_bytes / 2 ** 30))

    gen = torch.Generator(device=dev)
    # All layers live in ONE device allocation (an arena), as a serving stack would hold its weights and
    # caches: physically contiguous memory is mapped with large page-table fragments, which keeps the
    # address-translation caches effective over a multi-GiB working set.  --no-arena allocates per tensor.
    nq_b, no_b = blk.packed_sizes()
    wq_elems = D * shape.n_qkv if args.row_major else nq_b // 2
    wo_elems = nq * d * D if args.row_major else no_b // 2
    kv_elems = B * nkv * S * d
    align = 2 ** 20                                              # elements: 2 MiB
    def up(n):
        return -(-n // align) * align
    per_layer = up(wq_elems) + up(wo_elems) + 2 * up(kv_elems)
    arena = None if args.no_arena else torch.empty((n_layers * per_layer,), dtype=torch.float16, device=dev)
    def carve(i, off, n, shape_):
        if arena is None:
            return torch.empty(shape_, dtype=torch.float16, device=dev)
        return arena[i * per_layer + off: i * per_layer + off + n].view(shape_)
    layers = []
    for i in range(n_layers):
        gen.manual_seed(1000 + i)
        w_qkv = (torch.randn((D, shape.n_qkv), generator=gen, device=dev) * 0.02).half()
        w_o = (torch.randn((nq * d, D), generator=gen, device=dev) * 0.02).half()
        kc = carve(i, up(wq_elems) + up(wo_elems), kv_elems, (B, nkv, S, d))
        vc = carve(i, up(wq_elems) + up(wo_elems) + up(kv_elems), kv_elems, (B, nkv, S, d))
        kc.zero_()
        vc.zero_()
        kc[:, :, :L] = torch.randn((B, nkv, L, d), generator=gen, device=dev).half()
        vc[:, :, :L] = torch.randn((B, nkv, L, d), generator=gen, device=dev).half()
        if i == 0 and not args.no_check:
            first_rowmajor = (w_qkv.clone(), w_o.clone())          # for the check after the timed region
        if args.row_major:
            wq_t = carve(i, 0, wq_elems, (D, shape.n_qkv))
            wo_t = carve(i, up(wq_elems), wo_elems, (nq * d, D))
            wq_t.copy_(w_qkv)
            wo_t.copy_(w_o)
        else:
            # weights are static: rearranged once, off the clock, into the library's packed layout
            wq_t = carve(i, 0, wq_elems, (wq_elems,))
            wo_t = carve(i, up(wq_elems), wo_elems, (wo_elems,))
            blk.pack_weights(w_qkv.data_ptr(), w_o.data_ptr(), wq_t.data_ptr(), wo_t.data_ptr(),
                             torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
        del w_qkv, w_o
        layers.append((wq_t, wo_t, kc, vc))
    gen.manual_seed(999)
    x = torch.randn((B, D), generator=gen, device=dev).half()
    out = torch.empty((B, D), dtype=torch.float16, device=dev)

    if args.calibrate_copy:
        src = torch.empty(2 ** 28, dtype=torch.float32, device=dev).normal_()      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    stream = torch.cuda.Stream(device=dev)
    ptrs = [(w.data_ptr(), o.data_ptr(), k.data_ptr(), v.data_ptr()) for (w, o, k, v) in layers]
    xp, op = x.data_ptr(), out.data_ptr()
    torch.cuda.synchronize()

    with torch.cuda.stream(stream):
        sh = stream.cuda_stream

        decode = blk.decode_block if args.row_major else blk.decode_block_packed
        if args.layer:
            gamma = (1.0 + 0.25 * torch.randn((D,), generator=gen, device=dev)).half()
            gp = gamma.data_ptr()

            def decode(B_, xp_, w, o, k, v, L_, op_, sh_):
                blk.decode_layer(B_, xp_, gp, 1e-5, True, not args.row_major, w, o, k, v, L_, op_, sh_)

        if args.ragged:
            rp = torch.tensor(row_pos, dtype=torch.int32, device=dev)
            rpp = rp.data_ptr()
            gp2 = gp if args.layer else 0

            def decode(B_, xp_, w, o, k, v, L_, op_, sh_):
                blk.decode_layer_rows(B_, xp_, gp2, 1e-5, args.layer, not args.row_major, w, o, k, v, rpp, L_, op_, sh_)

        def step(i):
            w, o, k, v = ptrs[i % n_layers]
            decode(B, xp, w, o, k, v, L, op, sh)

        for i in range(args.warmup):
            step(i)
        blk.status(sh)
        plain = False
        if args.stack:
            args.steps = max(1, args.steps // n_layers) * n_layers
            n_passes = args.steps // n_layers
            out2 = torch.empty_like(out)
            cols = list(zip(*ptrs))

            def one_pass():
                blk.decode_stack(B, xp, [gp] * n_layers if args.layer else None, 1e-5, bool(args.layer), not args.row_major,
                                 cols[0], cols[1], cols[2], cols[3], L, out2.data_ptr(), sh)

            one_pass()
            blk.status(sh)

            def timed_region(first_step):
                for _ in range(n_passes):
                    one_pass()
        elif args.graph:
            # one pass over the layers becomes one graph launch; a timed "step" still is one kernel
            args.steps = max(1, args.steps // n_layers) * n_layers
            graph = torch.cuda.CUDAGraph()
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=stream):
                csh = torch.cuda.current_stream().cuda_stream
                for i in range(n_layers):
                    w, o, k, v = ptrs[i]
                    decode(B, xp, w, o, k, v, L, op, csh)
            n_replays = args.steps // n_layers
            graph.replay()
            torch.cuda.synchronize()

            def timed_region(first_step):
                for _ in range(n_replays):
                    graph.replay()
        else:
            plain = not (args.layer or args.ragged)

            def timed_region(first_step):
                for i in range(args.steps):
                    step(first_step + i)
        # timed region: exactly `steps` launches between two events on the launch stream
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        ev0.record(stream)
        timed_region(args.warmup)
        ev1.record(stream)
        torch.cuda.synchronize()
        blk.status(sh)
        ms_total = ev0.elapsed_time(ev1)
        rep_us = [ms_total / args.steps * 1e3]
        for r in range(1, args.reps):
            ea, eb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ea.record(stream)
            timed_region(args.warmup + r * args.steps)
            eb.record(stream)
            torch.cuda.synchronize()
            rep_us.append(ea.elapsed_time(eb) / args.steps * 1e3)
        blk.status(sh)
        one_launch = None
        if plain and d == 128 and not args.sweep and not args.no_stack_line:
            # the same layers once more with ONE launch per pass (cf_decode_stack): reported beside the headline,
            # never as `value`
            out2 = torch.empty_like(out)
            cols = list(zip(*ptrs))

            def one_pass():
                blk.decode_stack(B, xp, None, 1e-5, False, not args.row_major, cols[0], cols[1], cols[2], cols[3], L,
                                 out2.data_ptr(), sh)

            one_pass()
            blk.status(sh)
            n_passes = max(1, args.steps // n_layers)
            ea, eb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            ea.record(stream)
            for _ in range(n_passes):
                one_pass()
            eb.record(stream)
            torch.cuda.synchronize()
            blk.status(sh)
            us_layer = ea.elapsed_time(eb) / (n_passes * n_layers) * 1e3
            one_launch = {"us_per_layer": us_layer, "layers_per_launch": n_layers, "passes": n_passes,
                          "achieved_GBps": alg_bytes / (us_layer * 1e-6) / 1e9,
                          "frac": alg_bytes / (us_layer * 1e-6) / 1e9 / HBM_PEAK_GBS, "kernel": "fused_decode_stack",
                          "what": "all layers of a pass in one launch (cf_decode_stack, every layer reads the hidden state "
                                  "the previous one wrote)"}
    assert torch.isfinite(out.float()).all(), "non-finite output"
    plan = blk.plan()
    check = None
    if not args.no_check and not args.ragged:
        # outside the timed region: the first layer once more, against the oracle
        with torch.cuda.stream(stream):
            step(0)
            blk.status(stream.cuda_stream)
        torch.cuda.synchronize()
        if args.layer:
            log("(check skipped: the oracle leg of bench.py covers the bare block)")
        else:
            check = check_against_oracle(shape, B, L, x, first_rowmajor[0], first_rowmajor[1], layers[0][2], layers[0][3], out)
            assert check["ok"], "the timed kernel disagrees with the oracle: %r" % (check,)

    ms_per_step = ms_total / args.steps
    us = ms_per_step * 1e3
    achieved = alg_bytes / (ms_per_step * 1e-3) / 1e9
    name = "%s_b%d_kv%d" % (shape.name, B, L)
    res = {
        "metric": METRIC, "value": us, "unit": "us/step", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 storage, f32 accumulate", "data": "synthetic",
        "config": {"workload": name, "d_model": D, "n_q_heads": nq, "n_kv_heads": nkv, "head_dim": d,
                   "batch": B, "kv_len": L, "layers_rotated": n_layers,
                   "weight_layout": "row-major" if args.row_major else "packed (per-head blocks, one-time rearrangement)",
                   "launch": ("one cf_decode_stack call per pass over the layers" if args.stack else
                              "graph replay of one pass over the layers" if args.graph else "stream launches"),
                   "fused_steps": "rmsnorm + block + residual" if args.layer else "block",
                   "row_lengths": row_pos if args.ragged else "all kv_len",
                   "plan": plan},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None if (args.layer or args.ragged or args.stack) else MEASURED_TRAFFIC.get(name),
                     "algorithmic_bytes": alg_bytes,
                     "kernel": "fused_decode_layer" if (args.layer or args.ragged) else
                               "fused_decode_stack" if (args.stack and d == 128) else "fused_decode_block"},
    }
    if args.reps > 1:
        import numpy as np
        res["repetitions"] = {"n": len(rep_us), "median_us": float(np.median(rep_us)),
                              "p10_us": float(np.percentile(rep_us, 10)), "p90_us": float(np.percentile(rep_us, 90))}
    if one_launch is not None:
        res["one_launch_stack"] = one_launch
    if check is not None:
        res["check"] = check
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(shape, B, L, args.cpu_seconds)
    blk.close()
    del layers, arena
    torch.cuda.empty_cache()
    return res


if __name__ == "__main__":
    main()
