"""GPU parity of the fused MLA decode block (cf_mla_decode) with the CPU oracle (oracle/mla_block.py), through
the C ABI.  cf_mla_decode has two kernels: up to batch 2 the head-team kernel, from batch 3 on (and whenever a limit
on the token ranges is set) the token-range kernel on MFMA tiles; cases of batch 1 and 2 run both.

Tolerance on the block output, as for the other block: max|err| <= 1e-2 * max|ref| + 1e-3 (fp16 storage, fp32
accumulation), plus relative RMS < 5e-3; the appended cache row within one fp16 ulp plus the fp32 accumulation error
of a d_model-term dot product; every other cache row bit-identical.
"""
import sys

import numpy as np
import pytest

import cf_inputs
from oracle import mla_block as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _log(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def run(shape, inp, pos, max_splits=0):
    from paper_2508_18850_amd import MlaBlock
    dev = torch.device("cuda:0")
    B = inp["batch"]
    blk = MlaBlock(shape.d_model, shape.n_heads, shape.nope_dim, shape.rope_dim, shape.kv_lora_rank, shape.v_head_dim,
                   B, inp["max_seq"], shape.rope_base)
    if max_splits:
        blk.set_splits(max_splits)
    st = torch.cuda.current_stream().cuda_stream
    t = {k: torch.from_numpy(inp[k]).to(dev) for k in ("x", "w_q", "w_kv", "w_up", "w_down", "w_o", "kv_cache")}
    out = torch.full((B, shape.d_model), float("nan"), dtype=torch.float16, device=dev)
    for _ in range(2):          # two calls in a row: the second must not be confused by the first one's slots
        blk.decode(B, t["x"].data_ptr(), t["w_q"].data_ptr(), t["w_kv"].data_ptr(), t["w_up"].data_ptr(),
                   t["w_down"].data_ptr(), t["w_o"].data_ptr(), t["kv_cache"].data_ptr(), pos, out.data_ptr(), st)
    blk.status(st)
    res = {"out": out.cpu().numpy(), "kv_cache": t["kv_cache"].cpu().numpy()}
    for what, (name, width) in enumerate((("q_lat", shape.kv_lora_rank), ("q_rope", shape.rope_dim), ("z", shape.kv_lora_rank))):
        res[name] = np.empty((B, shape.n_heads, width), dtype=np.float32)
        blk.debug_export(what, res[name], st)
    blk.close()
    return res


def check(res, ref, inp, pos, label):
    out = res["out"].astype(np.float64)
    mref = np.abs(ref["out"]).max()
    err = np.abs(out - ref["out"]).max()
    rel_rms = np.sqrt(np.mean((out - ref["out"]) ** 2) / np.mean(ref["out"] ** 2))
    _log("%s: max|err| %.3e tol %.3e max|ref| %.3e rel-rms %.2e" % (label, err, 1e-2 * mref + 1e-3, mref, rel_rms))
    assert np.isfinite(out).all()
    assert err <= 1e-2 * mref + 1e-3
    assert rel_rms < 5e-3
    # Stage by stage (Alg. 4): the absorbed query and its rotary part are sums of fp16 products in fp32, compared at the
    # accuracy of such sums; z, a convex combination of fp16 rows, at the block's tolerance.
    for name in ("q_lat", "q_rope", "z"):
        got, want = res[name].astype(np.float64), ref[name]
        e, m = np.abs(got - want).max(), np.abs(want).max()
        tol_s = (1e-2 if name == "z" else 2e-3) * m + 1e-3
        _log("   %s: max|err| %.3e tol %.3e" % (name, e, tol_s))
        assert np.isfinite(got).all() and e <= tol_s, name
    got = res["kv_cache"][:, pos].astype(np.float64)
    bad = np.abs(got - ref["kv_new"]) > np.abs(ref["kv_new"]) * 2.0 ** -10 + 2e-5
    assert not bad.any(), float(np.abs(got - ref["kv_new"])[bad].max())
    before, after = inp["kv_cache"].view(np.uint16).copy(), res["kv_cache"].view(np.uint16).copy()
    before[:, pos] = 0
    after[:, pos] = 0
    assert np.array_equal(before, after), "cache rows other than pos were modified"


def oracle(shape, inp, pos):
    return orc.mla_decode_block(inp["x"], inp["w_q"], inp["w_kv"], inp["w_up"], inp["w_down"], inp["w_o"],
                                inp["kv_cache"], pos, shape.n_heads, shape.nope_dim, shape.rope_dim, shape.kv_lora_rank,
                                shape.v_head_dim, shape.rope_base)


def both_kernels(batch):
    """Range limits to run a case with: 0 = the library's choice (the head-team kernel at batch 1), 32 = the
    token-range kernel with its default ranges."""
    return (0, 32) if batch <= 1 else (0,)


CASES = [
    # name, shape, batch, cached tokens
    ("one_head", cf_inputs.MlaShape("s", 96, 1, 16, 64, 512, 32, 10000.0, 0), 1, 17),
    ("two_heads_b3", cf_inputs.MlaShape("s", 64, 2, 32, 64, 512, 16, 10000.0, 0), 3, 37),
    ("wide_b4", cf_inputs.MlaShape("s", 512, 16, 128, 64, 512, 128, 500000.0, 0), 4, 300),
    ("five_heads_b2", cf_inputs.MlaShape("s", 320, 5, 48, 64, 512, 64, 10000.0, 0), 2, 129),
    # the 16-row batch tile (batch 5..16): fewer rows than the tile, the full tile, one head with many batch rows
    ("two_heads_b7", cf_inputs.MlaShape("s", 64, 2, 32, 64, 512, 16, 10000.0, 0), 7, 150),
    ("wide_b16", cf_inputs.MlaShape("s", 512, 16, 128, 64, 512, 128, 500000.0, 0), 16, 300),
    ("one_head_b16", cf_inputs.MlaShape("s", 96, 1, 16, 64, 512, 32, 10000.0, 0), 16, 40),
    ("five_heads_b9", cf_inputs.MlaShape("s", 320, 5, 48, 64, 512, 64, 10000.0, 0), 9, 700),
]


@pytest.mark.parametrize("name,shape,batch,kv_len", CASES)
def test_small_shapes_match_oracle(name, shape, batch, kv_len):
    _log("mla case %s B=%d L=%d" % (name, batch, kv_len))
    ref = None
    for max_splits in both_kernels(batch):
        inp = cf_inputs.make_mla_inputs(shape, seed=61, batch=batch, kv_len=kv_len)
        ref = ref or oracle(shape, inp, kv_len)
        check(run(shape, inp, kv_len, max_splits), ref, inp, kv_len, "%s (range limit %d)" % (name, max_splits))


@pytest.mark.parametrize("pos", [0, 1, 15, 16, 17, 63, 64, 65, 127, 128, 129])
def test_edge_positions(pos):
    """Empty cache, fewer tokens than members of a team, the boundaries of the token split and of the 64-row tile."""
    shape = cf_inputs.MlaShape("s", 128, 2, 32, 64, 512, 32, 10000.0, 0)
    for batch in (1, 2):
        for max_splits in both_kernels(batch):
            inp = cf_inputs.make_mla_inputs(shape, seed=62 + pos, batch=batch, kv_len=pos)
            check(run(shape, inp, pos, max_splits), oracle(shape, inp, pos), inp, pos,
                  "pos %d batch %d (range limit %d)" % (pos, batch, max_splits))


@pytest.mark.parametrize("max_splits,kv_len,batch", [(1, 700, 2), (3, 700, 2), (32, 700, 1), (5, 1000, 6), (1, 129, 16)])
def test_forced_token_ranges(max_splits, kv_len, batch):
    """One range with several tiles of 128 rows, ranges that end inside a tile, many short ranges, ranges of a 16-row batch."""
    shape = cf_inputs.MlaShape("s", 256, 4, 64, 64, 512, 64, 10000.0, 0)
    inp = cf_inputs.make_mla_inputs(shape, seed=90 + max_splits, batch=batch, kv_len=kv_len)
    check(run(shape, inp, kv_len, max_splits), oracle(shape, inp, kv_len), inp, kv_len,
          "splits<=%d L=%d B=%d" % (max_splits, kv_len, batch))


def test_planted_row_is_selected():
    """A cached row that matches head 0's absorbed query dominates its softmax, wherever it sits in the token split."""
    shape = cf_inputs.MlaShape("s", 128, 2, 32, 64, 512, 32, 10000.0, 0)
    for where in (0, 63, 199):
        inp = cf_inputs.make_mla_inputs(shape, seed=70, batch=1, kv_len=200)
        ref0 = oracle(shape, inp, 200)
        target = np.concatenate([ref0["q_lat"][0, 0], ref0["q_rope"][0, 0]])
        inp["kv_cache"][0, where] = (target * 80.0 / np.linalg.norm(target)).astype(np.float16)
        ref = oracle(shape, inp, 200)
        for max_splits in both_kernels(1):
            mine = dict(inp, kv_cache=inp["kv_cache"].copy())
            check(run(shape, mine, 200, max_splits), ref, mine, 200, "planted at %d (range limit %d)" % (where, max_splits))


def test_full_size_deepseek_v2_lite_shape():
    shape = cf_inputs.MLA_SHAPES["deepseek_v2_lite"]
    ref = None
    for max_splits in both_kernels(1):
        inp = cf_inputs.make_mla_inputs(shape, seed=1000)
        ref = ref or oracle(shape, inp, shape.kv_len)
        check(run(shape, inp, shape.kv_len, max_splits), ref, inp, shape.kv_len, "%s (range limit %d)" % (shape.name, max_splits))


@pytest.mark.parametrize("batch,kv_len", [(16, 4096), (4, 4096), (16, 1000)])
def test_full_size_deepseek_v2_lite_shape_batched(batch, kv_len):
    """The batch of the paper's Appendix C (16) and batch 4 in the configuration bench_mla.py times, and a cache length
    that is no multiple of the tile."""
    shape = cf_inputs.MLA_SHAPES["deepseek_v2_lite"]
    inp = cf_inputs.make_mla_inputs(shape, seed=1001, batch=batch, kv_len=kv_len)
    check(run(shape, inp, kv_len), oracle(shape, inp, kv_len), inp, kv_len, "%s B=%d L=%d" % (shape.name, batch, kv_len))


@pytest.mark.parametrize("batch", [1, 5])
def test_captured_launch_replays(batch):
    """The launch stamp is counted on the device, so a launch recorded once in a HIP graph stays valid on every replay
    (batch 1: the head-team kernel, batch 5: the token-range kernel): three replays, with eager launches and
    synchronisation between them, each bit for bit the eager result, output and appended row."""
    from paper_2508_18850_amd import MlaBlock
    shape, pos = cf_inputs.MlaShape("s", 320, 5, 48, 64, 512, 64, 10000.0, 0), 200
    inp = cf_inputs.make_mla_inputs(shape, seed=90 + batch, batch=batch, kv_len=pos)
    dev = torch.device("cuda:0")
    blk = MlaBlock(shape.d_model, shape.n_heads, shape.nope_dim, shape.rope_dim, shape.kv_lora_rank, shape.v_head_dim,
                   batch, inp["max_seq"], shape.rope_base)
    t = {k: torch.from_numpy(inp[k]).to(dev) for k in ("x", "w_q", "w_kv", "w_up", "w_down", "w_o", "kv_cache")}
    out = torch.full((batch, shape.d_model), float("nan"), dtype=torch.float16, device=dev)
    s = torch.cuda.Stream()

    def launch(stream):
        blk.decode(batch, t["x"].data_ptr(), t["w_q"].data_ptr(), t["w_kv"].data_ptr(), t["w_up"].data_ptr(),
                   t["w_down"].data_ptr(), t["w_o"].data_ptr(), t["kv_cache"].data_ptr(), pos, out.data_ptr(), stream)

    with torch.cuda.stream(s):
        launch(s.cuda_stream)
        blk.status(s.cuda_stream)
    torch.cuda.synchronize()
    eager, row_eager = out.clone(), t["kv_cache"][:, pos].clone()
    ref = oracle(shape, inp, pos)
    assert np.abs(eager.cpu().numpy().astype(np.float64) - ref["out"]).max() <= 1e-2 * np.abs(ref["out"]).max() + 1e-3
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        launch(torch.cuda.current_stream().cuda_stream)
    for rep in range(3):
        out.fill_(float("nan"))
        t["kv_cache"][:, pos].zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        blk.status(0)
        assert torch.equal(out, eager), "replay %d" % rep
        assert torch.equal(t["kv_cache"][:, pos], row_eager), "replay %d" % rep
        launch(torch.cuda.current_stream().cuda_stream)          # eager launches move the device-side count on as well
        launch(torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        blk.status(0)
    blk.close()


def test_unsupported_shapes_and_bad_arguments_are_refused():
    from paper_2508_18850_amd import MlaBlock, CfError
    with pytest.raises(CfError) as e:
        MlaBlock(2048, 16, 128, 64, 256, 128, 1, 64, 10000.0)          # kv_lora_rank the kernel is not written for
    assert e.value.code == -2
    with pytest.raises(CfError) as e:
        MlaBlock(2048, 32, 128, 64, 512, 128, 1, 64, 10000.0)          # more heads than teams fit
    assert e.value.code == -2
    blk = MlaBlock(128, 2, 32, 64, 512, 32, 2, 64, 10000.0)
    a = torch.zeros(1 << 20, dtype=torch.float16, device="cuda")
    p = a.data_ptr()
    assert blk.decode_rc(3, p, p, p, p, p, p, p, 5, p) == -1           # batch above max_batch
    assert blk.decode_rc(1, p, p, p, p, p, p, p, 64, p) == -1          # pos outside the cache
    assert blk.decode_rc(1, p + 2, p, p, p, p, p, p, 5, p) == -1       # misaligned pointer
    assert blk.decode_rc(1, 0, p, p, p, p, p, p, 5, p) == -1           # null pointer
    with pytest.raises(CfError):
        blk.set_splits(33)
    with pytest.raises(CfError):
        blk.debug_export(0, np.empty((1, 2, 512), dtype=np.float32))   # before any call
    blk.close()
    with pytest.raises(CfError) as e:
        MlaBlock(2048, 16, 128, 64, 512, 128, 17, 64, 10000.0)         # batch above the 16-row tile
    assert e.value.code == -2
