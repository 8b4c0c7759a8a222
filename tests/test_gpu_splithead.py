"""GPU parity of the SplitHead variant (cf_splithead_decode; paper Appendix B, Alg. 5) with the CPU oracle of the
decode block, through the C ABI.  Alg. 5 computes the same block as Alg. 3 with the work divided along the head
dimension, so the oracle is the same one (oracle/decode_block.py, its C twin for the large shape); that Alg. 5, taken
step by step, is that function is pinned on the CPU (oracle/splithead_block.py, tests/test_oracle_splithead.py), and one
case here compares with that execution directly.

Bar, as for the other kernel: max|err| <= 1e-2 * max|ref| + 1e-3 on the output (fp16 storage, fp32 accumulation;
the order of the atomic additions over the heads is not fixed, which stays far inside this), relative RMS < 5e-3;
the appended K/V rows within one fp16 ulp plus the fp32 accumulation error of a d_model-term dot product; every other
cache row bit-identical.
"""
import sys

import numpy as np
import pytest

import cf_inputs
from oracle import decode_block as orc
from oracle import c_oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _log(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def run(shape, inp, pos, team, calls=2, spin_us=None):
    from paper_2508_18850_amd import SplitHeadBlock
    dev = torch.device("cuda:0")
    blk = SplitHeadBlock(shape.d_model, shape.n_q_heads, shape.head_dim, inp["max_seq"], shape.rope_base, team)
    if spin_us is not None:
        blk.set_spin_limit(spin_us)
    st = torch.cuda.current_stream().cuda_stream
    t = {k: torch.from_numpy(inp[k]).to(dev) for k in ("x", "w_qkv", "w_o", "k_cache", "v_cache")}
    w_members = torch.full_like(t["w_qkv"], float("nan"))
    blk.pack(t["w_qkv"].data_ptr(), w_members.data_ptr(), st)
    out = torch.full((1, shape.d_model), float("nan"), dtype=torch.float16, device=dev)
    for _ in range(calls):      # calls in a row: accumulator, counters and slots of one call must not leak into the next
        out.fill_(float("nan"))
        blk.decode(t["x"].data_ptr(), w_members.data_ptr(), t["w_o"].data_ptr(), t["k_cache"].data_ptr(),
                   t["v_cache"].data_ptr(), pos, out.data_ptr(), st)
    try:
        blk.status(st)
    finally:
        res = {"out": out.cpu().numpy(), "k_cache": t["k_cache"].cpu().numpy(), "v_cache": t["v_cache"].cpu().numpy()}
        blk.close()
    return res


def check(res, ref, inp, pos, label):
    out = res["out"].astype(np.float64)
    mref = np.abs(ref["out"]).max()
    err = np.abs(out - ref["out"]).max()
    tol = 1e-2 * mref + 1e-3
    rel_rms = np.sqrt(np.mean((out - ref["out"]) ** 2) / np.mean(ref["out"] ** 2))
    _log("%s: max|err| %.3e tol %.3e max|ref| %.3e rel-rms %.2e" % (label, err, tol, mref, rel_rms))
    assert np.isfinite(out).all()
    assert err <= tol
    assert rel_rms < 5e-3
    for cache, refrow in (("k_cache", ref["k_rot"]), ("v_cache", ref["v_new"])):
        got = res[cache][:, :, pos, :].astype(np.float64)
        bad = np.abs(got - refrow) > np.abs(refrow) * 2.0 ** -10 + 2e-5
        assert not bad.any(), (cache, float(np.abs(got - refrow)[bad].max()))
        before, after = inp[cache].view(np.uint16).copy(), res[cache].view(np.uint16).copy()
        before[:, :, pos, :] = 0
        after[:, :, pos, :] = 0
        assert np.array_equal(before, after), cache + ": rows other than pos were modified"


def oracle(inp, shape, pos, use_c=False):
    fn = c_oracle.decode_block if use_c else orc.decode_block
    return fn(inp["x"], inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], pos, shape.n_q_heads,
              shape.n_kv_heads, shape.head_dim, shape.rope_base)


def mha(d_model, heads, head_dim, base=10000.0):
    return cf_inputs.BlockShape("s", d_model, heads, heads, head_dim, base, 0)


CASES = [
    # name, shape, team size, cached tokens: empty cache, one cached row, a ragged count, several load batches, a
    # head count that is not a multiple of 8 (plain workgroup order), d_model that no 512 x 8 tile divides
    ("tiny_n2_empty", cf_inputs.SHAPES["tiny"], 2, 0),
    ("tiny_n4_one", cf_inputs.SHAPES["tiny"], 4, 1),
    ("tiny_n4", cf_inputs.SHAPES["tiny"], 4, 256),
    ("tiny_n2", cf_inputs.SHAPES["tiny"], 2, 77),
    ("d128_n8", mha(1024, 16, 128, 500000.0), 8, 333),
    ("d128_n4_5heads", mha(264, 5, 128), 4, 1000),
    ("d128_n2_ragged_d", mha(4104, 3, 128), 2, 45),
    ("d128_n8_long", mha(512, 8, 128), 8, 9000),
]


@pytest.mark.parametrize("name,shape,team,kv_len", CASES)
def test_small_shapes_match_oracle(name, shape, team, kv_len):
    _log("splithead case %s N=%d L=%d" % (name, team, kv_len))
    inp = cf_inputs.make_inputs(shape, seed=71, batch=1, kv_len=kv_len)
    check(run(shape, inp, kv_len, team), oracle(inp, shape, kv_len), inp, kv_len, name)


@pytest.mark.parametrize("team", [2, 4, 8])
def test_pack_gives_the_documented_layout(team):
    """cf_splithead_pack: [head][member][d_model][q lo | q hi | k lo | k hi | v lo | v hi], a member's dimensions as in
    oracle/splithead_block.block_dims (bit-exact: the values are only moved)."""
    from oracle import splithead_block as sh
    from paper_2508_18850_amd import SplitHeadBlock
    D, nh, d = 72, 3, 128
    rng = np.random.Generator(np.random.PCG64(team))
    w = rng.standard_normal((D, 3 * nh * d)).astype(np.float16)
    want = np.empty((nh, team, D, 3 * d // team), dtype=np.float16)
    for i in range(nh):
        for b in range(team):
            dims = sh.block_dims(b, team, d)
            want[i, b] = np.concatenate([w[:, which * nh * d + i * d + dims] for which in range(3)], axis=1)
    blk = SplitHeadBlock(D, nh, d, 16, 10000.0, team)
    st = torch.cuda.current_stream().cuda_stream
    src = torch.from_numpy(w).cuda()
    dst = torch.full_like(src, float("nan"))
    blk.pack(src.data_ptr(), dst.data_ptr(), st)
    blk.status(st)
    got = dst.cpu().numpy().reshape(want.shape)
    blk.close()
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))


def test_matches_the_block_by_block_execution_of_alg5():
    """The same bar against the oracle that takes Alg. 5's steps block by block (oracle/splithead_block.py)."""
    from oracle import splithead_block as sh
    shape = cf_inputs.SHAPES["tiny"]
    _log("splithead vs Alg. 5 oracle")
    inp = cf_inputs.make_inputs(shape, seed=13, batch=1, kv_len=77)
    ref = sh.splithead_decode_block(inp["x"], inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], 77,
                                    shape.n_q_heads, shape.head_dim, shape.rope_base, 4)
    check(run(shape, inp, 77, 4), ref, inp, 77, "alg5")


def test_headline_shape_matches_oracle():
    """Llama-2-7B shape, 4096 cached tokens, 8 workgroups per head: the configuration the comparison is timed on."""
    shape = cf_inputs.SHAPES["llama2_7b"]
    _log("splithead llama2_7b N=8 L=4096")
    inp = cf_inputs.make_inputs(shape, seed=3, batch=1, kv_len=4096)
    check(run(shape, inp, 4096, 8, calls=3), oracle(inp, shape, 4096, use_c=True), inp, 4096, "llama2_7b")


def test_long_cache_matches_oracle():
    """The longest cached length of the sweep the comparison is run on (16384 tokens: four load batches per thread in
    the score and P.V stages, 64 KiB of scores in LDS)."""
    shape = cf_inputs.SHAPES["llama2_7b"]
    _log("splithead llama2_7b N=8 L=16384")
    inp = cf_inputs.make_inputs(shape, seed=4, batch=1, kv_len=16384)
    check(run(shape, inp, 16384, 8, calls=2), oracle(inp, shape, 16384, use_c=True), inp, 16384, "llama2_7b_16k")


def test_same_result_as_the_split_token_kernel():
    """The two dataflows are the same function: their outputs agree to the fp16 rounding of the result and the
    difference of two fp32 summation orders (2 fp16 ulps of the largest output allowed)."""
    from paper_2508_18850_amd import DecodeBlock
    shape = mha(1024, 16, 128)
    inp = cf_inputs.make_inputs(shape, seed=9, batch=1, kv_len=700)
    _log("splithead vs split token")
    got = run(shape, inp, 700, 8)["out"].astype(np.float64)
    dev = torch.device("cuda:0")
    blk = DecodeBlock(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, 1, inp["max_seq"], shape.rope_base)
    st = torch.cuda.current_stream().cuda_stream
    t = {k: torch.from_numpy(inp[k]).to(dev) for k in ("x", "w_qkv", "w_o", "k_cache", "v_cache")}
    out = torch.empty((1, shape.d_model), dtype=torch.float16, device=dev)
    blk.decode_block(1, t["x"].data_ptr(), t["w_qkv"].data_ptr(), t["w_o"].data_ptr(), t["k_cache"].data_ptr(),
                     t["v_cache"].data_ptr(), 700, out.data_ptr(), st)
    blk.status(st)
    want = out.cpu().numpy().astype(np.float64)
    blk.close()
    assert np.abs(got - want).max() <= 2 * 2.0 ** -10 * np.abs(want).max()


def test_captured_launch_replays():
    """The launch stamp is counted on the device, so a launch recorded once in a HIP graph stays valid on every replay:
    three replays, with eager launches and synchronisation between them, each compared with the oracle (the atomic
    additions over the heads make the last bits vary, so not bit for bit) and each appended row with the eager one."""
    from paper_2508_18850_amd import SplitHeadBlock
    shape, team, pos = mha(1024, 16, 128), 4, 300
    inp = cf_inputs.make_inputs(shape, seed=77, batch=1, kv_len=pos)
    ref = oracle(inp, shape, pos)
    dev = torch.device("cuda:0")
    blk = SplitHeadBlock(shape.d_model, shape.n_q_heads, shape.head_dim, inp["max_seq"], shape.rope_base, team)
    t = {k: torch.from_numpy(inp[k]).to(dev) for k in ("x", "w_qkv", "w_o", "k_cache", "v_cache")}
    w_members = torch.empty_like(t["w_qkv"])
    out = torch.full((1, shape.d_model), float("nan"), dtype=torch.float16, device=dev)
    s = torch.cuda.Stream()

    def launch(stream):
        blk.decode(t["x"].data_ptr(), w_members.data_ptr(), t["w_o"].data_ptr(), t["k_cache"].data_ptr(),
                   t["v_cache"].data_ptr(), pos, out.data_ptr(), stream)

    with torch.cuda.stream(s):
        blk.pack(t["w_qkv"].data_ptr(), w_members.data_ptr(), s.cuda_stream)
        launch(s.cuda_stream)
        blk.status(s.cuda_stream)
    torch.cuda.synchronize()
    k_eager = t["k_cache"][:, :, pos].clone()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        launch(torch.cuda.current_stream().cuda_stream)
    for rep in range(3):
        out.fill_(float("nan"))
        t["k_cache"][:, :, pos].zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        blk.status(0)
        res = {"out": out.cpu().numpy(), "k_cache": t["k_cache"].cpu().numpy(), "v_cache": t["v_cache"].cpu().numpy()}
        check(res, ref, inp, pos, "replay %d" % rep)
        assert torch.equal(t["k_cache"][:, :, pos], k_eager)
        launch(torch.cuda.current_stream().cuda_stream)          # eager launches move the device-side count on as well
        launch(torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        blk.status(0)
    blk.close()


def test_unsupported_and_invalid_arguments():
    from paper_2508_18850_amd import SplitHeadBlock, CfError
    for args, code in (((512, 8, 64, 256, 10000.0, 8), -2),      # 64 / (2 * 8) = 4 dimensions per half: below one 16-byte piece
                       ((512, 8, 64, 256, 10000.0, 3), -2),      # team size not 2, 4 or 8
                       ((4096, 64, 128, 256, 10000.0, 8), -2),   # 512 workgroups cannot be resident
                       ((4096, 32, 128, 40000, 10000.0, 8), -2),  # the scores of 40000 tokens do not fit in LDS
                       ((4096, 32, 96, 256, 10000.0, 2), -2),
                       ((4096, 0, 128, 256, 10000.0, 2), -1)):
        with pytest.raises(CfError) as e:
            SplitHeadBlock(*args)
        assert e.value.code == code, args
    blk = SplitHeadBlock(512, 8, 64, 256, 10000.0, 4)
    a = torch.zeros(1 << 20, dtype=torch.float16, device="cuda")
    p = a.data_ptr()
    assert blk.decode_rc(p, p, p, p, p, 256, p) == -1            # pos == max_seq
    assert blk.decode_rc(p, p, p, p, p, -1, p) == -1
    assert blk.decode_rc(0, p, p, p, p, 3, p) == -1              # null pointer
    assert blk.decode_rc(p + 2, p, p, p, p, 3, p) == -1          # misaligned
    blk.close()


def test_forced_timeout_is_reported_and_the_handle_recovers():
    """With the limit -1 the peers of member 0 are absent and its waits give up at the first look, whatever the timing:
    the launch still ends (no wait is unbounded), cf_splithead_status reports CF_ETIMEOUT and clears the workspace, and
    the next call is correct."""
    from paper_2508_18850_amd import SplitHeadBlock, CfError
    shape = mha(2048, 32, 128)
    inp = cf_inputs.make_inputs(shape, seed=5, batch=1, kv_len=200)
    dev = torch.device("cuda:0")
    blk = SplitHeadBlock(shape.d_model, shape.n_q_heads, shape.head_dim, inp["max_seq"], shape.rope_base, 8)
    st = torch.cuda.current_stream().cuda_stream
    t = {k: torch.from_numpy(inp[k]).to(dev) for k in ("x", "w_qkv", "w_o", "k_cache", "v_cache")}
    w_members = torch.empty_like(t["w_qkv"])
    blk.pack(t["w_qkv"].data_ptr(), w_members.data_ptr(), st)
    out = torch.empty((1, shape.d_model), dtype=torch.float16, device=dev)
    args = (t["x"].data_ptr(), w_members.data_ptr(), t["w_o"].data_ptr(), t["k_cache"].data_ptr(), t["v_cache"].data_ptr(),
            200, out.data_ptr(), st)
    blk.set_spin_limit(-1)          # members 1.. of every team leave at once, member 0 gives up at its first look
    _log("splithead forced timeout")
    blk.decode(*args)
    with pytest.raises(CfError) as e:
        blk.status(st)
    assert e.value.code == -5
    blk.set_spin_limit(2000000)
    blk.decode(*args)
    blk.status(st)
    res = {"out": out.cpu().numpy(), "k_cache": t["k_cache"].cpu().numpy(), "v_cache": t["v_cache"].cpu().numpy()}
    blk.close()
    check(res, oracle(inp, shape, 200), inp, 200, "after timeout")
