"""GPU parity: the fused HIP decode block against the CPU oracle, through the C ABI.

Tolerance on the block output (fp16 storage, fp32 accumulation):
    max|err| <= 1e-2 * max|ref| + 1e-3
plus tighter stage-wise checks (rotated queries, per-head attention vectors,
appended cache rows), because the absolute term above is loose for outputs of
magnitude ~0.1.
"""
import dataclasses
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


class Runner:
    """Uploads one case, runs the library, downloads everything the checks need."""

    def __init__(self, shape, batch, max_seq, debug=True):
        from paper_2508_18850_amd import DecodeBlock
        self.shape, self.batch, self.max_seq = shape, batch, max_seq
        self.blk = DecodeBlock(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, batch, max_seq,
                               shape.rope_base, debug=debug)
        self.stream = torch.cuda.current_stream().cuda_stream

    def run(self, inp, pos, out_fill=None, packed=False):
        dev = torch.device("cuda:0")
        t = {k: torch.from_numpy(inp[k]).to(dev) for k in ("x", "w_qkv", "w_o", "k_cache", "v_cache")}
        out = torch.empty((self.batch, self.shape.d_model), dtype=torch.float16, device=dev)
        if out_fill is not None:
            out.fill_(out_fill)
        if packed:
            nq_bytes, no_bytes = self.blk.packed_sizes()
            wq_p = torch.full((nq_bytes // 2,), float("nan"), dtype=torch.float16, device=dev)
            wo_p = torch.full((no_bytes // 2,), float("nan"), dtype=torch.float16, device=dev)
            self.blk.pack_weights(t["w_qkv"].data_ptr(), t["w_o"].data_ptr(), wq_p.data_ptr(), wo_p.data_ptr(),
                                  self.stream)
            self.packed = (wq_p, wo_p)
            self.blk.decode_block_packed(self.batch, t["x"].data_ptr(), wq_p.data_ptr(), wo_p.data_ptr(),
                                         t["k_cache"].data_ptr(), t["v_cache"].data_ptr(), pos, out.data_ptr(),
                                         self.stream)
        else:
            self.blk.decode_block(self.batch, t["x"].data_ptr(), t["w_qkv"].data_ptr(), t["w_o"].data_ptr(),
                                  t["k_cache"].data_ptr(), t["v_cache"].data_ptr(), pos, out.data_ptr(), self.stream)
        self.blk.status(self.stream)
        res = {"out": out.cpu().numpy(), "k_cache": t["k_cache"].cpu().numpy(), "v_cache": t["v_cache"].cpu().numpy()}
        shp = (self.batch, self.shape.n_q_heads, self.shape.head_dim)
        for what, key in ((0, "q_rot"), (1, "attn")):
            a = np.empty(shp, dtype=np.float32)
            self.blk.debug_export(what, a, self.stream)
            res[key] = a
        return res


def oracle(inp, shape, pos, use_c=False):
    fn = c_oracle.decode_block if use_c else orc.decode_block
    return fn(inp["x"], inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], pos,
              shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_base)


def check(res, ref, inp, pos, label):
    out = res["out"].astype(np.float64)
    mref = np.abs(ref["out"]).max()
    err = np.abs(out - ref["out"]).max()
    tol = 1e-2 * mref + 1e-3
    rel_rms = np.sqrt(np.mean((out - ref["out"]) ** 2) / np.mean(ref["out"] ** 2))
    _log("%s: max|err| %.3e tol %.3e max|ref| %.3e rel-rms %.2e" % (label, err, tol, mref, rel_rms))
    assert np.isfinite(out).all()
    assert err <= tol
    assert rel_rms < 5e-3                      # fp16 output rounding alone is ~3e-4
    # stage-wise: fp32 on-chip values against the fp64 oracle
    for key, rtol in (("q_rot", 2e-5), ("attn", 2e-4)):
        e = np.abs(res[key].astype(np.float64) - ref[key]).max()
        assert e <= rtol * np.abs(ref[key]).max() + 1e-6, (key, e)
    # appended rows: fp16 rounding of the oracle's values (1 ulp of fp16 relative slack) on top of the
    # fp32 accumulation error of a d_model-term dot product (sqrt(n) * 2^-24 * sqrt(n) * rms(term):
    # about 5e-6 for n = 4096..8192 and these distributions; 2e-5 allowed); all other rows untouched
    for cache, refrow in (("k_cache", ref["k_rot"]), ("v_cache", ref["v_new"])):
        got = res[cache][:, :, pos, :].astype(np.float64)
        bad = np.abs(got - refrow) > np.abs(refrow) * 2.0 ** -10 + 2e-5
        assert not bad.any(), (cache, float(np.abs(got - refrow)[bad].max()))
        before = inp[cache].view(np.uint16).copy()
        after = res[cache].view(np.uint16).copy()
        before[:, :, pos, :] = 0
        after[:, :, pos, :] = 0
        assert np.array_equal(before, after), cache + ": rows other than pos were modified"


SMALL = cf_inputs.BlockShape("small", 264, 4, 2, 64, 10000.0, 77)


@pytest.mark.parametrize("name,shape,batch,kv_len", [
    ("tiny", cf_inputs.SHAPES["tiny"], 1, 256),
    ("ragged_d64_g2_b3", SMALL, 3, 77),
    ("d128_g4_b2", cf_inputs.BlockShape("s", 1024, 16, 4, 128, 500000.0, 333), 2, 333),
    ("d128_g8_b1", cf_inputs.BlockShape("s", 512, 16, 2, 128, 10000.0, 1000), 1, 1000),
    ("d128_g1_b16", cf_inputs.BlockShape("s", 512, 8, 8, 128, 10000.0, 130), 16, 130),
    ("d64_g8_b5", cf_inputs.BlockShape("s", 256, 8, 1, 64, 10000.0, 45), 5, 45),
])
@pytest.mark.parametrize("packed", [False, True])
def test_small_shapes_match_oracle(name, shape, batch, kv_len, packed):
    _log("case %s B=%d L=%d packed=%s" % (name, batch, kv_len, packed))
    inp = cf_inputs.make_inputs(shape, seed=11, batch=batch, kv_len=kv_len)
    r = Runner(shape, batch, inp["max_seq"])
    res = r.run(inp, kv_len, out_fill=float("nan"), packed=packed)
    _log("plan %s" % r.blk.plan())
    check(res, oracle(inp, shape, kv_len), inp, kv_len, name)
    if packed:
        # the packed buffers are a pure rearrangement of the weights: per-head blocks of W_qkv (padded),
        # [head][512-column chunk][row][512] tiles of W_o, zero-filled past d_model (bit-exact)
        D, nq, d = shape.d_model, shape.n_q_heads, shape.head_dim
        wq_p, wo_p = (a.cpu().numpy().view(np.uint16) for a in r.packed)
        want_q = inp["w_qkv"].view(np.uint16).reshape(D, shape.n_qkv // d, d).transpose(1, 0, 2)
        nblk, pad = shape.n_qkv // d, 128                  # each block is followed by 256 zero bytes
        got_q = wq_p.reshape(nblk, D * d + pad)
        assert np.array_equal(got_q[:, :D * d].reshape(want_q.shape), want_q)
        assert not got_q[:, D * d:].any()
        nch = (D + 511) // 512
        padded = np.zeros((nq * d, nch * 512), dtype=np.uint16)
        padded[:, :D] = inp["w_o"].view(np.uint16)
        want_o = padded.reshape(nq, d, nch, 512).transpose(0, 2, 1, 3)
        assert np.array_equal(wo_p.reshape(want_o.shape), want_o)


@pytest.mark.parametrize("pos", [0, 1, 2, 31, 32, 33, 255])
def test_edge_positions(pos):
    """Empty cache (KV length 1 = the V projection), fewer tokens than splits,
    one wave-step boundary, and the last row of the cache capacity."""
    shape = cf_inputs.SHAPES["tiny"]
    _log("edge pos=%d" % pos)
    inp = cf_inputs.make_inputs(shape, seed=3, kv_len=pos, max_seq=256)
    r = Runner(shape, 1, 256)
    res = r.run(inp, pos)
    ref = oracle(inp, shape, pos)
    check(res, ref, inp, pos, "pos=%d" % pos)
    if pos == 0:
        y = inp["x"].astype(np.float64) @ inp["w_qkv"].astype(np.float64)
        v = y[:, (shape.n_q_heads + shape.n_kv_heads) * shape.head_dim:]
        want = v @ inp["w_o"].astype(np.float64)            # MHA: concat of v_new per head is v itself
        assert np.abs(res["out"].astype(np.float64) - want).max() <= 1e-2 * np.abs(want).max() + 1e-3


def test_repeated_calls_and_decode_sequence():
    """Three consecutive steps on one handle: each step's appended row is read by the next."""
    shape = dataclasses.replace(cf_inputs.SHAPES["tiny"], n_kv_heads=4)
    L = 100
    inp = cf_inputs.make_inputs(shape, seed=5, batch=2, kv_len=L, max_seq=128)
    r = Runner(shape, 2, 128)
    cur = dict(inp)
    rng = np.random.default_rng(0)
    for step in range(3):
        _log("sequence step %d" % step)
        pos = L + step
        cur["x"] = rng.standard_normal(inp["x"].shape).astype(np.float16)
        ref = oracle(cur, shape, pos)
        res = r.run(cur, pos)
        check(res, ref, cur, pos, "step%d" % step)
        cur["k_cache"], cur["v_cache"] = res["k_cache"], res["v_cache"]   # carry the GPU-written cache forward


def test_planted_dominant_keys():
    """A key that dominates the softmax at the first cached token, at a split
    boundary, at the last cached token and at the NEW token must select its value."""
    shape = cf_inputs.SHAPES["tiny"]
    L = 256
    inp = cf_inputs.make_inputs(shape, seed=8, kv_len=L)
    base = oracle(inp, shape, L)
    r = Runner(shape, 1, inp["max_seq"])
    for t in (0, 63, 64, L - 1):
        _log("planted key at %d" % t)
        mod = dict(inp)
        kc = inp["k_cache"].copy()
        for h in range(shape.n_kv_heads):
            q = base["q_rot"][0, h]
            kc[0, h, t] = (60.0 * q / (q @ q) * np.sqrt(shape.head_dim)).astype(np.float16)
        mod["k_cache"] = kc
        ref = oracle(mod, shape, L)
        res = r.run(mod, L)
        check(res, ref, mod, L, "planted@%d" % t)
        assert np.abs(res["attn"][0] - inp["v_cache"][0, :, t].astype(np.float64)).max() < 1e-3
    # new token dominant: scale x so that q.k_new is huge compared with cached scores
    _log("planted key at the new token")
    mod = dict(inp)
    mod["x"] = (inp["x"].astype(np.float32) * 12.0).astype(np.float16)
    mod["w_qkv"] = inp["w_qkv"].copy()
    nq, nkv, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    mod["w_qkv"][:, nq * d:(nq + nkv) * d] = mod["w_qkv"][:, :nq * d]      # k_new == q  ->  score |q|^2/sqrt(d)
    ref = oracle(mod, shape, L)
    res = r.run(mod, L)
    check(res, ref, mod, L, "planted@new")
    w_new_min = min(orc.attention_weights(ref["q_rot"][0, h], np.concatenate(
        [mod["k_cache"][0, h, :L].astype(np.float64), ref["k_rot"][0, h][None]], 0))[-1] for h in range(nq))
    assert w_new_min > 0.99


def test_error_paths_do_not_launch():
    from paper_2508_18850_amd import DecodeBlock, CfError
    shape = cf_inputs.SHAPES["tiny"]
    blk = DecodeBlock(shape.d_model, 8, 8, 64, 2, 128, 10000.0)
    buf = torch.zeros(1 << 20, dtype=torch.float16, device="cuda:0")
    p = buf.data_ptr()
    assert blk.decode_block_rc(3, p, p, p, p, p, 0, p) == -1          # batch > max_batch
    assert blk.decode_block_rc(1, p, p, p, p, p, 128, p) == -1        # pos == max_seq
    assert blk.decode_block_rc(1, p, p, p, p, p, -1, p) == -1
    assert blk.decode_block_rc(1, p + 2, p, p, p, p, 0, p) == -1      # misaligned
    assert blk.decode_block_rc(1, 0, p, p, p, p, 0, p) == -1          # null
    with pytest.raises(CfError):
        DecodeBlock(512, 8, 8, 96, 1, 128, 10000.0)                    # head_dim not compiled
    with pytest.raises(CfError):
        DecodeBlock(512, 8, 3, 64, 1, 128, 10000.0)                    # n_q % n_kv != 0
    blk.status()
    blk.close()


def _device_case(shape, batch, kv_len, seed):
    inp = cf_inputs.make_inputs(shape, seed=seed, batch=batch, kv_len=kv_len, poison=False)
    dev = torch.device("cuda:0")
    t = {k: torch.from_numpy(inp[k]).to(dev) for k in ("x", "w_qkv", "w_o", "k_cache", "v_cache")}
    out = torch.empty((batch, shape.d_model), dtype=torch.float16, device=dev)
    return inp, t, out


def test_spin_limit_reports_timeout_and_handle_recovers():
    """A spin limit of zero makes the bounded waits give up at their first unsuccessful look: the kernel
    still ends, cf_status reports CF_ETIMEOUT, and the next call on the same handle is correct."""
    from paper_2508_18850_amd import DecodeBlock, CfError
    shape = cf_inputs.SHAPES["llama2_7b"]
    L = 1024
    inp, t, out = _device_case(shape, 1, L, seed=77)
    blk = DecodeBlock(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, 1, inp["max_seq"],
                      shape.rope_base)
    args = (1, t["x"].data_ptr(), t["w_qkv"].data_ptr(), t["w_o"].data_ptr(), t["k_cache"].data_ptr(),
            t["v_cache"].data_ptr(), L, out.data_ptr(), 0)
    blk.set_tuning(0, 0, 0, -1)                   # give up at the first failed look
    _log("launch with a zero spin limit")
    blk.decode_block(*args)
    with pytest.raises(CfError) as ei:
        blk.status()
    assert ei.value.code == -5
    blk.set_tuning(0, 0, 0, 2000000)              # back to 2 s
    _log("launch with the normal spin limit")
    blk.decode_block(*args)
    blk.status()
    ref = oracle(inp, shape, L, use_c=True)
    got = out.cpu().numpy().astype(np.float64)
    assert np.abs(got - ref["out"]).max() <= 1e-2 * np.abs(ref["out"]).max() + 1e-3
    blk.close()


def test_many_launches_are_bitwise_reproducible():
    """300 launches on one handle with changing positions and batch sizes (launch stamps keep
    counting, the split plan changes): the same call always gives the same bits."""
    shape = cf_inputs.BlockShape("s", 1024, 16, 4, 128, 10000.0, 600)
    inp, t, out = _device_case(shape, 4, 600, seed=5)
    from paper_2508_18850_amd import DecodeBlock
    blk = DecodeBlock(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, 4, inp["max_seq"],
                      shape.rope_base)
    k0, v0 = t["k_cache"].clone(), t["v_cache"].clone()
    first = {}
    cases = [(1, 600), (4, 37), (2, 599), (4, 600), (3, 0), (1, 1)]
    for i in range(300):
        b, pos = cases[i % len(cases)]
        t["k_cache"].copy_(k0)
        t["v_cache"].copy_(v0)
        out.fill_(float("nan"))
        blk.decode_block(b, t["x"].data_ptr(), t["w_qkv"].data_ptr(), t["w_o"].data_ptr(), t["k_cache"].data_ptr(),
                         t["v_cache"].data_ptr(), pos, out.data_ptr(), torch.cuda.current_stream().cuda_stream)
        got = out[:b].cpu().numpy().view(np.uint16).copy()
        if (b, pos) in first:
            assert np.array_equal(got, first[(b, pos)]), "launch %d differs for batch %d pos %d" % (i, b, pos)
        else:
            first[(b, pos)] = got
    blk.status()
    for (b, pos), bits in first.items():
        sub = {k: (inp[k][:b] if k in ("x", "k_cache", "v_cache") else inp[k]) for k in inp if k not in ("shape",)}
        ref = orc.decode_block(sub["x"], inp["w_qkv"], inp["w_o"], sub["k_cache"], sub["v_cache"], pos,
                               shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_base)["out"]
        got = bits.view(np.float16).astype(np.float64)
        assert np.abs(got - ref).max() <= 1e-2 * np.abs(ref).max() + 1e-3, (b, pos)
    blk.close()


@pytest.mark.parametrize("heads,workgroups", [(32, 32), (32, 64), (32, 128), (32, 256), (64, 64), (64, 128), (64, 256),
                                              (128, 128), (128, 256)])
def test_team_sizes_and_head_counts(heads, workgroups):
    """The team size (workgroups per head: 1, 2, 4, 8; the paper's cluster size) against the head count, as in the
    sweep of the paper's evaluation with varying cluster sizes and numbers of heads: every combination the sweep
    times gives the oracle's result (packed and row-major weights)."""
    shape = cf_inputs.BlockShape("s", 512, heads, heads, 128, 10000.0, 300)
    _log("heads=%d workgroups=%d" % (heads, workgroups))
    inp = cf_inputs.make_inputs(shape, seed=40 + heads, batch=1, kv_len=300)
    ref = oracle(inp, shape, 300)
    for packed in (False, True):
        r = Runner(shape, 1, inp["max_seq"])
        r.blk.set_tuning(workgroups=workgroups)
        res = r.run(inp, 300, packed=packed)
        plan = r.blk.plan()                     # the plan of the call just made
        assert plan["workgroups"] == workgroups and plan["team_size"] == workgroups // heads
        check(res, ref, inp, 300, "heads%d_w%d_%s" % (heads, workgroups, "packed" if packed else "rows"))
        r.blk.close()


@pytest.mark.parametrize("batch", [3, 5, 6, 12])
def test_batches_that_do_not_divide_the_team(batch):
    """Batches between the powers of two on a grouped-query shape with 32 workgroups per KV head: the plan keeps the
    attention items (batch rows x KV splits) within one per member, and the result is the oracle's."""
    shape = cf_inputs.BlockShape("s", 1024, 32, 8, 128, 500000.0, 2100)
    _log("batch %d" % batch)
    inp = cf_inputs.make_inputs(shape, seed=70 + batch, batch=batch, kv_len=2100)
    r = Runner(shape, batch, inp["max_seq"])
    res = r.run(inp, 2100, out_fill=float("nan"), packed=True)
    plan = r.blk.plan()
    _log("plan %s" % plan)
    assert plan["kv_splits"] * batch <= plan["team_size"], plan
    check(res, oracle(inp, shape, 2100), inp, 2100, "b%d" % batch)
    r.blk.close()


@pytest.mark.parametrize("d_model,nq,nkv,hd", [(520, 4, 2, 64), (1032, 3, 3, 128)])
def test_pack_weights_gives_the_documented_layout(d_model, nq, nkv, hd):
    """cf_pack_weights, bit-exact (the values are only moved): W_qkv_packed [(n_q + 2 n_kv)][d_model][head_dim], every
    block followed by 256 zero bytes; W_o_packed [n_q][ceil(d_model / 512)][head_dim][512], zero past d_model."""
    from paper_2508_18850_amd import DecodeBlock
    rng = np.random.Generator(np.random.PCG64(d_model))
    nqkv = (nq + 2 * nkv) * hd
    w_qkv = rng.standard_normal((d_model, nqkv)).astype(np.float16)
    w_o = rng.standard_normal((nq * hd, d_model)).astype(np.float16)
    blk = DecodeBlock(d_model, nq, nkv, hd, 1, 16, 10000.0)
    st = torch.cuda.current_stream().cuda_stream
    qb, ob = blk.packed_sizes()
    nblk, nch = nq + 2 * nkv, -(-d_model // 512)
    assert qb == nblk * (d_model * hd * 2 + 256) and ob == nq * nch * hd * 512 * 2
    a, b = torch.from_numpy(w_qkv).cuda(), torch.from_numpy(w_o).cuda()
    pa = torch.full((qb // 2,), float("nan"), dtype=torch.float16, device="cuda")
    pb = torch.full((ob // 2,), float("nan"), dtype=torch.float16, device="cuda")
    blk.pack_weights(a.data_ptr(), b.data_ptr(), pa.data_ptr(), pb.data_ptr(), st)
    blk.status(st)
    got_q = pa.cpu().numpy().view(np.uint16).reshape(nblk, d_model * hd + 128)
    got_o = pb.cpu().numpy().view(np.uint16).reshape(nq, nch, hd, 512)
    blk.close()
    for j in range(nblk):
        want = np.ascontiguousarray(w_qkv[:, j * hd:(j + 1) * hd]).view(np.uint16).reshape(-1)
        assert np.array_equal(got_q[j, :d_model * hd], want), j
        assert not got_q[j, d_model * hd:].any(), "padding is not zero"
    for i in range(nq):
        for c in range(nch):
            cols = min(512, d_model - 512 * c)
            want = w_o[i * hd:(i + 1) * hd, 512 * c:512 * c + cols].view(np.uint16)
            assert np.array_equal(got_o[i, c, :, :cols], want), (i, c)
            assert not got_o[i, c, :, cols:].any(), "columns past d_model are not zero"
