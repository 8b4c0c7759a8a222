"""cf_decode_stack through the C ABI: a stack of layers in one call, the hidden state handed from layer to layer.

Checks: (1) the result and every appended cache row are bit-identical to the same layers enqueued one by one with
cf_decode_layer (with RMSNorm or residual, or head_dim 64, the stack is the same launches with the library's buffers in
between; the bare block with head_dim 128 runs all layers in ONE launch, the hidden state handed on inside the kernel);
(2) every layer on its own: the oracle applied to the fp16 hidden state the GPU fed that layer, against what the GPU
made of it, at the block tolerance max|err| <= 1e-2 * max|ref| + 1e-3 (not widened: both start from the same input);
(3) bad arguments are refused before anything is enqueued.
"""
import sys

import numpy as np
import pytest

import cf_inputs
from oracle import decode_block as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _log(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def make_layers(shape, n_layers, batch, kv_len, seed):
    layers = [cf_inputs.make_inputs(shape, seed=seed + l, batch=batch, kv_len=kv_len) for l in range(n_layers)]
    rng = np.random.Generator(np.random.PCG64(seed + 100))
    gammas = [(1.0 + 0.25 * rng.standard_normal(shape.d_model)).astype(np.float16) for _ in range(n_layers)]
    return layers, gammas


def oracle_layer(shape, inp, gamma, eps, residual, pos, x):
    """One layer of the oracle on the hidden state x (fp16 array)."""
    args = (inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], pos, shape.n_q_heads, shape.n_kv_heads,
            shape.head_dim, shape.rope_base)
    if gamma is None:
        ref = orc.decode_block(x, *args)
        if residual:
            ref["out"] = ref["out"] + x.astype(np.float64)
    else:
        ref = orc.decode_layer(x, gamma, eps, *args)
        if not residual:
            ref["out"] = ref["out"] - x.astype(np.float64)
    return ref


def check_layers(shape, layers, gammas, eps, residual, pos, hidden, caches):
    """hidden[l]: the fp16 input of layer l as the GPU had it (hidden[n] = the result); caches[l]: (k, v) after the run."""
    for l, inp in enumerate(layers):
        ref = oracle_layer(shape, inp, None if gammas is None else gammas[l], eps, residual, pos, hidden[l])
        got = hidden[l + 1].astype(np.float64)
        err = np.abs(got - ref["out"]).max()
        tol = 1e-2 * np.abs(ref["out"]).max() + 1e-3
        _log("   layer %d: max|err| %.3e tol %.3e max|ref| %.3e" % (l, err, tol, np.abs(ref["out"]).max()))
        assert np.isfinite(got).all() and err <= tol, (l, err, tol)
        k_row = caches[l][0][:, :, pos, :].astype(np.float64)
        v_row = caches[l][1][:, :, pos, :].astype(np.float64)
        assert (np.abs(k_row - ref["k_rot"]) <= np.abs(ref["k_rot"]) * 2.0 ** -10 + 2e-5).all(), l
        assert (np.abs(v_row - ref["v_new"]) <= np.abs(ref["v_new"]) * 2.0 ** -10 + 2e-5).all(), l


S64 = cf_inputs.BlockShape("s64", 512, 8, 4, 64, 10000.0, 0)
# head_dim 128 without RMSNorm and residual: all layers in one launch
M128 = cf_inputs.BlockShape("mha128", 512, 4, 4, 128, 10000.0, 0)
G2 = cf_inputs.BlockShape("gqa2", 512, 4, 2, 128, 10000.0, 0)
G4 = cf_inputs.BlockShape("gqa4", 1024, 8, 2, 128, 500000.0, 0)
G8 = cf_inputs.BlockShape("gqa8", 1024, 8, 1, 128, 10000.0, 0)


@pytest.mark.parametrize("shape,norm,residual,packed,batch,n_layers,pos", [
    (S64, True, 1, True, 2, 4, 150), (S64, False, 0, False, 1, 4, 150), (S64, True, 1, False, 4, 4, 150),
    (S64, False, 1, True, 1, 4, 150),
    (M128, False, 0, True, 1, 5, 150), (M128, False, 0, False, 3, 4, 97), (M128, False, 0, True, 9, 3, 150),
    (G2, False, 0, True, 1, 4, 300), (G2, False, 0, False, 4, 3, 31), (G4, False, 0, True, 1, 4, 333),
    (G4, False, 0, True, 2, 3, 0), (G4, False, 0, False, 16, 3, 70), (G8, False, 0, True, 1, 4, 257),
    (G8, False, 0, True, 4, 3, 64), (M128, False, 0, True, 1, 1, 150)],
    ids=lambda v: getattr(v, "name", None))
def test_stack_matches_single_calls_and_oracle(shape, norm, residual, packed, batch, n_layers, pos):
    from paper_2508_18850_amd import DecodeBlock
    eps = 1e-5
    _log("stack %s norm=%s residual=%d packed=%s batch=%d layers=%d pos=%d" % (shape.name, norm, residual, packed, batch,
                                                                            n_layers, pos))
    layers, gammas = make_layers(shape, n_layers, batch, pos, seed=300)
    if not norm:
        gammas = None
    dev = torch.device("cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    blk = DecodeBlock(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, batch, layers[0]["max_seq"],
                      shape.rope_base)

    def upload():
        t = []
        for l, inp in enumerate(layers):
            d = {k: torch.from_numpy(inp[k]).to(dev) for k in ("w_qkv", "w_o", "k_cache", "v_cache")}
            d["g"] = torch.from_numpy(gammas[l]).to(dev) if norm else None
            if packed:
                nq, no = blk.packed_sizes()
                wq = torch.empty((nq // 2,), dtype=torch.float16, device=dev)
                wo = torch.empty((no // 2,), dtype=torch.float16, device=dev)
                blk.pack_weights(d["w_qkv"].data_ptr(), d["w_o"].data_ptr(), wq.data_ptr(), wo.data_ptr(), st)
                d["w_qkv"], d["w_o"] = wq, wo
            t.append(d)
        return t

    x = torch.from_numpy(layers[0]["x"]).to(dev)
    # the stack in one call
    a = upload()
    out_a = torch.full((batch, shape.d_model), float("nan"), dtype=torch.float16, device=dev)
    blk.decode_stack(batch, x.data_ptr(), [d["g"].data_ptr() for d in a] if norm else None, eps, residual, packed,
                     [d["w_qkv"].data_ptr() for d in a], [d["w_o"].data_ptr() for d in a],
                     [d["k_cache"].data_ptr() for d in a], [d["v_cache"].data_ptr() for d in a], pos, out_a.data_ptr(), st)
    blk.status(st)
    # the same layers one by one
    b = upload()
    bufs = [torch.empty_like(out_a) for _ in range(n_layers)]
    cur = x
    for l, d in enumerate(b):
        dst = bufs[l]
        blk.decode_layer(batch, cur.data_ptr(), d["g"].data_ptr() if norm else 0, eps, residual, packed, d["w_qkv"].data_ptr(),
                         d["w_o"].data_ptr(), d["k_cache"].data_ptr(), d["v_cache"].data_ptr(), pos, dst.data_ptr(), st)
        cur = dst
    blk.status(st)
    got = out_a.cpu().numpy()
    assert np.array_equal(got.view(np.uint16), cur.cpu().numpy().view(np.uint16))
    for da, db in zip(a, b):
        for c in ("k_cache", "v_cache"):
            assert np.array_equal(da[c].cpu().numpy().view(np.uint16), db[c].cpu().numpy().view(np.uint16))
    assert np.array_equal(x.cpu().numpy().view(np.uint16), layers[0]["x"].view(np.uint16)), "x was modified"
    # the oracle, every layer from the hidden state the GPU gave it (the stack's own hidden states are those of the
    # single calls: the results are bit-identical, layer by layer by induction)
    hidden = [layers[0]["x"]] + [t.cpu().numpy() for t in bufs]
    caches = [(d["k_cache"].cpu().numpy(), d["v_cache"].cpu().numpy()) for d in a]
    check_layers(shape, layers, gammas, eps, residual, pos, hidden, caches)
    blk.close()


def test_more_layers_than_one_launch_holds():
    """95 layers of a small head_dim-128 block: two launches (88 + 7), chained through the library's buffers; against the
    same layers one by one (bit-identical) and, for three of the layers, against the oracle."""
    from paper_2508_18850_amd import DecodeBlock
    shape = cf_inputs.BlockShape("deep", 256, 2, 2, 128, 10000.0, 0)
    n_layers, pos, batch = 95, 21, 1
    base = cf_inputs.make_inputs(shape, seed=900, batch=batch, kv_len=pos)
    rng = np.random.Generator(np.random.PCG64(901))
    dev = torch.device("cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    blk = DecodeBlock(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, batch, base["max_seq"], shape.rope_base)
    # the output projection scaled so that the hidden state keeps its size through 95 blocks without a residual path
    host = []
    for l in range(n_layers):
        host.append({"w_qkv": (rng.standard_normal(base["w_qkv"].shape, dtype=np.float32) * 0.02).astype(np.float16),
                     "w_o": (rng.standard_normal(base["w_o"].shape, dtype=np.float32) * 0.06).astype(np.float16),
                     "k_cache": base["k_cache"].copy(), "v_cache": base["v_cache"].copy()})

    def upload():
        return [{k: torch.from_numpy(v).to(dev) for k, v in h.items()} for h in host]

    x = torch.from_numpy(base["x"]).to(dev)
    a = upload()
    out_a = torch.full((batch, shape.d_model), float("nan"), dtype=torch.float16, device=dev)
    blk.decode_stack(batch, x.data_ptr(), None, 0.0, 0, 0, [d["w_qkv"].data_ptr() for d in a], [d["w_o"].data_ptr() for d in a],
                     [d["k_cache"].data_ptr() for d in a], [d["v_cache"].data_ptr() for d in a], pos, out_a.data_ptr(), st)
    blk.status(st)
    b = upload()
    bufs = [torch.empty_like(out_a) for _ in range(n_layers)]
    cur = x
    for l, d in enumerate(b):
        blk.decode_block(batch, cur.data_ptr(), d["w_qkv"].data_ptr(), d["w_o"].data_ptr(), d["k_cache"].data_ptr(),
                         d["v_cache"].data_ptr(), pos, bufs[l].data_ptr(), st)
        cur = bufs[l]
    blk.status(st)
    assert np.array_equal(out_a.cpu().numpy().view(np.uint16), cur.cpu().numpy().view(np.uint16))
    for da, db in zip(a, b):
        for c in ("k_cache", "v_cache"):
            assert np.array_equal(da[c].cpu().numpy().view(np.uint16), db[c].cpu().numpy().view(np.uint16))
    hidden = [base["x"]] + [t.cpu().numpy() for t in bufs]
    assert np.isfinite(hidden[-1]).all() and np.abs(hidden[-1].astype(np.float64)).max() > 1e-3, "the hidden state died out"
    for l in (0, 87, 94):
        ref = orc.decode_block(hidden[l], host[l]["w_qkv"], host[l]["w_o"], host[l]["k_cache"], host[l]["v_cache"], pos,
                               shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_base)["out"]
        err = np.abs(hidden[l + 1].astype(np.float64) - ref).max()
        assert err <= 1e-2 * np.abs(ref).max() + 1e-3, (l, err)
    blk.close()


def test_bad_arguments_enqueue_nothing():
    from paper_2508_18850_amd import DecodeBlock
    shape = cf_inputs.SHAPES["tiny"]
    inp = cf_inputs.make_inputs(shape, seed=1, batch=1, kv_len=20)
    dev = torch.device("cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    blk = DecodeBlock(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, 1, inp["max_seq"], shape.rope_base)
    t = {k: torch.from_numpy(inp[k]).to(dev) for k in ("x", "w_qkv", "w_o", "k_cache", "v_cache")}
    out = torch.zeros((1, shape.d_model), dtype=torch.float16, device=dev)
    p = {k: v.data_ptr() for k, v in t.items()}
    two = lambda k: [p[k], p[k]]
    args = lambda **kw: dict(dict(batch=1, x=p["x"], norm_weights=None, eps=0.0, residual=0, packed=0, w_qkv=two("w_qkv"),
                                  w_o=two("w_o"), k_cache=two("k_cache"), v_cache=two("v_cache"), pos=20,
                                  out=out.data_ptr(), stream=st), **kw)
    assert blk.decode_stack_rc(**args(out=p["x"])) == -1                      # x and out are the same buffer
    assert blk.decode_stack_rc(**args(w_o=[p["w_o"], 0])) == -1               # null pointer in the second layer
    assert blk.decode_stack_rc(**args(k_cache=[p["k_cache"], p["k_cache"] + 2])) == -1     # misaligned
    assert blk.decode_stack_rc(**args(pos=inp["max_seq"])) == -1
    blk.status(st)
    for c in ("k_cache", "v_cache"):                                          # nothing ran: the caches are untouched
        assert np.array_equal(t[c].cpu().numpy().view(np.uint16), inp[c].view(np.uint16))
    assert blk.decode_stack_rc(**args()) == 0
    blk.status(st)
    assert torch.isfinite(out.float()).all()
    blk.close()


def test_full_size_stack_of_two_layers():
    """Llama-2-7B shape, 4096 cached tokens, RMSNorm and residual, packed weights: two layers in one call against the
    C oracle applied layer by layer."""
    from oracle import c_oracle
    from paper_2508_18850_amd import DecodeBlock
    shape = cf_inputs.SHAPES["llama2_7b"]
    n_layers, pos, eps, batch = 2, 4096, 1e-5, 1
    _log("full-size stack")
    layers, gammas = make_layers(shape, n_layers, batch, pos, seed=7000)
    dev = torch.device("cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    blk = DecodeBlock(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, batch, layers[0]["max_seq"],
                      shape.rope_base)
    dv = []
    for l, inp in enumerate(layers):
        d = {k: torch.from_numpy(inp[k]).to(dev) for k in ("w_qkv", "w_o", "k_cache", "v_cache")}
        nq, no = blk.packed_sizes()
        wq = torch.empty((nq // 2,), dtype=torch.float16, device=dev)
        wo = torch.empty((no // 2,), dtype=torch.float16, device=dev)
        blk.pack_weights(d["w_qkv"].data_ptr(), d["w_o"].data_ptr(), wq.data_ptr(), wo.data_ptr(), st)
        d["w_qkv"], d["w_o"], d["g"] = wq, wo, torch.from_numpy(gammas[l]).to(dev)
        dv.append(d)
    x = torch.from_numpy(layers[0]["x"]).to(dev)
    out = torch.full((batch, shape.d_model), float("nan"), dtype=torch.float16, device=dev)
    blk.decode_stack(batch, x.data_ptr(), [d["g"].data_ptr() for d in dv], eps, 1, 1, [d["w_qkv"].data_ptr() for d in dv],
                     [d["w_o"].data_ptr() for d in dv], [d["k_cache"].data_ptr() for d in dv],
                     [d["v_cache"].data_ptr() for d in dv], pos, out.data_ptr(), st)
    blk.status(st)
    got = out.cpu().numpy().astype(np.float64)
    # the hidden state between the two layers as the GPU had it: the first layer alone (bit-identical to the stack's)
    mid = torch.full((batch, shape.d_model), float("nan"), dtype=torch.float16, device=dev)
    kc0 = torch.from_numpy(layers[0]["k_cache"]).to(dev)
    vc0 = torch.from_numpy(layers[0]["v_cache"]).to(dev)
    blk.decode_layer(batch, x.data_ptr(), dv[0]["g"].data_ptr(), eps, 1, 1, dv[0]["w_qkv"].data_ptr(), dv[0]["w_o"].data_ptr(),
                     kc0.data_ptr(), vc0.data_ptr(), pos, mid.data_ptr(), st)
    blk.status(st)
    blk.close()
    hidden = [layers[0]["x"], mid.cpu().numpy(), out.cpu().numpy()]
    for l, inp in enumerate(layers):
        ref = c_oracle.decode_layer(hidden[l], gammas[l], eps, inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], pos,
                                    shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_base)["out"]
        err = np.abs(hidden[l + 1].astype(np.float64) - ref).max()
        tol = 1e-2 * np.abs(ref).max() + 1e-3
        _log("full-size stack, layer %d: max|err| %.3e tol %.3e max|ref| %.3e" % (l, err, tol, np.abs(ref).max()))
        assert np.isfinite(got).all() and err <= tol


def test_full_size_bare_stack_in_one_launch():
    """Llama-2-7B shape, 4096 cached tokens, the bare block, packed weights: three layers in one launch, bit-identical to
    the same layers enqueued one by one, every layer against the C oracle from the hidden state the GPU gave it."""
    from oracle import c_oracle
    from paper_2508_18850_amd import DecodeBlock
    shape = cf_inputs.SHAPES["llama2_7b"]
    n_layers, pos, batch = 3, 4096, 1
    _log("full-size bare stack")
    layers, _ = make_layers(shape, n_layers, batch, pos, seed=7100)
    for inp in layers[1:]:                      # (no residual path: keep the hidden state at the size of an input)
        inp["w_o"] = (inp["w_o"].astype(np.float32) * 16.0).astype(np.float16)
    layers[0]["w_o"] = (layers[0]["w_o"].astype(np.float32) * 16.0).astype(np.float16)
    dev = torch.device("cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    blk = DecodeBlock(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, batch, layers[0]["max_seq"],
                      shape.rope_base)

    def upload():
        dv = []
        for inp in layers:
            d = {k: torch.from_numpy(inp[k]).to(dev) for k in ("w_qkv", "w_o", "k_cache", "v_cache")}
            nq, no = blk.packed_sizes()
            wq = torch.empty((nq // 2,), dtype=torch.float16, device=dev)
            wo = torch.empty((no // 2,), dtype=torch.float16, device=dev)
            blk.pack_weights(d["w_qkv"].data_ptr(), d["w_o"].data_ptr(), wq.data_ptr(), wo.data_ptr(), st)
            d["w_qkv"], d["w_o"] = wq, wo
            dv.append(d)
        return dv

    x = torch.from_numpy(layers[0]["x"]).to(dev)
    a = upload()
    out = torch.full((batch, shape.d_model), float("nan"), dtype=torch.float16, device=dev)
    blk.decode_stack(batch, x.data_ptr(), None, 0.0, 0, 1, [d["w_qkv"].data_ptr() for d in a], [d["w_o"].data_ptr() for d in a],
                     [d["k_cache"].data_ptr() for d in a], [d["v_cache"].data_ptr() for d in a], pos, out.data_ptr(), st)
    blk.status(st)
    b = upload()
    bufs = [torch.empty_like(out) for _ in range(n_layers)]
    cur = x
    for l, d in enumerate(b):
        blk.decode_block_packed(batch, cur.data_ptr(), d["w_qkv"].data_ptr(), d["w_o"].data_ptr(), d["k_cache"].data_ptr(),
                                d["v_cache"].data_ptr(), pos, bufs[l].data_ptr(), st)
        cur = bufs[l]
    blk.status(st)
    assert np.array_equal(out.cpu().numpy().view(np.uint16), cur.cpu().numpy().view(np.uint16))
    for da, db in zip(a, b):
        for c in ("k_cache", "v_cache"):
            assert torch.equal(da[c].view(torch.int16), db[c].view(torch.int16))
    blk.close()
    hidden = [layers[0]["x"]] + [t.cpu().numpy() for t in bufs]
    for l, inp in enumerate(layers):
        ref = c_oracle.decode_block(hidden[l], inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], pos,
                                    shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_base)["out"]
        err = np.abs(hidden[l + 1].astype(np.float64) - ref).max()
        tol = 1e-2 * np.abs(ref).max() + 1e-3
        _log("full-size bare stack, layer %d: max|err| %.3e tol %.3e max|ref| %.3e" % (l, err, tol, np.abs(ref).max()))
        assert np.isfinite(hidden[l + 1]).all() and err <= tol
