"""cf_decode_stack through the C ABI: a stack of layers in one call, the hidden state handed from layer to layer.

Checks: (1) the result and every appended cache row are bit-identical to the same layers enqueued one by one with
cf_decode_layer (the stack is the same launches with the library's buffers in between); (2) the result matches the
oracle applied layer by layer, each layer's input being the fp16 rounding of the previous oracle output, within the
block tolerance (max|err| <= 1e-2 * max|ref| + 1e-3) widened by the number of layers, since each layer starts from a
slightly different fp16 input; (3) bad arguments are refused before anything is enqueued.
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


def oracle_chain(shape, layers, gammas, eps, residual, pos):
    x = layers[0]["x"]
    rows = []
    for l, inp in enumerate(layers):
        args = (inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], pos, shape.n_q_heads, shape.n_kv_heads,
                shape.head_dim, shape.rope_base)
        if gammas is None:
            ref = orc.decode_block(x, *args)
            if residual:
                ref["out"] = ref["out"] + x.astype(np.float64)
        else:
            ref = orc.decode_layer(x, gammas[l], eps, *args)
            if not residual:
                ref["out"] = ref["out"] - x.astype(np.float64)
        rows.append((ref["k_rot"], ref["v_new"]))
        out = ref["out"]
        x = out.astype(np.float16)
    return out, rows


@pytest.mark.parametrize("norm,residual,packed,batch", [(True, 1, True, 2), (False, 0, False, 1), (True, 1, False, 4),
                                                         (False, 1, True, 1)])
def test_stack_matches_single_calls_and_oracle(norm, residual, packed, batch):
    from paper_2508_18850_amd import DecodeBlock
    shape = cf_inputs.BlockShape("s", 512, 8, 4, 64, 10000.0, 0)
    n_layers, pos, eps = 4, 150, 1e-5
    _log("stack norm=%s residual=%d packed=%s batch=%d" % (norm, residual, packed, batch))
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
    bufs = [torch.empty_like(out_a) for _ in range(2)]
    cur = x
    for l, d in enumerate(b):
        dst = bufs[l & 1]
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
    # the oracle, layer by layer
    ref, rows = oracle_chain(shape, layers, gammas, eps, residual, pos)
    err = np.abs(got.astype(np.float64) - ref).max()
    tol = n_layers * (1e-2 * np.abs(ref).max() + 1e-3)
    _log("stack: max|err| %.3e tol %.3e max|ref| %.3e" % (err, tol, np.abs(ref).max()))
    assert np.isfinite(got).all() and err <= tol
    # first layer's appended rows: its input is exact, so the single-layer bound holds
    k0 = a[0]["k_cache"].cpu().numpy()[:, :, pos, :].astype(np.float64)
    assert (np.abs(k0 - rows[0][0]) <= np.abs(rows[0][0]) * 2.0 ** -10 + 2e-5).all()
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
    blk.close()
    cur = layers[0]["x"]
    for l, inp in enumerate(layers):
        ref = c_oracle.decode_layer(cur, gammas[l], eps, inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], pos,
                                    shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_base)["out"]
        cur = ref.astype(np.float16)
    err = np.abs(got - ref).max()
    tol = n_layers * (1e-2 * np.abs(ref).max() + 1e-3)
    _log("full-size stack: max|err| %.3e tol %.3e max|ref| %.3e" % (err, tol, np.abs(ref).max()))
    assert np.isfinite(got).all() and err <= tol
