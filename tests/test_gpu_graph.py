"""The decode call under HIP graph capture: a stack of layers captured once and replayed.

cf_decode_block allocates nothing, synchronises nothing and keeps its launch counter on the device (every workgroup
counts its own launches), so a captured launch stays valid on every replay.  The test replays a graph of several
layers three times, with eager work and synchronisation between the replays, and compares every replay with the eager
result (bit-identical: same kernel, same plan, same inputs).
"""
import numpy as np
import pytest

import cf_inputs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def test_captured_stack_replays_like_eager_launches():
    from paper_2508_18850_amd import DecodeBlock
    shape, batch, kv_len, n_layers = cf_inputs.BlockShape("s", 1024, 16, 4, 128, 10000.0, 300), 2, 300, 3
    dev = torch.device("cuda:0")
    blk = DecodeBlock(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, batch,
                      cf_inputs.default_max_seq(kv_len), shape.rope_base)
    layers = []
    for i in range(n_layers):
        inp = cf_inputs.make_inputs(shape, seed=50 + i, batch=batch, kv_len=kv_len, poison=False)
        layers.append({k: torch.from_numpy(inp[k]).to(dev) for k in ("w_qkv", "w_o", "k_cache", "v_cache")})
    x = torch.from_numpy(cf_inputs.make_inputs(shape, seed=49, batch=batch, kv_len=kv_len)["x"]).to(dev)
    bufs = [torch.empty_like(x) for _ in range(2)]

    def stack(stream):
        # layer i reads the previous layer's output (ping-pong buffers) and appends to its own cache
        src = x
        for i, lay in enumerate(layers):
            dst = bufs[i % 2]
            blk.decode_block(batch, src.data_ptr(), lay["w_qkv"].data_ptr(), lay["w_o"].data_ptr(),
                             lay["k_cache"].data_ptr(), lay["v_cache"].data_ptr(), kv_len, dst.data_ptr(), stream)
            src = dst
        return src

    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        eager = stack(s.cuda_stream).clone()
        blk.status(s.cuda_stream)
        appended = [lay["k_cache"][:, :, kv_len].clone() for lay in layers]
    torch.cuda.synchronize()
    assert torch.isfinite(eager.float()).all()

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        out = stack(torch.cuda.current_stream().cuda_stream)
    for rep in range(3):
        out.fill_(float("nan"))
        for lay in layers:
            lay["k_cache"][:, :, kv_len].zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        blk.status(0)
        assert torch.equal(out, eager), "replay %d differs from the eager launches" % rep
        for lay, want in zip(layers, appended):
            assert torch.equal(lay["k_cache"][:, :, kv_len], want)
        # eager work between the replays (an eager launch moves the launch counters on as well)
        again = stack(torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert torch.equal(again, eager)
    blk.close()
