"""cf_decode_block_static (the entry point for callers that cannot allocate) against cf_decode_block.

Both run the same kernel with the same work plan and fixed-order reductions, so the results must agree bit for bit;
they are also held to the block tolerance against the oracle.  Two calls in a row on the shared scratch array, the
second with a smaller input and another number of workgroups (the launch counters are re-aligned in between), then a
third one back at the first shape.
"""
import sys

import numpy as np
import pytest

import cf_inputs
from oracle import decode_block as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _case(shape, batch, kv_len, seed):
    from paper_2508_18850_amd import CfConfig, DecodeBlock, decode_block_static
    print("static entry point: %s batch %d kv %d seed %d" % (shape.name, batch, kv_len, seed), flush=True)
    sys.stdout.flush()
    dev = torch.device("cuda:0")
    inp = cf_inputs.make_inputs(shape, seed=seed, batch=batch, kv_len=kv_len)
    S = inp["max_seq"]
    stream = torch.cuda.current_stream().cuda_stream
    ref = orc.decode_block(inp["x"], inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], kv_len,
                           shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_base)

    def upload():
        return {k: torch.from_numpy(inp[k]).to(dev) for k in ("x", "w_qkv", "w_o", "k_cache", "v_cache")}

    # the existing entry point
    t = upload()
    out_h = torch.full((batch, shape.d_model), float("nan"), dtype=torch.float16, device=dev)
    blk = DecodeBlock(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, batch, S, shape.rope_base)
    blk.decode_block(batch, t["x"].data_ptr(), t["w_qkv"].data_ptr(), t["w_o"].data_ptr(), t["k_cache"].data_ptr(),
                     t["v_cache"].data_ptr(), kv_len, out_h.data_ptr(), stream)
    blk.status(stream)
    want = {"out": out_h.cpu().numpy(), "k": t["k_cache"].cpu().numpy(), "v": t["v_cache"].cpu().numpy()}
    blk.close()

    # the entry point under test: no handle, nothing allocated by the library
    t = upload()
    out_s = torch.full((batch, shape.d_model), float("nan"), dtype=torch.float16, device=dev)
    cfg = CfConfig(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, batch, S, shape.rope_base, 0)
    decode_block_static(cfg, batch, t["x"].data_ptr(), t["w_qkv"].data_ptr(), t["w_o"].data_ptr(),
                        t["k_cache"].data_ptr(), t["v_cache"].data_ptr(), kv_len, out_s.data_ptr(), stream)
    torch.cuda.synchronize()
    got = {"out": out_s.cpu().numpy(), "k": t["k_cache"].cpu().numpy(), "v": t["v_cache"].cpu().numpy()}

    assert np.array_equal(got["out"].view(np.uint16), want["out"].view(np.uint16)), "out differs from cf_decode_block"
    assert np.array_equal(got["k"].view(np.uint16), want["k"].view(np.uint16)), "k_cache differs from cf_decode_block"
    assert np.array_equal(got["v"].view(np.uint16), want["v"].view(np.uint16)), "v_cache differs from cf_decode_block"
    err = np.abs(got["out"].astype(np.float64) - ref["out"]).max()
    tol = 1e-2 * np.abs(ref["out"]).max() + 1e-3
    assert err <= tol, (err, tol)


def test_static_entry_point_two_calls_then_back():
    big = cf_inputs.BlockShape("static_a", 1024, 8, 8, 128, 10000.0, 300)         # 256 workgroups
    small = cf_inputs.BlockShape("static_b", 384, 6, 6, 64, 10000.0, 37)          # 252 workgroups (6 KV heads)
    _case(big, 2, 300, 11)
    _case(small, 1, 37, 12)
    _case(big, 2, 300, 13)


def test_static_entry_point_refuses_what_does_not_fit():
    from paper_2508_18850_amd import CfConfig, CfError, decode_block_static
    dev = torch.device("cuda:0")
    buf = torch.zeros((1 << 16,), dtype=torch.float16, device=dev)
    p = buf.data_ptr()
    # Llama-2-70B shape at batch 8: 64 heads x 8 rows x 8192 columns of per-head partial outputs alone are 33.5 MB
    cfg = CfConfig(8192, 64, 8, 128, 8, 64, 10000.0, 0)
    with pytest.raises(CfError) as e:
        decode_block_static(cfg, 8, p, p, p, p, p, 8, p, torch.cuda.current_stream().cuda_stream)
    assert e.value.code == -6
    with pytest.raises(CfError) as e:      # bad shape: refused before anything else
        decode_block_static(CfConfig(1000, 8, 8, 100, 1, 64, 10000.0, 0), 1, p, p, p, p, p, 8, p, 0)
    assert e.value.code in (-1, -2)
