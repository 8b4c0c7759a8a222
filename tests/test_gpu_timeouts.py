"""The bounded waits of the kernels, forced from the host: with a wait limit of zero every wait gives up at its first
unsuccessful look (a limit of a microsecond is not enough to be sure: most waits are over by the second look), the
kernel still runs to its end, the status call reports CF_ETIMEOUT and clears the exchange state, and the next call
with the normal limit is correct again.
"""
import numpy as np
import pytest

import cf_inputs
from oracle import decode_block as orc
from oracle import mla_block as morc
from oracle import cluster_collectives as oc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

CF_ETIMEOUT = -5


def test_decode_block_reports_a_timeout_and_recovers():
    from paper_2508_18850_amd import DecodeBlock, CfError
    from oracle import c_oracle
    shape = cf_inputs.SHAPES["llama2_7b"]
    batch, kv_len = 1, shape.kv_len
    inp = cf_inputs.make_inputs(shape, seed=90, batch=batch, kv_len=kv_len, poison=False)
    dev = torch.device("cuda:0")
    blk = DecodeBlock(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, batch, inp["max_seq"], shape.rope_base)
    st = torch.cuda.current_stream().cuda_stream
    t = {k: torch.from_numpy(inp[k]).to(dev) for k in ("x", "w_qkv", "w_o", "k_cache", "v_cache")}
    out = torch.empty((batch, shape.d_model), dtype=torch.float16, device=dev)

    def call():
        blk.decode_block(batch, t["x"].data_ptr(), t["w_qkv"].data_ptr(), t["w_o"].data_ptr(), t["k_cache"].data_ptr(),
                         t["v_cache"].data_ptr(), kv_len, out.data_ptr(), st)

    blk.set_tuning(spin_limit_us=-1)
    call()
    with pytest.raises(CfError) as e:
        blk.status(st)
    assert e.value.code == CF_ETIMEOUT
    blk.set_tuning(spin_limit_us=2000000)
    call()
    blk.status(st)
    ref = c_oracle.decode_block(inp["x"], inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], kv_len,
                                shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_base)["out"]
    err = np.abs(out.cpu().numpy().astype(np.float64) - ref).max()
    assert err <= 1e-2 * np.abs(ref).max() + 1e-3
    blk.close()


def test_team_collectives_report_a_timeout_and_recover():
    from paper_2508_18850_amd import TeamCollectives, TEAM_SUM, TEAM_ROUNDS, CfError
    tc = TeamCollectives(64, 65536)
    host = np.random.Generator(np.random.PCG64(3)).standard_normal((8, 8, 65536)).astype(np.float32)
    src = torch.from_numpy(host).cuda()
    dst = torch.empty_like(src)
    st = torch.cuda.current_stream().cuda_stream
    tc.set_spin_limit(0)
    tc.reduce(8, 8, TEAM_SUM, src.data_ptr(), dst.data_ptr(), 65536, TEAM_ROUNDS, st)
    with pytest.raises(CfError) as e:
        tc.status(st)
    assert e.value.code == CF_ETIMEOUT
    tc.set_spin_limit(2000000)
    tc.reduce(8, 8, TEAM_SUM, src.data_ptr(), dst.data_ptr(), 65536, TEAM_ROUNDS, st)
    tc.status(st)
    want, _ = oc.cluster_reduce([host[0, b] for b in range(8)], "sum")
    tol = 8 * 2.0 ** -24 * np.abs(host[0]).sum(axis=0) + 1e-30
    assert np.all(np.abs(dst[0, 0].cpu().numpy().astype(np.float64) - want[0]) <= tol)
    tc.close()


def test_mla_block_reports_a_timeout_and_recovers():
    from paper_2508_18850_amd import MlaBlock, CfError
    shape = cf_inputs.MlaShape("s", 512, 16, 128, 64, 512, 128, 10000.0, 0)
    inp = cf_inputs.make_mla_inputs(shape, seed=91, batch=1, kv_len=1500, poison=False)
    dev = torch.device("cuda:0")
    blk = MlaBlock(shape.d_model, shape.n_heads, shape.nope_dim, shape.rope_dim, shape.kv_lora_rank, shape.v_head_dim, 1,
                   inp["max_seq"], shape.rope_base)
    st = torch.cuda.current_stream().cuda_stream
    t = {k: torch.from_numpy(inp[k]).to(dev) for k in ("x", "w_q", "w_kv", "w_up", "w_down", "w_o", "kv_cache")}
    out = torch.empty((1, shape.d_model), dtype=torch.float16, device=dev)

    def call():
        blk.decode(1, t["x"].data_ptr(), t["w_q"].data_ptr(), t["w_kv"].data_ptr(), t["w_up"].data_ptr(),
                   t["w_down"].data_ptr(), t["w_o"].data_ptr(), t["kv_cache"].data_ptr(), 1500, out.data_ptr(), st)

    blk.set_spin_limit(0)
    call()
    with pytest.raises(CfError) as e:
        blk.status(st)
    assert e.value.code == CF_ETIMEOUT
    blk.set_spin_limit(2000000)
    call()
    blk.status(st)
    ref = morc.mla_decode_block(inp["x"], inp["w_q"], inp["w_kv"], inp["w_up"], inp["w_down"], inp["w_o"], inp["kv_cache"],
                                1500, shape.n_heads, shape.nope_dim, shape.rope_dim, shape.kv_lora_rank, shape.v_head_dim,
                                shape.rope_base)["out"]
    err = np.abs(out.cpu().numpy().astype(np.float64) - ref).max()
    assert err <= 1e-2 * np.abs(ref).max() + 1e-3
    blk.close()
