"""GPU parity of cf_decode_layer (RMSNorm in front of the block, residual connection behind it, fused into the
same kernel) against the CPU oracle's decode_layer, through the C ABI.

Tolerance: that of the block (max|err| <= 1e-2 * max|ref| + 1e-3 on the output plus the stage-wise checks of
test_gpu_parity.check).  The mean square of a row is a fp32 sum of D squares (relative error ~1e-7), far
inside the stage-wise bound of 2e-5 on the rotated queries.
"""
import numpy as np
import pytest

import cf_inputs
from oracle import decode_block as orc
from oracle import c_oracle
from test_gpu_parity import check, _log

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def gamma_for(shape, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    return (1.0 + 0.25 * rng.standard_normal(shape.d_model)).astype(np.float16)


def run_layer(shape, batch, inp, pos, gamma, eps, residual, packed):
    from paper_2508_18850_amd import DecodeBlock
    dev = torch.device("cuda:0")
    blk = DecodeBlock(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, batch, inp["max_seq"],
                      shape.rope_base, debug=True)
    st = torch.cuda.current_stream().cuda_stream
    t = {k: torch.from_numpy(inp[k]).to(dev) for k in ("x", "w_qkv", "w_o", "k_cache", "v_cache")}
    g = torch.from_numpy(gamma).to(dev) if gamma is not None else None
    out = torch.full((batch, shape.d_model), float("nan"), dtype=torch.float16, device=dev)
    wq, wo = t["w_qkv"], t["w_o"]
    if packed:
        nq_bytes, no_bytes = blk.packed_sizes()
        wq = torch.empty((nq_bytes // 2,), dtype=torch.float16, device=dev)
        wo = torch.empty((no_bytes // 2,), dtype=torch.float16, device=dev)
        blk.pack_weights(t["w_qkv"].data_ptr(), t["w_o"].data_ptr(), wq.data_ptr(), wo.data_ptr(), st)
    blk.decode_layer(batch, t["x"].data_ptr(), g.data_ptr() if g is not None else 0, eps, residual, packed,
                     wq.data_ptr(), wo.data_ptr(), t["k_cache"].data_ptr(), t["v_cache"].data_ptr(), pos,
                     out.data_ptr(), st)
    blk.status(st)
    res = {"out": out.cpu().numpy(), "k_cache": t["k_cache"].cpu().numpy(), "v_cache": t["v_cache"].cpu().numpy()}
    for what, key in ((0, "q_rot"), (1, "attn")):
        a = np.empty((batch, shape.n_q_heads, shape.head_dim), dtype=np.float32)
        blk.debug_export(what, a, st)
        res[key] = a
    assert np.array_equal(t["x"].cpu().numpy().view(np.uint16), inp["x"].view(np.uint16)), "x was modified"
    blk.close()
    return res


def reference(shape, inp, pos, gamma, eps, residual, use_c=False):
    args = (inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], pos, shape.n_q_heads, shape.n_kv_heads,
            shape.head_dim, shape.rope_base)
    if gamma is None:
        ref = (c_oracle.decode_block if use_c else orc.decode_block)(inp["x"], *args)
        if residual:
            ref["out"] = ref["out"] + inp["x"].astype(np.float64)
        return ref
    ref = (c_oracle.decode_layer if use_c else orc.decode_layer)(inp["x"], gamma, eps, *args)
    if not residual:
        ref["out"] = ref["out"] - inp["x"].astype(np.float64)
    return ref


SHAPES = [
    ("tiny", cf_inputs.SHAPES["tiny"], 1, 256),
    ("ragged_d64_g2_b3", cf_inputs.BlockShape("small", 264, 4, 2, 64, 10000.0, 77), 3, 77),
    ("d128_g4_b4", cf_inputs.BlockShape("s", 1024, 16, 4, 128, 500000.0, 333), 4, 333),
    ("d128_g1_b16", cf_inputs.BlockShape("s", 512, 8, 8, 128, 10000.0, 130), 16, 130),
    ("d128_g8_b5", cf_inputs.BlockShape("s", 2048, 16, 2, 128, 10000.0, 45), 5, 45),
]


@pytest.mark.parametrize("name,shape,batch,kv_len", SHAPES)
@pytest.mark.parametrize("packed", [False, True])
@pytest.mark.parametrize("norm,residual", [(True, True), (True, False), (False, True)])
def test_layer_matches_oracle(name, shape, batch, kv_len, packed, norm, residual):
    _log("layer case %s B=%d L=%d packed=%s norm=%s residual=%s" % (name, batch, kv_len, packed, norm, residual))
    inp = cf_inputs.make_inputs(shape, seed=23, batch=batch, kv_len=kv_len)
    # rows of different scale, so that a wrong or shared normalisation factor shows
    scale = np.array([0.25 * (b + 1) for b in range(batch)], dtype=np.float32)[:, None]
    inp["x"] = (inp["x"].astype(np.float32) * scale).astype(np.float16)
    gamma = gamma_for(shape, 5) if norm else None
    eps = 1e-5
    res = run_layer(shape, batch, inp, kv_len, gamma, eps, residual, packed)
    check(res, reference(shape, inp, kv_len, gamma, eps, residual), inp, kv_len, name)


def test_large_eps_and_zero_row():
    # a zero row normalises to zero (eps keeps the factor finite); a large eps changes the factor visibly
    shape, batch, kv_len = cf_inputs.BlockShape("s", 512, 8, 2, 64, 10000.0, 50), 2, 50
    inp = cf_inputs.make_inputs(shape, seed=3, batch=batch, kv_len=kv_len)
    inp["x"][1] = 0
    gamma = gamma_for(shape, 6)
    for eps in (1e-6, 0.5):
        res = run_layer(shape, batch, inp, kv_len, gamma, eps, True, True)
        check(res, reference(shape, inp, kv_len, gamma, eps, True), inp, kv_len, "eps=%g" % eps)


@pytest.mark.parametrize("workload,batch", [("llama2_7b", 1), ("llama3_8b", 4)])
def test_full_size_layer(workload, batch):
    """The configuration the bench times (packed weights), with normalisation and residual, against the C oracle."""
    shape = cf_inputs.SHAPES[workload]
    _log("full-size layer %s B=%d" % (workload, batch))
    inp = cf_inputs.make_inputs(shape, seed=1000, batch=batch)
    gamma = gamma_for(shape, 7)
    res = run_layer(shape, batch, inp, shape.kv_len, gamma, 1e-5, True, True)
    check(res, reference(shape, inp, shape.kv_len, gamma, 1e-5, True, use_c=True), inp, shape.kv_len, workload)


def test_layer_arguments_are_checked():
    from paper_2508_18850_amd import DecodeBlock
    shape = cf_inputs.SHAPES["tiny"]
    blk = DecodeBlock(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, 1, 64, shape.rope_base)
    a = torch.zeros(1 << 20, dtype=torch.float16, device="cuda")
    p = a.data_ptr()
    assert blk.decode_layer_rc(1, p, p, -1.0, 1, 0, p, p, p, p, 3, p + 4096) == -1            # negative eps
    assert blk.decode_layer_rc(1, p, p, float("nan"), 1, 0, p, p, p, p, 3, p + 4096) == -1    # eps not a number
    assert blk.decode_layer_rc(1, p, p + 2, 1e-5, 1, 0, p, p, p, p, 3, p + 4096) == -1        # misaligned weight
    assert blk.decode_layer_rc(1, p, p, 1e-5, 1, 0, p, p, p, p, 3, p) == -1                   # out == x with residual
    blk.close()


# ---------------------------------------------------------------------------------------------------
# rows with positions of their own (cf_decode_layer_rows)
# ---------------------------------------------------------------------------------------------------

def run_rows(shape, batch, inp, row_pos, max_pos, gamma, eps, residual, packed, kv_splits=0):
    from paper_2508_18850_amd import DecodeBlock
    dev = torch.device("cuda:0")
    blk = DecodeBlock(shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, batch, inp["max_seq"],
                      shape.rope_base, debug=True)
    if kv_splits:
        blk.set_tuning(kv_splits=kv_splits)
    st = torch.cuda.current_stream().cuda_stream
    t = {k: torch.from_numpy(inp[k]).to(dev) for k in ("x", "w_qkv", "w_o", "k_cache", "v_cache")}
    g = torch.from_numpy(gamma).to(dev) if gamma is not None else None
    rp = torch.tensor(list(row_pos), dtype=torch.int32, device=dev)
    out = torch.full((batch, shape.d_model), float("nan"), dtype=torch.float16, device=dev)
    wq, wo = t["w_qkv"], t["w_o"]
    if packed:
        nq_bytes, no_bytes = blk.packed_sizes()
        wq = torch.empty((nq_bytes // 2,), dtype=torch.float16, device=dev)
        wo = torch.empty((no_bytes // 2,), dtype=torch.float16, device=dev)
        blk.pack_weights(t["w_qkv"].data_ptr(), t["w_o"].data_ptr(), wq.data_ptr(), wo.data_ptr(), st)
    blk.decode_layer_rows(batch, t["x"].data_ptr(), g.data_ptr() if g is not None else 0, eps, residual, packed,
                          wq.data_ptr(), wo.data_ptr(), t["k_cache"].data_ptr(), t["v_cache"].data_ptr(),
                          rp.data_ptr(), max_pos, out.data_ptr(), st)
    blk.status(st)
    res = {"out": out.cpu().numpy(), "k_cache": t["k_cache"].cpu().numpy(), "v_cache": t["v_cache"].cpu().numpy()}
    for what, key in ((0, "q_rot"), (1, "attn")):
        a = np.empty((batch, shape.n_q_heads, shape.head_dim), dtype=np.float32)
        blk.debug_export(what, a, st)
        res[key] = a
    plan = blk.plan()
    _log("plan %s" % plan)
    blk.close()
    res["plan"] = plan
    return res


def check_rows(res, ref, inp, row_pos, label):
    """test_gpu_parity.check row by row (each row has its own appended cache row)."""
    for b, pos in enumerate(row_pos):
        one = {k: v[b:b + 1] for k, v in res.items() if k != "plan"}
        refb = {k: v[b:b + 1] for k, v in ref.items()}
        inpb = {k: inp[k][b:b + 1] for k in ("k_cache", "v_cache")}
        check(one, refb, inpb, pos, "%s row %d pos %d" % (label, b, pos))


ROW_CASES = [
    # name, shape, positions of the rows (capacity = max + a few rows)
    ("d64_g2", cf_inputs.BlockShape("small", 264, 4, 2, 64, 10000.0, 77), [77, 0, 5]),
    ("d128_g4", cf_inputs.BlockShape("s", 1024, 16, 4, 128, 500000.0, 333), [1, 333, 332, 100]),
    ("d128_g1_b16", cf_inputs.BlockShape("s", 512, 8, 8, 128, 10000.0, 130),
     [130, 129, 1, 0, 64, 65, 33, 32, 31, 2, 100, 17, 130, 77, 3, 128]),
    ("d128_g8_b2", cf_inputs.BlockShape("s", 2048, 16, 2, 128, 10000.0, 1000), [1000, 250]),
    ("d128_g1_b1", cf_inputs.BlockShape("s", 512, 8, 8, 128, 10000.0, 300), [123]),      # bound above the only row
]


@pytest.mark.parametrize("name,shape,row_pos", ROW_CASES)
@pytest.mark.parametrize("packed", [False, True])
@pytest.mark.parametrize("layer", [True, False])
def test_rows_with_own_positions_match_oracle(name, shape, row_pos, packed, layer):
    batch, max_pos = len(row_pos), shape.kv_len
    _log("rows case %s pos=%s packed=%s layer=%s" % (name, row_pos, packed, layer))
    inp = cf_inputs.make_inputs(shape, seed=31, batch=batch, kv_len=max_pos)
    # cached rows at and beyond a row's own position must never be read: poison them
    for b, pos in enumerate(row_pos):
        inp["k_cache"][b, :, pos:] = np.nan
        inp["v_cache"][b, :, pos:] = np.nan
    gamma = gamma_for(shape, 9) if layer else None
    res = run_rows(shape, batch, inp, row_pos, max_pos, gamma, 1e-5, layer, packed)
    ref = orc.decode_rows(inp["x"], gamma, 1e-5, inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], row_pos,
                          shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_base)
    check_rows(res, ref, inp, row_pos, name)


def test_rows_when_a_workgroup_handles_several_rows():
    """More (row, split) items than workgroups in a team: a workgroup goes from one row to another and has to
    rebuild its RoPE table for the other row's position."""
    shape = cf_inputs.BlockShape("s", 512, 8, 8, 128, 10000.0, 130)
    row_pos = [130, 129, 1, 0, 64, 65, 33, 32, 31, 2, 100, 17, 130, 77, 3, 128]
    inp = cf_inputs.make_inputs(shape, seed=32, batch=16, kv_len=130)
    gamma = gamma_for(shape, 10)
    res = run_rows(shape, 16, inp, row_pos, 130, gamma, 1e-5, True, True, kv_splits=4)
    assert 16 * res["plan"]["kv_splits"] > res["plan"]["team_size"], res["plan"]
    ref = orc.decode_rows(inp["x"], gamma, 1e-5, inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], row_pos,
                          shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_base)
    check_rows(res, ref, inp, row_pos, "several rows per workgroup")


def test_full_size_rows():
    """Llama-3-8B shape, four rows of different lengths (packed weights), against the C oracle row by row."""
    shape = cf_inputs.SHAPES["llama3_8b"]
    row_pos = [shape.kv_len, shape.kv_len // 2 + 3, 17, shape.kv_len - 1]
    inp = cf_inputs.make_inputs(shape, seed=1001, batch=4)
    for b, pos in enumerate(row_pos):
        inp["k_cache"][b, :, pos:] = np.nan
        inp["v_cache"][b, :, pos:] = np.nan
    gamma = gamma_for(shape, 8)
    res = run_rows(shape, 4, inp, row_pos, shape.kv_len, gamma, 1e-5, True, True)
    ref = orc.decode_rows(inp["x"], gamma, 1e-5, inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], row_pos,
                          shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_base,
                          layer_fn=c_oracle.decode_layer, block_fn=c_oracle.decode_block)
    check_rows(res, ref, inp, row_pos, "llama3_8b rows")


def test_row_positions_outside_the_bound_are_clamped():
    # an entry above max_pos is read as max_pos, a negative one as 0: the kernel stays inside its buffers
    shape = cf_inputs.BlockShape("s", 512, 8, 2, 64, 10000.0, 40)
    inp = cf_inputs.make_inputs(shape, seed=4, batch=2, kv_len=40)
    res = run_rows(shape, 2, inp, [10 ** 6, -5], 40, None, 0.0, False, False)
    ref = orc.decode_rows(inp["x"], None, 0.0, inp["w_qkv"], inp["w_o"], inp["k_cache"], inp["v_cache"], [40, 0],
                          shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_base)
    check_rows(res, ref, inp, [40, 0], "clamped")
