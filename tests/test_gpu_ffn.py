"""GPU parity of the fused feed-forward block (cf_ffn_*) against oracle/ffn_block.py, through the C ABI.

Tolerance as for the decode block (fp16 storage, fp32 accumulation): max|err| <= 1e-2 * max|ref| + 1e-3, plus a
relative RMS bound, since the absolute term is loose for small outputs."""
import sys

import numpy as np
import pytest

import cf_inputs
from oracle import ffn_block as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _run(shape, batch, act, seed, max_batch=None, scale_rows=False, calls=1):
    from paper_2508_18850_amd import FfnBlock
    print("ffn case: %s d_model %d d_ff %d batch %d act %d seed %d" % (shape.name, shape.d_model, shape.d_ff, batch, act, seed),
          flush=True)
    sys.stdout.flush()
    dev = torch.device("cuda:0")
    inp = cf_inputs.make_ffn_inputs(shape, seed=seed, batch=batch)
    if scale_rows:      # rows of different scale, so that a row mixed up with another shows
        inp["z"] = (inp["z"].astype(np.float32) * (1.0 + np.arange(batch, dtype=np.float32))[:, None]).astype(np.float16)
    ref = orc.ffn_block(inp["z"], inp["w1"], inp["w2"], inp["w3"], act)["out"]
    t = {k: torch.from_numpy(inp[k]).to(dev) for k in ("z", "w1", "w2", "w3")}
    out = torch.full((batch, shape.d_model), float("nan"), dtype=torch.float16, device=dev)
    blk = FfnBlock(shape.d_model, shape.d_ff, max_batch or batch, act)
    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(calls):
        out.fill_(float("nan"))
        blk.decode(batch, t["z"].data_ptr(), t["w1"].data_ptr(), t["w2"].data_ptr(), t["w3"].data_ptr(), out.data_ptr(), stream)
        blk.status(stream)
    got = out.cpu().numpy().astype(np.float64)
    blk.close()
    assert np.isfinite(got).all()
    err = np.abs(got - ref).max()
    tol = 1e-2 * np.abs(ref).max() + 1e-3
    rel_rms = np.sqrt(((got - ref) ** 2).mean() / (ref ** 2).mean())
    print("   max|err| %.3e (tol %.3e), rel rms %.3e, max|ref| %.3e" % (err, tol, rel_rms, np.abs(ref).max()), flush=True)
    assert err <= tol, (err, tol)
    assert rel_rms < 5e-3, rel_rms


SMALL = [
    cf_inputs.FfnShape("f_a", 512, 1376),          # one piece per row, rows dealt to wavefronts
    cf_inputs.FfnShape("f_b", 1024, 700),          # two pieces per row; uneven rows per workgroup
    cf_inputs.FfnShape("f_c", 1000, 300),          # d_model not a multiple of 512 (ragged last piece)
    cf_inputs.FfnShape("f_d", 4096, 520),          # eight pieces: one per wavefront
    cf_inputs.FfnShape("f_e", 6144, 264),          # twelve pieces, two column blocks per thread
    cf_inputs.FfnShape("f_f", 8192, 256),          # sixteen pieces; one row per workgroup
    cf_inputs.FfnShape("f_g", 256, 100),           # fewer hidden units than compute units
]


@pytest.mark.parametrize("shape", SMALL, ids=[s.name for s in SMALL])
@pytest.mark.parametrize("act", [0, 1])
def test_small_shapes(shape, act):
    _run(shape, 1, act, seed=100 + act)


@pytest.mark.parametrize("batch", [2, 3, 4])
def test_batches(batch):
    """Batch 2 to 4 on the MFMA kernel, except for the last shape, whose 100 workgroups are not a multiple of 16: there
    the vector kernel runs its 2-row and 4-row tiles."""
    _run(SMALL[1], batch, 0, seed=200 + batch, scale_rows=True)
    _run(SMALL[4], batch, 1, seed=210 + batch, scale_rows=True, max_batch=4)
    _run(SMALL[6], batch, 0, seed=215 + batch, scale_rows=True, max_batch=4)


@pytest.mark.parametrize("shape", SMALL[:6], ids=[s.name for s in SMALL[:6]])
@pytest.mark.parametrize("batch", [5, 16])
def test_tile_kernel_small_shapes(shape, batch):
    """Batch above 1 runs the MFMA kernel: ragged d_model, one to twelve column pieces, one to four column groups per
    slice, slices of hidden units that end inside a 32-unit step."""
    _run(shape, batch, batch % 2, seed=220 + batch, scale_rows=True)


@pytest.mark.parametrize("batch", [7, 9, 12])
def test_tile_kernel_batches(batch):
    _run(cf_inputs.FfnShape("f_h", 2048, 2500), batch, 0, seed=230 + batch, scale_rows=True, max_batch=16)


def test_two_calls_in_a_row_and_a_smaller_batch():
    _run(SMALL[0], 2, 0, seed=300, max_batch=4, calls=3)


def test_both_kernels_on_one_handle():
    """A handle for batch 16 runs the MFMA kernel at batch 6 and the vector kernel at batch 1, on the same slots."""
    _run(SMALL[1], 6, 0, seed=310, max_batch=16, calls=2)
    _run(SMALL[1], 1, 0, seed=311, max_batch=16, calls=2)


@pytest.mark.parametrize("name", ["llama2_7b", "llama3_8b", "llama2_70b"])
def test_full_size(name):
    _run(cf_inputs.FFN_SHAPES[name], 1, 0, seed=400)


def test_full_size_batch4():
    _run(cf_inputs.FFN_SHAPES["llama2_7b"], 4, 0, seed=401, scale_rows=True)


@pytest.mark.parametrize("name,batch", [("llama2_7b", 2), ("llama2_7b", 16), ("llama3_8b", 8), ("llama2_70b", 16)])
def test_full_size_tile_kernel(name, batch):
    _run(cf_inputs.FFN_SHAPES[name], batch, 0, seed=402, scale_rows=True)


@pytest.mark.parametrize("batch", [1, 6])
def test_captured_launch_replays(batch):
    """The launch stamp is counted on the device, so a launch recorded once in a HIP graph stays valid on every replay
    (batch 1: the vector kernel, batch 6: the MFMA kernel): three replays, with eager launches and synchronisation
    between them, each bit for bit the eager result (all sums are taken in a fixed order)."""
    from paper_2508_18850_amd import FfnBlock
    dev = torch.device("cuda:0")
    shape = SMALL[1]
    inp = cf_inputs.make_ffn_inputs(shape, seed=600 + batch, batch=batch)
    t = {k: torch.from_numpy(inp[k]).to(dev) for k in ("z", "w1", "w2", "w3")}
    out = torch.full((batch, shape.d_model), float("nan"), dtype=torch.float16, device=dev)
    blk = FfnBlock(shape.d_model, shape.d_ff, batch, 0)
    s = torch.cuda.Stream()

    def launch(stream):
        blk.decode(batch, t["z"].data_ptr(), t["w1"].data_ptr(), t["w2"].data_ptr(), t["w3"].data_ptr(), out.data_ptr(), stream)

    with torch.cuda.stream(s):
        launch(s.cuda_stream)
        blk.status(s.cuda_stream)
    torch.cuda.synchronize()
    eager = out.clone()
    ref = orc.ffn_block(inp["z"], inp["w1"], inp["w2"], inp["w3"], 0)["out"]
    assert np.abs(eager.cpu().numpy().astype(np.float64) - ref).max() <= 1e-2 * np.abs(ref).max() + 1e-3
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        launch(torch.cuda.current_stream().cuda_stream)
    for rep in range(3):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        blk.status(0)
        assert torch.equal(out, eager), "replay %d" % rep
        launch(torch.cuda.current_stream().cuda_stream)          # eager launches move the device-side count on as well
        launch(torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        blk.status(0)
    blk.close()


def test_closed_forms_on_the_gpu():
    """W1 = 0 gives sigma(0) = 0 everywhere: out = 0; z = 0 likewise."""
    from paper_2508_18850_amd import FfnBlock
    dev = torch.device("cuda:0")
    shape = SMALL[1]
    inp = cf_inputs.make_ffn_inputs(shape, seed=500, batch=1)
    stream = torch.cuda.current_stream().cuda_stream
    blk = FfnBlock(shape.d_model, shape.d_ff, 1, 0)
    for zero in ("w1", "z", "w2"):
        t = {k: torch.from_numpy(inp[k]).to(dev) for k in ("z", "w1", "w2", "w3")}
        t[zero].zero_()
        out = torch.full((1, shape.d_model), float("nan"), dtype=torch.float16, device=dev)
        blk.decode(1, t["z"].data_ptr(), t["w1"].data_ptr(), t["w2"].data_ptr(), t["w3"].data_ptr(), out.data_ptr(), stream)
        blk.status(stream)
        assert (out.cpu().numpy() == 0).all(), zero
    blk.close()


def test_refused_arguments():
    from paper_2508_18850_amd import CfError, FfnBlock
    dev = torch.device("cuda:0")
    for args in ((1004, 64, 1, 0), (512, 64, 1, 7), (512, 0, 1, 0)):
        with pytest.raises(CfError) as e:
            FfnBlock(*args)
        assert e.value.code == -1
    for args in ((512, 64, 17, 0), (16384, 64, 1, 0), (512, 100, 5, 0)):
        with pytest.raises(CfError) as e:
            FfnBlock(*args)
        assert e.value.code == -2
    blk = FfnBlock(512, 64, 2, 0)
    buf = torch.zeros((1 << 16,), dtype=torch.float16, device=dev)
    p = buf.data_ptr()
    assert blk.decode_rc(3, p, p, p, p, p, 0) == -1
    assert blk.decode_rc(0, p, p, p, p, p, 0) == -1
    assert blk.decode_rc(1, p + 2, p, p, p, p, 0) == -1
    assert blk.decode_rc(1, p, p, p, 0, p, 0) == -1
    blk.close()
