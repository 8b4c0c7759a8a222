"""GPU parity at the full sizes of the benchmark configurations, in the launch
configuration bench.py times (default plan).  The whole output is compared with
the oracle; the plain C oracle (pinned against the numpy one) is used where the
numpy one would need many seconds."""
import numpy as np
import pytest

import cf_inputs
from test_gpu_parity import Runner, oracle, check, _log

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def run_case(shape, batch, kv_len, seed, use_c=True, packed=True):
    _log("full-size %s B=%d L=%d packed=%s" % (shape.name, batch, kv_len, packed))
    inp = cf_inputs.make_inputs(shape, seed=seed, batch=batch, kv_len=kv_len)
    r = Runner(shape, batch, inp["max_seq"])
    res = r.run(inp, kv_len, out_fill=float("nan"), packed=packed)
    _log("plan %s" % r.blk.plan())
    ref = oracle(inp, shape, kv_len, use_c=use_c)
    check(res, ref, inp, kv_len, "%s B=%d L=%d" % (shape.name, batch, kv_len))
    r.blk.close()


@pytest.mark.parametrize("packed", [True, False])
def test_llama2_7b_kv4096_numpy_oracle(packed):
    run_case(cf_inputs.SHAPES["llama2_7b"], 1, 4096, seed=1000, use_c=False, packed=packed)


@pytest.mark.parametrize("kv_len", [1024, 2048, 8192, 16384, 32768])
def test_llama2_7b_long_context_sweep(kv_len):
    run_case(cf_inputs.SHAPES["llama2_7b"], 1, kv_len, seed=2000 + kv_len // 1024)


@pytest.mark.parametrize("batch", [1, 4, 16])
def test_llama3_8b_gqa(batch):
    run_case(cf_inputs.SHAPES["llama3_8b"], batch, 8192, seed=3000 + batch)


def test_llama2_70b_gqa_kv32768():
    run_case(cf_inputs.SHAPES["llama2_70b"], 1, 32768, seed=4000)


def test_mha_64_heads_kv4096():
    """64 heads x 128 at d_model 8192: the shape of the team-size sweep that runs at 4 workgroups per head."""
    run_case(cf_inputs.SHAPES["mha_64h"], 1, 4096, seed=5000)
