"""The layer on the library's own device scratch (moe_layer_static, for callers that cannot allocate):
same result bits as moe_layer with a caller workspace, on two calls in a row, the second with a smaller
input; sizes beyond the scratch array are refused."""
import numpy as np
import pytest
import torch

import paper_2411_11217_amd as M
from moe_workloads import CONFIGS, MoEConfig, scaled
from util import Case, assert_close, say

pytestmark = pytest.mark.gpu


def run_both(case: Case):
    cfg = case.cfg
    y_ref, ws = M.moe_layer(case.shape, case.x, case.Wr, case.pw.table_dev, case.pw.pages_dev, bias=case.bias)
    y = torch.full((cfg.T, cfg.H), float("nan"), dtype=torch.float32, device="cuda")
    before = torch.cuda.memory_allocated()
    M.moe_layer_static(case.shape, case.x, case.Wr, case.pw.table_dev, case.pw.pages_dev, y, bias=case.bias)
    assert torch.cuda.memory_allocated() == before         # nothing went through torch's allocator either
    torch.cuda.synchronize()
    return y, y_ref


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_scratch_layer_equals_workspace_layer_twice(dtype):
    big = MoEConfig("static_a", dtype, T=300, H=512, F=1024, E=8, k=2, page_bytes=128 * 1024, seed=11)
    small = scaled(big, name="static_b", T=77, seed=12)
    assert M.workspace_layout(M.make_shape(big.T, big.H, big.F, big.E, big.k, big.dtype, big.page_bytes)).total <= M.STATIC_SCRATCH_BYTES
    for cfg in (big, small):                               # the second call finds the first call's leftovers in the scratch
        case = Case(cfg)
        y, y_ref = run_both(case)
        assert torch.equal(y, y_ref), cfg.name
        ref = case.oracle_layer()
        got = y.cpu().numpy()
        assert_close(got, ref["y"], cfg.dtype, cfg.name + " y against the oracle")
        say(f"    {cfg.name}: bit-identical to moe_layer")


def test_static_scratch_layer_refuses_sizes_beyond_its_array():
    cfg = scaled(CONFIGS["c2_mixtral8x7b_t256"], T=512)
    s = M.make_shape(cfg.T, cfg.H, cfg.F, cfg.E, cfg.k, cfg.dtype, cfg.page_bytes)
    assert M.workspace_layout(s).total > M.STATIC_SCRATCH_BYTES
    x = torch.zeros((cfg.T, cfg.H), dtype=torch.bfloat16, device="cuda")
    Wr = torch.zeros((cfg.E, cfg.H), dtype=torch.bfloat16, device="cuda")
    gu, d = M.pages_required(s)
    table = torch.zeros((cfg.E, gu + d), dtype=torch.int32, device="cuda")
    pool = torch.zeros((1, cfg.page_bytes), dtype=torch.uint8, device="cuda")
    y = torch.zeros((cfg.T, cfg.H), dtype=torch.float32, device="cuda")
    with pytest.raises(M.MoEError) as ei:
        M.moe_layer_static(s, x, Wr, table, pool, y)
    assert ei.value.status == -3                           # MOE_ERR_WORKSPACE_TOO_SMALL, named in the message
    assert "workspace" in str(ei.value).lower()
