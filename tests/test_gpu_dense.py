"""GPU parity of the dense neighbours of the layer (paged linear map, residual + RMS norm, cast) against
oracle/dense.py, through the C ABI, and of the two task calls against the sequence of their stages."""
import numpy as np
import pytest
import torch

import paper_2411_11217_amd as M
from moe_workloads import MoEConfig, scaled
from oracle import dense
from util import Case, assert_close, assert_h_close, say, shape_of, assert_status_clean

pytestmark = pytest.mark.gpu


def bits(t: torch.Tensor) -> np.ndarray:
    return t.cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def paged_linear(ls, W, extra=3, seed=0):
    """Pages of one dense matrix at shuffled slots of a pool of its own; -> (table_dev, pool_dev)."""
    n = M.linear_pages_required(ls)
    slots = torch.randperm(n + extra, generator=torch.Generator().manual_seed(seed))[:n].to(torch.int32)
    pool = torch.zeros((n + extra, ls.page_bytes), dtype=torch.uint8)
    M.linear_pack(ls, W, slots, pool)
    return slots.cuda(), pool.cuda()


@pytest.mark.parametrize("T,K,N,page", [
    (300, 256, 384, 3 * 16384),        # ragged rows, odd number of 128-wide column tiles, tiles not dividing pages evenly
    (64, 128, 128, 16384),             # smallest shape: one column tile, 4 half-steps
    (270, 256, 256, 16384),            # one tall row tile: the 14 rows behind the first 256 ride along
    (800, 512, 384, 2 * 16384),        # three full row tiles, the last one with 32 more rows
    (1000, 1024, 2048, 1 << 20),       # several row and column tiles
    (4096, 4096, 4096, 2 << 20),       # the O projection of the Mixtral-8x7B shape: 256-wide column tiles
])
def test_linear_matches_the_oracle(T, K, N, page):
    g = torch.Generator().manual_seed(T + K)
    x = torch.randn((T, K), generator=g).to(torch.bfloat16)
    W = (torch.randn((N, K), generator=g) * 0.02).to(torch.bfloat16)
    ls = M.make_linear_shape(T, K, N, page)
    table, pool = paged_linear(ls, W)
    status = torch.zeros(4, dtype=torch.int32, device="cuda")
    out = M.moe_linear(ls, x.cuda(), table, pool, status=status)
    torch.cuda.synchronize()
    assert_status_clean(status.cpu().tolist())
    rows = np.arange(T) if T * K * N < 2e9 else np.unique(np.r_[0, T - 1, 255, 256, np.random.default_rng(0).integers(0, T, 60)])
    ref = dense.linear(bits(x)[rows], bits(W))
    assert_close(out.cpu().numpy()[rows], ref, "bf16", f"linear {T}x{K}x{N}")


def test_linear_empty_and_errors():
    ls = M.make_linear_shape(0, 128, 128, 16384)
    lib = M.binding._lib()
    import ctypes
    assert lib.moe_linear(ctypes.byref(ls), None, None, None, 0, None, None, 0, None, None) == 0          # T == 0: nothing to do
    bad = M.make_linear_shape(8, 100, 128, 16384)
    assert lib.moe_linear(ctypes.byref(bad), None, None, None, 0, None, None, 0, None, None) == M.binding.ERR_INVALID_ARG
    ok = M.make_linear_shape(8, 128, 128, 16384)
    fake = ctypes.c_void_p(256)
    assert lib.moe_linear(ctypes.byref(ok), fake, fake, fake, 1, fake, fake, 4, None, None) == M.binding.ERR_WORKSPACE_TOO_SMALL


@pytest.mark.parametrize("T,H,with_hidden", [(37, 256, True), (5, 8192, True), (64, 4096, False), (3, 4, True)])
def test_add_rmsnorm_matches_the_oracle(T, H, with_hidden):
    g = torch.Generator().manual_seed(H)
    hidden = torch.randn((T, H), generator=g) * 3.0 if with_hidden else None
    delta = torch.randn((T, H), generator=g)
    gamma = 1.0 + 0.1 * torch.randn((H,), generator=g)
    eps = 1e-5
    hs, x = M.moe_add_rmsnorm(None if hidden is None else hidden.cuda(), delta.cuda(), gamma.cuda(), eps)
    torch.cuda.synchronize()
    s_ref, x_ref = dense.add_rmsnorm(None if hidden is None else hidden.numpy(), delta.numpy(), gamma.numpy(), eps)
    assert_close(hs.cpu().numpy(), s_ref, "f32", "residual stream")
    assert_h_close(x.float().cpu().numpy(), dense.bf16_bits_to_f64(x_ref), "bf16", "normalised rows")
    _, x2 = M.moe_add_rmsnorm(None if hidden is None else hidden.cuda(), delta.cuda(), gamma.cuda(), eps, want_hidden=False)
    assert torch.equal(x, x2)


def test_cast_is_round_to_nearest_even_bit_exact():
    g = torch.Generator().manual_seed(9)
    v = torch.randn((1 << 16,), generator=g) * 10.0
    v[:6] = torch.tensor([0.0, -0.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, float("inf"), 3.3895e38])
    got = M.moe_cast_bf16(v.cuda())
    torch.cuda.synchronize()
    want = dense.f64_to_bf16_bits(v.double().numpy())          # float32 values are exact in float64: one rounding
    assert np.array_equal(bits(got), want)
    assert np.array_equal(bits(got), bits(v.to(torch.bfloat16)))


def test_post_and_pre_attention_tasks_equal_their_stages_and_the_oracle():
    cfg = scaled(MoEConfig("t1", "bf16", T=200, H=256, F=384, E=4, k=2, page_bytes=64 * 1024, seed=31))
    case = Case(cfg)
    s = case.shape
    g = torch.Generator().manual_seed(5)
    Ka, Nq = 384, 640                                                         # attention width, QKV width
    attn = torch.randn((s.T, Ka), generator=g).to(torch.bfloat16)
    hidden = torch.randn((s.T, s.H), generator=g) * 2.0
    Wo = (torch.randn((s.H, Ka), generator=g) * 0.05).to(torch.bfloat16)
    Wqkv = (torch.randn((Nq, s.H), generator=g) * 0.05).to(torch.bfloat16)
    g1 = 1.0 + 0.1 * torch.randn((s.H,), generator=g)
    g2 = 1.0 + 0.1 * torch.randn((s.H,), generator=g)
    eps = 1e-5
    o_shape = M.make_linear_shape(s.T, Ka, s.H, s.page_bytes)
    q_shape = M.make_linear_shape(s.T, s.H, Nq, s.page_bytes)
    # one pool: the experts' pages, then Wo's, then Wqkv's
    n_exp, n_o, n_q = case.pw.pool_pages, M.linear_pages_required(o_shape), M.linear_pages_required(q_shape)
    pool = torch.zeros((n_exp + n_o + n_q, s.page_bytes), dtype=torch.uint8)
    pool[:n_exp] = case.pw.pages_dev.cpu()
    o_table = torch.arange(n_exp, n_exp + n_o, dtype=torch.int32)
    q_table = torch.arange(n_exp + n_o, n_exp + n_o + n_q, dtype=torch.int32)
    M.linear_pack(o_shape, Wo, o_table, pool)
    M.linear_pack(q_shape, Wqkv, q_table, pool)
    pool_d, o_table_d, q_table_d = pool.cuda(), o_table.cuda(), q_table.cuda()

    hidden_mid, x_moe, y, ws = M.moe_post_attention(s, o_shape, attn.cuda(), hidden.cuda(), o_table_d, g1.cuda(), eps,
                                                    case.Wr, case.pw.table_dev, pool_d)
    hidden_out, x_norm, qkv, qkv16 = M.moe_pre_attention(q_shape, hidden_mid, y, g2.cuda(), eps, q_table_d, pool_d)
    torch.cuda.synchronize()
    # the tasks are exactly their stages
    o = M.moe_linear(o_shape, attn.cuda(), o_table_d, pool_d)
    hm2, x2 = M.moe_add_rmsnorm(hidden.cuda(), o, g1.cuda(), eps)
    y2, _ = M.moe_layer(s, x2, case.Wr, case.pw.table_dev, pool_d)
    ho2, xn2 = M.moe_add_rmsnorm(hm2, y2, g2.cuda(), eps)
    q2 = M.moe_linear(q_shape, xn2, q_table_d, pool_d)
    torch.cuda.synchronize()
    for a, b, name in ((hidden_mid, hm2, "hidden_mid"), (x_moe, x2, "x_moe"), (y, y2, "y"), (hidden_out, ho2, "hidden_out"),
                       (x_norm, xn2, "x_norm"), (qkv, q2, "qkv"), (qkv16, M.moe_cast_bf16(q2), "qkv bf16")):
        assert torch.equal(a, b), name
    # and every stage matches the oracle when fed the GPU's upstream result (a rounding flip must not cascade)
    o_ref = dense.linear(bits(attn), bits(Wo))
    assert_close(o.cpu().numpy(), o_ref, "bf16", "O projection")
    s_ref, x_ref = dense.add_rmsnorm(hidden.numpy(), o.cpu().numpy(), g1.numpy(), eps)
    assert_close(hidden_mid.cpu().numpy(), s_ref, "f32", "hidden + o")
    assert_h_close(x_moe.float().cpu().numpy(), dense.bf16_bits_to_f64(x_ref), "bf16", "x_moe")
    import oracle
    v = case.view
    ref = oracle.layer(bits(x_moe), v["Wr"], v["W1"], v["W3"], v["W2"], cfg.k, 1)
    same = (ref["gap_next"] >= 1e-4)
    say(f"    near-tie tokens excluded: {int((~same).sum())}")
    assert_close(y.cpu().numpy()[same], ref["y"][same], "bf16", "MoE layer on the GPU's x_moe")
    s2_ref, xn_ref = dense.add_rmsnorm(hidden_mid.cpu().numpy(), y.cpu().numpy(), g2.numpy(), eps)
    assert_h_close(x_norm.float().cpu().numpy(), dense.bf16_bits_to_f64(xn_ref), "bf16", "x_norm")
    assert_close(qkv.cpu().numpy(), dense.linear(bits(x_norm), bits(Wqkv)), "bf16", "QKV projection")
