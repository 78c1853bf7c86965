"""GPU parity: every stage of the HIP path against the CPU oracle, element by
element, on the same seeded inputs, through the C ABI.  Stage tests feed each
GPU stage the ORACLE's upstream results so that a near tie in the router cannot
cascade; the layer test runs the fused call end to end."""
import numpy as np
import pytest
import torch

import oracle
import paper_2411_11217_amd as M
from moe_workloads import CONFIGS, MoEConfig, scaled
from util import Case, assert_close, assert_h_close, check_permutation_valid, compare_routing, say, shape_of, assert_status_clean

pytestmark = pytest.mark.gpu

C1 = CONFIGS["c1_tiny_f32"]
# reduced bf16 cases: several row tiles of 256 with ragged tails, several column tiles,
# an odd number of 128-wide column tiles in the down projection (H = 384), k in {1,2,4}
MED = {
    "bf16_two_experts_ragged": MoEConfig("m1", "bf16", T=700, H=256, F=384, E=2, k=1, page_bytes=64 * 1024, seed=21),
    "bf16_top2_of_4": MoEConfig("m2", "bf16", T=333, H=384, F=512, E=4, k=2, page_bytes=48 * 1024, seed=22),
    "bf16_top4_of_16": MoEConfig("m3", "bf16", T=200, H=256, F=256, E=16, k=4, page_bytes=32 * 1024, seed=23),
    "f32_top2_of_5": MoEConfig("m4", "f32", T=150, H=128, F=256, E=5, k=2, page_bytes=96 * 1024, seed=24),
    "bf16_skewed": MoEConfig("m5", "bf16", T=600, H=256, F=256, E=8, k=2, page_bytes=64 * 1024, seed=25,
                             bias=((0, 3.0), (7, -3.0))),
}


def _dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def _dev_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def run_stagewise(case: Case):
    cfg, s = case.cfg, case.shape
    ref = case.oracle_layer()
    # ---- a1 route
    ids, w, logits = M.moe_route(s, case.x, case.Wr, bias=case.bias, want_logits=True)
    torch.cuda.synchronize()
    np.testing.assert_allclose(logits.cpu().numpy(), ref["logits"], rtol=0, atol=2e-5 * max(1.0, np.abs(ref["logits"]).max()))
    compare_routing(cfg, ids.cpu().numpy(), w.cpu().numpy(), ref)
    # ---- a2 permute on the oracle's ids: bit exact
    pm = M.moe_permute(s, _dev_i32(ref["ids"]), x=case.x, topk_w=_dev_f32(ref["w"]))
    torch.cuda.synchronize()
    for name in ("counts", "offsets", "row_src", "row_of"):
        assert np.array_equal(pm[name].cpu().numpy(), ref[name]), name
    xp = pm["x_perm"].cpu()
    xp_bits = xp.view(torch.int16).numpy().view(np.uint16) if cfg.dtype == "bf16" else xp.numpy()
    assert np.array_equal(xp_bits, ref["x_perm"]), "x_perm"
    assert np.array_equal(pm["row_w"].cpu().numpy(), ref["w"].astype(np.float32).reshape(-1)[ref["row_src"]])
    # ---- a3 expert FFN on the oracle's permuted rows
    v = case.view
    h_ref, o_ref = oracle.expert_ffn(ref["x_perm"], ref["offsets"], v["W1"], v["W3"], v["W2"], cfg.dtype_code)
    xperm_dev = case.x[torch.from_numpy(ref["row_src"] // cfg.k).long().cuda()].contiguous()
    status = torch.zeros(4, dtype=torch.int32, device="cuda")
    h, out = M.moe_expert_ffn(s, xperm_dev, _dev_i32(ref["offsets"]), case.pw.table_dev, case.pw.pages_dev, status=status)
    torch.cuda.synchronize()
    assert_status_clean(status.cpu().tolist())
    assert_h_close(h.float().cpu().numpy(), h_ref, cfg.dtype, "h")
    assert_close(out.cpu().numpy(), o_ref, cfg.dtype, "expert out")
    # with the gate weight fused into the epilogue
    rw = ref["w"].reshape(-1)[ref["row_src"]]
    _, out_w = M.moe_expert_ffn(s, xperm_dev, _dev_i32(ref["offsets"]), case.pw.table_dev, case.pw.pages_dev,
                                row_w=_dev_f32(rw))
    assert_close(out_w.cpu().numpy(), o_ref * rw[:, None], cfg.dtype, "expert out * w")
    # ---- a4 combine on the oracle's expert outputs
    o_dev = _dev_f32(o_ref)
    y = M.moe_combine(s, o_dev, _dev_i32(ref["row_of"]), topk_w=_dev_f32(ref["w"]))
    y_ref = oracle.combine(o_dev.cpu().numpy().astype(np.float64), ref["row_of"], cfg.k, w=ref["w"].astype(np.float32))
    assert_close(y.cpu().numpy(), y_ref, "f32", "combine")
    y1 = M.moe_combine(s, o_dev, _dev_i32(ref["row_of"]), topk_w=None)
    assert_close(y1.cpu().numpy(), oracle.combine(o_dev.cpu().numpy().astype(np.float64), ref["row_of"], cfg.k), "f32",
                 "combine (unweighted)")
    return ref


def run_layer(case: Case, ref=None):
    cfg, s = case.cfg, case.shape
    ref = ref or case.oracle_layer()
    y, ws = M.moe_layer(s, case.x, case.Wr, case.pw.table_dev, case.pw.pages_dev, bias=case.bias)
    torch.cuda.synchronize()
    assert_status_clean(ws.view("status").cpu().tolist())
    ids = ws.view("topk_ids").cpu().numpy()
    same = compare_routing(cfg, ids, ws.view("topk_w").cpu().numpy(), ref, "layer route")
    pm = {n: ws.view(n).cpu().numpy() for n in ("counts", "offsets", "row_src", "row_of")}
    check_permutation_valid(ids, cfg.E, cfg.k, pm)               # valid for the ids the GPU chose
    if same.all() and (ids == ref["ids"]).all():
        for n in pm:
            assert np.array_equal(pm[n], ref[n]), n
    assert (np.abs(pm["counts"].astype(np.int64) - ref["counts"]).sum()) <= 2 * int((~same).sum())
    assert_close(y.cpu().numpy()[same], ref["y"][same], cfg.dtype, "layer y")
    return y, ws


@pytest.mark.parametrize("down_cols", [0, 1, 2])
def test_expert_ffn_row_counts_across_the_tile_variants(down_cols):
    # (the gate/up launch takes the same choice of column tiles as the down launch: by grid size, narrow, wide)
    """Segments of 1 .. 300 rows, one per expert, on both sides of every threshold of the bf16 kernel's row-tile
    variants (32, 64, 128, 192 rows, the 256-row tile boundary, tiles that take a remainder of up to 32 rows along) and an
    empty one, against the oracle row by row; with the tall tiles switched off every bit stays the same."""
    counts = [1, 16, 17, 32, 33, 0, 64, 65, 127, 128, 129, 160, 192, 193, 255, 256, 257, 300, 31, 449, 272, 273, 288, 289, 532,
              544, 576, 577, 800, 863, 865, 1061]
    E, H, F = len(counts), 256, 384
    cfg = MoEConfig("rows", "bf16", T=sum(counts), H=H, F=F, E=E, k=1, page_bytes=64 * 1024, seed=77)
    case = Case(cfg, shuffle_pages=True, extra_pages=1)
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    v = case.view
    x_bits = v["x"]                                     # [T, H] in the oracle's storage form; k = 1: rows are tokens
    h_ref, o_ref = oracle.expert_ffn(x_bits, offsets, v["W1"], v["W3"], v["W2"], cfg.dtype_code)
    M.set_option("down_cols", down_cols)
    M.set_option("gate_cols", down_cols)
    try:
        status = torch.zeros(4, dtype=torch.int32, device="cuda")
        h, out = M.moe_expert_ffn(case.shape, case.x, _dev_i32(offsets), case.pw.table_dev, case.pw.pages_dev, status=status)
        torch.cuda.synchronize()
    finally:
        M.set_option("down_cols", 0)
        M.set_option("gate_cols", 0)
    assert_status_clean(status.cpu().tolist())
    M.set_option("down_cols", down_cols)
    M.set_option("gate_cols", down_cols)
    M.set_option("tall_tiles", 0)
    try:
        h0, out0 = M.moe_expert_ffn(case.shape, case.x, _dev_i32(offsets), case.pw.table_dev, case.pw.pages_dev, status=status)
        torch.cuda.synchronize()
    finally:
        M.set_option("down_cols", 0)
        M.set_option("gate_cols", 0)
        M.set_option("tall_tiles", 1)
    assert torch.equal(h0, h) and torch.equal(out0, out)
    for e, c in enumerate(counts):
        if c == 0:
            continue
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        assert_h_close(h.float().cpu().numpy()[lo:hi], h_ref[lo:hi], "bf16", f"h, expert {e} with {c} rows")
        assert_close(out.cpu().numpy()[lo:hi], o_ref[lo:hi], "bf16", f"out, expert {e} with {c} rows")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("T,H,E,k", [(1, 128, 1, 1), (17, 128, 3, 3), (100, 384, 16, 4), (33, 1024, 17, 2), (250, 256, 32, 8),
                                     (47, 640, 33, 5), (130, 2048, 64, 64), (2000, 512, 8, 2)])
def test_router_shapes(T, H, E, k, dtype):
    # token counts off the 16-token blocks, fewer 64-element units than wavefronts, every expert-padding bound, a bias
    bias = ((0, 0.5), (E - 1, -0.25)) if E > 1 else ((0, 1.0),)
    cfg = MoEConfig("route", dtype, T=T, H=H, F=128, E=E, k=k, page_bytes=64 * 1024, seed=40 + E, bias=bias)
    case = Case(cfg)
    ref = case.oracle_route()
    ids, w, logits = M.moe_route(case.shape, case.x, case.Wr, bias=case.bias, want_logits=True)
    torch.cuda.synchronize()
    np.testing.assert_allclose(logits.cpu().numpy(), ref["logits"], rtol=0, atol=2e-5 * max(1.0, np.abs(ref["logits"]).max()))
    compare_routing(cfg, ids.cpu().numpy(), w.cpu().numpy(), ref)


@pytest.mark.parametrize("T,E,k", [(1, 1, 1), (1000, 1, 1), (512, 3, 2), (513, 3, 2), (4096, 8, 2), (16384, 64, 1),
                                   (5000, 16, 4), (40000, 64, 2), (131072, 8, 2), (140000, 5, 2)])
def test_permutation_block_counts(T, E, k):
    # one block (no count kernel), up to 256 blocks (each placing block sums the block counts), more (scan kernel)
    rng = np.random.default_rng(T + E)
    skew = rng.random(E) ** 3 + 1e-3                      # some experts rare, some popular
    ids = np.stack([rng.choice(E, size=k, replace=False, p=skew / skew.sum()) for _ in range(T)]).astype(np.int32)
    w = rng.random((T, k), dtype=np.float32)
    ref = oracle.permute(ids, E)
    s = M.MoEShape(T, 128, 128, E, k, M.DTYPE_BF16, 16384)
    pm = M.moe_permute(s, _dev_i32(ids), topk_w=_dev_f32(w))
    torch.cuda.synchronize()
    for name in ("counts", "offsets", "row_src", "row_of"):
        assert np.array_equal(pm[name].cpu().numpy(), ref[name]), name
    assert np.array_equal(pm["row_w"].cpu().numpy(), w.reshape(-1)[ref["row_src"]])


def test_c1_stagewise_and_layer():
    case = Case(C1)
    ref = run_stagewise(case)
    run_layer(case, ref)


@pytest.mark.parametrize("name", list(MED))
@pytest.mark.parametrize("down_cols", [2, 1, 0])
def test_reduced_cases_stagewise_and_layer(name, down_cols):
    # 256- and 128-wide column tiles of the down projection (0: chosen by grid size)
    say(f"  case {name} down_cols {down_cols}")
    M.set_option("down_cols", down_cols)
    try:
        case = Case(MED[name], shuffle_pages=True, extra_pages=3)
        ref = run_stagewise(case)
        run_layer(case, ref)
    finally:
        M.set_option("down_cols", 0)


@pytest.mark.parametrize("name", ["bf16_top2_of_4", "bf16_two_experts_ragged", "f32_top2_of_5"])
@pytest.mark.parametrize("option,default,other", [("xcd_remap", 1, 0), ("fuse_gather", 1, 0), ("half_tiles", 1, 0), ("tall_tiles", 1, 0),
                                                  ("down_cols", 0, 1), ("down_cols", 0, 2), ("chunked", 32, 0), ("chunked", 32, 8),
                                                  ("tall_first", 1, 0), ("balance", 1, 0), ("gate_cols", 0, 1), ("gate_cols", 0, 2)])
def test_kernel_options_give_identical_bits(option, default, other, name):
    # which block computes which tile, the tile variant, and who gathers the rows of x do not change any arithmetic
    case = Case(MED[name])
    y1, _ = M.moe_layer(case.shape, case.x, case.Wr, case.pw.table_dev, case.pw.pages_dev)
    M.set_option(option, other)
    try:
        y0, _ = M.moe_layer(case.shape, case.x, case.Wr, case.pw.table_dev, case.pw.pages_dev)
    finally:
        M.set_option(option, default)
    assert torch.equal(y0, y1)


@pytest.mark.parametrize("seed", range(8))
def test_random_shapes_and_routings_against_the_oracle(seed):
    # seeded random layer shapes with a random router bias (uneven segments of every length up to a few row tiles)
    rng = np.random.default_rng(1000 + seed)
    E = int(rng.integers(1, 13))
    k = int(rng.integers(1, min(E, 4) + 1))
    T = int(rng.integers(1, 1400))
    H = int(rng.choice([128, 256, 384]))
    F = int(rng.choice([128, 256, 640]))
    bias = tuple((e, float(rng.normal(0.0, 0.35))) for e in range(E)) if E > 1 else ()
    cfg = MoEConfig(f"rand{seed}", "bf16", T=T, H=H, F=F, E=E, k=k, page_bytes=int(rng.choice([16384, 49152, 65536])),
                    seed=50 + seed, bias=bias)
    say(f"    T={T} H={H} F={F} E={E} k={k} page={cfg.page_bytes}")
    case = Case(cfg, shuffle_pages=bool(seed & 1), extra_pages=seed % 3)
    y, ws = run_layer(case)
    say(f"    counts: {ws.view('counts').cpu().tolist()}")


def test_page_indirection_is_invisible():
    """Shuffling the physical page slots (table updated with them) leaves every bit of the output unchanged."""
    cfg = MED["bf16_top2_of_4"]
    a = Case(cfg)
    b = Case(cfg, shuffle_pages=True, extra_pages=7, inputs=a.inp)
    ya, _ = M.moe_layer(a.shape, a.x, a.Wr, a.pw.table_dev, a.pw.pages_dev)
    yb, _ = M.moe_layer(b.shape, b.x, b.Wr, b.pw.table_dev, b.pw.pages_dev)
    assert not torch.equal(a.pw.table_dev, b.pw.table_dev)
    assert torch.equal(ya, yb)
    # run-to-run bit identity (no order-dependent atomics anywhere on the path)
    ya2, ws = M.moe_layer(a.shape, a.x, a.Wr, a.pw.table_dev, a.pw.pages_dev)
    assert torch.equal(ya, ya2)


def test_non_resident_page_is_flagged_not_followed():
    cfg = MED["bf16_top2_of_4"]
    case = Case(cfg)
    table = case.pw.table_host.clone()
    table[1, 2] = -1
    with pytest.raises(M.MoEError) as ei:
        M.page_table_validate(case.shape, table, case.pw.pool_pages)
    assert ei.value.status == -4
    # the kernels guard the entry themselves: no fault, status bit set
    y, ws = M.moe_layer(case.shape, case.x, case.Wr, table.cuda(), case.pw.pages_dev)
    torch.cuda.synchronize()
    assert ws.view("status").cpu()[0].item() & 1 == 1
    table[1, 2] = case.pw.pool_pages + 5
    y, ws = M.moe_layer(case.shape, case.x, case.Wr, table.cuda(), case.pw.pages_dev)
    torch.cuda.synchronize()
    assert ws.view("status").cpu()[0].item() & 1 == 1


@pytest.mark.parametrize("kw", [
    dict(T=1), dict(T=5, k=1), dict(T=64, E=4, k=4), dict(T=257, E=1, k=1), dict(T=255, E=3, k=2),
    dict(T=513, E=2, k=2), dict(T=40, E=64, k=8, H=128, F=128),
], ids=lambda kw: "-".join(f"{a}{b}" for a, b in kw.items()))
def test_edge_shapes(kw):
    base = dict(T=64, H=256, F=256, E=8, k=2)
    base.update(kw)
    cfg = MoEConfig("edge", "bf16", page_bytes=64 * 1024, seed=31, **base)
    case = Case(cfg)
    ref = run_stagewise(case)
    run_layer(case, ref)


def test_empty_batch_is_a_noop():
    cfg = MoEConfig("empty", "bf16", T=0, H=128, F=128, E=4, k=2, page_bytes=16384, seed=1)
    s = shape_of(cfg)
    x = torch.empty((0, 128), dtype=torch.bfloat16, device="cuda")
    Wr = torch.zeros((4, 128), dtype=torch.bfloat16, device="cuda")
    ids, w, _ = M.moe_route(s, x, Wr)
    assert ids.shape == (0, 2)
    pm = M.moe_permute(s, ids, x=x, topk_w=w)
    torch.cuda.synchronize()
    assert pm["counts"].cpu().tolist() == [0, 0, 0, 0] and pm["offsets"].cpu().tolist() == [0] * 5


def test_all_tokens_to_one_expert_and_empty_experts():
    cfg = MoEConfig("one", "bf16", T=300, H=256, F=256, E=4, k=1, page_bytes=64 * 1024, seed=33, bias=((2, 50.0),))
    case = Case(cfg)
    ref = run_stagewise(case)
    assert ref["counts"].tolist() == [0, 0, 300, 0]
    run_layer(case, ref)


def test_expert_with_more_row_tiles_than_the_tile_order_cuts_into_row_blocks():
    # 70000 of 70400 rows go to one expert: 273 row tiles, beyond the 256 up to which the tile order cuts an expert into row
    # blocks (it falls back to single column-tile groups there), next to experts with a handful of rows; the XCDs' shares
    # of such a launch differ, so blocks take tiles of other XCDs
    cfg = MoEConfig("tallest", "bf16", T=70400, H=128, F=128, E=4, k=1, page_bytes=16384, seed=35, bias=((1, 0.8),))
    case = Case(cfg)
    ref = run_stagewise(case)
    counts = ref["counts"].tolist()
    assert counts[1] > 256 * 256 and sum(counts) == 70400 and 0 < min(counts) < 2000, counts
    run_layer(case, ref)


def test_identical_experts_and_single_expert_invariants():
    """With identical experts the output does not depend on routing; with one expert the layer is a dense SwiGLU FFN."""
    cfg = MED["bf16_top2_of_4"]
    case = Case(cfg, identical_experts=True)
    y, _ = M.moe_layer(case.shape, case.x, case.Wr, case.pw.table_dev, case.pw.pages_dev)
    Wr2 = torch.randn(case.Wr.shape, generator=torch.Generator().manual_seed(7)).to(torch.bfloat16).cuda()
    y2, ws2 = M.moe_layer(case.shape, case.x, Wr2, case.pw.table_dev, case.pw.pages_dev)
    dense_cfg = scaled(cfg, E=1, k=1)
    inp1 = {k: (v[:1].contiguous() if k in ("W1", "W3", "W2", "Wr") else v) for k, v in case.inp.items()}
    dense = Case(dense_cfg, inputs=inp1)
    yd, _ = M.moe_layer(dense.shape, dense.x, dense.Wr, dense.pw.table_dev, dense.pw.pages_dev)
    ref = dense.oracle_layer()
    assert_close(yd.cpu().numpy(), ref["y"], "bf16", "dense (E=1)")
    assert_close(y.cpu().numpy(), ref["y"], "bf16", "identical experts vs dense")
    assert_close(y2.cpu().numpy(), ref["y"], "bf16", "identical experts, other router")
    w = ws2.view("topk_w").cpu().numpy()
    np.testing.assert_allclose(w.sum(axis=1), 1.0, atol=1e-5)
    assert ws2.view("counts").cpu().numpy().sum() == cfg.T * cfg.k


def test_streamed_pages_match_resident_pages_bitwise():
    cfg = scaled(MED["bf16_top4_of_16"], T=300)
    res = Case(cfg)
    y_res, ws_res = M.moe_layer(res.shape, res.x, res.Wr, res.pw.table_dev, res.pw.pages_dev)
    torch.cuda.synchronize()
    host = M.PagedWeights(res.shape, res.inp["W1"], res.inp["W3"], res.inp["W2"],
                          order=torch.Generator().manual_seed(3), extra_pages=4, pin=True)
    st = M.Streamer(res.shape, host.pages_host, host.table_host)
    try:
        for _ in range(2):          # the second call reuses slots that the first one filled
            y_st, ws_st = M.moe_layer_streamed(st, res.x, res.Wr)
            torch.cuda.synchronize()
            assert_status_clean(ws_st.view("status").cpu().tolist())
            assert torch.equal(y_st, y_res)
        x_perm = res.x[ws_res.view("row_src").long() // cfg.k].contiguous()   # moe_layer gathered inside its GEMM
        h, out = M.moe_expert_ffn_streamed(st, x_perm, ws_res.view("offsets"), row_w=ws_res.view("row_w"))
        torch.cuda.synchronize()
        assert torch.equal(out, ws_res.view("out")) and torch.equal(h, ws_res.view("h"))
    finally:
        st.close()
    ref = res.oracle_layer()
    assert_close(y_res.cpu().numpy(), ref["y"], "bf16", "streamed case vs oracle")


@pytest.mark.parametrize("resident", ["none", "some", "all"])
def test_multi_layer_weight_paging_matches_resident_layers_bitwise(resident):
    """Three layers, four micro-batches, two passes (the second starts with the first layer already
    prefetched): every output equals moe_layer on that layer's resident pages, bit for bit."""
    base = scaled(MED["bf16_top2_of_4"], T=96)
    s = shape_of(base)
    gu, d = M.pages_required(s)
    ppe = gu + d
    n_res = {"none": 0, "some": gu // 2 + 1, "all": ppe}[resident]
    L, n = 3, 4
    cases = [Case(scaled(base, seed=base.seed + 10 * l)) for l in range(L)]
    hosts = [M.PagedWeights(s, c.inp["W1"], c.inp["W3"], c.inp["W2"], order=torch.Generator().manual_seed(40 + l),
                            extra_pages=2, pin=True) for l, c in enumerate(cases)]
    g = torch.Generator().manual_seed(77)
    x_host = [[torch.randn((s.T, s.H), generator=g).to(torch.bfloat16).pin_memory() for _ in range(n)] for _ in range(L)]
    want = [[M.moe_layer(s, x_host[l][j].cuda(), cases[l].Wr, cases[l].pw.table_dev, cases[l].pw.pages_dev)[0]
             for j in range(n)] for l in range(L)]
    torch.cuda.synchronize()
    pipe = M.Pipeline(s, [(h.pages_host, h.table_host) for h in hosts], n_res, max_micro_batches=n)
    try:
        for rep in range(2):
            y = [[torch.zeros((s.T, s.H), dtype=torch.float32, device="cuda") for _ in range(n)] for _ in range(L)]
            ws = pipe.run(x_host, [c.Wr for c in cases], y)
            torch.cuda.synchronize()
            assert_status_clean(ws.view("status").cpu().tolist())
            for l in range(L):
                for j in range(n):
                    assert torch.equal(y[l][j], want[l][j]), (resident, rep, l, j)
    finally:
        pipe.close()
    ref = cases[0].oracle_layer()
    y0, _ = M.moe_layer(s, cases[0].x, cases[0].Wr, cases[0].pw.table_dev, cases[0].pw.pages_dev)
    assert_close(y0.cpu().numpy(), ref["y"], "bf16", "paging case, layer 0 vs oracle")


def test_layer_can_be_captured_in_a_hip_graph_and_replayed():
    """The layer call only launches kernels (status words are cleared by a kernel, not a memset), so it can be
    captured; every replay, with eager work in between, equals the eager result."""
    case = Case(MED["bf16_top2_of_4"])
    s = case.shape
    ws = M.Workspace(s)
    y = torch.empty((s.T, s.H), dtype=torch.float32, device="cuda")
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        M.moe_layer(s, case.x, case.Wr, case.pw.table_dev, case.pw.pages_dev, workspace=ws, y=y, stream=st)
        st.synchronize()
        want = y.clone()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            M.moe_layer(s, case.x, case.Wr, case.pw.table_dev, case.pw.pages_dev, workspace=ws, y=y, stream=st)
        for rep in range(4):
            y.zero_()
            ws.buf.zero_()
            (case.x.float() @ case.x.float().T).sum().item()       # eager work and a synchronisation between replays
            g.replay()
            st.synchronize()
            assert torch.equal(y, want), rep
