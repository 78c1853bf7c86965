"""Pins of the CPU oracle against things other than itself.

The paper prints no worked numeric example of an MoE layer, so the pins are
what the definition and the mathematics fix: library routines on special cases
(numpy float64 matmul, scipy softmax, numpy stable sort, torch's bfloat16
conversion), brute force on tiny inputs, closed forms and invariants.  The last
tests plant plausible mistakes into copies of the inputs and check that a pin
notices each of them.
"""
import numpy as np
import pytest
import scipy.special
import torch

import oracle
from moe_workloads import CONFIGS, MoEConfig, make_activations, make_inputs, make_router, bias_vector, oracle_view, scaled


def _views(inp):
    return {k: oracle_view(v) for k, v in inp.items()}


def _f64(t):
    return t.to(torch.float64).numpy()


def _dense_swiglu_f64(x, W1, W3, W2, dtype):
    """Three plain float64 matrix products (numpy) around the SwiGLU product."""
    g = x @ W1.T
    u = x @ W3.T
    h = g / (1.0 + np.exp(-g)) * u
    if dtype == 1:
        h = torch.from_numpy(h).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    else:
        h = h.astype(np.float32).astype(np.float64)
    return h, h @ W2.T


TINY = MoEConfig("tiny", "f32", T=37, H=64, F=96, E=5, k=2, page_bytes=65536, seed=11)
TINY_BF16 = scaled(TINY, dtype="bf16", seed=12)


# ---------------------------------------------------------------- storage type

def test_round_bf16_known_values():
    # spacing of bfloat16 in [1,2) is 2^-7
    assert oracle.round_bf16(1.0) == 1.0
    assert oracle.round_bf16(1 + 2**-8) == 1.0                      # tie -> even mantissa
    assert oracle.round_bf16(1 + 3 * 2**-8) == 1 + 2**-6            # tie -> even mantissa
    assert oracle.round_bf16(1 + 2**-8 + 2**-40) == 1 + 2**-7       # just above the tie (a float32 detour would lose this)
    assert oracle.round_bf16(-(1 + 2**-8 + 2**-40)) == -(1 + 2**-7)
    assert oracle.round_bf16(255.5) == 256.0                        # carries into the next binade
    assert oracle.round_bf16(2.0**-133) == 2.0**-133                # smallest subnormal
    assert oracle.round_bf16(2.0**-135) == 0.0
    assert oracle.round_bf16(0.0) == 0.0


def test_round_bf16_matches_torch_on_float32_inputs():
    rng = np.random.default_rng(0)
    v = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))).astype(np.float32)
    want = torch.from_numpy(v).to(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([oracle.round_bf16(float(a)) for a in v])
    assert np.array_equal(got, want)


# ---------------------------------------------------------------- a1 router

@pytest.mark.parametrize("cfg", [TINY, TINY_BF16], ids=["f32", "bf16"])
def test_logits_match_numpy_matmul(cfg):
    x, Wr = make_activations(cfg), make_router(cfg)
    bias = np.linspace(-1, 1, cfg.E)
    out = oracle.route(oracle_view(x), oracle_view(Wr), cfg.k, cfg.dtype_code, bias=bias)
    want = _f64(x) @ _f64(Wr).T + bias[None, :]
    np.testing.assert_allclose(out["logits"], want, rtol=0, atol=1e-12)


def test_topk_brute_force_with_exact_ties():
    # integer-valued inputs make equal logits common; lower index must win
    rng = np.random.default_rng(3)
    T, H, E = 200, 4, 7
    x = rng.integers(-2, 3, size=(T, H)).astype(np.float32)
    Wr = rng.integers(-1, 2, size=(E, H)).astype(np.float32)
    logits = x.astype(np.float64) @ Wr.astype(np.float64).T
    assert (np.sort(logits, axis=1)[:, 1:] == np.sort(logits, axis=1)[:, :-1]).any()
    for k in (1, 2, 3, 7):
        out = oracle.route(x, Wr, k, 0)
        for t in range(T):
            order = sorted(range(E), key=lambda e: (-logits[t, e], e))   # full sort with index tie-break
            assert list(out["ids"][t]) == order[:k]


def test_gate_weights_closed_forms():
    cfg = TINY
    x, Wr = oracle_view(make_activations(cfg)), oracle_view(make_router(scaled(cfg, seed=5)))
    Wr = (Wr * 50).astype(np.float32)                                # spread the logits
    for k in (1, 2, 3, cfg.E):
        out = oracle.route(x, Wr, k, 0)
        np.testing.assert_allclose(out["w"].sum(axis=1), 1.0, rtol=0, atol=1e-12)
        assert (out["w"] > 0).all()
        assert (np.diff(out["w"], axis=1) <= 0).all()               # listed by descending logit
    assert np.array_equal(oracle.route(x, Wr, 1, 0)["w"], np.ones((cfg.T, 1)))
    full = oracle.route(x, Wr, cfg.E, 0)
    sm = scipy.special.softmax(full["logits"], axis=1)               # k == E: the plain softmax
    np.testing.assert_allclose(full["w"], np.take_along_axis(sm, full["ids"], axis=1), rtol=1e-12, atol=0)
    # k < E: softmax over all E, renormalised over the selected ones
    out = oracle.route(x, Wr, 2, 0)
    sel = np.take_along_axis(sm, out["ids"], axis=1)
    np.testing.assert_allclose(out["w"], sel / sel.sum(axis=1, keepdims=True), rtol=1e-12, atol=0)


def test_gaps_reported():
    x = np.array([[1.0, 0.0]], np.float32)
    Wr = np.array([[3.0, 0], [1.0, 0], [2.5, 0], [1.0, 0]], np.float32)
    out = oracle.route(x, Wr, 2, 0)
    assert list(out["ids"][0]) == [0, 2]
    assert out["gap_next"][0] == 1.5 and out["gap_inner"][0] == 0.5
    out = oracle.route(x, Wr, 4, 0)
    assert list(out["ids"][0]) == [0, 2, 1, 3]
    assert np.isinf(out["gap_next"][0]) and out["gap_inner"][0] == 0.0


# ---------------------------------------------------------------- a2 permutation

@pytest.mark.parametrize("T,k,E", [(1, 1, 1), (5, 2, 3), (300, 2, 8), (257, 4, 16), (64, 8, 8)])
def test_permutation_is_stable_sort(T, k, E):
    rng = np.random.default_rng(T * 131 + k)
    ids = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    out = oracle.permute(ids, E)
    R = T * k
    flat = ids.reshape(-1)
    assert np.array_equal(out["counts"], np.bincount(flat, minlength=E))
    assert out["counts"].sum() == R and out["offsets"][0] == 0 and out["offsets"][E] == R
    assert np.array_equal(out["offsets"][1:], np.cumsum(out["counts"]))
    assert np.array_equal(out["row_src"], np.argsort(flat, kind="stable"))
    assert np.array_equal(out["row_of"][out["row_src"]], np.arange(R))
    assert np.array_equal(np.sort(out["row_src"]), np.arange(R))
    e_of_row = flat[out["row_src"]]
    assert (np.diff(e_of_row) >= 0).all()
    for e in range(E):
        seg = out["row_src"][out["offsets"][e]:out["offsets"][e + 1]]
        assert (np.diff(seg // k) > 0).all()                        # token index strictly increasing


def test_permute_empty_expert_and_all_to_one():
    ids = np.zeros((9, 1), np.int32) + 2
    out = oracle.permute(ids, 4)
    assert list(out["counts"]) == [0, 0, 9, 0] and list(out["offsets"]) == [0, 0, 0, 9, 9]
    assert np.array_equal(out["row_src"], np.arange(9))


def test_gather_rows_is_a_copy():
    cfg = TINY_BF16
    x = oracle_view(make_activations(cfg))
    row_src = np.random.default_rng(1).permutation(cfg.T * cfg.k).astype(np.int32)
    xp = oracle.gather_rows(x, row_src, cfg.k, 1)
    assert np.array_equal(xp, x[row_src // cfg.k])


# ---------------------------------------------------------------- a3 expert FFN

@pytest.mark.parametrize("cfg", [TINY, TINY_BF16], ids=["f32", "bf16"])
def test_single_expert_is_dense_swiglu(cfg):
    cfg1 = scaled(cfg, E=1, k=1)
    inp = make_inputs(cfg1)
    v = _views(inp)
    out = oracle.layer(v["x"], v["Wr"], v["W1"], v["W3"], v["W2"], 1, cfg1.dtype_code)
    assert (out["ids"] == 0).all() and np.array_equal(out["w"], np.ones((cfg1.T, 1)))
    h_ref, y_ref = _dense_swiglu_f64(_f64(inp["x"]), _f64(inp["W1"][0]), _f64(inp["W3"][0]), _f64(inp["W2"][0]),
                                     cfg1.dtype_code)
    h, o = oracle.expert_ffn(v["x"], np.array([0, cfg1.T], np.int32), v["W1"], v["W3"], v["W2"], cfg1.dtype_code)
    # h is a rounded quantity: all but a vanishing share of elements are equal bit for bit
    # (the reference rounds through float32 for bf16, which can move a value sitting on a tie)
    assert (h != h_ref).mean() < 1e-3
    np.testing.assert_allclose(o, y_ref, rtol=0, atol=2e-5 * np.abs(y_ref).max())
    np.testing.assert_allclose(out["y"], y_ref, rtol=0, atol=2e-5 * np.abs(y_ref).max())


@pytest.mark.parametrize("cfg", [TINY, TINY_BF16], ids=["f32", "bf16"])
def test_per_expert_segments_use_their_own_weights(cfg):
    inp = make_inputs(cfg)
    v = _views(inp)
    out = oracle.layer(v["x"], v["Wr"], v["W1"], v["W3"], v["W2"], cfg.k, cfg.dtype_code)
    _, o = oracle.expert_ffn(out["x_perm"], out["offsets"], v["W1"], v["W3"], v["W2"], cfg.dtype_code)
    xp = _f64(inp["x"])[out["row_src"] // cfg.k]
    for e in range(cfg.E):
        lo, hi = out["offsets"][e], out["offsets"][e + 1]
        _, ref = _dense_swiglu_f64(xp[lo:hi], _f64(inp["W1"][e]), _f64(inp["W3"][e]), _f64(inp["W2"][e]), cfg.dtype_code)
        np.testing.assert_allclose(o[lo:hi], ref, rtol=0, atol=2e-5 * max(np.abs(ref).max(), 1e-30))
    # the full layer against a per-token loop over numpy products
    y_ref = np.zeros((cfg.T, cfg.H))
    for t in range(cfg.T):
        for s in range(cfg.k):
            e = out["ids"][t, s]
            _, oo = _dense_swiglu_f64(_f64(inp["x"])[t:t + 1], _f64(inp["W1"][e]), _f64(inp["W3"][e]),
                                      _f64(inp["W2"][e]), cfg.dtype_code)
            y_ref[t] += out["w"][t, s] * oo[0]
    np.testing.assert_allclose(out["y"], y_ref, rtol=0, atol=2e-5 * np.abs(y_ref).max())


@pytest.mark.parametrize("cfg", [TINY, TINY_BF16], ids=["f32", "bf16"])
def test_identical_experts_make_output_routing_independent(cfg):
    inp = make_inputs(cfg, identical_experts=True)
    v = _views(inp)
    out = oracle.layer(v["x"], v["Wr"], v["W1"], v["W3"], v["W2"], cfg.k, cfg.dtype_code)
    _, dense = _dense_swiglu_f64(_f64(inp["x"]), _f64(inp["W1"][0]), _f64(inp["W3"][0]), _f64(inp["W2"][0]),
                                 cfg.dtype_code)
    np.testing.assert_allclose(out["y"], dense, rtol=0, atol=2e-5 * np.abs(dense).max())
    # another router: different routing, same output
    Wr2 = oracle_view(make_router(scaled(cfg, seed=99)))
    out2 = oracle.layer(v["x"], Wr2, v["W1"], v["W3"], v["W2"], cfg.k, cfg.dtype_code)
    assert not np.array_equal(out["ids"], out2["ids"])
    np.testing.assert_allclose(out2["y"], out["y"], rtol=0, atol=1e-12)


def test_w2_linearity_and_row_weight():
    cfg = TINY
    inp = make_inputs(cfg)
    v = _views(inp)
    out = oracle.layer(v["x"], v["Wr"], v["W1"], v["W3"], v["W2"], cfg.k, 0)
    out2 = oracle.layer(v["x"], v["Wr"], v["W1"], v["W3"], (v["W2"] * 2).astype(np.float32), cfg.k, 0)
    assert np.array_equal(out2["y"], 2 * out["y"])                  # power-of-two scaling is exact
    rw = np.random.default_rng(0).uniform(0.1, 1, cfg.R)
    _, o = oracle.expert_ffn(out["x_perm"], out["offsets"], v["W1"], v["W3"], v["W2"], 0, want_h=False)
    _, ow = oracle.expert_ffn(out["x_perm"], out["offsets"], v["W1"], v["W3"], v["W2"], 0, row_w=rw, want_h=False)
    np.testing.assert_allclose(ow, o * rw[:, None], rtol=1e-15, atol=0)
    sel = np.array([5, 0, cfg.R - 1], np.int32)
    _, osel = oracle.expert_ffn(out["x_perm"], out["offsets"], v["W1"], v["W3"], v["W2"], 0, sel=sel, want_h=False)
    assert np.array_equal(osel, o[sel])


# ---------------------------------------------------------------- a4 combine

def test_combine_closed_forms():
    rng = np.random.default_rng(2)
    T, k, H, E = 23, 3, 16, 6
    ids = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    pm = oracle.permute(ids, E)
    w = rng.uniform(0.1, 1, (T, k))
    w /= w.sum(axis=1, keepdims=True)
    y = oracle.combine(np.ones((T * k, H)), pm["row_of"], k, w)
    np.testing.assert_allclose(y, 1.0, rtol=0, atol=1e-15)          # weights of a token sum to 1
    # row r carries the value r: y[t] = sum_s w[t,s] * row_of[t,s]
    o = np.repeat(np.arange(T * k, dtype=np.float64)[:, None], H, axis=1)
    y = oracle.combine(o, pm["row_of"], k, w)
    np.testing.assert_allclose(y[:, 0], (w * pm["row_of"].reshape(T, k)).sum(axis=1), rtol=1e-14)
    # unweighted form
    y = oracle.combine(o, pm["row_of"], k, None)
    np.testing.assert_allclose(y[:, 0], pm["row_of"].reshape(T, k).sum(axis=1), rtol=1e-14)
    # one-hot rows recover the gate weights
    o = np.zeros((T * k, H))
    t0, s0 = 7, 1
    o[pm["row_of"][t0 * k + s0], :] = 1.0
    y = oracle.combine(o, pm["row_of"], k, w)
    assert np.allclose(y[t0], w[t0, s0]) and np.count_nonzero(y) == H


# ---------------------------------------------------------------- workloads

def test_counts_sum_and_c1_statistics():
    cfg = CONFIGS["c1_tiny_f32"]
    v = _views(make_inputs(cfg))
    out = oracle.layer(v["x"], v["Wr"], v["W1"], v["W3"], v["W2"], cfg.k, 0)
    assert out["counts"].sum() == cfg.T * cfg.k
    # weights N(0, 0.02), x N(0,1): output scale ~ sqrt(F) * 0.02 * (|silu(g) u| scale) -- a coarse sanity band
    assert 0.005 < out["y"].std() < 0.05


def test_c4_router_bias_gives_the_stated_skew():
    cfg = CONFIGS["c4_mixtral8x22b_t8192_skew"]
    x, Wr, b = make_activations(cfg), make_router(cfg), bias_vector(cfg)
    out = oracle.route(oracle_view(x), oracle_view(Wr), cfg.k, 1, bias=b.numpy())
    share = oracle.permute(out["ids"], cfg.E)["counts"] / float(cfg.R)
    assert 0.38 <= share[0] <= 0.42, share
    assert 0.0 < share[7] < 0.02, share


def test_near_tie_rate_is_small_on_c3_shape():
    cfg = scaled(CONFIGS["c3_mixtral8x7b_t4096"], T=1024)
    out = oracle.route(oracle_view(make_activations(cfg)), oracle_view(make_router(cfg)), cfg.k, 1)
    assert (out["gap_next"] < 1e-4).mean() < 0.01


# ---------------------------------------------------------------- planted mistakes
# Each plants one plausible slip into what the ORACLE is given (on the CPU) and
# checks that the independent reference used above would notice it.

def _layer_vs_dense_err(cfg, mutate):
    cfg1 = scaled(cfg, E=1, k=1)
    inp = make_inputs(cfg1)
    v = _views(inp)
    W1, W3, W2 = mutate(v["W1"], v["W3"], v["W2"])
    out = oracle.layer(v["x"], v["Wr"], W1, W3, W2, 1, cfg1.dtype_code)
    _, y_ref = _dense_swiglu_f64(_f64(inp["x"]), _f64(inp["W1"][0]), _f64(inp["W3"][0]), _f64(inp["W2"][0]),
                                 cfg1.dtype_code)
    return np.abs(out["y"] - y_ref).max() / np.abs(y_ref).max()


def test_planted_mistakes_are_caught():
    assert _layer_vs_dense_err(TINY, lambda a, b, c: (a, b, c)) < 1e-4
    assert _layer_vs_dense_err(TINY, lambda a, b, c: (b, a, c)) > 1e-2            # gate and up swapped
    assert _layer_vs_dense_err(TINY, lambda a, b, c: (a, b, -c)) > 1e-2           # sign
    assert _layer_vs_dense_err(TINY, lambda a, b, c: (a[:, ::-1].copy(), b, c)) > 1e-2   # wrong row index
    sq = scaled(TINY, F=64)                                                      # square W2 so a transpose fits
    assert _layer_vs_dense_err(sq, lambda a, b, c: (a, b, np.ascontiguousarray(c.transpose(0, 2, 1)))) > 1e-2


def test_c1_golden_fixture_unchanged():
    import importlib.util
    import json
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_c1_golden", os.path.join(here, "make_c1_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    got = mod.compute()
    with open(os.path.join(here, "c1_oracle.json")) as f:
        want = json.load(f)
    for key in ("counts", "ids_first8", "row_src_first16"):
        assert got[key] == want[key], key
    for key in ("w_first4", "y_first4x4", "y_sum", "y_abs_sum"):
        np.testing.assert_allclose(np.array(got[key]), np.array(want[key]), rtol=1e-12, atol=0)
