"""The Hierarchical Roofline Model tool against the paper's equations (section 3, Eqs. 7-11, and the
per-layer latency model of section 4.2) and against this library's own measurements."""
import math

import pytest

from paper_2411_11217_amd import hrm


def test_three_roofs_and_reduction_to_the_plain_roofline():
    # Eq. 7 is the minimum of the three roofs; without a slower level it is Eq. 8
    assert hrm.attainable_hrm(100.0, 10.0, 4.0, 1.0, 30.0) == 30.0       # link roof
    assert hrm.attainable_hrm(100.0, 10.0, 4.0, 1.0, 50.0) == 40.0       # GPU memory roof
    assert hrm.attainable_hrm(100.0, 10.0, 20.0, 1.0, 500.0) == 100.0    # compute roof
    for i in (0.5, 3.0, 10.0, 40.0):
        assert hrm.attainable_hrm(100.0, 10.0, i, math.inf, 1.0) == hrm.attainable(100.0, 10.0, i) == min(100.0, 10.0 * i)


def test_turning_points_and_balance_point():
    hw = hrm.Hardware(p_g=1000.0, b_g=50.0, b_cg=2.0, p_c=40.0, b_c=10.0)
    # P1 (Eq. 9): the link roof meets what the host attains by itself
    i1 = hrm.turning_point_p1(hw)
    assert i1 == 20.0
    assert hw.b_cg * i1 == pytest.approx(hrm.attainable(hw.p_c, hw.b_c, i1))
    assert hw.b_cg * (i1 * 0.9) < hrm.attainable(hw.p_c, hw.b_c, i1 * 0.9)      # below P1 the host wins
    # P2 (Eq. 10): the link roof meets what the GPU attains at its own intensity
    for i_gpu in (4.0, 20.0, 100.0):
        i2 = hrm.turning_point_p2(hw, i_gpu)
        assert hw.b_cg * i2 == pytest.approx(hrm.attainable(hw.p_g, hw.b_g, i_gpu))
        assert hrm.attainable_hrm(hw.p_g, hw.b_g, i_gpu, hw.b_cg, i2 * 0.5) == pytest.approx(hw.b_cg * i2 * 0.5)
    # balance point (Eq. 11)
    assert hw.b_g * 4.0 == pytest.approx(hw.b_cg * hrm.balance_intensity(hw, 4.0))
    # a link faster than host memory: moving data always pays
    assert hrm.turning_point_p1(hrm.Hardware(1.0, 1.0, b_cg=20.0, p_c=40.0, b_c=10.0)) == 0.0


def test_layer_counts():
    L = hrm.MIXTRAL_8X7B
    assert L.weight_bytes == 3 * 8 * 4096 * 14336 * 2
    assert L.flops(4096) == 6 * 8192 * 4096 * 14336 + 2 * 4096 * 4096 * 8
    # with many rows every expert is touched: the GPU bytes contain all the weights once
    assert L.gpu_bytes(4096) == pytest.approx(L.weight_bytes + 2 * 4096 * 4096 * 2 + 2 * 8192 * 4096 * 2
                                              + 2 * 8192 * 14336 * 2 + 8 * 8192 * 4096 + 4 * 4096 * 4096, rel=1e-9)
    # one token with k = 2 touches (in expectation) fewer than two experts' weights
    assert L.gpu_bytes(1) < 2 * 3 * 4096 * 14336 * 2 * 1.01


def test_latency_model_properties():
    L, hw = hrm.DBRX, hrm.MI355X_MEASURED
    prev = None
    for step in range(11):
        r = hrm.layer_latency(L, hw, 16384, 4096, step / 10)
        assert r["T"] == max(r["comm"], r["T_gpu"])
        # the bytes that cross the link for the layer: the non-resident weights and every token's hidden state
        assert r["comm"] == pytest.approx(((1 - step / 10) * L.weight_bytes + 16384 * L.h1 * L.dt) / hw.b_cg)
        w_only = hrm.layer_latency(L, hw, 16384, 4096, step / 10, hidden_from_host=False)
        assert w_only["comm"] == pytest.approx((1 - step / 10) * L.weight_bytes / hw.b_cg) and w_only["T_gpu"] == r["T_gpu"]
        if prev is not None:
            assert r["T"] <= prev + 1e-12            # keeping more weights on the GPU never hurts
        prev = r["T"]
    # T_gpu does not depend on r_w; N not a multiple of mu adds one short kernel execution
    a = hrm.layer_latency(L, hw, 16384, 4096, 0.0)["T_gpu"]
    b = hrm.layer_latency(L, hw, 16384 + 100, 4096, 1.0)["T_gpu"]
    assert b > a and b - a == pytest.approx(max(L.flops(100) / hw.p_g, L.gpu_bytes(100) / hw.b_g))
    # link-bound operational intensity with respect to the host data is 2 * N * k / (n_e * dt)
    assert hrm.layer_latency(L, hw, 16384, 4096, 0.0)["I_link"] == pytest.approx(2 * 16384 * 4 / (16 * 2), rel=1e-3)


def test_crossover_micro_batch_is_the_ridge():
    L, hw = hrm.MIXTRAL_8X7B, hrm.MI355X_MEASURED
    mu = hrm.crossover_micro_batch(L, hw)
    assert L.flops(mu) / hw.p_g >= L.gpu_bytes(mu) / hw.b_g
    assert L.flops(mu - 1) / hw.p_g < L.gpu_bytes(mu - 1) / hw.b_g
    # if only the weights counted, the ridge would be n_e * dt * p_g / (2 * k * b_g) tokens
    closed = L.n_e * L.dt * hw.p_g / (2 * L.k * hw.b_g)
    assert closed < mu < 1.15 * closed
    # the two resident workloads of this repository sit on either side of it
    assert 256 < mu < 4096


# (layer, N, mu, r_w, hidden states cross the link, measured ms per layer on one MI355X, tolerance):
# bench.py (inputs resident) and bench.py --pipeline (hidden states copied from the host)
MEASURED = [
    (hrm.MIXTRAL_8X7B, 256, 256, 1.0, False, 0.53, 0.05),
    (hrm.MIXTRAL_8X7B, 4096, 4096, 1.0, False, 2.24, 0.05),
    (hrm.MIXTRAL_8X22B, 8192, 8192, 1.0, False, 7.48, 0.08),
    (hrm.DBRX, 16384, 4096, 0.0, True, 115.3, 0.03),
    (hrm.DBRX, 16384, 4096, 48 / 95, True, 59.0, 0.03),
    (hrm.DBRX, 16384, 4096, 76 / 95, True, 26.2, 0.03),     # next to the turning point: link time = 1.25 x GPU time
    (hrm.DBRX, 16384, 4096, 1.0, True, 21.9, 0.08),
]


@pytest.mark.parametrize("layer,N,mu,r_w,hidden,measured_ms,tol", MEASURED)
def test_model_with_measured_rates_predicts_the_measured_latency(layer, N, mu, r_w, hidden, measured_ms, tol):
    r = hrm.layer_latency(layer, hrm.MI355X_MEASURED, N, mu, r_w, hidden_from_host=hidden)
    assert r["T"] * 1e3 == pytest.approx(measured_ms, rel=tol)
    # and the nominal peaks are an upper bound on what was measured
    assert hrm.layer_latency(layer, hrm.MI355X_PEAK, N, mu, r_w, hidden_from_host=hidden)["T"] * 1e3 < measured_ms


def test_policy_search_respects_memory_and_finds_the_balance():
    L = hrm.DBRX
    # plenty of GPU memory: compute bound, with the smallest resident fraction that gets there
    pol, rec = hrm.best_policy(L, hrm.MI355X_MEASURED, 16384, [1024, 4096], n_layers=40)
    assert rec["bound"] == "gpu" and pol["r_w"] == pytest.approx(0.85)
    assert hrm.layer_latency(L, hrm.MI355X_MEASURED, 16384, pol["mu"], 0.80)["bound"] == "link"
    # 96 GB for 40 layers (236 GiB of weights): only part fits; the search keeps as much resident as fits
    small = hrm.Hardware(p_g=1.05e15, b_g=5.0e12, b_cg=55.7e9, m_g=96e9)
    pol, rec = hrm.best_policy(L, small, 16384, [1024, 4096], n_layers=40)
    assert 0.0 < pol["r_w"] < 1.0 and rec["bound"] == "link"
    assert pol["gpu_bytes_needed"] <= small.m_g
    worse = hrm.layer_latency(L, small, 16384, pol["mu"], pol["r_w"] - 0.05)
    assert worse["T"] > rec["T"]
    # nothing fits: no policy
    none, _ = hrm.best_policy(L, hrm.Hardware(1e15, 5e12, 55e9, m_g=1e9), 16384, [4096])
    assert none is None
