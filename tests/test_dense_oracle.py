"""Pins of the oracle for the dense neighbours of the layer (oracle/dense.py): closed forms, special
cases, hand loops on tiny inputs and library routines (torch CPU float64)."""
import numpy as np
import torch

from oracle import dense, round_bf16


def bits(t: torch.Tensor) -> np.ndarray:
    return t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_bf16_round_trip_and_ties():
    v = np.array([0.0, 1.0, -2.5, 3.0e38, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -30])
    b = dense.f64_to_bf16_bits(v)
    back = dense.bf16_bits_to_f64(b)
    assert back[0] == 0.0 and back[1] == 1.0 and back[2] == -2.5
    assert back[4] == 1.0                       # exact tie: to even (mantissa 0)
    assert back[5] == 1.0 + 2.0 ** -6           # exact tie: to even (mantissa 2)
    assert back[6] == 1.0 + 2.0 ** -7           # just above the tie: up (no double rounding through float32)
    for x in np.random.default_rng(0).standard_normal(200):
        assert dense.bf16_bits_to_f64(dense.f64_to_bf16_bits(np.array([x])))[0] == round_bf16(float(x))
    # every bf16 value survives the round trip
    allbits = np.arange(0, 0x7f80, 37, dtype=np.uint16)
    assert np.array_equal(dense.f64_to_bf16_bits(dense.bf16_bits_to_f64(allbits)), allbits)


def test_linear_is_the_plain_sum_and_matches_torch():
    g = torch.Generator().manual_seed(0)
    x = torch.randn((5, 24), generator=g).to(torch.bfloat16)
    W = (torch.randn((7, 24), generator=g) * 0.1).to(torch.bfloat16)
    y = dense.linear(bits(x), bits(W))
    hand = np.zeros((5, 7))
    for t in range(5):
        for n in range(7):
            for k in range(24):
                hand[t, n] += float(x[t, k]) * float(W[n, k])
    assert np.allclose(y, hand, rtol=0, atol=1e-12)
    lib = torch.nn.functional.linear(x.double(), W.double()).numpy()
    assert np.allclose(y, lib, rtol=0, atol=1e-12)
    # an identity weight returns the input; a transposed operand would not (W is [N][K], not [K][N])
    eye = torch.eye(24).to(torch.bfloat16)
    assert np.array_equal(dense.linear(bits(x), bits(eye)), x.double().numpy())
    W2 = torch.zeros((3, 24)); W2[1, 5] = 2.0
    assert np.array_equal(dense.linear(bits(x), bits(W2))[:, 1], 2.0 * x.double().numpy()[:, 5])


def test_rmsnorm_closed_forms_and_library():
    H = 32
    gamma = np.linspace(0.5, 1.5, H)
    # a constant row c: s / sqrt(c^2 + eps) * gamma
    s, xb = dense.add_rmsnorm(None, np.full((1, H), -3.0), gamma, eps=0.25)
    want = -3.0 / np.sqrt(9.25) * gamma
    assert np.array_equal(s, np.full((1, H), -3.0))
    assert np.array_equal(dense.bf16_bits_to_f64(xb)[0], [round_bf16(v) for v in want])
    # with eps = 0 the result does not depend on the row's scale, and gamma = 1 gives unit RMS
    rng = np.random.default_rng(1)
    v = rng.standard_normal((4, H))
    _, a = dense.add_rmsnorm(None, v, np.ones(H), 0.0)
    _, b = dense.add_rmsnorm(None, 8.0 * v, np.ones(H), 0.0)       # power of two: no rounding difference
    assert np.array_equal(a, b)
    assert np.allclose(np.sqrt(np.mean(dense.bf16_bits_to_f64(a) ** 2, axis=1)), 1.0, atol=5e-3)
    # the residual is added before the norm
    h, d = rng.standard_normal((4, H)), rng.standard_normal((4, H))
    s, xb = dense.add_rmsnorm(h, d, gamma, 1e-5)
    assert np.array_equal(s, h + d)
    s2, xb2 = dense.add_rmsnorm(None, h + d, gamma, 1e-5)
    assert np.array_equal(xb, xb2)
    # library routine
    lib = torch.nn.functional.rms_norm(torch.from_numpy(h + d), (H,), torch.from_numpy(gamma), 1e-5).numpy()
    assert np.abs(dense.bf16_bits_to_f64(xb) - lib).max() <= np.abs(lib).max() * 2.0 ** -8
    # eps matters: a dropped eps changes a tiny row completely
    _, tiny = dense.add_rmsnorm(None, np.full((1, H), 1e-4), np.ones(H), 1.0)
    assert np.allclose(dense.bf16_bits_to_f64(tiny), 1e-4, rtol=1e-2)
