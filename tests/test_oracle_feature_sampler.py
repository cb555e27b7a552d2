"""CPU pins of the oracle's Feature Sampler (no GPU): a hand-worked case, the library's SiLU and
linear layers, the cases where the gate closes or saturates, and linearity in the feature."""
import numpy as np
import torch

import oracle


def test_hand_worked_case():
    # Hd = 2, I = 3.  f = (1, 2), e = (ln 3, 0):  up = (1, 2, 3), gate = (ln 3, 0, -ln 3)
    # SiLU(ln 3) = ln3 * 3/4, SiLU(0) = 0, SiLU(-ln 3) = -ln3 / 4
    f = np.array([[1.0, 2.0]])
    e = np.array([[np.log(3.0), 0.0]])
    w_up = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]])
    w_gate = np.array([[1.0, 0.0], [0.0, 1.0], [-1.0, 5.0]])
    w_down = np.array([[1.0, 1.0, 1.0], [2.0, 0.0, -4.0]])
    l3 = np.log(3.0)
    s = np.array([0.75 * l3 * 1.0, 0.0, -0.25 * l3 * 3.0])
    expect = np.array([[s.sum() + 1.0, 2.0 * s[0] - 4.0 * s[2] + 2.0]])
    np.testing.assert_allclose(oracle.feature_sampler(f, e, w_up, w_gate, w_down), expect, rtol=1e-12)
    np.testing.assert_allclose(oracle.feature_sampler(f, e, w_up, w_gate, w_down, residual=False), expect - f, rtol=1e-12, atol=1e-15)


def test_against_library_layers():
    rng = np.random.default_rng(1)
    rows, Hd, I = 5, 24, 56
    f, e = rng.standard_normal((rows, Hd)), rng.standard_normal((rows, Hd))
    wu, wg, wd = rng.standard_normal((I, Hd)), rng.standard_normal((I, Hd)), rng.standard_normal((Hd, I))
    T = lambda a: torch.from_numpy(a)
    F = torch.nn.functional
    ref = F.linear(F.silu(F.linear(T(e), T(wg))) * F.linear(T(f), T(wu)), T(wd)) + T(f)
    np.testing.assert_allclose(oracle.feature_sampler(f, e, wu, wg, wd), ref.numpy(), rtol=1e-12, atol=1e-12)


def test_closed_gate_leaves_the_residual_and_open_gate_is_linear():
    rng = np.random.default_rng(2)
    rows, Hd, I = 3, 8, 16
    f = rng.standard_normal((rows, Hd))
    wu, wd = rng.standard_normal((I, Hd)), rng.standard_normal((Hd, I))
    # e = 0: every gate is SiLU(0) = 0
    out = oracle.feature_sampler(f, np.zeros((rows, Hd)), wu, rng.standard_normal((I, Hd)), wd)
    np.testing.assert_array_equal(out, f)
    # a gate far in the linear range: SiLU(g) -> g, so eta = W_down (g * (W_up f)) + f
    e = np.ones((rows, Hd))
    wg = np.full((I, Hd), 10.0)            # gate = 80 everywhere
    out = oracle.feature_sampler(f, e, wu, wg, wd)
    np.testing.assert_allclose(out, (80.0 * (f @ wu.T)) @ wd.T + f, rtol=1e-12)
    # linear in f for a fixed e
    e = rng.standard_normal((rows, Hd))
    wg = rng.standard_normal((I, Hd))
    a = oracle.feature_sampler(f, e, wu, wg, wd)
    b = oracle.feature_sampler(3.0 * f, e, wu, wg, wd)
    np.testing.assert_allclose(b, 3.0 * a, rtol=1e-12)


def test_tile_order_of_the_weights_element_by_element():
    """The packed order against its definition, one element at a time, on a matrix whose entries
    name their own position; a ragged last tile row is padded with zeros."""
    N, K = 40, 96
    w = (np.arange(N)[:, None] * 1000 + np.arange(K)[None, :]).astype(np.float64)
    p = oracle.pack_weight(w)
    assert p.shape == (48 * K,)
    S = K // 32
    for t in range(3):
        for s_ in range(S):
            for n in range(16):
                for g in range(4):
                    for j in range(8):
                        row, col = 16 * t + n, 32 * s_ + 8 * g + j
                        got = p[((t * S + s_) * 64 + n + 16 * g) * 8 + j]
                        assert got == (w[row, col] if row < N else 0.0)
