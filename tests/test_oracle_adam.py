"""Pins for the oracle's Adam block (Algorithm 2, update lines; Sec. 4.2 N_t equation)."""
import numpy as np
import pytest
import torch

from conftest import golden
from oracle import galore_oracle as orc


def test_hand_computed_scalar_steps():
    rows = golden("adam_scalar_steps.txt")
    M = np.zeros((1, 1))
    V = np.zeros((1, 1))
    for k, R, m_ref, v_ref, _mh, _vh, n_ref in rows:
        N = orc.adam(np.array([[R]]), M, V, 0.9, 0.999, 1e-8, int(k))
        assert M[0, 0] == pytest.approx(m_ref, rel=1e-8)
        assert V[0, 0] == pytest.approx(v_ref, rel=1e-8)
        assert N[0, 0] == pytest.approx(n_ref, rel=2e-8)


def test_constant_gradient_closed_form():
    # R = x at every step => Mhat = x, Vhat = x^2, N = x / (|x| + eps) for all k.
    x = np.array([[0.3, -1.7, 2.5e-3, 40.0]])
    M = np.zeros_like(x)
    V = np.zeros_like(x)
    eps = 1e-8
    for k in range(1, 30):
        N = orc.adam(x, M, V, 0.9, 0.999, eps, k)
        np.testing.assert_allclose(N, x / (np.abs(x) + eps), rtol=1e-12)
        np.testing.assert_allclose(M, x * (1 - 0.9 ** k), rtol=1e-12)
        np.testing.assert_allclose(V, x * x * (1 - 0.999 ** k), rtol=1e-12)


def test_stored_moments_are_not_bias_corrected():
    # After one step from zero the stored first moment must be (1-b1) R, not R.
    R = np.array([[2.0]])
    M = np.zeros((1, 1)); V = np.zeros((1, 1))
    orc.adam(R, M, V, 0.9, 0.999, 1e-8, 1)
    assert M[0, 0] == pytest.approx(0.2, rel=1e-14)
    assert V[0, 0] == pytest.approx(0.004, rel=1e-13)


def test_eps_outside_the_square_root():
    # With V tiny the two placements differ a lot: eps = 1e-2, R = 1e-3 at k = 1 gives
    # N = 1e-3 / (1e-3 + 1e-2) under Algorithm 2; sqrt(V + eps) would give ~1e-2.
    R = np.array([[1e-3]])
    M = np.zeros((1, 1)); V = np.zeros((1, 1))
    N = orc.adam(R, M, V, 0.9, 0.999, 1e-2, 1)
    assert N[0, 0] == pytest.approx(1e-3 / (1e-3 + 1e-2), rel=1e-12)


@pytest.mark.parametrize("seed", [0, 1])
def test_matches_library_adam_over_many_steps(seed):
    # torch.optim.Adam (fp64, CPU) is the library statement of the same update; with lr = 1
    # and a parameter starting at 0, minus its parameter increment per step equals N.
    rng = np.random.default_rng(seed)
    shape = (5, 7)
    p = torch.zeros(shape, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([p], lr=1.0, betas=(0.9, 0.999), eps=1e-8)
    M = np.zeros(shape); V = np.zeros(shape)
    for k in range(1, 25):
        R = rng.standard_normal(shape) * (10.0 ** rng.integers(-3, 2))
        before = p.detach().clone().numpy()
        p.grad = torch.from_numpy(R.copy())
        opt.step()
        N_lib = before - p.detach().numpy()
        N = orc.adam(R, M, V, 0.9, 0.999, 1e-8, k)
        np.testing.assert_allclose(N, N_lib, rtol=1e-9, atol=1e-12)
        st = opt.state[p]
        np.testing.assert_allclose(M, st["exp_avg"].numpy(), rtol=1e-12, atol=1e-300)
        np.testing.assert_allclose(V, st["exp_avg_sq"].numpy(), rtol=1e-12, atol=1e-300)
