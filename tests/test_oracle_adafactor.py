"""Pins for the oracle's Adafactor block: Adafactor with first-order statistics as the optimizer of the projected
gradient (Sec. 4.3 and Sec. 5 of the paper name it and print no equations, so parity with the paper is unpinned; the
routine is pinned to the published Adafactor update through torch's implementation, closed forms and a hand-worked step)."""
import numpy as np
import pytest
import torch

from conftest import golden
from oracle import galore_oracle as orc


def _state(shape):
    return np.zeros(shape), np.zeros(shape[0]), np.zeros(shape[1])


def test_hand_worked_two_steps_with_momentum_and_clipping():
    R = np.array([[3.0, 1.0], [1.0, 1.0]])
    M, rowv, colv = _state(R.shape)
    for k, n11, n12, n21, n22 in golden("adafactor_hand.txt"):
        N = orc.adafactor(R, M, rowv, colv, 0.5, int(k), eps1=0.0)
        np.testing.assert_allclose(N, [[n11, n12], [n21, n22]], rtol=1e-13)
        np.testing.assert_allclose(rowv, [10.0, 2.0], rtol=1e-14)
        np.testing.assert_allclose(colv, [10.0, 2.0], rtol=1e-14)


@pytest.mark.parametrize("shape", [(5, 7), (7, 5), (6, 6)])
def test_library_adafactor_without_momentum(shape):
    # torch.optim.Adafactor is the same published update (row / column means instead of sums: the same quotient),
    # without momentum.  With eps2 = 1 and a parameter of RMS below 1 its step size is min(lr, 1 / sqrt(k)) = lr, so
    # W_k - W_{k-1} = -lr * Uhat_k, which is -lr * N_k of the oracle at b1 = 0.
    g = torch.Generator().manual_seed(3)
    W0 = (torch.randn(*shape, generator=g, dtype=torch.float64) * 0.1)
    w = torch.nn.Parameter(W0.clone())
    lr = 1e-2
    opt = torch.optim.Adafactor([w], lr=lr, beta2_decay=-0.8, eps=(1e-30, 1.0), d=1.0, weight_decay=0.0)
    W = W0.numpy().copy()
    M, rowv, colv = _state(shape)
    for k in range(1, 8):
        G = torch.randn(*shape, generator=g, dtype=torch.float64) * (0.5 + k)      # scale changes so the decay matters
        w.grad = G.clone()
        opt.step()
        N = orc.adafactor(G.numpy(), M, rowv, colv, 0.0, k)
        W -= lr * N
        np.testing.assert_allclose(W, w.detach().numpy(), rtol=0, atol=1e-13)


def test_rank_one_magnitudes_give_the_sign_matrix():
    # |R_ij| = a_i b_j: the factored second moment is exact at k = 1, U = sign(R), RMS(U) = 1, nothing is clipped
    rng = np.random.default_rng(0)
    a, b = rng.uniform(0.1, 3.0, 6), rng.uniform(0.1, 3.0, 9)
    sgn = rng.choice([-1.0, 1.0], (6, 9))
    R = sgn * np.outer(a, b)
    M, rowv, colv = _state(R.shape)
    N = orc.adafactor(R, M, rowv, colv, 0.0, 1, eps1=0.0)
    np.testing.assert_allclose(N, sgn, rtol=1e-13)
    np.testing.assert_allclose(rowv, a * a * np.sum(b * b), rtol=1e-13)     # which index carries which statistic
    np.testing.assert_allclose(colv, b * b * np.sum(a * a), rtol=1e-13)


def test_first_step_is_invariant_to_the_scale_of_the_gradient():
    rng = np.random.default_rng(1)
    R = rng.standard_normal((4, 11))
    outs = []
    for c in (1.0, 1e-3, 250.0):
        M, rowv, colv = _state(R.shape)
        outs.append(orc.adafactor(c * R, M, rowv, colv, 0.9, 1, eps1=0.0))
    np.testing.assert_allclose(outs[1], outs[0], rtol=1e-12)
    np.testing.assert_allclose(outs[2], outs[0], rtol=1e-12)


def test_constant_gradient_momentum_sum_and_clipped_rms():
    # the same R at every step keeps the statistics where the first step put them, so Uhat is the same every time and
    # M_k = (1 - b1^k) Uhat; with clipping engaged RMS(Uhat) = d exactly
    rng = np.random.default_rng(2)
    R = rng.standard_normal((5, 8)) * np.array([[10.0], [1.0], [0.1], [1.0], [3.0]])
    M0, r0, c0 = _state(R.shape)
    Uhat = orc.adafactor(R, M0, r0, c0, 0.0, 1)
    rms = np.sqrt(np.mean(Uhat ** 2))
    assert rms == pytest.approx(1.0, rel=1e-12)          # this R is not of rank-one magnitudes: RMS(U) > 1 before clipping
    M, rowv, colv = _state(R.shape)
    for k in range(1, 7):
        N = orc.adafactor(R, M, rowv, colv, 0.9, k)
        np.testing.assert_allclose(N, (1 - 0.9 ** k) * Uhat, rtol=1e-12)
        np.testing.assert_allclose(rowv, r0, rtol=1e-13)


def test_clip_threshold_and_unclipped_case():
    R = np.array([[2.0, 1.0], [1.0, 2.0]])      # U^2 = (1.6, 0.4, 0.4, 1.6): RMS exactly 1, untouched at d = 1
    M, rowv, colv = _state(R.shape)
    N = orc.adafactor(R, M, rowv, colv, 0.0, 1, eps1=0.0)
    np.testing.assert_allclose(N ** 2, [[1.6, 0.4], [0.4, 1.6]], rtol=1e-13)
    M, rowv, colv = _state(R.shape)
    N = orc.adafactor(R, M, rowv, colv, 0.0, 1, eps1=0.0, clip_d=0.5)      # threshold 0.5: scaled to RMS 0.5
    np.testing.assert_allclose(N ** 2, [[0.4, 0.1], [0.1, 0.4]], rtol=1e-13)


def test_transposed_problem_swaps_the_statistics():
    rng = np.random.default_rng(4)
    R = rng.standard_normal((3, 10))
    Ma, ra, ca = _state(R.shape)
    Mb, rb, cb = _state(R.T.shape)
    for k in (1, 2, 3):
        Rk = R * k
        Na = orc.adafactor(Rk, Ma, ra, ca, 0.8, k)
        Nb = orc.adafactor(np.ascontiguousarray(Rk.T), Mb, rb, cb, 0.8, k)
        np.testing.assert_allclose(Nb, Na.T, rtol=1e-12)
        np.testing.assert_allclose(rb, ca, rtol=1e-13)
        np.testing.assert_allclose(cb, ra, rtol=1e-13)


def test_zero_gradient_is_finite():
    M, rowv, colv = _state((3, 4))
    N = orc.adafactor(np.zeros((3, 4)), M, rowv, colv, 0.9, 1)
    assert np.all(N == 0.0) and np.all(np.isfinite(rowv)) and np.all(np.isfinite(colv))


@pytest.mark.parametrize("shape", [(6, 10), (10, 6)])
def test_full_rank_identity_projector_is_the_library_optimizer(shape):
    # r = min(m, n) with P = I, alpha = 1, b1 = 0: the GaLore step with Adafactor is torch's Adafactor on W itself
    # (Sec. 3.3: GaLore at full rank follows the original trajectory).  fp32 storage of the state on the oracle's side.
    m, n = shape
    r = min(m, n)
    g = torch.Generator().manual_seed(5)
    W0 = torch.randn(m, n, generator=g, dtype=torch.float64) * 0.1
    w = torch.nn.Parameter(W0.clone())
    lr = 5e-3
    opt = torch.optim.Adafactor([w], lr=lr, beta2_decay=-0.8, eps=(1e-30, 1.0), d=1.0, weight_decay=0.0)
    t = orc.GaLoreAdafactorTensor(W0.numpy(), r, scale=1.0, beta1=0.0, dtype="f32", auto_refresh=False)
    t.set_projector(np.eye(r))
    for k in range(1, 6):
        G = torch.randn(m, n, generator=g, dtype=torch.float64)
        w.grad = G.clone()
        opt.step()
        t.step(G.numpy(), lr)
        np.testing.assert_allclose(t.W, w.detach().numpy(), rtol=0, atol=5e-7)
