"""Pins for the oracle's projection, projection-back and whole step (Algorithm 2)."""
import numpy as np
import pytest
import torch

from conftest import golden
from oracle import galore_oracle as orc


def _orth(n, seed):
    q, r = np.linalg.qr(np.random.default_rng(seed).standard_normal((n, n)))
    return q * np.sign(np.diag(r))


def test_projection_matches_library_matmul_both_sides():
    rng = np.random.default_rng(0)
    G = rng.standard_normal((6, 11))
    P = rng.standard_normal((6, 4))
    np.testing.assert_allclose(orc.project(P, G), P.T @ G, rtol=1e-13, atol=1e-13)
    Gt = rng.standard_normal((11, 6))
    Q = rng.standard_normal((6, 4))
    np.testing.assert_allclose(orc.project(Q, Gt), Gt @ Q, rtol=1e-13, atol=1e-13)


def test_projection_single_entry_indices():
    # One non-zero in P and in G: R[i, j] = P[k, i] G[k, j] pins every index of the left form.
    P = np.zeros((3, 2)); G = np.zeros((3, 5))
    P[2, 1] = 3.0; G[2, 4] = 5.0
    R = orc.project(P, G)
    want = np.zeros((2, 5)); want[1, 4] = 15.0
    np.testing.assert_array_equal(R, want)
    Q = np.zeros((3, 2)); G2 = np.zeros((5, 3))
    Q[1, 0] = 2.0; G2[4, 1] = 7.0
    want = np.zeros((5, 2)); want[4, 0] = 14.0
    np.testing.assert_array_equal(orc.project(Q, G2), want)


def test_apply_update_matches_library_matmul_both_sides():
    rng = np.random.default_rng(1)
    W = rng.standard_normal((5, 9)); P = rng.standard_normal((5, 3)); N = rng.standard_normal((3, 9))
    want = W - 0.1 * 0.25 * (P @ N)
    np.testing.assert_allclose(orc.apply_update(W.copy(), P, N, 0.1, 0.25), want, rtol=1e-13)
    W = rng.standard_normal((9, 5)); Q = rng.standard_normal((5, 3)); N = rng.standard_normal((9, 3))
    want = W - 0.1 * 0.25 * (N @ Q.T)
    np.testing.assert_allclose(orc.apply_update(W.copy(), Q, N, 0.1, 0.25), want, rtol=1e-13)


def test_full_rank_projection_round_trip_is_identity():
    # Sec. 3.3: with r = min(m, n) and rho = identity, P P^T G = G for any orthogonal P.
    rng = np.random.default_rng(2)
    for (m, n) in [(7, 12), (12, 7)]:
        G = rng.standard_normal((m, n))
        k = min(m, n)
        P = _orth(k, 5)
        R = orc.project(P, G)
        W = np.zeros((m, n))
        orc.apply_update(W, P, R, lr=-1.0, alpha=1.0)  # W <- 0 + P R
        np.testing.assert_allclose(W, G, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("shape", [(6, 10), (10, 6), (8, 8)])
def test_identity_projector_reduces_to_library_adam(shape):
    # r = min(m,n), P = I  =>  GaLore's trajectory is plain Adam with step size lr*alpha.
    m, n = shape
    k = min(m, n)
    rng = np.random.default_rng(7)
    W0 = rng.standard_normal(shape) * 0.02
    lr, alpha = 1e-2, 0.25
    t = orc.GaLoreTensor(W0, rank=k, scale=alpha, dtype="f64", auto_refresh=False)
    t.proj = np.eye(k)
    p = torch.tensor(W0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([p], lr=lr * alpha, betas=(0.9, 0.999), eps=1e-8)
    for step in range(12):
        G = rng.standard_normal(shape)
        p.grad = torch.from_numpy(G.copy())
        opt.step()
        _step_f64(t, G, lr)
        np.testing.assert_allclose(t.W, p.detach().numpy(), rtol=1e-10, atol=1e-13)


def _step_f64(t, G, lr):
    """GaLoreTensor.step without storage rounding (dtype 'f64' keeps W; M, V rounding to fp32 is
    bypassed by redoing the step from the pieces)."""
    R = orc.project(t.proj, G)
    N = orc.adam(R, t.M, t.V, t.beta1, t.beta2, t.eps, t.t + 1)
    orc.apply_update(t.W, t.proj, N, lr, t.alpha, t.wd)
    t.t += 1
    return N


def test_signed_permutation_projector_equals_scaled_adam():
    # Adam is entry-wise, so a signed permutation as P gives exactly the plain Adam update.
    rng = np.random.default_rng(8)
    m, n = 5, 9
    perm = rng.permutation(m)
    P = np.zeros((m, m))
    P[perm, np.arange(m)] = rng.choice([-1.0, 1.0], m)
    W0 = rng.standard_normal((m, n))
    a = orc.GaLoreTensor(W0, rank=m, dtype="f64", auto_refresh=False); a.proj = P
    b = orc.GaLoreTensor(W0, rank=m, dtype="f64", auto_refresh=False); b.proj = np.eye(m)
    for _ in range(5):
        G = rng.standard_normal((m, n))
        _step_f64(a, G, 1e-2); _step_f64(b, G, 1e-2)
    np.testing.assert_allclose(a.W, b.W, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("shape", [(8, 14), (14, 8)])
def test_update_lies_in_projector_span_and_has_norm_of_N(shape):
    m, n = shape
    k, r = min(m, n), 3
    rng = np.random.default_rng(9)
    P = _orth(k, 11)[:, :r]
    W0 = rng.standard_normal(shape)
    t = orc.GaLoreTensor(W0, rank=r, dtype="f64", auto_refresh=False); t.proj = P
    lr = 3e-2
    N = _step_f64(t, rng.standard_normal(shape), lr)
    dW = t.W - W0
    if m <= n:
        np.testing.assert_allclose((np.eye(m) - P @ P.T) @ dW, 0, atol=1e-14)
    else:
        np.testing.assert_allclose(dW @ (np.eye(n) - P @ P.T), 0, atol=1e-14)
    assert np.linalg.norm(dW) == pytest.approx(lr * 0.25 * np.linalg.norm(N), rel=1e-12)


def test_update_opposes_the_gradient():
    # Descent direction: <W1 - W0, G> < 0 (the caller passes +grad and the update is subtracted).
    rng = np.random.default_rng(10)
    G = rng.standard_normal((6, 9))
    t = orc.GaLoreTensor(np.zeros((6, 9)), rank=4, dtype="f64", update_gap=10)
    t.step(G, 1e-2)
    assert np.sum(t.W * G) < 0


def test_weight_decay_hand_value_and_alpha_one_library_adamw():
    (W0, G, lr, alpha, wd, W1), = golden("weight_decay_hand.txt")
    t = orc.GaLoreTensor(np.array([[W0]]), rank=1, scale=alpha, weight_decay=wd, dtype="f64",
                         auto_refresh=False)
    t.proj = np.array([[1.0]])
    _step_f64(t, np.array([[G]]), lr)
    assert t.W[0, 0] == pytest.approx(W1, rel=1e-12)
    # alpha = 1, P = I: decoupled decay coincides with the library's AdamW.
    rng = np.random.default_rng(12)
    W0 = rng.standard_normal((4, 6))
    t = orc.GaLoreTensor(W0, rank=4, scale=1.0, weight_decay=0.1, dtype="f64", auto_refresh=False)
    t.proj = np.eye(4)
    p = torch.tensor(W0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([p], lr=1e-2, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.1)
    for _ in range(6):
        G = rng.standard_normal((4, 6))
        p.grad = torch.from_numpy(G.copy()); opt.step()
        _step_f64(t, G, 1e-2)
    np.testing.assert_allclose(t.W, p.detach().numpy(), rtol=1e-11)


def test_refresh_cadence_and_moments_survive_refresh():
    # t mod T == 0 with t starting at 0: refresh on calls 0 and T; moments are not reset.
    rng = np.random.default_rng(13)
    t = orc.GaLoreTensor(rng.standard_normal((6, 8)), rank=2, update_gap=3, dtype="f32")
    seen = []
    for step in range(7):
        before = None if t.proj is None else t.proj.copy()
        M_before = t.M.copy()
        t.step(rng.standard_normal((6, 8)), 1e-3)
        changed = before is None or not np.array_equal(before, t.proj)
        seen.append(changed)
        if step == 3:
            assert np.abs(M_before).max() > 0  # state carried into the refresh step
    assert seen == [True, False, False, True, False, False, True]
    assert t.t == 7


def test_storage_rounding_of_state():
    rng = np.random.default_rng(14)
    t = orc.GaLoreTensor(rng.standard_normal((6, 8)) * 0.02, rank=2, update_gap=3, dtype="bf16")
    t.step(rng.standard_normal((6, 8)), 1e-3)
    for a, dt in ((t.W, torch.bfloat16), (t.proj, torch.bfloat16), (t.M, torch.float32), (t.V, torch.float32)):
        back = torch.from_numpy(a).to(dt).to(torch.float64).numpy()
        np.testing.assert_array_equal(a, back)


def test_optimizer_state_element_count():
    # Sec. 4.2: GaLore keeps mr + 2nr state elements for an m x n weight (m <= n).
    m, n, r = 6, 10, 3
    t = orc.GaLoreTensor(np.zeros((m, n)), rank=r, update_gap=1, dtype="f32")
    t.step(np.random.default_rng(0).standard_normal((m, n)), 1e-3)
    assert t.proj.size + t.M.size + t.V.size == m * r + 2 * n * r
