"""Pins for the oracle's two-sided rule (Definition 3.6, Sec. 3.3): G~ = P rho(P^T G Q) Q^T with rho = Adam,
P = [u_1..u_r], Q = [v_1..v_r] of G = U S V^T."""
import numpy as np
import pytest
import torch

from conftest import golden
from oracle import galore_oracle as orc


def _orth(n, seed):
    q, r = np.linalg.qr(np.random.default_rng(seed).standard_normal((n, n)))
    return q * np.sign(np.diag(r))


def test_hand_worked_step():
    R, M, V, N, *W1 = golden("two_sided_hand.txt")[0]
    G = np.array([[1.0, 2.0, 3.0], [4.0, 5.0, 6.0]])
    P = np.array([[0.6], [0.8]])
    Q = np.array([[0.0], [0.6], [0.8]])
    t = orc.GaLoreTensorTwoSided(np.zeros((2, 3)), 1, scale=0.25, dtype="f64", auto_refresh=False)
    t.set_projectors(P, Q)
    t.step(G, 0.1)
    assert t.last_R.shape == (1, 1)
    np.testing.assert_allclose(t.last_R[0, 0], R, rtol=1e-14)
    np.testing.assert_allclose(t.M[0, 0], M, rtol=1e-7)     # the moments are stored in fp32
    np.testing.assert_allclose(t.V[0, 0], V, rtol=1e-7)
    np.testing.assert_allclose(t.last_N[0, 0], N, rtol=1e-14)
    np.testing.assert_allclose(t.W.reshape(-1), W1, rtol=1e-13, atol=1e-18)


def test_projection_single_entry_indices():
    # One non-zero in each of P, G, Q: R[a, b] = P[i, a] G[i, j] Q[j, b] pins every index and both transposes.
    P = np.zeros((3, 2)); G = np.zeros((3, 4)); Q = np.zeros((4, 2))
    P[2, 1] = 2.0; G[2, 3] = 5.0; Q[3, 0] = 7.0
    want = np.zeros((2, 2)); want[1, 0] = 70.0
    np.testing.assert_array_equal(orc.project_two_sided(P, G, Q), want)
    # and the way back: W[i, j] -= P[i, a] N[a, b] Q[j, b]
    N = np.zeros((2, 2)); N[1, 0] = 3.0
    W = orc.apply_two_sided(np.zeros((3, 4)), P, N, Q, lr=1.0, alpha=1.0)
    want = np.zeros((3, 4)); want[2, 3] = -42.0
    np.testing.assert_array_equal(W, want)


def test_matches_library_matmul():
    rng = np.random.default_rng(3)
    for (m, n, r) in [(6, 11, 4), (11, 6, 3), (7, 7, 7)]:
        G = rng.standard_normal((m, n)); P = rng.standard_normal((m, r)); Q = rng.standard_normal((n, r))
        np.testing.assert_allclose(orc.project_two_sided(P, G, Q), P.T @ G @ Q, rtol=1e-12, atol=1e-12)
        N = rng.standard_normal((r, r)); W = rng.standard_normal((m, n))
        want = (1 - 0.1 * 0.5) * W - 0.1 * 0.25 * (P @ N @ Q.T)
        np.testing.assert_allclose(orc.apply_two_sided(W.copy(), P, N, Q, 0.1, 0.25, 0.5), want, rtol=1e-12, atol=1e-13)


def test_full_rank_identity_regulariser_reproduces_the_gradient():
    # Sec. 3.3 ("Difference between GaLore and LoRA"): with r = min(m, n) and rho = identity,
    # P P^T G Q Q^T = G.  For m != n the square factor is orthogonal and the other one is the
    # exact singular-vector block of G, so the statement holds for the projectors of the SVD equation.
    rng = np.random.default_rng(4)
    for (m, n) in [(6, 6), (5, 9), (9, 5)]:
        G = rng.standard_normal((m, n))
        r = min(m, n)
        P, Q, s = orc.projector_pair(G, r)
        R = orc.project_two_sided(P, G, Q)
        np.testing.assert_allclose(R, np.diag(s[:r]), atol=1e-10)          # R = S_r: diagonal, descending, positive
        W = orc.apply_two_sided(np.zeros((m, n)), P, R, Q, lr=-1.0, alpha=1.0)
        np.testing.assert_allclose(W, G, rtol=1e-10, atol=1e-10)


def test_identity_projectors_reduce_to_library_adam():
    # m = n = r, P = Q = I: R = G and the rule is plain Adam with learning rate lr * alpha.
    n, lr, alpha = 6, 1e-2, 0.25
    rng = np.random.default_rng(5)
    W0 = rng.standard_normal((n, n))
    t = orc.GaLoreTensorTwoSided(W0, n, scale=alpha, dtype="f64", auto_refresh=False)
    t.set_projectors(np.eye(n), np.eye(n))
    w = torch.tensor(W0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([w], lr=lr * alpha, betas=(0.9, 0.999), eps=1e-8)
    for k in range(12):
        G = rng.standard_normal((n, n)) * (1 + k)
        # the step from its pieces, without the class's rounding of the stored moments to fp32
        R = orc.project_two_sided(t.P, G, t.Q)
        N = orc.adam(R, t.M, t.V, t.beta1, t.beta2, t.eps, k + 1)
        orc.apply_two_sided(t.W, t.P, N, t.Q, lr, t.alpha)
        w.grad = torch.tensor(G)
        opt.step()
    np.testing.assert_allclose(t.W, w.detach().numpy(), rtol=1e-10, atol=1e-12)


def test_signed_permutations_commute_with_the_entrywise_map():
    # P, Q signed permutation blocks: R is a signed sub-block of G, Adam acts entry-wise, so the update is
    # alpha * Adam on those entries put back in place, zero elsewhere.
    rng = np.random.default_rng(6)
    m, n, r = 5, 7, 3
    rows, cols = [4, 0, 2], [6, 1, 3]
    sp, sq = np.array([1.0, -1.0, 1.0]), np.array([-1.0, -1.0, 1.0])
    P = np.zeros((m, r)); Q = np.zeros((n, r))
    P[rows, range(r)] = sp; Q[cols, range(r)] = sq
    G = rng.standard_normal((m, n))
    t = orc.GaLoreTensorTwoSided(np.zeros((m, n)), r, scale=0.5, dtype="f64", auto_refresh=False)
    t.set_projectors(P, Q)
    t.step(G, 0.1)
    sub = G[np.ix_(rows, cols)]
    n_sub = sub / (np.abs(sub) + 1e-8)                     # first Adam step: N = g / (|g| + eps)
    want = np.zeros((m, n)); want[np.ix_(rows, cols)] = -0.1 * 0.5 * n_sub
    np.testing.assert_allclose(t.W, want, rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("shape", [(8, 12, 3), (12, 8, 4)])
def test_update_lies_in_both_spans_and_has_norm_of_N(shape):
    m, n, r = shape
    rng = np.random.default_rng(7)
    P, Q = _orth(m, 1)[:, :r], _orth(n, 2)[:, :r]
    t = orc.GaLoreTensorTwoSided(rng.standard_normal((m, n)), r, scale=0.25, dtype="f64", auto_refresh=False)
    t.set_projectors(P, Q)
    W0 = t.W.copy()
    t.step(rng.standard_normal((m, n)), 0.05)
    dW = t.W - W0
    np.testing.assert_allclose((np.eye(m) - P @ P.T) @ dW, 0, atol=1e-14)
    np.testing.assert_allclose(dW @ (np.eye(n) - Q @ Q.T), 0, atol=1e-14)
    np.testing.assert_allclose(np.linalg.norm(dW), 0.05 * 0.25 * np.linalg.norm(t.last_N), rtol=1e-12)


def test_projector_pair_against_known_factors_and_lapack():
    # G built from explicit orthogonal factors and distinct singular values: ground truth by construction.
    m, n, r = 8, 12, 3
    U, Vf = _orth(m, 11), _orth(n, 12)
    s = np.array([9.0, 6.5, 4.0, 2.5, 1.2, 0.7, 0.3, 0.1])
    G = U @ np.diag(s) @ Vf[:, :m].T
    P, Q, sig = orc.projector_pair(G, r)
    np.testing.assert_allclose(sig, s, rtol=1e-11)
    for i in range(r):
        sgn = np.sign(P[:, i] @ U[:, i])
        np.testing.assert_allclose(P[:, i], sgn * U[:, i], atol=1e-10)
        np.testing.assert_allclose(Q[:, i], sgn * Vf[:, i], atol=1e-10)     # the SAME sign: the pair belongs together
    np.testing.assert_allclose(Q.T @ Q, np.eye(r), atol=1e-12)
    # leading part of G (Sec. 3.3, SVD equation) and Eckart-Young residual
    lead = P @ np.diag(sig[:r]) @ Q.T
    np.testing.assert_allclose(np.linalg.norm(G - lead) ** 2, (s[r:] ** 2).sum(), rtol=1e-10)
    # LAPACK, tall input
    rng = np.random.default_rng(13)
    G2 = rng.standard_normal((12, 7))
    P2, Q2, s2 = orc.projector_pair(G2, 4)
    Ul, sl, Vtl = np.linalg.svd(G2, full_matrices=False)
    np.testing.assert_allclose(s2, sl, rtol=1e-11)
    for i in range(4):
        sgn = np.sign(P2[:, i] @ Ul[:, i])
        np.testing.assert_allclose(P2[:, i], sgn * Ul[:, i], atol=1e-9)
        np.testing.assert_allclose(Q2[:, i], sgn * Vtl[i], atol=1e-9)
    np.testing.assert_allclose(P2.T @ P2, np.eye(4), atol=1e-12)
    # the block of the short side is the one-sided projector of Algorithm 2 (Q for a tall G, P for a wide one)
    np.testing.assert_array_equal(Q2, orc.projector(G2, 4)[0])
    np.testing.assert_array_equal(P, orc.projector(G, r)[0])


def test_projector_pair_rejects_zero_singular_value():
    G = np.outer([1.0, 2.0, 3.0], [1.0, 0.0, -1.0, 2.0])   # rank 1
    with pytest.raises(RuntimeError):
        orc.projector_pair(G, 2)
