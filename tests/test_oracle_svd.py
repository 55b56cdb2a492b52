"""Pins for the oracle's Jacobi SVD and projector choice (Sec. 3.3 SVD equation; Algorithm 2)."""
import numpy as np
import pytest

from oracle import galore_oracle as orc


def _householder(v):
    v = np.asarray(v, dtype=np.float64)
    return np.eye(len(v)) - 2.0 * np.outer(v, v) / (v @ v)


def _known_svd(m, n):
    """G = U diag(s) V^T from explicitly built orthogonal factors (products of reflectors of
    simple integer vectors), distinct singular values: the decomposition is known by construction."""
    U = _householder(np.arange(1, m + 1)) @ _householder([(-1) ** i * (i % 3 + 1) for i in range(m)])
    V = _householder(np.arange(n, 0, -1)) @ _householder([(i * i) % 5 + 1 for i in range(n)])
    k = min(m, n)
    s = np.array([2.0 ** (k - i) + i for i in range(k)])  # strictly decreasing, all distinct
    G = (U[:, :k] * s) @ V[:, :k].T
    return G, U, s, V


@pytest.mark.parametrize("shape", [(8, 12), (12, 8)])
@pytest.mark.parametrize("r", [1, 3, 8])
def test_brute_force_known_factors(shape, r):
    m, n = shape
    G, U, s, V = _known_svd(m, n)
    proj, sig = orc.projector(G, r)
    np.testing.assert_allclose(sig, s, rtol=1e-12)
    truth = U[:, :r] if m <= n else V[:, :r]
    assert proj.shape == truth.shape
    # columns equal the true singular vectors up to the canonical sign
    for c in range(r):
        col = truth[:, c]
        col = col * np.sign(col[np.argmax(np.abs(col))])
        np.testing.assert_allclose(proj[:, c], col, atol=1e-11)


def test_orthonormal_columns_within_1e6():
    rng = np.random.default_rng(0)
    for (m, n, r) in [(40, 64, 16), (64, 40, 16), (33, 33, 33)]:
        proj, _ = orc.projector(rng.standard_normal((m, n)), r)
        assert np.abs(proj.T @ proj - np.eye(r)).max() <= 1e-6
        assert np.abs(proj.T @ proj - np.eye(r)).max() <= 1e-12


@pytest.mark.parametrize("shape,r", [((30, 50), 7), ((50, 30), 7), ((17, 23), 17)])
def test_against_lapack_svd(shape, r):
    rng = np.random.default_rng(1)
    m, n = shape
    # well-separated spectrum so individual vectors are well conditioned
    k = min(m, n)
    U, _ = np.linalg.qr(rng.standard_normal((m, k)))
    V, _ = np.linalg.qr(rng.standard_normal((n, k)))
    s = 1.5 ** -np.arange(k)
    G = (U * s) @ V.T
    proj, sig = orc.projector(G, r)
    Ul, Sl, Vlt = np.linalg.svd(G, full_matrices=False)
    np.testing.assert_allclose(sig, Sl, rtol=1e-9, atol=1e-14)
    ref = Ul[:, :r] if m <= n else Vlt[:r].T
    np.testing.assert_allclose(proj @ proj.T, ref @ ref.T, atol=1e-9)
    np.testing.assert_allclose(np.abs(np.sum(proj * ref, axis=0)), 1.0, atol=1e-9)


def test_eckart_young_residual_and_diagonalisation():
    rng = np.random.default_rng(2)
    G = rng.standard_normal((20, 35))
    r = 6
    P, sig = orc.projector(G, r)
    resid = np.linalg.norm(G - P @ (P.T @ G)) ** 2
    assert resid == pytest.approx(np.sum(sig[r:] ** 2), rel=1e-10)
    D = P.T @ G @ G.T @ P
    np.testing.assert_allclose(D, np.diag(sig[:r] ** 2), atol=1e-9)
    assert np.all(np.diff(sig) <= 1e-14)


def test_sign_convention_and_negated_gradient():
    rng = np.random.default_rng(3)
    G = rng.standard_normal((9, 13))
    P, _ = orc.projector(G, 4)
    for c in range(4):
        assert P[np.argmax(np.abs(P[:, c])), c] > 0
    # the paper feeds -grad to the SVD; the projector must not depend on that sign
    P2, _ = orc.projector(-G, 4)
    np.testing.assert_allclose(P, P2, atol=1e-12)


def test_rank_deficient_input():
    rng = np.random.default_rng(4)
    A = rng.standard_normal((10, 3)) @ rng.standard_normal((3, 15))
    P, sig = orc.projector(A, 3)
    assert np.all(sig[3:] < 1e-10 * sig[0])
    np.testing.assert_allclose(P @ (P.T @ A), A, atol=1e-10)


def _degenerate(m, n):
    rng = np.random.default_rng(6)
    cases = {"zero": np.zeros((m, n)), "rank2": rng.standard_normal((m, 2)) @ rng.standard_normal((2, n)),
             "constant": np.ones((m, n))}
    z = rng.standard_normal((m, n)); z[:, n // 3:] = 0.0
    cases["zero_columns"] = z          # rank n // 3 < m: a null space on the short side
    z = rng.standard_normal((m, n)); z[m // 3:] = 0.0
    cases["zero_rows"] = z
    z = np.zeros((m, n)); z[3, 7] = 2.0
    cases["single_entry"] = z
    return cases


@pytest.mark.parametrize("name", ["zero", "rank2", "constant", "zero_columns", "zero_rows", "single_entry"])
@pytest.mark.parametrize("shape", [(40, 90), (90, 40)])
def test_null_spaces_against_lapack(name, shape):
    # Matrices with a null space on the short side: rows that belong to zero singular values hold
    # rounding noise, which the stopping rule has to leave alone (it used to rotate them for ever).
    # Singular values against LAPACK's; the vectors of a null space are arbitrary, so for them only
    # orthonormality and the captured energy (Eckart-Young: sum of the r largest sigma^2) are fixed.
    m, n = shape
    G = _degenerate(m, n)[name]
    r = 12
    P, sig = orc.projector(G, r)
    sv = np.linalg.svd(G, compute_uv=False)
    np.testing.assert_allclose(sig[:len(sv)], sv, atol=1e-12 * max(sv[0], 1.0))
    assert np.abs(P.T @ P - np.eye(r)).max() <= 1e-12
    captured = np.linalg.norm(P.T @ G if m <= n else G @ P) ** 2
    np.testing.assert_allclose(captured, np.sum(sv[:r] ** 2), rtol=1e-10, atol=1e-300)


def test_transposed_input_swaps_sides():
    rng = np.random.default_rng(5)
    G = rng.standard_normal((7, 11))
    P, s1 = orc.projector(G, 3)       # left vectors of G
    Q, s2 = orc.projector(G.T, 3)     # right vectors of G^T = left vectors of G
    np.testing.assert_allclose(s1, s2, rtol=1e-12)
    np.testing.assert_allclose(P, Q, atol=1e-11)
