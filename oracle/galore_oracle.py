"""Python face of the CPU oracle (test infrastructure, never the product path).

Loads ``libgalore_oracle.so`` (plain C, fp64, built from ``galore_oracle.c`` in
this directory) and composes its routines into one GaLore step in the order of
Algorithm 2 of arXiv 2403.03507.  Only the tests, the smoke check and the
benchmark's cpu_baseline leg use this module.  It imports nothing from the HIP
package.

Readings of the paper taken here (the paper is silent or inconsistent):
  * M and V have the shape of R = P^T G (Algorithm 2 prints n x r for the
    initial moments but r x n for R).
  * The refresh test uses the 0-based counter t (first step refreshes); the
    bias correction uses k = t + 1, and corrected moments are temporaries.
  * eps is added after the square root of the corrected second moment
    (Algorithm 2 / the N_t equation, not the form in Sec. 3.1).
  * The caller passes the positive gradient and the update is subtracted; the
    paper negates the gradient and adds.  Same trajectory.
  * m > n mirrors Algorithm 2 with Q = V[:, :r], R = G Q, update N Q^T
    (Sec. 4.2, one-sided projection rule).
  * M and V are kept as they are when the projector changes.
  * Weight decay, not printed in the paper, is decoupled and not scaled by
    alpha: W <- (1 - lr*wd) W - lr*alpha*P N.  Parity unpinned beyond wd = 0.
  * Storage: the algorithm's state lives in the caller's dtypes, so after each
    step W and the projector are rounded (nearest-even) to the weight dtype and
    M, V to fp32; all arithmetic in between is fp64.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "galore_oracle.c")
_LIB = os.path.join(_HERE, "libgalore_oracle.so")


def build(force=False):
    """Compile the C oracle with gcc (OpenMP on outer loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_lib = None
_dp = ctypes.POINTER(ctypes.c_double)
_i64 = ctypes.c_int64
_f64 = ctypes.c_double


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        L = _lib
        L.oracle_num_threads.restype = ctypes.c_int
        L.oracle_set_num_threads.argtypes = [ctypes.c_int]
        L.oracle_round_bf16.argtypes = [_dp, _i64]
        L.oracle_round_f32.argtypes = [_dp, _i64]
        L.oracle_project_left.argtypes = [_dp, _dp, _dp, _i64, _i64, _i64]
        L.oracle_project_right.argtypes = [_dp, _dp, _dp, _i64, _i64, _i64]
        L.oracle_adam.argtypes = [_dp, _dp, _dp, _dp, _i64, _f64, _f64, _f64, _i64]
        L.oracle_adafactor.argtypes = [_dp, _dp, _dp, _dp, _dp, _i64, _i64, _f64, _f64, _f64, _f64, _i64]
        L.oracle_apply_left.argtypes = [_dp, _dp, _dp, _i64, _i64, _i64, _f64, _f64, _f64]
        L.oracle_apply_right.argtypes = [_dp, _dp, _dp, _i64, _i64, _i64, _f64, _f64, _f64]
        L.oracle_top_left_singular_vectors.argtypes = [_dp, _i64, _i64, _i64, _dp, _dp, _f64, ctypes.c_int]
        L.oracle_top_left_singular_vectors.restype = ctypes.c_int
        L.oracle_projector.argtypes = [_dp, _i64, _i64, _i64, _dp, _dp, _f64, ctypes.c_int]
        L.oracle_projector.restype = ctypes.c_int
        L.oracle_project_two_sided.argtypes = [_dp, _dp, _dp, _dp, _i64, _i64, _i64]
        L.oracle_apply_two_sided.argtypes = [_dp, _dp, _dp, _dp, _i64, _i64, _i64, _f64, _f64, _f64]
        L.oracle_projector_pair.argtypes = [_dp, _i64, _i64, _i64, _dp, _dp, _dp, _f64, ctypes.c_int]
        L.oracle_projector_pair.restype = ctypes.c_int
    return _lib


def _c(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a


def _p(a):
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_dp)


def num_threads():
    return int(lib().oracle_num_threads())


def set_num_threads(n):
    """Threads of the oracle's parallel loops from now on (for timing; results do not depend on it)."""
    lib().oracle_set_num_threads(int(n))


def round_storage(x, dtype):
    """Nearest-even rounding of an fp64 array to 'f32' or 'bf16' values (kept as fp64)."""
    y = _c(x).copy()
    if dtype == "bf16":
        lib().oracle_round_bf16(_p(y), y.size)
    elif dtype == "f32":
        lib().oracle_round_f32(_p(y), y.size)
    elif dtype != "f64":
        raise ValueError(dtype)
    return y


def project(proj, G):
    """R = P^T G (m <= n) or G Q (m > n)."""
    G = _c(G)
    proj = _c(proj)
    m, n = G.shape
    r = proj.shape[1]
    if m <= n:
        assert proj.shape[0] == m
        R = np.empty((r, n))
        lib().oracle_project_left(_p(proj), _p(G), _p(R), m, n, r)
    else:
        assert proj.shape[0] == n
        R = np.empty((m, r))
        lib().oracle_project_right(_p(G), _p(proj), _p(R), m, n, r)
    return R


def project_left(P, G):
    """R (r x n) = P^T G whatever the shape of G (used on column subsets of a LEFT tensor)."""
    G, P = _c(G), _c(P)
    (m, n), r = G.shape, P.shape[1]
    assert P.shape[0] == m
    R = np.empty((r, n))
    lib().oracle_project_left(_p(P), _p(G), _p(R), m, n, r)
    return R


def project_right(Q, G):
    """R (m x r) = G Q whatever the shape of G (used on row subsets of a RIGHT tensor)."""
    G, Q = _c(G), _c(Q)
    (m, n), r = G.shape, Q.shape[1]
    assert Q.shape[0] == n
    R = np.empty((m, r))
    lib().oracle_project_right(_p(G), _p(Q), _p(R), m, n, r)
    return R


def apply_left(W, P, N, lr, alpha, weight_decay=0.0):
    """In place W <- (1 - lr*wd) W - lr*alpha * P N, whatever the shape of W."""
    P, N = _c(P), _c(N)
    (m, n), r = W.shape, P.shape[1]
    assert P.shape[0] == m and N.shape == (r, n)
    lib().oracle_apply_left(_p(W), _p(P), _p(N), m, n, r, lr, alpha, weight_decay)
    return W


def apply_right(W, Q, N, lr, alpha, weight_decay=0.0):
    """In place W <- (1 - lr*wd) W - lr*alpha * N Q^T, whatever the shape of W."""
    Q, N = _c(Q), _c(N)
    (m, n), r = W.shape, Q.shape[1]
    assert Q.shape[0] == n and N.shape == (m, r)
    lib().oracle_apply_right(_p(W), _p(N), _p(Q), m, n, r, lr, alpha, weight_decay)
    return W


def adam(R, M, V, beta1, beta2, eps, k):
    """In-place moment update; returns N.  k is the 1-based step number."""
    R = _c(R)
    assert M.shape == R.shape and V.shape == R.shape
    N = np.empty_like(R)
    lib().oracle_adam(_p(R), _p(M), _p(V), _p(N), R.size, beta1, beta2, eps, int(k))
    return N


ADAFACTOR_DECAY_POW, ADAFACTOR_EPS1, ADAFACTOR_CLIP = -0.8, 1e-30, 1.0   # the publication's constants


def adafactor(R, M, rowv, colv, beta1, k, decay_pow=ADAFACTOR_DECAY_POW, eps1=ADAFACTOR_EPS1, clip_d=ADAFACTOR_CLIP):
    """Adafactor with first-order statistics on the projected gradient (see oracle_adafactor): updates M
    (R's shape), rowv (rows) and colv (cols) in place and returns N.  k is the 1-based step number."""
    R = _c(R)
    rows, cols = R.shape
    assert M.shape == R.shape and rowv.shape == (rows,) and colv.shape == (cols,)
    N = np.empty_like(R)
    lib().oracle_adafactor(_p(R), _p(M), _p(rowv), _p(colv), _p(N), rows, cols, beta1, decay_pow, eps1, clip_d, int(k))
    return N


def apply_update(W, proj, N, lr, alpha, weight_decay=0.0):
    """In place: W <- (1 - lr*wd) W - lr*alpha * (P N  or  N Q^T)."""
    m, n = W.shape
    proj = _c(proj)
    N = _c(N)
    r = proj.shape[1]
    if m <= n:
        assert N.shape == (r, n)
        lib().oracle_apply_left(_p(W), _p(proj), _p(N), m, n, r, lr, alpha, weight_decay)
    else:
        assert N.shape == (m, r)
        lib().oracle_apply_right(_p(W), _p(N), _p(proj), m, n, r, lr, alpha, weight_decay)
    return W


def top_left_singular_vectors(A, r, tol=1e-12, max_sweeps=60):
    A = _c(A)
    p, q = A.shape
    U = np.empty((p, r))
    s = np.empty(p)
    sweeps = lib().oracle_top_left_singular_vectors(_p(A), p, q, r, _p(U), _p(s), tol, max_sweeps)
    if sweeps < 0:
        raise RuntimeError("Jacobi SVD did not converge")
    return U, s


def projector(G, r, tol=1e-12, max_sweeps=60):
    """P = U[:, :r] (m <= n) or Q = V[:, :r] (m > n), plus all singular values."""
    G = _c(G)
    m, n = G.shape
    k = min(m, n)
    proj = np.empty((k, r))
    s = np.empty(k)
    sweeps = lib().oracle_projector(_p(G), m, n, r, _p(proj), _p(s), tol, max_sweeps)
    if sweeps < 0:
        raise RuntimeError("Jacobi SVD did not converge")
    return proj, s


def project_two_sided(P, G, Q):
    """R (r x r) = P^T G Q  (Definition 3.6)."""
    P, G, Q = _c(P), _c(G), _c(Q)
    (m, n), r = G.shape, P.shape[1]
    assert P.shape == (m, r) and Q.shape == (n, r)
    R = np.empty((r, r))
    lib().oracle_project_two_sided(_p(P), _p(G), _p(Q), _p(R), m, n, r)
    return R


def apply_two_sided(W, P, N, Q, lr, alpha, weight_decay=0.0):
    """In place W <- (1 - lr*wd) W - lr*alpha * P N Q^T  (Definition 3.6, N r x r)."""
    P, N, Q = _c(P), _c(N), _c(Q)
    (m, n), r = W.shape, P.shape[1]
    assert P.shape == (m, r) and Q.shape == (n, r) and N.shape == (r, r)
    lib().oracle_apply_two_sided(_p(W), _p(P), _p(N), _p(Q), m, n, r, lr, alpha, weight_decay)
    return W


def projector_pair(G, r, tol=1e-12, max_sweeps=60):
    """P = [u_1..u_r], Q = [v_1..v_r] of G = U S V^T (Sec. 3.3), paired signs, plus the singular values."""
    G = _c(G)
    m, n = G.shape
    P, Q, s = np.empty((m, r)), np.empty((n, r)), np.empty(min(m, n))
    rc = lib().oracle_projector_pair(_p(G), m, n, r, _p(P), _p(Q), _p(s), tol, max_sweeps)
    if rc == -2:
        raise RuntimeError("singular value r is zero: the right vector is not determined")
    if rc < 0:
        raise RuntimeError("Jacobi SVD did not converge")
    return P, Q, s


class GaLoreTensorTwoSided:
    """One weight matrix under the two-sided rule of Definition 3.6 with rho = Adam (the update block of
    Algorithm 2 applied to the r x r matrix R = P^T G Q); fp64 arithmetic, storage-dtype state."""

    def __init__(self, W, rank, update_gap=200, scale=0.25, beta1=0.9, beta2=0.999,
                 eps=1e-8, weight_decay=0.0, dtype="f32", auto_refresh=True):
        self.dtype = dtype
        self.W = round_storage(W, dtype)
        self.m, self.n = self.W.shape
        self.r = int(rank)
        assert 1 <= self.r <= min(self.m, self.n)
        self.T = int(update_gap)
        self.alpha, self.beta1, self.beta2 = float(scale), float(beta1), float(beta2)
        self.eps, self.wd = float(eps), float(weight_decay)
        self.auto_refresh = auto_refresh
        self.M = np.zeros((self.r, self.r))
        self.V = np.zeros((self.r, self.r))
        self.P = self.Q = self.sigma = None
        self.t = 0
        self.last_R = self.last_N = None

    def refresh(self, G):
        P, Q, s = projector_pair(G, self.r)
        self.P, self.Q, self.sigma = round_storage(P, self.dtype), round_storage(Q, self.dtype), s
        return self.P, self.Q

    def set_projectors(self, P, Q):
        self.P, self.Q = round_storage(P, self.dtype), round_storage(Q, self.dtype)

    def step(self, G, lr):
        G = round_storage(G, self.dtype)
        if self.auto_refresh and self.t % self.T == 0:
            self.refresh(G)
        R = project_two_sided(self.P, G, self.Q)
        N = adam(R, self.M, self.V, self.beta1, self.beta2, self.eps, self.t + 1)
        self.last_R, self.last_N = R, N
        apply_two_sided(self.W, self.P, N, self.Q, lr, self.alpha, self.wd)
        self.W = round_storage(self.W, self.dtype)
        self.M = round_storage(self.M, "f32")
        self.V = round_storage(self.V, "f32")
        self.t += 1
        return self.W


class GaLoreTensor:
    """One weight matrix under Algorithm 2, fp64 arithmetic, storage-dtype state."""

    def __init__(self, W, rank, update_gap=200, scale=0.25, beta1=0.9, beta2=0.999,
                 eps=1e-8, weight_decay=0.0, dtype="f32", auto_refresh=True):
        self.dtype = dtype
        self.W = round_storage(W, dtype)
        self.m, self.n = self.W.shape
        self.r = int(rank)
        assert 1 <= self.r <= min(self.m, self.n)
        self.T = int(update_gap)
        self.alpha, self.beta1, self.beta2 = float(scale), float(beta1), float(beta2)
        self.eps, self.wd = float(eps), float(weight_decay)
        self.auto_refresh = auto_refresh
        self.left = self.m <= self.n
        shape = (self.r, self.n) if self.left else (self.m, self.r)
        self.M = np.zeros(shape)
        self.V = np.zeros(shape)
        self.proj = None
        self.sigma = None
        self.t = 0
        self.last_R = None
        self.last_N = None

    def refresh(self, G):
        P, s = projector(G, self.r)
        self.proj = round_storage(P, self.dtype)
        self.sigma = s
        return self.proj

    def set_projector(self, proj):
        self.proj = round_storage(proj, self.dtype)

    def step(self, G, lr):
        G = round_storage(G, self.dtype)
        if self.auto_refresh and self.t % self.T == 0:
            self.refresh(G)
        R = project(self.proj, G)
        N = adam(R, self.M, self.V, self.beta1, self.beta2, self.eps, self.t + 1)
        self.last_R, self.last_N = R, N
        apply_update(self.W, self.proj, N, lr, self.alpha, self.wd)
        self.W = round_storage(self.W, self.dtype)
        self.M = round_storage(self.M, "f32")
        self.V = round_storage(self.V, "f32")
        self.t += 1
        return self.W


class GaLoreAdafactorTensor:
    """One weight matrix under Algorithm 2 with Adafactor (first-order statistics on) in place of Adam as the
    optimizer of the projected gradient: fp64 arithmetic, storage-dtype state (W, P in the tensor's dtype; M,
    the row and the column statistics fp32)."""

    def __init__(self, W, rank, update_gap=200, scale=0.25, beta1=0.9, weight_decay=0.0, dtype="f32", auto_refresh=True):
        self.dtype = dtype
        self.W = round_storage(W, dtype)
        self.m, self.n = self.W.shape
        self.r = int(rank)
        assert 1 <= self.r <= min(self.m, self.n)
        self.T, self.alpha, self.beta1, self.wd = int(update_gap), float(scale), float(beta1), float(weight_decay)
        self.auto_refresh = auto_refresh
        self.left = self.m <= self.n
        shape = (self.r, self.n) if self.left else (self.m, self.r)
        self.M = np.zeros(shape)
        self.rowv = np.zeros(shape[0])
        self.colv = np.zeros(shape[1])
        self.proj = None
        self.t = 0

    def refresh(self, G):
        P, _ = projector(G, self.r)
        self.proj = round_storage(P, self.dtype)
        return self.proj

    def set_projector(self, proj):
        self.proj = round_storage(proj, self.dtype)

    def step(self, G, lr):
        G = round_storage(G, self.dtype)
        if self.auto_refresh and self.t % self.T == 0:
            self.refresh(G)
        R = project(self.proj, G)
        N = adafactor(R, self.M, self.rowv, self.colv, self.beta1, self.t + 1)
        self.last_R, self.last_N = R, N
        apply_update(self.W, self.proj, N, lr, self.alpha, self.wd)
        self.W = round_storage(self.W, self.dtype)
        self.M = round_storage(self.M, "f32")
        self.rowv = round_storage(self.rowv, "f32")
        self.colv = round_storage(self.colv, "f32")
        self.t += 1
        return self.W
