"""GPU parity of the three per-step stages against the fp64 oracle, element by element.

Stages are called through the C ABI (galore_transpose / galore_project / galore_adam /
galore_project_back), which
run the same kernels galore_step runs.  Shapes span several 128x128 tiles, ragged tails, odd
sizes that force the unaligned load path, padded leading dimensions and both orientations.
"""
import numpy as np
import pytest
import torch

from helpers import TDT, TOL, dev, f32, relF, strided, to64

B1, B2, EPS = f32(0.9), f32(0.999), f32(1e-8)
from oracle import galore_oracle as orc
from paper_2403_03507_amd import binding as gb
from paper_2403_03507_amd import workloads as wl

pytestmark = pytest.mark.gpu

SHAPES = [  # (m, n, r)
    (512, 1376, 128),   # 60M gate/up
    (1376, 512, 128),   # 60M down (RIGHT)
    (512, 512, 128),
    (256, 300, 96),     # ragged n, not a multiple of 8
    (130, 257, 33),     # odd everything: unaligned path, partial tiles in every dimension
    (257, 130, 33),     # same, RIGHT
    (64, 64, 64),       # r = m = n, single partial tile
    (1, 5, 1),          # degenerate: one row
    (300, 1000, 300),   # r = m
    # r a multiple of 64 with an odd row length of W: the any-alignment variant of the large-tile weight update
    # (16-byte pieces at element alignment, the piece across a row's end element by element)
    (128, 333, 64),
    (64, 1021, 64),
    (1021, 65, 64),     # RIGHT
    (515, 67, 64),      # RIGHT, ragged last tile row
]


def _transposed(P):
    """The projector's transposed copy, made by the library's own transpose stage."""
    Pt = torch.empty(P.shape[1], P.shape[0], dtype=P.dtype, device=P.device)
    gb.galore_transpose(P, Pt)
    return Pt


def _long_by_r(N, m, n):
    """Device copy of N in the layout the back-projection reads: (long side) x r."""
    return (N.t().contiguous() if m <= n else N).cuda()


def _inputs(m, n, r, dtype, seed):
    k = min(m, n)
    G = wl.GradientSource(m, n, seed, "lowrank", dtype=dtype, signal_rank=min(8, k), noise=0.05).grad(0)
    P = wl.random_orthonormal(k, r, seed + 1).to(TDT[dtype])
    W = wl.make_weight(m, n, seed + 2, dtype)
    return W, G, P


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", SHAPES)
def test_project(shape, dtype):
    m, n, r = shape
    _, G, P = _inputs(m, n, r, dtype, 11)
    R_ref = orc.project(to64(P), to64(G))
    R = torch.full(R_ref.shape, float("nan"), dtype=torch.float32, device="cuda")
    gb.galore_project(_transposed(P.cuda()), G.cuda(), R)
    torch.cuda.synchronize()
    assert relF(to64(R), R_ref) <= 1e-5
    scale = np.abs(R_ref).max() + 1e-30
    assert np.abs(to64(R) - R_ref).max() <= 2e-5 * scale + 1e-6 * np.sqrt(max(m, n))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("pad", [8, 3])
def test_project_with_padded_leading_dimensions(dtype, pad):
    for (m, n, r) in [(200, 328, 40), (328, 200, 40)]:
        _, G, P = _inputs(m, n, r, dtype, 12)
        R_ref = orc.project(to64(P), to64(G))
        R = torch.empty(R_ref.shape, dtype=torch.float32, device="cuda")
        gb.galore_project(strided(_transposed(P.cuda()), pad), strided(G.cuda(), pad), R)
        torch.cuda.synchronize()
        assert relF(to64(R), R_ref) <= 1e-5


@pytest.mark.parametrize("transpose_n", [False, True])
@pytest.mark.parametrize("n_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("count_shape", [(128, 1376), (33, 257), (1, 3), (7, 1), (256, 4096), (64, 200), (72, 136)])
def test_adam(count_shape, n_dtype, transpose_n):
    rng = np.random.default_rng(5)
    shape = count_shape
    M = np.zeros(shape); V = np.zeros(shape)
    Md = torch.zeros(shape, dtype=torch.float32, device="cuda")
    Vd = torch.zeros(shape, dtype=torch.float32, device="cuda")
    Nd = torch.empty(shape[::-1] if transpose_n else shape, dtype=TDT[n_dtype], device="cuda")
    big = np.zeros(shape)
    for k in range(1, 5):
        R32 = (rng.standard_normal(shape) * 10.0 ** rng.integers(-4, 1, shape)).astype(np.float32)
        big = np.maximum(big, np.abs(R32))  # running size of the terms that entered M
        N_ref = orc.adam(R32.astype(np.float64), M, V, B1, B2, EPS, k)
        gb.galore_adam(torch.from_numpy(R32).cuda(), Md, Vd, Nd, transpose_n, 0.9, 0.999, 1e-8, k)
        torch.cuda.synchronize()
        N_dev = to64(Nd).T if transpose_n else to64(Nd)
        assert relF(to64(Md), M) <= 1e-6 and relF(to64(Vd), V) <= 1e-6
        # M is a sum that can cancel: bound the error by the size of the terms, not of the result
        assert np.all(np.abs(to64(Md) - M) <= 3e-7 * big + 1e-30)
        np.testing.assert_allclose(to64(Vd), V, rtol=2e-6, atol=1e-30)
        rel = 5e-6 if n_dtype == "f32" else 2.0 ** -8
        assert relF(N_dev, N_ref) <= rel
        assert np.all(np.abs(N_dev - N_ref) <= rel * np.abs(N_ref) + 1e-5)
        # oracle state follows fp32 storage, like the device state
        M[:] = orc.round_storage(M, "f32"); V[:] = orc.round_storage(V, "f32")


def test_adam_bias_correction_at_large_k():
    shape = (16, 64)
    rng = np.random.default_rng(6)
    M0 = rng.standard_normal(shape).astype(np.float32); V0 = (rng.standard_normal(shape) ** 2).astype(np.float32)
    R32 = rng.standard_normal(shape).astype(np.float32)
    for k in (7, 200, 100000):
        M = M0.astype(np.float64); V = V0.astype(np.float64)
        N_ref = orc.adam(R32.astype(np.float64), M, V, B1, B2, EPS, k)
        Md = torch.from_numpy(M0.copy()).cuda(); Vd = torch.from_numpy(V0.copy()).cuda()
        Nd = torch.empty(shape, dtype=torch.float32, device="cuda")
        gb.galore_adam(torch.from_numpy(R32).cuda(), Md, Vd, Nd, False, 0.9, 0.999, 1e-8, k)
        np.testing.assert_allclose(to64(Nd), N_ref, rtol=5e-6, atol=1e-12)


def _offset_view(t, pad=3):
    """t inside a wider buffer that starts one element into its allocation (leading dimension cols + pad, rows at
    arbitrary element offsets), NaN everywhere outside the matrix."""
    rows, cols = t.shape
    buf = torch.full((rows * (cols + pad) + 1,), float("nan"), dtype=t.dtype, device=t.device)
    v = buf[1:].view(rows, cols + pad)[:, :cols]
    v.copy_(t)
    v._buf = buf
    return v


def _check_project_back(m, n, r, dtype, seed=13, view=None, wd=0.1):
    """W <- (1 - lr wd) W - lr alpha (P N | N Q^T) on the device against the oracle, every entry."""
    W, _, P = _inputs(m, n, r, dtype, seed)
    rng = np.random.default_rng(seed + 1)
    nshape = (r, n) if m <= n else (m, r)
    N = torch.from_numpy(rng.uniform(-1, 1, nshape)).to(TDT[dtype])
    lr, alpha, wd = f32(1e-2), 0.25, f32(wd)
    W_ref = to64(W).copy()
    orc.apply_update(W_ref, to64(P), to64(N), lr, alpha, wd)
    Wd = W.cuda().clone() if view is None else view(W.cuda())
    gb.galore_project_back(P.cuda(), _long_by_r(N, m, n), Wd, lr, alpha, wd)
    torch.cuda.synchronize()
    assert relF(to64(Wd), W_ref) <= TOL[dtype]
    if dtype == "f32":
        np.testing.assert_allclose(to64(Wd), W_ref, rtol=1e-5, atol=1e-7)
    else:
        # bf16 storage: every entry within one bf16 ulp of the rounded oracle value.  Where the update cancels the
        # weight almost exactly the fp32 rounding of the r-term accumulation (worst case r 2^-24 of the terms' size),
        # not the ulp of the tiny result, bounds the difference.
        W_r = orc.round_storage(W_ref, "bf16")
        ulp = np.maximum(np.abs(W_r), 2.0 ** -126) * 2.0 ** -7
        cancel = r * 2.0 ** -24 * (np.abs(to64(W)) + np.abs(W_ref - to64(W)))
        assert np.all(np.abs(to64(Wd) - W_r) <= ulp + cancel)
        assert np.mean(to64(Wd) == W_r) >= 0.98
        if m * n >= 64:
            assert np.mean(to64(Wd) != to64(W)) > 0.5      # the update is far above an ulp here: it must show
    return Wd


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", SHAPES)
def test_project_back(shape, dtype):
    _check_project_back(*shape, dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_project_back_padded_weight(dtype):
    for (m, n, r) in [(200, 328, 40), (328, 200, 40), (128, 333, 64), (1021, 65, 64)]:
        Wd = _check_project_back(m, n, r, dtype, seed=15, view=lambda w: strided(w, 5), wd=0.0)
        assert torch.all(torch.isnan(Wd._base[:, n:]))  # padding untouched (the helper fills it with NaN)


@pytest.mark.parametrize("shape", [(128, 333, 64), (64, 1021, 64), (1021, 65, 64), (515, 67, 64), (192, 520, 128), (200, 328, 40)])
def test_project_back_weight_at_element_alignment_bf16(shape):
    # W one element into its allocation with an odd leading dimension: no row starts on a 4-byte boundary.  Every
    # entry is checked, and nothing outside the matrix may be written (the surroundings hold NaN).
    m, n, r = shape
    Wd = _check_project_back(m, n, r, "bf16", seed=17, view=_offset_view)
    body = Wd._buf[1:].view(m, -1)
    assert torch.isnan(Wd._buf[0]) and torch.isnan(body[:, n:]).all()


def test_project_back_llama1b_odd_row_length_full_size_bf16():
    # The 1B stack's 2048 x 5461 gate/up matrix at its rank (512) and the 5461 x 2048 down matrix: the any-alignment
    # weight update at the size the benchmark runs it (8 x 22 tiles, 8 K steps), every entry against the oracle.
    _check_project_back(2048, 5461, 512, "bf16", seed=19)
    _check_project_back(5461, 2048, 512, "bf16", seed=23)


def test_round_trip_identity_full_rank():
    # Sec. 3.3: r = min(m, n), identity in place of Adam  =>  P (P^T G) = G.
    m, n = 96, 200
    G = wl.GradientSource(m, n, 3, "lowrank", signal_rank=8, noise=0.05).grad(0)
    P = wl.random_orthonormal(m, m, 4)
    R = torch.empty(m, n, dtype=torch.float32, device="cuda")
    gb.galore_project(_transposed(P.cuda()), G.cuda(), R)
    W = torch.zeros(m, n, dtype=torch.float32, device="cuda")
    gb.galore_project_back(P.cuda(), R.t().contiguous(), W, -1.0, 1.0, 0.0)
    torch.cuda.synchronize()
    assert relF(to64(W), to64(G)) <= 1e-5


@pytest.mark.parametrize("r", [64, 192, 320])
@pytest.mark.parametrize("shape", [(4160, 4360), (4360, 4160)])
def test_more_tiles_than_compute_units_ragged_bf16(shape, r):
    # 17 x 18 = 306 tiles of 256 x 256 with partial tiles on both edges: every workgroup of the
    # persistent large-tile kernel walks more than one tile; r = 64 / 192 / 320 gives 1 / 3 / 5
    # K steps in the back-projection, i.e. its peeled last steps with and without the pipelined loop.
    m, n = shape
    W, G, P = _inputs(m, n, r, "bf16", 21)
    R_ref = orc.project(to64(P), to64(G))
    R = torch.full(R_ref.shape, float("nan"), dtype=torch.float32, device="cuda")
    gb.galore_project(_transposed(P.cuda()), G.cuda(), R)
    torch.cuda.synchronize()
    assert relF(to64(R), R_ref) <= 1e-5
    rng = np.random.default_rng(22)
    nshape = (r, n) if m <= n else (m, r)
    N = torch.from_numpy(rng.uniform(-1, 1, nshape)).to(torch.bfloat16)
    lr, alpha, wd = f32(1e-2), 0.25, f32(0.1)
    W_ref = to64(W).copy()
    orc.apply_update(W_ref, to64(P), to64(N), lr, alpha, wd)
    Wd = W.cuda().clone()
    gb.galore_project_back(P.cuda(), _long_by_r(N, m, n), Wd, lr, alpha, wd)
    torch.cuda.synchronize()
    W_r = orc.round_storage(W_ref, "bf16")
    ulp = np.maximum(np.abs(W_r), 2.0 ** -126) * 2.0 ** -7
    # among 18 M entries a few updates cancel the weight almost exactly; there the fp32 rounding of
    # the r-term accumulation (worst case r 2^-24 of the terms' size), not the bf16 ulp of the tiny
    # result, bounds the difference
    cancel = r * 2.0 ** -24 * (np.abs(to64(W)) + np.abs(W_ref - to64(W)))
    assert np.all(np.abs(to64(Wd) - W_r) <= ulp + cancel)
    assert np.mean(to64(Wd) == W_r) >= 0.98
