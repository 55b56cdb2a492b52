"""C-ABI checks that need no GPU: the library loads, exports what the header declares, and
rejects bad arguments on the host before anything is launched."""
import ctypes
import os
import re

import pytest
import torch

from conftest import ROOT
from paper_2403_03507_amd import binding as gb


def _declared():
    text = open(os.path.join(ROOT, "include", "galore.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(galore_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = gb.lib()
    names = _declared()
    assert len(names) >= 12
    for n in names:
        assert hasattr(L, n), n
    assert sorted(gb.EXPORTS) == names


def test_status_strings():
    L = gb.lib()
    assert L.galore_status_string(0) == b"ok"
    assert L.galore_status_string(4) == b"rank out of range"


def _hp(**kw):
    return gb.make_hparams(kw.pop("rank", 4), **kw)


def _fake_state(k, r, l, left=True, dtype=gb.GALORE_F32, ptr=4096):
    mshape = (r, l) if left else (l, r)
    return gb.galore_state(gb.galore_tensor(ptr, k, r, r, dtype),
                           gb.galore_tensor(ptr, mshape[0], mshape[1], mshape[1], gb.GALORE_F32),
                           gb.galore_tensor(ptr, mshape[0], mshape[1], mshape[1], gb.GALORE_F32),
                           gb.galore_tensor(ptr, r, k, k, dtype))


def _status(fn, *a, **k):
    with pytest.raises(gb.GaloreError) as e:
        fn(*a, **k)
    return e.value.status


def test_workspace_bytes_counts_the_padded_gradient_copy():
    # a bf16 tensor with rows <= cols, rows % 64 == 0 and cols % 8 != 0 is projected from a copy of G
    # whose rows are padded to a multiple of 8: the step then needs R (r x 100008 fp32), N (r x 100003 bf16)
    # and the copy (64 x 100008 bf16); the same shape in fp32, transposed, with rows % 64 != 0 or with
    # cols % 8 == 0 needs no copy.  (Short, very wide tensors: there the step's need exceeds the refresh's.)
    hp = _hp(rank=8, refresh_iters=1)
    al = lambda x: (x + 255) // 256 * 256
    step = lambda m, n, pad, esz: al(8 * (pad if pad else n) * 4) + al(8 * n * esz) + (al(m * pad * esz) if pad else 0)
    ws = lambda m, n, dt: gb.galore_workspace_bytes(hp, [gb.shape_desc(m, n, dt)])
    assert ws(64, 100003, torch.bfloat16) == step(64, 100003, 100008, 2)
    assert ws(64, 100008, torch.bfloat16) == step(64, 100008, 0, 2)
    assert ws(64, 100003, torch.float32) == step(64, 100003, 0, 4)
    assert ws(100003, 64, torch.bfloat16) == step(64, 100003, 0, 2)
    assert ws(72, 100003, torch.bfloat16) == step(72, 100003, 0, 2)


def test_workspace_bytes_formula_and_errors():
    w = [gb.shape_desc(8, 16, torch.float32)]
    need = gb.galore_workspace_bytes(_hp(rank=4), w)
    assert need >= 4 * 16 * 4 * 2 and need % 256 == 0
    assert _status(gb.galore_workspace_bytes, _hp(rank=9), w) == 4          # rank > min(m, n)
    assert _status(gb.galore_workspace_bytes, _hp(rank=0), w) == 4
    assert _status(gb.galore_workspace_bytes, _hp(update_gap=0), w) == 1
    assert _status(gb.galore_workspace_bytes, _hp(beta1=1.0), w) == 1
    assert _status(gb.galore_workspace_bytes, _hp(refresh_iters=0), w) == 1
    assert _status(gb.galore_workspace_bytes, _hp(refresh_warm_iters=-1), w) == 1
    bad = [gb.galore_tensor(None, 8, 16, 12, 0)]                               # ld < cols
    assert _status(gb.galore_workspace_bytes, _hp(), bad) == 2
    bad = [gb.galore_tensor(None, 8, 16, 16, 7)]                               # unknown dtype
    assert _status(gb.galore_workspace_bytes, _hp(), bad) == 3


def test_init_validation_happens_before_any_device_work():
    hp = _hp(rank=4)
    w = [gb.shape_desc(8, 16, torch.float32)]
    ok_state = _fake_state(8, 4, 16)
    ws = 1 << 20
    # NULL workspace, misaligned workspace, too-small workspace
    assert _status(gb.galore_init, hp, w, [ok_state], 0, ws, stream=ctypes.c_void_p(None)) == 1
    assert _status(gb.galore_init, hp, w, [ok_state], 4096 + 8, ws, stream=ctypes.c_void_p(None)) == 5
    assert _status(gb.galore_init, hp, w, [ok_state], 4096, 256, stream=ctypes.c_void_p(None)) == 6
    # projector of the wrong shape / dtype
    s = _fake_state(8, 4, 16); s.proj.rows = 16
    assert _status(gb.galore_init, hp, w, [s], 4096, ws, stream=ctypes.c_void_p(None)) == 2
    s = _fake_state(8, 4, 16, dtype=gb.GALORE_BF16)
    assert _status(gb.galore_init, hp, w, [s], 4096, ws, stream=ctypes.c_void_p(None)) == 3
    # transposed projector copy: wrong shape / missing
    s = _fake_state(8, 4, 16); s.proj_t.rows, s.proj_t.cols, s.proj_t.ld = 8, 4, 4
    assert _status(gb.galore_init, hp, w, [s], 4096, ws, stream=ctypes.c_void_p(None)) == 2
    s = _fake_state(8, 4, 16); s.proj_t.data = None
    assert _status(gb.galore_init, hp, w, [s], 4096, ws, stream=ctypes.c_void_p(None)) == 1
    # moments: wrong orientation, wrong dtype, misaligned, NULL
    s = _fake_state(8, 4, 16, left=False)
    assert _status(gb.galore_init, hp, w, [s], 4096, ws, stream=ctypes.c_void_p(None)) == 2
    s = _fake_state(8, 4, 16); s.m.dtype = gb.GALORE_BF16
    assert _status(gb.galore_init, hp, w, [s], 4096, ws, stream=ctypes.c_void_p(None)) == 3
    s = _fake_state(8, 4, 16); s.v.data = 4096 + 4
    assert _status(gb.galore_init, hp, w, [s], 4096, ws, stream=ctypes.c_void_p(None)) == 5
    s = _fake_state(8, 4, 16); s.m.data = None
    assert _status(gb.galore_init, hp, w, [s], 4096, ws, stream=ctypes.c_void_p(None)) == 1
    # tall tensor: projector lives on the column side
    wt = [gb.shape_desc(16, 8, torch.float32)]
    s = _fake_state(8, 4, 16, left=True)   # moments given as r x rows: wrong for a RIGHT tensor
    assert _status(gb.galore_init, hp, wt, [s], 4096, ws, stream=ctypes.c_void_p(None)) == 2
    assert "moments" in gb.lib().galore_last_error(None).decode()


def test_stateless_calls_validate_shapes():
    L = gb.lib()
    T = gb.galore_tensor
    P = T(4096, 8, 4, 4, 0); Pt = T(4096, 4, 8, 8, 0); G = T(4096, 8, 16, 16, 0); R = T(4096, 4, 16, 16, 0)
    bad_R = T(4096, 16, 4, 4, 0)
    assert L.galore_project(ctypes.byref(Pt), ctypes.byref(G), ctypes.byref(bad_R), None) == 2
    assert L.galore_project(ctypes.byref(P), ctypes.byref(G), ctypes.byref(R), None) in (2, 4)   # untransposed projector
    Gb = T(4096, 8, 16, 16, 1)
    assert L.galore_project(ctypes.byref(Pt), ctypes.byref(Gb), ctypes.byref(R), None) == 3
    assert L.galore_project(None, ctypes.byref(G), ctypes.byref(R), None) == 1
    P9 = T(4096, 9, 8, 8, 0)
    assert L.galore_project(ctypes.byref(P9), ctypes.byref(G), ctypes.byref(R), None) == 4
    M = T(4096, 4, 16, 16, 0)
    assert L.galore_adam(ctypes.byref(R), ctypes.byref(M), ctypes.byref(M), ctypes.byref(M), 0, 0.9, 0.999, 1e-8, 0, None) == 1
    Mb = T(4096, 4, 16, 16, 1)
    assert L.galore_adam(ctypes.byref(R), ctypes.byref(Mb), ctypes.byref(M), ctypes.byref(M), 0, 0.9, 0.999, 1e-8, 1, None) == 3
    assert L.galore_adam(ctypes.byref(R), ctypes.byref(M), ctypes.byref(M), ctypes.byref(M), 1, 0.9, 0.999, 1e-8, 1, None) == 2  # N not transposed
    W = T(4096, 8, 16, 16, 0); N = T(4096, 4, 16, 16, 0)
    assert L.galore_project_back(ctypes.byref(P), ctypes.byref(N), ctypes.byref(W), 1e-3, 0.25, 0.0, None) == 2  # N must be 16 x 4
    assert L.galore_transpose(ctypes.byref(P), ctypes.byref(P), None) == 2


def test_null_context_calls():
    L = gb.lib()
    assert L.galore_step(None, None, None, 0, 0, 0.0) == 1
    assert L.galore_refresh_subspace(None, None, 0, 0) == 1
    assert L.galore_set_step(None, 0, 0) == 1
    L.galore_destroy(None)


def test_init_rejects_malformed_8bit_moment_state():
    hp = _hp(rank=4)
    w = [gb.shape_desc(8, 512, torch.float32)]
    ws = 1 << 22

    def q8_state():
        s = _fake_state(8, 4, 512)
        s.m.dtype = s.v.dtype = gb.GALORE_U8
        s.m_scale = gb.galore_tensor(4096, 4, 2, 2, gb.GALORE_F32)
        s.v_scale = gb.galore_tensor(4096, 4, 2, 2, gb.GALORE_F32)
        return s

    s = q8_state(); s.v.dtype = gb.GALORE_F32                    # one moment 8-bit, the other fp32
    assert _status(gb.galore_init, hp, w, [s], 4096, ws, stream=ctypes.c_void_p(None)) == 3
    s = q8_state(); s.m_scale.cols = s.m_scale.ld = 3            # wrong number of blocks per row
    assert _status(gb.galore_init, hp, w, [s], 4096, ws, stream=ctypes.c_void_p(None)) == 2
    s = q8_state(); s.v_scale.data = None
    assert _status(gb.galore_init, hp, w, [s], 4096, ws, stream=ctypes.c_void_p(None)) == 1
    s = q8_state(); s.m_scale.dtype = gb.GALORE_BF16
    assert _status(gb.galore_init, hp, w, [s], 4096, ws, stream=ctypes.c_void_p(None)) == 3
    # rows of the moment matrix that are not a multiple of 256 long
    w2 = [gb.shape_desc(8, 300, torch.float32)]
    s = _fake_state(8, 4, 300); s.m.dtype = s.v.dtype = gb.GALORE_U8
    assert _status(gb.galore_init, hp, w2, [s], 4096, ws, stream=ctypes.c_void_p(None)) == 9
    # 8-bit codes are a moment format only
    wq = [gb.shape_desc(8, 512, gb.GALORE_U8)]
    assert _status(gb.galore_workspace_bytes, hp, wq) == 3


def _two_sided_call(hp, w, g, st, ws_ptr, ws_bytes, t=0):
    L = gb.lib()
    gb._check(L.galore_two_sided_step(ctypes.byref(hp), ctypes.byref(w) if w is not None else None,
                                      ctypes.byref(g) if g is not None else None, ctypes.byref(st), t, 1e-3,
                                      ws_ptr, ws_bytes, None))


def test_two_sided_validation_happens_before_any_device_work():
    hp = _hp(rank=4, auto_refresh=False)
    m, n, r = 8, 16, 4
    w = gb.galore_tensor(4096, m, n, n, gb.GALORE_F32)
    g = gb.galore_tensor(4096, m, n, n, gb.GALORE_F32)

    def state():
        return gb.galore_two_sided_state(gb.galore_tensor(4096, m, r, r, gb.GALORE_F32), gb.galore_tensor(4096, n, r, r, gb.GALORE_F32),
                                         gb.galore_tensor(4096, r, r, r, gb.GALORE_F32), gb.galore_tensor(4096, r, r, r, gb.GALORE_F32))
    need = gb.galore_two_sided_workspace_bytes(hp, gb.shape_desc(m, n, torch.float32))
    assert need % 256 == 0 and need >= (r * m + 2 * r * n + 2 * r * r + n * r) * 4
    assert _status(gb.galore_two_sided_workspace_bytes, _hp(rank=9), gb.shape_desc(m, n, torch.float32)) == 4
    assert _status(_two_sided_call, hp, w, None, state(), 4096, need) == 1                  # G NULL
    assert _status(_two_sided_call, hp, w, g, state(), 0, need) == 6                         # workspace NULL
    assert _status(_two_sided_call, hp, w, g, state(), 4096 + 8, need) == 5                  # misaligned
    assert _status(_two_sided_call, hp, w, g, state(), 4096, need - 256) == 6                # too small
    assert _status(_two_sided_call, hp, w, g, state(), 4096, need, t=-1) == 1
    bad = gb.galore_tensor(4096, m, n + 1, n + 1, gb.GALORE_F32)
    assert _status(_two_sided_call, hp, w, bad, state(), 4096, need) == 2                   # G shape
    bad = gb.galore_tensor(4096, m, n, n, gb.GALORE_BF16)
    assert _status(_two_sided_call, hp, w, bad, state(), 4096, need) == 3                   # G dtype
    s = state(); s.q.rows = m
    assert _status(_two_sided_call, hp, w, g, s, 4096, need) == 7                            # Q is cols(W) x rank
    s = state(); s.p.dtype = gb.GALORE_BF16
    assert _status(_two_sided_call, hp, w, g, s, 4096, need) == 3
    s = state(); s.m.dtype = gb.GALORE_BF16
    assert _status(_two_sided_call, hp, w, g, s, 4096, need) == 3                            # moments are fp32
    s = state(); s.v.cols = r + 1; s.v.ld = r + 1
    assert _status(_two_sided_call, hp, w, g, s, 4096, need) == 7                            # moments are rank x rank
    assert _status(_two_sided_call, _hp(rank=9, auto_refresh=False), w, g, state(), 4096, need) == 4


def _adafactor_call(hp, w, g, st, ws_ptr, ws_bytes, t=0):
    L = gb.lib()
    gb._check(L.galore_adafactor_step(ctypes.byref(hp), ctypes.byref(w) if w is not None else None,
                                      ctypes.byref(g) if g is not None else None, ctypes.byref(st), t, 1e-3,
                                      ws_ptr, ws_bytes, None))


@pytest.mark.parametrize("shape", [(8, 16), (16, 8)])
def test_adafactor_validation_happens_before_any_device_work(shape):
    hp = _hp(rank=4, auto_refresh=False)
    m, n = shape
    r = 4
    k, rows, cols = min(m, n), (r if m <= n else m), (n if m <= n else r)      # R, M: r x n (m <= n) or m x r
    w = gb.galore_tensor(4096, m, n, n, gb.GALORE_F32)
    g = gb.galore_tensor(4096, m, n, n, gb.GALORE_F32)

    def state():
        return gb.galore_adafactor_state(gb.galore_tensor(4096, k, r, r, gb.GALORE_F32), gb.galore_tensor(4096, rows, cols, cols, gb.GALORE_F32),
                                         gb.galore_tensor(4096, 1, rows, rows, gb.GALORE_F32), gb.galore_tensor(4096, 1, cols, cols, gb.GALORE_F32))
    need = gb.galore_adafactor_workspace_bytes(hp, gb.shape_desc(m, n, torch.float32))
    assert need % 256 == 0 and need >= (r * k + 2 * rows * cols) * 4          # transposed projector, R, N
    assert _status(gb.galore_adafactor_workspace_bytes, _hp(rank=9), gb.shape_desc(m, n, torch.float32)) == 4
    assert _status(_adafactor_call, hp, w, None, state(), 4096, need) == 1                  # G NULL
    assert _status(_adafactor_call, hp, w, g, state(), 0, need) == 6                         # workspace NULL
    assert _status(_adafactor_call, hp, w, g, state(), 4096 + 8, need) == 5                  # misaligned
    assert _status(_adafactor_call, hp, w, g, state(), 4096, need - 256) == 6                # too small
    assert _status(_adafactor_call, hp, w, g, state(), 4096, need, t=-1) == 1
    bad = gb.galore_tensor(4096, m, n + 1, n + 1, gb.GALORE_F32)
    assert _status(_adafactor_call, hp, w, bad, state(), 4096, need) == 2                   # G shape
    s = state(); s.proj.rows = k + 1
    assert _status(_adafactor_call, hp, w, g, s, 4096, need) == 7                            # projector is min(rows, cols) x rank
    s = state(); s.proj.dtype = gb.GALORE_BF16
    assert _status(_adafactor_call, hp, w, g, s, 4096, need) == 3
    s = state(); s.m.rows = rows + 1
    assert _status(_adafactor_call, hp, w, g, s, 4096, need) == 7                            # M has R's shape
    s = state(); s.row.cols = rows + 1; s.row.ld = rows + 1
    assert _status(_adafactor_call, hp, w, g, s, 4096, need) == 7                            # one row statistic per row of M
    s = state(); s.col.dtype = gb.GALORE_BF16
    assert _status(_adafactor_call, hp, w, g, s, 4096, need) == 3                            # statistics are fp32
    # the stage call: shapes, dtypes, step number, workspace
    L = gb.lib()
    R = gb.galore_tensor(4096, rows, cols, cols, gb.GALORE_F32)
    st = state()

    def stage(R=R, M=st.m, row=st.row, col=st.col, N=None, beta1=0.9, k=1, ws=4096, nbytes=1 << 20):
        N = N if N is not None else gb.galore_tensor(4096, rows, cols, cols, gb.GALORE_F32)
        gb._check(L.galore_adafactor(ctypes.byref(R), ctypes.byref(M), ctypes.byref(row), ctypes.byref(col), ctypes.byref(N),
                                     beta1, k, ws, nbytes, None))
    assert _status(stage, k=0) == 1
    assert _status(stage, beta1=1.0) == 1
    assert _status(stage, nbytes=16) == 6
    assert _status(stage, N=gb.galore_tensor(4096, rows, cols + 1, cols + 1, gb.GALORE_F32)) == 2
    assert _status(stage, R=gb.galore_tensor(4096, rows, cols, cols, gb.GALORE_BF16)) == 3
