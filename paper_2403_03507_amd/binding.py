"""ctypes face of ``libgalore.so`` (the C ABI in ``include/galore.h``).

Argument marshalling only: every step of the optimizer runs inside the HIP library.
PyTorch is used for device memory and for the current HIP stream.  There is no fallback:
if the library is missing this module raises.
"""
import ctypes
import os

import torch  # also loads the HIP runtime the library binds to

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgalore.so")

GALORE_OK = 0
STATUS_NAMES = {0: "OK", 1: "INVALID_ARG", 2: "SHAPE", 3: "DTYPE", 4: "RANK", 5: "ALIGN",
                6: "WORKSPACE", 7: "STATE", 8: "HIP", 9: "UNIMPLEMENTED"}
GALORE_F32, GALORE_BF16, GALORE_U8 = 0, 1, 2
_DTYPES = {torch.float32: GALORE_F32, torch.bfloat16: GALORE_BF16, torch.uint8: GALORE_U8}


class galore_tensor(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("ld", ctypes.c_int64), ("dtype", ctypes.c_int32)]


class galore_state(ctypes.Structure):
    _fields_ = [("proj", galore_tensor), ("m", galore_tensor), ("v", galore_tensor), ("proj_t", galore_tensor),
                ("m_scale", galore_tensor), ("v_scale", galore_tensor)]


class galore_two_sided_state(ctypes.Structure):
    _fields_ = [("p", galore_tensor), ("q", galore_tensor), ("m", galore_tensor), ("v", galore_tensor)]


class galore_adafactor_state(ctypes.Structure):
    _fields_ = [("proj", galore_tensor), ("m", galore_tensor), ("row", galore_tensor), ("col", galore_tensor)]


class galore_hparams(ctypes.Structure):
    _fields_ = [("rank", ctypes.c_int32), ("update_gap", ctypes.c_int32), ("scale", ctypes.c_float),
                ("beta1", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float),
                ("weight_decay", ctypes.c_float), ("refresh_iters", ctypes.c_int32),
                ("auto_refresh", ctypes.c_int32), ("refresh_warm_iters", ctypes.c_int32), ("seed", ctypes.c_uint64)]


class GaloreError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("galore status %d (%s): %s" % (status, STATUS_NAMES.get(status, "?"), message))
        self.status = status


EXPORTS = ["galore_status_string", "galore_workspace_bytes", "galore_init", "galore_step", "galore_step_static",
           "galore_refresh_subspace", "galore_get_step", "galore_set_step", "galore_last_error",
           "galore_destroy", "galore_transpose", "galore_project", "galore_adam", "galore_adam_q8", "galore_project_back",
           "galore_profile_start", "galore_profile_stop", "galore_set_concurrency",
           "galore_set_call_overlap", "galore_set_fused_adam", "galore_join", "galore_get_stream",
           "galore_two_sided_workspace_bytes", "galore_two_sided_step", "galore_two_sided_refresh",
           "galore_adafactor_workspace_bytes", "galore_adafactor_step", "galore_adafactor_refresh", "galore_adafactor"]
STAGES = ["project_left", "project_right", "adam", "back", "transpose", "refresh"]

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libgalore.so is not built: run `python -m paper_2403_03507_amd.build` "
                               "(or __graft_entry__.build()) first")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
        tp, sp, hp = ctypes.POINTER(galore_tensor), ctypes.POINTER(galore_state), ctypes.POINTER(galore_hparams)
        L.galore_status_string.argtypes = [ctypes.c_int]
        L.galore_status_string.restype = ctypes.c_char_p
        L.galore_workspace_bytes.argtypes = [hp, tp, i32, ctypes.POINTER(ctypes.c_size_t)]
        L.galore_init.argtypes = [ctypes.POINTER(vp), hp, tp, sp, i32, vp, ctypes.c_size_t, vp]
        L.galore_step.argtypes = [vp, tp, tp, i32, i32, f32]
        L.galore_step_static.argtypes = [vp, tp, tp, i32, i32, f32]
        L.galore_refresh_subspace.argtypes = [vp, tp, i32, i32]
        L.galore_get_step.argtypes = [vp, i32, ctypes.POINTER(i64)]
        L.galore_set_step.argtypes = [vp, i32, i64]
        L.galore_last_error.argtypes = [vp]
        L.galore_last_error.restype = ctypes.c_char_p
        L.galore_destroy.argtypes = [vp]
        L.galore_destroy.restype = None
        L.galore_transpose.argtypes = [tp, tp, vp]
        L.galore_project.argtypes = [tp, tp, tp, vp]
        L.galore_adam.argtypes = [tp, tp, tp, tp, i32, f32, f32, f32, i64, vp]
        L.galore_adam_q8.argtypes = [tp, tp, tp, tp, tp, tp, i32, f32, f32, f32, i64, vp]
        L.galore_project_back.argtypes = [tp, tp, tp, f32, f32, f32, vp]
        L.galore_set_concurrency.argtypes = [vp, i32]
        L.galore_set_call_overlap.argtypes = [vp, i32]
        L.galore_set_fused_adam.argtypes = [vp, i32]
        L.galore_join.argtypes = [vp]
        L.galore_get_stream.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_void_p)]
        tsp = ctypes.POINTER(galore_two_sided_state)
        L.galore_two_sided_workspace_bytes.argtypes = [hp, tp, ctypes.POINTER(ctypes.c_size_t)]
        L.galore_two_sided_step.argtypes = [hp, tp, tp, tsp, i64, f32, vp, ctypes.c_size_t, vp]
        L.galore_two_sided_refresh.argtypes = [hp, tp, tsp, vp, ctypes.c_size_t, vp]
        afp = ctypes.POINTER(galore_adafactor_state)
        L.galore_adafactor_workspace_bytes.argtypes = [hp, tp, ctypes.POINTER(ctypes.c_size_t)]
        L.galore_adafactor_step.argtypes = [hp, tp, tp, afp, i64, f32, vp, ctypes.c_size_t, vp]
        L.galore_adafactor_refresh.argtypes = [hp, tp, afp, vp, ctypes.c_size_t, vp]
        L.galore_adafactor.argtypes = [tp, tp, tp, tp, tp, f32, i64, vp, ctypes.c_size_t, vp]
        L.galore_profile_start.argtypes = [vp]
        L.galore_profile_stop.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
        _lib = L
    return _lib


def _check(status, ctx=None):
    if status != GALORE_OK:
        msg = lib().galore_last_error(ctx)
        raise GaloreError(status, msg.decode() if msg else "")


def desc(t):
    """galore_tensor view of a 2-D torch tensor with unit column stride."""
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError("need a 2-D row-major tensor")
    return galore_tensor(t.data_ptr(), t.shape[0], t.shape[1], t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1]),
                         _DTYPES[t.dtype])


def shape_desc(rows, cols, dtype, ld=None, data=None):
    return galore_tensor(data, rows, cols, cols if ld is None else ld, _DTYPES[dtype] if not isinstance(dtype, int) else dtype)


def _arr(items, typ):
    if isinstance(items, ctypes.Array) and items._type_ is typ:
        return items      # marshalled once by the caller (tensor_array): per-layer calls of small stacks are host-bound
    return (typ * len(items))(*items)


def tensor_array(descs):
    """A C array of galore_tensor for the list arguments of galore_step / galore_refresh_subspace, built once
    and reused while the tensors stay where they are."""
    return _arr(list(descs), galore_tensor)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_hparams(rank, update_gap=200, scale=0.25, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0,
                 refresh_iters=6, auto_refresh=True, seed=0, refresh_warm_iters=0):
    return galore_hparams(rank, update_gap, scale, beta1, beta2, eps, weight_decay, refresh_iters,
                          1 if auto_refresh else 0, refresh_warm_iters, seed)


# ---- the C calls, same names -------------------------------------------------------------------

def galore_workspace_bytes(hp, w_descs):
    out = ctypes.c_size_t(0)
    _check(lib().galore_workspace_bytes(ctypes.byref(hp), _arr(w_descs, galore_tensor), len(w_descs), ctypes.byref(out)))
    return out.value


def galore_init(hp, w_descs, states, workspace_ptr, workspace_bytes, stream=None):
    ctx = ctypes.c_void_p(None)
    st = lib().galore_init(ctypes.byref(ctx), ctypes.byref(hp), _arr(w_descs, galore_tensor), _arr(states, galore_state),
                           len(w_descs), ctypes.c_void_p(workspace_ptr), workspace_bytes,
                           stream if stream is not None else _stream())
    _check(st)
    return ctx


def galore_step(ctx, w_descs, g_descs, first, count, lr):
    _check(lib().galore_step(ctx, _arr(w_descs, galore_tensor), _arr(g_descs, galore_tensor), first, count, lr), ctx)


def galore_step_static(ctx, w_descs, g_descs, first, count, lr):
    _check(lib().galore_step_static(ctx, _arr(w_descs, galore_tensor), _arr(g_descs, galore_tensor), first, count, lr), ctx)


def galore_refresh_subspace(ctx, g_descs, first, count):
    _check(lib().galore_refresh_subspace(ctx, _arr(g_descs, galore_tensor), first, count), ctx)


def galore_get_step(ctx, tensor):
    t = ctypes.c_int64(0)
    _check(lib().galore_get_step(ctx, tensor, ctypes.byref(t)))
    return t.value


def galore_set_step(ctx, tensor, t):
    _check(lib().galore_set_step(ctx, tensor, t), ctx)


def galore_destroy(ctx):
    lib().galore_destroy(ctx)


def galore_transpose(src, dst):
    _check(lib().galore_transpose(ctypes.byref(desc(src)), ctypes.byref(desc(dst)), _stream()))


def galore_project(proj_t, G, R):
    _check(lib().galore_project(ctypes.byref(desc(proj_t)), ctypes.byref(desc(G)), ctypes.byref(desc(R)), _stream()))


def galore_adam(R, M, V, N, transpose_n, beta1, beta2, eps, k):
    _check(lib().galore_adam(ctypes.byref(desc(R)), ctypes.byref(desc(M)), ctypes.byref(desc(V)), ctypes.byref(desc(N)),
                             1 if transpose_n else 0, beta1, beta2, eps, k, _stream()))


def galore_adam_q8(R, Mc, Vc, Ms, Vs, N, transpose_n, beta1, beta2, eps, k):
    _check(lib().galore_adam_q8(ctypes.byref(desc(R)), ctypes.byref(desc(Mc)), ctypes.byref(desc(Vc)), ctypes.byref(desc(Ms)),
                                ctypes.byref(desc(Vs)), ctypes.byref(desc(N)), 1 if transpose_n else 0, beta1, beta2, eps, k,
                                _stream()))


def galore_project_back(proj, N, W, lr, scale, weight_decay=0.0):
    _check(lib().galore_project_back(ctypes.byref(desc(proj)), ctypes.byref(desc(N)), ctypes.byref(desc(W)), lr, scale,
                                     weight_decay, _stream()))


def galore_set_concurrency(ctx, lanes):
    _check(lib().galore_set_concurrency(ctx, lanes), ctx)


def galore_set_call_overlap(ctx, on):
    _check(lib().galore_set_call_overlap(ctx, int(on)), ctx)  # False/0 off, True/1/2 two calls in flight, 3 three


def galore_set_fused_adam(ctx, on):
    _check(lib().galore_set_fused_adam(ctx, 1 if on else 0), ctx)


def galore_join(ctx):
    _check(lib().galore_join(ctx), ctx)


def galore_get_stream(ctx, which):
    out = ctypes.c_void_p(None)
    _check(lib().galore_get_stream(ctx, which, ctypes.byref(out)), ctx)
    return out.value


def galore_profile_start(ctx):
    _check(lib().galore_profile_start(ctx), ctx)


def galore_profile_stop(ctx):
    """-> {stage name: (milliseconds, launches)}"""
    n = len(STAGES)
    ms = (ctypes.c_double * n)()
    cnt = (ctypes.c_int64 * n)()
    _check(lib().galore_profile_stop(ctx, ms, cnt), ctx)
    return {STAGES[i]: (ms[i], cnt[i]) for i in range(n)}


def galore_two_sided_workspace_bytes(hp, w_desc):
    out = ctypes.c_size_t(0)
    _check(lib().galore_two_sided_workspace_bytes(ctypes.byref(hp), ctypes.byref(w_desc), ctypes.byref(out)))
    return out.value


def galore_two_sided_step(hp, W, G, state, t, lr, workspace):
    _check(lib().galore_two_sided_step(ctypes.byref(hp), ctypes.byref(desc(W)), ctypes.byref(desc(G)), ctypes.byref(state),
                                       int(t), lr, workspace.data_ptr(), workspace.numel(), _stream()))


def galore_two_sided_refresh(hp, G, state, workspace):
    _check(lib().galore_two_sided_refresh(ctypes.byref(hp), ctypes.byref(desc(G)), ctypes.byref(state),
                                          workspace.data_ptr(), workspace.numel(), _stream()))


class GaLoreTwoSided:
    """One weight matrix under the two-sided rule (Definition 3.6): owns P, Q, the r x r moments and the
    workspace (torch memory) and keeps the step count; all arithmetic happens in the library."""

    def __init__(self, weight, rank, device="cuda", **hparams):
        m, n = weight.shape
        self.hp = make_hparams(rank, **hparams)
        self.P = torch.zeros(m, rank, dtype=weight.dtype, device=device)
        self.Q = torch.zeros(n, rank, dtype=weight.dtype, device=device)
        self.M = torch.zeros(rank, rank, dtype=torch.float32, device=device)
        self.V = torch.zeros(rank, rank, dtype=torch.float32, device=device)
        nbytes = galore_two_sided_workspace_bytes(self.hp, shape_desc(m, n, weight.dtype))
        self.workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
        self.t = 0

    def state(self):
        return galore_two_sided_state(desc(self.P), desc(self.Q), desc(self.M), desc(self.V))

    def refresh(self, grad):
        galore_two_sided_refresh(self.hp, grad, self.state(), self.workspace)

    def step(self, weight, grad, lr):
        galore_two_sided_step(self.hp, weight, grad, self.state(), self.t, lr, self.workspace)
        self.t += 1


def galore_adafactor_workspace_bytes(hp, w_desc):
    out = ctypes.c_size_t(0)
    _check(lib().galore_adafactor_workspace_bytes(ctypes.byref(hp), ctypes.byref(w_desc), ctypes.byref(out)))
    return out.value


def galore_adafactor_step(hp, W, G, state, t, lr, workspace):
    _check(lib().galore_adafactor_step(ctypes.byref(hp), ctypes.byref(desc(W)), ctypes.byref(desc(G)), ctypes.byref(state),
                                       int(t), lr, workspace.data_ptr(), workspace.numel(), _stream()))


def galore_adafactor_refresh(hp, G, state, workspace):
    _check(lib().galore_adafactor_refresh(ctypes.byref(hp), ctypes.byref(desc(G)), ctypes.byref(state),
                                          workspace.data_ptr(), workspace.numel(), _stream()))


def galore_adafactor(R, M, row, col, N, beta1, k, workspace):
    """Stage call: the Adafactor update block on the projected gradient R; row, col are 1-D fp32 tensors."""
    _check(lib().galore_adafactor(ctypes.byref(desc(R)), ctypes.byref(desc(M)), ctypes.byref(desc(row.view(1, -1))),
                                  ctypes.byref(desc(col.view(1, -1))), ctypes.byref(desc(N)), beta1, int(k),
                                  workspace.data_ptr(), workspace.numel(), _stream()))


class GaLoreAdafactor:
    """One weight matrix under GaLore with Adafactor (first-order statistics on): owns the projector, the first
    moment, the row and column statistics and the workspace (torch memory) and keeps the step count; all arithmetic
    happens in the library."""

    def __init__(self, weight, rank, device="cuda", **hparams):
        m, n = weight.shape
        self.hp = make_hparams(rank, **hparams)
        shape = (rank, n) if m <= n else (m, rank)
        self.proj = torch.zeros(min(m, n), rank, dtype=weight.dtype, device=device)
        self.M = torch.zeros(*shape, dtype=torch.float32, device=device)
        self.row = torch.zeros(shape[0], dtype=torch.float32, device=device)
        self.col = torch.zeros(shape[1], dtype=torch.float32, device=device)
        nbytes = galore_adafactor_workspace_bytes(self.hp, shape_desc(m, n, weight.dtype))
        self.workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
        self.t = 0

    def state(self):
        return galore_adafactor_state(desc(self.proj), desc(self.M), desc(self.row.view(1, -1)), desc(self.col.view(1, -1)))

    def refresh(self, grad):
        galore_adafactor_refresh(self.hp, grad, self.state(), self.workspace)

    def step(self, weight, grad, lr):
        galore_adafactor_step(self.hp, weight, grad, self.state(), self.t, lr, self.workspace)
        self.t += 1


class GaLore:
    """Owns the device memory of a tensor list's optimizer state (allocated with torch) and a
    library context bound to torch's current stream.  All arithmetic happens in the library."""

    def __init__(self, weights, rank, device="cuda", workspace_bytes=None, moments="f32", workspace_factor=1, **hparams):
        """moments: "f32" (Algorithm 2 as printed) or "q8" (8-bit codes + one fp32 scale per 256 elements).
        workspace_factor: multiples of galore_workspace_bytes to allocate when workspace_bytes is not given;
        with as many multiples as calls in flight, overlapped calls (set_call_overlap) also overlap their subspace refreshes."""
        assert moments in ("f32", "q8")
        self.moments = moments
        self.hp = make_hparams(rank, **hparams)
        self.shapes = [(w.shape[0], w.shape[1]) for w in weights]
        self.dtypes = [w.dtype for w in weights]
        self.proj, self.M, self.V, self.proj_t = [], [], [], []
        self.M_scale, self.V_scale = [], []
        for (m, n), dt in zip(self.shapes, self.dtypes):
            k, l = (m, n) if m <= n else (n, m)
            self.proj.append(torch.zeros(k, rank, dtype=dt, device=device))
            self.proj_t.append(torch.empty(rank, k, dtype=dt, device=device))
            shape = (rank, l) if m <= n else (l, rank)
            mdt = torch.float32 if moments == "f32" else torch.uint8
            self.M.append(torch.empty(shape, dtype=mdt, device=device))
            self.V.append(torch.empty(shape, dtype=mdt, device=device))
            if moments == "q8":
                self.M_scale.append(torch.empty(shape[0], shape[1] // 256, dtype=torch.float32, device=device))
                self.V_scale.append(torch.empty(shape[0], shape[1] // 256, dtype=torch.float32, device=device))
        w_descs = [shape_desc(m, n, dt) for (m, n), dt in zip(self.shapes, self.dtypes)]
        if workspace_bytes is None:
            workspace_bytes = int(workspace_factor) * galore_workspace_bytes(self.hp, w_descs)
        self.workspace = torch.empty(max(workspace_bytes, 256), dtype=torch.uint8, device=device)
        none = galore_tensor(None, 0, 0, 0, GALORE_F32)
        states = [galore_state(desc(p), desc(m), desc(v), desc(pt),
                               desc(self.M_scale[i]) if moments == "q8" else none,
                               desc(self.V_scale[i]) if moments == "q8" else none)
                  for i, (p, m, v, pt) in enumerate(zip(self.proj, self.M, self.V, self.proj_t))]
        self.ctx = galore_init(self.hp, w_descs, states, self.workspace.data_ptr(), workspace_bytes)

    def step(self, weights, grads, lr, first=0):
        galore_step(self.ctx, [desc(w) for w in weights], [desc(g) for g in grads], first, len(weights), lr)

    def step_static(self, weights, grads, lr, first=0):
        """galore_step with the transients in the library's static device array (allocates nothing)."""
        galore_step_static(self.ctx, [desc(w) for w in weights], [desc(g) for g in grads], first, len(weights), lr)

    def set_call_overlap(self, on):
        galore_set_call_overlap(self.ctx, on)

    def set_fused_adam(self, on):
        galore_set_fused_adam(self.ctx, on)

    def join(self):
        galore_join(self.ctx)

    def library_streams(self):
        """The library's three streams as torch streams (for Tensor.record_stream)."""
        return [torch.cuda.ExternalStream(galore_get_stream(self.ctx, i)) for i in range(3)]

    def refresh(self, grads, first=0):
        galore_refresh_subspace(self.ctx, [desc(g) for g in grads], first, len(grads))

    def get_step(self, i):
        return galore_get_step(self.ctx, i)

    def set_step(self, i, t):
        galore_set_step(self.ctx, i, t)

    def close(self):
        if self.ctx is not None:
            galore_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
