"""Python face of the 8-bit-moment oracle (test infrastructure, never the product path).

Loads ``libq8_oracle.so`` (plain C, built from ``q8_oracle.c`` in this directory with floating
point contraction off, so every fp32 operation of the definition is rounded exactly once) and
wraps one Adam step with 8-bit block-wise moments: ``adam_q8_def`` is the definition (fp64),
``adam_q8`` the second checker that replays one stated fp32 operation sequence.  Parity unpinned by
the paper: the number format is this build's own definition, stated in the header of ``q8_oracle.c``.  Imports nothing
from the HIP package.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "q8_oracle.c")
_LIB = os.path.join(_HERE, "libq8_oracle.so")
BLOCK = 256


def build(force=False):
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-std=c11",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None
_f32p = ctypes.POINTER(ctypes.c_float)
_u8p = ctypes.POINTER(ctypes.c_uint8)
_f64p = ctypes.POINTER(ctypes.c_double)
_i64 = ctypes.c_int64
_f32 = ctypes.c_float


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        L = _lib
        L.oracle_q8_decode_table.argtypes = [ctypes.c_int, _f64p]
        for name in ("oracle_q8_encode_m_array", "oracle_q8_encode_v_array"):
            getattr(L, name).argtypes = [_f32p, _f32p, _u8p, _i64]
        for name in ("oracle_q8_decode_m_array", "oracle_q8_decode_v_array"):
            getattr(L, name).argtypes = [_u8p, _f32p, _f32p, _i64]
        L.oracle_adam_q8.argtypes = [_f32p, _u8p, _u8p, _f32p, _f32p, _f32p, _i64] + [_f32] * 7
        L.oracle_adam_q8_def.argtypes = [_f32p, _u8p, _u8p, _f32p, _f32p, _f64p, _f64p, _f64p, _i64,
                                         ctypes.c_double, ctypes.c_double, ctypes.c_double, _i64]
    return _lib


def _f(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _u(a):
    return np.ascontiguousarray(a, dtype=np.uint8)


def decode_table(is_v):
    out = np.zeros(256 if is_v else 128, dtype=np.float64)
    lib().oracle_q8_decode_table(1 if is_v else 0, out.ctypes.data_as(_f64p))
    return out


def _bcast(scale, n):
    s = _f(scale)
    return _f(np.broadcast_to(s, (n,))) if s.size != n else s.reshape(-1)


def encode(x, scale, is_v):
    x = _f(x).reshape(-1)
    s = _bcast(scale, x.size)
    out = np.zeros(x.size, dtype=np.uint8)
    fn = lib().oracle_q8_encode_v_array if is_v else lib().oracle_q8_encode_m_array
    fn(x.ctypes.data_as(_f32p), s.ctypes.data_as(_f32p), out.ctypes.data_as(_u8p), x.size)
    return out


def decode(codes, scale, is_v):
    c = _u(codes).reshape(-1)
    s = _bcast(scale, c.size)
    out = np.zeros(c.size, dtype=np.float32)
    fn = lib().oracle_q8_decode_v_array if is_v else lib().oracle_q8_decode_m_array
    fn(c.ctypes.data_as(_u8p), s.ctypes.data_as(_f32p), out.ctypes.data_as(_f32p), c.size)
    return out


def n_blocks(count):
    return (count + BLOCK - 1) // BLOCK


def bias_corrections(beta1, beta2, k):
    """1 / (1 - beta^k), formed in fp64 and rounded to fp32 (they cross the C ABI as fp32)."""
    return (np.float32(1.0 / (1.0 - float(np.float32(beta1)) ** k)), np.float32(1.0 / (1.0 - float(np.float32(beta2)) ** k)))


def adam_q8(R, Mc, Vc, Ms, Vs, beta1, beta2, eps, k):
    """One step on the flattened row-major R.  Mc, Vc (uint8), Ms, Vs (fp32 per block) are updated
    in place; returns N (fp32)."""
    R = _f(R).reshape(-1)
    assert Mc.dtype == np.uint8 and Vc.dtype == np.uint8 and Ms.dtype == np.float32 and Vs.dtype == np.float32
    assert Mc.size == R.size and Vc.size == R.size and Ms.size == n_blocks(R.size) and Vs.size == n_blocks(R.size)
    N = np.zeros(R.size, dtype=np.float32)
    b1, b2 = np.float32(beta1), np.float32(beta2)
    ic1, ic2 = bias_corrections(beta1, beta2, k)
    lib().oracle_adam_q8(R.ctypes.data_as(_f32p), Mc.ctypes.data_as(_u8p), Vc.ctypes.data_as(_u8p),
                         Ms.ctypes.data_as(_f32p), Vs.ctypes.data_as(_f32p), N.ctypes.data_as(_f32p), R.size,
                         b1, b2, np.float32(1.0) - b1, np.float32(1.0) - b2, np.float32(eps), ic1, ic2)
    return N


def adam_q8_def(R, Mc, Vc, Ms, Vs, beta1, beta2, eps, k):
    """THE DEFINITION of the step (fp64, see the header of q8_oracle.c) on the flattened row-major R.
    Mc, Vc (uint8), Ms, Vs (fp32 per block) are updated in place; returns (N, Ym, Yv) in fp64: the
    normalised update and the quotients |m| / scale, v / scale the new codes were chosen from.
    beta1, beta2, eps are used as given (pass the fp32-representable numbers an fp32 interface sees)."""
    R = _f(R).reshape(-1)
    assert Mc.dtype == np.uint8 and Vc.dtype == np.uint8 and Ms.dtype == np.float32 and Vs.dtype == np.float32
    assert Mc.size == R.size and Vc.size == R.size and Ms.size == n_blocks(R.size) and Vs.size == n_blocks(R.size)
    N, Ym, Yv = (np.zeros(R.size, dtype=np.float64) for _ in range(3))
    lib().oracle_adam_q8_def(R.ctypes.data_as(_f32p), Mc.ctypes.data_as(_u8p), Vc.ctypes.data_as(_u8p),
                             Ms.ctypes.data_as(_f32p), Vs.ctypes.data_as(_f32p), N.ctypes.data_as(_f64p),
                             Ym.ctypes.data_as(_f64p), Yv.ctypes.data_as(_f64p), R.size,
                             float(beta1), float(beta2), float(eps), int(k))
    return N, Ym, Yv


def midpoints(is_v):
    """Decision boundaries of the encoder: midpoints between consecutive magnitudes in use (fp64, exact)."""
    t = decode_table(is_v)
    t = t[t >= 0]
    return 0.5 * (t[1:] + t[:-1])
