"""CPU oracle for the integer-only inference path (test infrastructure only).

Thin numpy/ctypes front end over ``hawq_oracle.c`` plus the network walk in
``oracle.resnet``.  Nothing in the product package imports this; it is used by
``tests/``, by the smoke check and by the benchmark's CPU-baseline leg.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hawq_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

U8, S8, U4, S4, S32 = 0, 1, 2, 3, 4
_NP = {U8: np.uint8, S8: np.int8, U4: np.uint8, S4: np.uint8, S32: np.int32}
OK, ERR_ARG, ERR_OVERFLOW, ERR_ALLOC = 0, 1, 2, 3


class OracleError(RuntimeError):
    def __init__(self, code, what):
        super().__init__("%s failed with oracle status %d" % (what, code))
        self.code = code


# how the C file is compiled (the benchmark's CPU-baseline record quotes this)
CFLAGS = ["-O2", "-ftree-vectorize", "-mavx2", "-fopenmp"]


def build(force=False):
    """Compile the C oracle with gcc (plain loops, OpenMP, no intrinsics)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc"] + CFLAGS + ["-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        i32, i64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
        _lib.oracle_rq.restype = i64
        _lib.oracle_rq.argtypes = [i64, i32, i32]
        _lib.oracle_rq_array.restype = None
        _lib.oracle_rq_array.argtypes = [vp, vp, vp, i64, vp]
        _lib.oracle_unpack.restype = None
        _lib.oracle_unpack.argtypes = [vp, ctypes.c_int, i64, vp]
        _lib.oracle_conv2d_int.restype = ctypes.c_int
        _lib.oracle_conv2d_int.argtypes = [i32] * 11 + [ctypes.c_int] * 4 + [vp] * 8 + [i32, i64, i64, vp]
        _lib.oracle_conv2d_dual_int.restype = ctypes.c_int
        _lib.oracle_conv2d_dual_int.argtypes = [vp, vp, i32] + [ctypes.c_int] * 5 + [vp] * 10 + [i32, i64, i64, vp]
        _lib.oracle_gemm_int.restype = ctypes.c_int
        _lib.oracle_gemm_int.argtypes = [i32] * 3 + [ctypes.c_int] * 3 + [vp] * 5 + [i32, i64, i64, vp]
        _lib.oracle_residual_add_dyadic.restype = ctypes.c_int
        _lib.oracle_residual_add_dyadic.argtypes = [i64, i32] + [ctypes.c_int] * 3 + [vp] * 6 + [i32, i64, i64, vp]
        _lib.oracle_avgpool_int.restype = ctypes.c_int
        _lib.oracle_avgpool_int.argtypes = [i32] * 4 + [ctypes.c_int] * 2 + [vp] * 3 + [i64, i64, vp]
        _lib.oracle_pool2d_sum_int.restype = ctypes.c_int
        _lib.oracle_pool2d_sum_int.argtypes = [i32] * 10 + [ctypes.c_int] * 2 + [vp] * 3 + [i64, i64, vp]
        _lib.oracle_concat_dyadic.restype = ctypes.c_int
        _lib.oracle_concat_dyadic.argtypes = [i64, i32, vp, vp, vp, vp, vp, ctypes.c_int, i64, i64, vp]
        _lib.oracle_maxpool_int.restype = ctypes.c_int
        _lib.oracle_maxpool_int.argtypes = [i32] * 4 + [ctypes.c_int] * 2 + [vp, i64, i64, vp]
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def nelems_to_bytes(n, dt):
    return n // 2 if dt in (U4, S4) else n


def _out(n_elems, dt, shape_last_is_channels):
    """Allocate an output array; 4-bit outputs are packed along the last axis."""
    shape = list(shape_last_is_channels)
    if dt in (U4, S4):
        shape[-1] //= 2
    return np.zeros(shape, dtype=_NP[dt])


def rq(t, b, c):
    """Dyadic requantisation of scalars or arrays: floor(t*b/2^c + 1/2)."""
    t = np.ascontiguousarray(np.broadcast_arrays(t, b, c)[0], dtype=np.int64)
    bb = np.ascontiguousarray(np.broadcast_to(b, t.shape), dtype=np.int32)
    cc = np.ascontiguousarray(np.broadcast_to(c, t.shape), dtype=np.int32)
    out = np.empty_like(t)
    lib().oracle_rq_array(_ptr(t), _ptr(bb), _ptr(cc), t.size, _ptr(out))
    return out


def unpack(a, dt, n=None):
    """Logical int32 values of a dense tensor stored as type dt (flat)."""
    a = np.ascontiguousarray(a)
    if n is None:
        n = a.size * (2 if dt in (U4, S4) else 1)
    out = np.empty(n, dtype=np.int32)
    lib().oracle_unpack(_ptr(a), dt, n, _ptr(out))
    return out


def conv2d_int(x, w, bias, b, c, *, N, H, W, C, K, R, S, stride, pad, x_dt, w_dt, y_dt,
               relu, y_lo, y_hi, residual=None, res_b=None, res_c=None, res_dt=U8):
    """One quantised conv layer; see ``oracle_conv2d_int`` in the C file.
    ``stride`` / ``pad`` are ints or (h, w) pairs.  Returns [N,P,Q,K] (packed along K
    for 4-bit outputs)."""
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    ph, pw = (pad, pad) if np.isscalar(pad) else pad
    P = (H + 2 * ph - R) // sh + 1
    Q = (W + 2 * pw - S) // sw + 1
    x = _c(x, _NP[x_dt]); w = _c(w, np.int8 if w_dt == S8 else _NP[w_dt])
    bias = _c(bias, np.int32); b = _c(b, np.int32); c = _c(c, np.uint8)
    residual = _c(residual, _NP[res_dt]) if residual is not None else None
    res_b = _c(res_b, np.int32); res_c = _c(res_c, np.uint8)
    assert x.size == nelems_to_bytes(N * H * W * C, x_dt), "x size"
    assert w.size == nelems_to_bytes(K * R * S * C, w_dt), "w size"
    assert bias.size == K and (b is None or (b.size == K and c.size == K))
    if residual is not None:
        assert residual.size == nelems_to_bytes(N * P * Q * K, res_dt), "residual size"
        assert res_b.size == K and res_c.size == K
    y = _out(N * P * Q * K, y_dt, (N, P, Q, K))
    st = lib().oracle_conv2d_int(N, H, W, C, K, R, S, sh, sw, ph, pw, x_dt, w_dt, y_dt, res_dt,
                                 _ptr(x), _ptr(w), _ptr(bias), _ptr(b), _ptr(c),
                                 _ptr(residual), _ptr(res_b), _ptr(res_c), int(relu), int(y_lo), int(y_hi), _ptr(y))
    if st != OK:
        raise OracleError(st, "oracle_conv2d_int")
    return y


def conv2d_dual_int(x, w, bias, b, c, xs, ws, bias_s, b_s, c_s, *, N, K, H, W, C, R, S, stride, pad, x_dt, w_dt,
                    Hs, Ws, Cs, Rs, Ss, stride_s, pad_s, xs_dt, ws_dt, y_dt, relu, y_lo, y_hi):
    """Block output with a convolution on both branches (main: x, w, ...; shortcut: xs, ws, ...), both INT32
    accumulators rescaled by their own dyadic number and added; see ``oracle_conv2d_dual_int``."""
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    x = _c(x, _NP[x_dt]); w = _c(w, np.int8 if w_dt == S8 else _NP[w_dt])
    xs = _c(xs, _NP[xs_dt]); ws = _c(ws, np.int8 if ws_dt == S8 else _NP[ws_dt])
    bias = _c(bias, np.int32); b = _c(b, np.int32); c = _c(c, np.uint8)
    bias_s = _c(bias_s, np.int32); b_s = _c(b_s, np.int32); c_s = _c(c_s, np.uint8)
    assert x.size == nelems_to_bytes(N * H * W * C, x_dt) and w.size == nelems_to_bytes(K * R * S * C, w_dt)
    assert xs.size == nelems_to_bytes(N * Hs * Ws * Cs, xs_dt) and ws.size == nelems_to_bytes(K * Rs * Ss * Cs, ws_dt)
    for a in (bias, b, c, bias_s, b_s, c_s):
        assert a.size == K
    dims = np.array([N, H, W, C, R, S, stride, stride, pad, pad], dtype=np.int32)
    dimss = np.array([Hs, Ws, Cs, Rs, Ss, stride_s, stride_s, pad_s, pad_s], dtype=np.int32)
    y = _out(N * P * Q * K, y_dt, (N, P, Q, K))
    st = lib().oracle_conv2d_dual_int(_ptr(dims), _ptr(dimss), K, x_dt, w_dt, xs_dt, ws_dt, y_dt,
                                      _ptr(x), _ptr(w), _ptr(bias), _ptr(b), _ptr(c),
                                      _ptr(xs), _ptr(ws), _ptr(bias_s), _ptr(b_s), _ptr(c_s),
                                      int(relu), int(y_lo), int(y_hi), _ptr(y))
    if st != OK:
        raise OracleError(st, "oracle_conv2d_dual_int")
    return y


def gemm_int(x, w, bias, b, c, *, M, N, K, x_dt, w_dt, y_dt, relu=0, y_lo=-(1 << 31), y_hi=(1 << 31) - 1):
    x = _c(x, _NP[x_dt]); w = _c(w, np.int8 if w_dt == S8 else _NP[w_dt])
    bias = _c(bias, np.int32); b = _c(b, np.int32); c = _c(c, np.uint8)
    assert x.size == nelems_to_bytes(M * K, x_dt) and w.size == nelems_to_bytes(N * K, w_dt)
    y = _out(M * N, y_dt, (M, N))
    st = lib().oracle_gemm_int(M, N, K, x_dt, w_dt, y_dt, _ptr(x), _ptr(w), _ptr(bias), _ptr(b), _ptr(c),
                               int(relu), int(y_lo), int(y_hi), _ptr(y))
    if st != OK:
        raise OracleError(st, "oracle_gemm_int")
    return y


def residual_add_dyadic(m, m_b, m_c, r, r_b, r_c, *, n_pixels, K, m_dt, r_dt, y_dt, relu, y_lo, y_hi):
    m = _c(m, _NP[m_dt]); r = _c(r, _NP[r_dt])
    m_b = _c(m_b, np.int32); m_c = _c(m_c, np.uint8); r_b = _c(r_b, np.int32); r_c = _c(r_c, np.uint8)
    assert m.size == nelems_to_bytes(n_pixels * K, m_dt) and r.size == nelems_to_bytes(n_pixels * K, r_dt)
    y = _out(n_pixels * K, y_dt, (n_pixels, K))
    st = lib().oracle_residual_add_dyadic(n_pixels, K, m_dt, r_dt, y_dt, _ptr(m), _ptr(m_b), _ptr(m_c),
                                          _ptr(r), _ptr(r_b), _ptr(r_c), int(relu), int(y_lo), int(y_hi), _ptr(y))
    if st != OK:
        raise OracleError(st, "oracle_residual_add_dyadic")
    return y


def avgpool_int(x, b, c, *, N, H, W, C, x_dt, y_dt, y_lo, y_hi):
    x = _c(x, _NP[x_dt]); b = _c(b, np.int32); c = _c(c, np.uint8)
    assert x.size == nelems_to_bytes(N * H * W * C, x_dt)
    y = _out(N * C, y_dt, (N, C))
    st = lib().oracle_avgpool_int(N, H, W, C, x_dt, y_dt, _ptr(x), _ptr(b), _ptr(c), int(y_lo), int(y_hi), _ptr(y))
    if st != OK:
        raise OracleError(st, "oracle_avgpool_int")
    return y


def maxpool_int(x, *, N, H, W, C, x_dt, y_dt, y_lo, y_hi):
    x = _c(x, _NP[x_dt])
    assert x.size == nelems_to_bytes(N * H * W * C, x_dt)
    P, Q = (H + 2 - 3) // 2 + 1, (W + 2 - 3) // 2 + 1
    y = _out(N * P * Q * C, y_dt, (N, P, Q, C))
    st = lib().oracle_maxpool_int(N, H, W, C, x_dt, y_dt, _ptr(x), int(y_lo), int(y_hi), _ptr(y))
    if st != OK:
        raise OracleError(st, "oracle_maxpool_int")
    return y


def pool2d_sum_int(x, b, c, *, N, H, W, C, R, S, stride, pad, x_dt, y_dt, y_lo=-(1 << 31), y_hi=(1 << 31) - 1):
    """Window sum carried in INT32 (raw sums with b = c = None and y_dt = S32), optionally followed by one dyadic
    rescale and clamp; see ``oracle_pool2d_sum_int``."""
    x = _c(x, _NP[x_dt]); b = _c(b, np.int32); c = _c(c, np.uint8)
    assert x.size == nelems_to_bytes(N * H * W * C, x_dt)
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    y = _out(N * P * Q * C, y_dt, (N, P, Q, C))
    st = lib().oracle_pool2d_sum_int(N, H, W, C, R, S, stride, stride, pad, pad, x_dt, y_dt, _ptr(x), _ptr(b), _ptr(c),
                                     int(y_lo), int(y_hi), _ptr(y))
    if st != OK:
        raise OracleError(st, "oracle_pool2d_sum_int")
    return y


def concat_dyadic(branches, *, n_pixels, y_dt, y_lo, y_hi):
    """branches: list of (q [n_pixels, K_i], dtype, b [K_i], c [K_i]); returns [n_pixels, sum K_i] (packed for 4-bit)."""
    n = len(branches)
    qs = [_c(q, _NP[dt]) for q, dt, _, _ in branches]
    bs = [_c(b, np.int32) for _, _, b, _ in branches]
    cs = [_c(c, np.uint8) for _, _, _, c in branches]
    K = np.array([b.size for b in bs], dtype=np.int32)
    for q, (_, dt, _, _), k in zip(qs, branches, K):
        assert q.size == nelems_to_bytes(n_pixels * int(k), dt)
    dts = (ctypes.c_int * n)(*[dt for _, dt, _, _ in branches])
    arr = lambda xs: (ctypes.c_void_p * n)(*[x.ctypes.data for x in xs])
    y = _out(n_pixels * int(K.sum()), y_dt, (n_pixels, int(K.sum())))
    st = lib().oracle_concat_dyadic(n_pixels, n, _ptr(K), dts, arr(qs), arr(bs), arr(cs), y_dt, int(y_lo), int(y_hi), _ptr(y))
    if st != OK:
        raise OracleError(st, "oracle_concat_dyadic")
    return y
