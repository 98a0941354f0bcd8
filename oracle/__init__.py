"""AdaFuse CPU oracle -- TEST INFRASTRUCTURE, not a product path.

numpy/ctypes front end of ``adafuse_oracle.c`` (plain C, fp64).  Only tests, the
smoke check and the bench's ``cpu_baseline`` leg may import this package; the
HIP path never does, and this package never imports the HIP path.

bf16 tensors travel as ``numpy.uint16`` bit patterns.
"""
import ctypes as C
import os

import numpy as np

from .build import build as _build, build_ubsan as _build_ubsan

_lib = None

_u16p = C.POINTER(C.c_uint16)
_i32p = C.POINTER(C.c_int32)
_f32p = C.POINTER(C.c_float)
_f64p = C.POINTER(C.c_double)
_i64p = C.POINTER(C.c_int64)


def lib():
    """Load (building with gcc if needed) the oracle shared library."""
    global _lib
    if _lib is None:
        path = _build_ubsan() if os.environ.get("ADAFUSE_ORACLE_UBSAN") == "1" else _build()
        L = C.CDLL(path)
        L.oracle_bf16_to_f64.restype = C.c_double
        L.oracle_bf16_to_f64.argtypes = [C.c_uint16]
        L.oracle_f64_to_bf16_rne.restype = C.c_uint16
        L.oracle_f64_to_bf16_rne.argtypes = [C.c_double]
        L.oracle_f64_to_bf16_rne_array.restype = None
        L.oracle_f64_to_bf16_rne_array.argtypes = [_f64p, _u16p, C.c_int64]
        L.oracle_bf16_to_f64_array.restype = None
        L.oracle_bf16_to_f64_array.argtypes = [_u16p, _f64p, C.c_int64]
        L.oracle_num_threads.restype = C.c_int
        L.oracle_pregate.restype = C.c_int
        L.oracle_pregate.argtypes = [_u16p, _u16p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                     _f64p, _f32p, _i32p, _f64p, _f32p]
        common = [_u16p, C.c_int64, _u16p, _u16p, C.c_int, C.c_int, C.c_int, C.c_int]
        L.oracle_merge_rows.restype = C.c_int
        L.oracle_merge_rows.argtypes = common + [_i32p, _f32p, C.c_int, C.c_float,
                                                 C.c_int, C.c_int, _u16p, C.c_int64]
        L.oracle_merge_rows_f64.restype = C.c_int
        L.oracle_merge_rows_f64.argtypes = common + [_i32p, _f32p, C.c_int, C.c_float,
                                                     C.c_int, C.c_int, _f64p, C.c_int64]
        L.oracle_inplace_swap_rows.restype = C.c_int
        L.oracle_inplace_swap_rows.argtypes = common + [_i32p, _f32p, C.c_int, _i32p, _f32p, C.c_int,
                                                        C.c_float, C.c_int, C.c_int, _u16p, C.c_int64]
        L.oracle_dynamic_adapter_forward.restype = C.c_int
        L.oracle_dynamic_adapter_forward.argtypes = common + [_i32p, _f32p, C.c_int, C.c_float, _f64p, _f64p]
        L.oracle_gemv_bf16.restype = C.c_int
        L.oracle_gemv_bf16.argtypes = [_u16p, C.c_int64, C.c_int, C.c_int, _f64p, _f64p]
        L.oracle_bf16_ulp_diff.restype = C.c_int
        L.oracle_bf16_ulp_diff.argtypes = [_u16p, _u16p, C.c_int64, _i64p, _i64p]
        _lib = L
    return _lib


def _arr(x, dtype):
    a = np.ascontiguousarray(x, dtype=dtype)
    return a


def _ptr(a, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle: {what}: invalid argument")


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def bf16_to_f64(bits):
    b = _arr(bits, np.uint16)
    out = np.empty(b.shape, np.float64)
    lib().oracle_bf16_to_f64_array(_ptr(b, C.c_uint16), _ptr(out, C.c_double), b.size)
    return out


def f64_to_bf16(x):
    a = _arr(x, np.float64)
    out = np.empty(a.shape, np.uint16)
    lib().oracle_f64_to_bf16_rne_array(_ptr(a, C.c_double), _ptr(out, C.c_uint16), a.size)
    return out


def pregate(hidden, w_router, k, gate_norm=0):
    """Router oracle.  hidden [T][d], w_router [E][d] (uint16 bf16 bits).

    Returns dict(logits f64 [T][E], logits32 f32, idx i32 [T][k], gates f64, gates32 f32).
    """
    h = _arr(hidden, np.uint16)
    w = _arr(w_router, np.uint16)
    if h.ndim != 2 or w.ndim != 2 or h.shape[1] != w.shape[1]:
        raise ValueError("oracle.pregate: hidden [T][d] and w_router [E][d] expected")
    T, d = h.shape
    E = w.shape[0]
    logits = np.empty((T, E), np.float64)
    logits32 = np.empty((T, E), np.float32)
    idx = np.empty((T, k), np.int32)
    gates = np.empty((T, k), np.float64)
    gates32 = np.empty((T, k), np.float32)
    rc = lib().oracle_pregate(_ptr(h, C.c_uint16), _ptr(w, C.c_uint16), T, d, E, k, gate_norm,
                              _ptr(logits, C.c_double), _ptr(logits32, C.c_float),
                              _ptr(idx, C.c_int32), _ptr(gates, C.c_double), _ptr(gates32, C.c_float))
    _check(rc, "pregate")
    return dict(logits=logits, logits32=logits32, idx=idx, gates=gates, gates32=gates32)


def _switch_common(w_base, a_bank, b_bank):
    w = _arr(w_base, np.uint16)
    a = _arr(a_bank, np.uint16)
    b = _arr(b_bank, np.uint16)
    if w.ndim != 2 or a.ndim != 3 or b.ndim != 3:
        raise ValueError("oracle: W [out][in], A [E][r][in], B [E][out][r] expected")
    out, in_ = w.shape
    E, r, in_a = a.shape
    if in_a != in_ or b.shape != (E, out, r):
        raise ValueError("oracle: bank shapes do not match W")
    return w, a, b, out, in_, E, r


def _sel(idx, gates):
    i = _arr(np.atleast_1d(idx), np.int32)
    g = _arr(np.atleast_1d(gates), np.float32)
    if i.shape != g.shape or i.ndim != 1:
        raise ValueError("oracle: idx and gates must be 1-D of equal length")
    return i, g


def merge(w_base, a_bank, b_bank, idx, gates, scale, rows=None, rounded=True):
    """W' = rn_bf16(W_base + s * sum_j g_j B_{e_j} A_{e_j}) for rows [r0,r1) (all rows if None).

    rounded=False returns the fp64 values before rounding.
    """
    w, a, b, out, in_, E, r = _switch_common(w_base, a_bank, b_bank)
    i, g = _sel(idx, gates)
    r0, r1 = (0, out) if rows is None else rows
    if rounded:
        res = np.empty((r1 - r0, in_), np.uint16)
        rc = lib().oracle_merge_rows(_ptr(w, C.c_uint16), in_, _ptr(a, C.c_uint16), _ptr(b, C.c_uint16),
                                     out, in_, E, r, _ptr(i, C.c_int32), _ptr(g, C.c_float), i.size,
                                     float(scale), r0, r1, _ptr(res, C.c_uint16), in_)
    else:
        res = np.empty((r1 - r0, in_), np.float64)
        rc = lib().oracle_merge_rows_f64(_ptr(w, C.c_uint16), in_, _ptr(a, C.c_uint16), _ptr(b, C.c_uint16),
                                         out, in_, E, r, _ptr(i, C.c_int32), _ptr(g, C.c_float), i.size,
                                         float(scale), r0, r1, _ptr(res, C.c_double), in_)
    _check(rc, "merge")
    return res


def inplace_swap(w_cur, a_bank, b_bank, idx_prev, gates_prev, idx_next, gates_next, scale, rows=None):
    """Paper-literal Eq.8 step: rn_bf16(W_cur - dW_prev + dW_next), one rounding."""
    w, a, b, out, in_, E, r = _switch_common(w_cur, a_bank, b_bank)
    ip, gp = _sel(idx_prev, gates_prev)
    inx, gn = _sel(idx_next, gates_next)
    r0, r1 = (0, out) if rows is None else rows
    res = np.empty((r1 - r0, in_), np.uint16)
    rc = lib().oracle_inplace_swap_rows(_ptr(w, C.c_uint16), in_, _ptr(a, C.c_uint16), _ptr(b, C.c_uint16),
                                        out, in_, E, r, _ptr(ip, C.c_int32), _ptr(gp, C.c_float), ip.size,
                                        _ptr(inx, C.c_int32), _ptr(gn, C.c_float), inx.size,
                                        float(scale), r0, r1, _ptr(res, C.c_uint16), in_)
    _check(rc, "inplace_swap")
    return res


def dynamic_adapter_forward(w_base, a_bank, b_bank, idx, gates, scale, x):
    """y = W_base x + s * sum_j g_j B_{e_j}(A_{e_j} x), fp64 (Eq.1/Eq.2)."""
    w, a, b, out, in_, E, r = _switch_common(w_base, a_bank, b_bank)
    i, g = _sel(idx, gates)
    xv = _arr(x, np.float64)
    if xv.shape != (in_,):
        raise ValueError("oracle: x must be [in]")
    y = np.empty(out, np.float64)
    rc = lib().oracle_dynamic_adapter_forward(_ptr(w, C.c_uint16), in_, _ptr(a, C.c_uint16), _ptr(b, C.c_uint16),
                                              out, in_, E, r, _ptr(i, C.c_int32), _ptr(g, C.c_float), i.size,
                                              float(scale), _ptr(xv, C.c_double), _ptr(y, C.c_double))
    _check(rc, "dynamic_adapter_forward")
    return y


def prefill(w_base, a_bank, b_bank, idx, gates, scale, x_bits, tokens=None):
    """Prefill of one adapted matrix (section "Decoding Phase": many tokens, each with its own
    pre-gated decision, adapters un-merged): row t of the result is Eq.2 for token t,
        y[t] = W_base x[t] + s * sum_j gates[t][j] * B_{idx[t][j]} (A_{idx[t][j]} x[t]),
    taken token by token with dynamic_adapter_forward.  x_bits [T][in] bf16 bit patterns,
    idx [T][k], gates [T][k] fp32.  tokens = the rows wanted (default: all); returns fp64
    [len(tokens)][out].
    """
    xb = _arr(x_bits, np.uint16)
    i2 = _arr(idx, np.int32)
    g2 = _arr(gates, np.float32)
    if xb.ndim != 2 or i2.ndim != 2 or i2.shape != g2.shape or i2.shape[0] != xb.shape[0]:
        raise ValueError("oracle.prefill: x [T][in], idx [T][k], gates [T][k] expected")
    rows = range(xb.shape[0]) if tokens is None else list(tokens)
    xs = bf16_to_f64(xb)
    return np.stack([dynamic_adapter_forward(w_base, a_bank, b_bank, i2[t], g2[t], scale, xs[t]) for t in rows]) \
        if len(rows) else np.empty((0, _arr(w_base, np.uint16).shape[0]), np.float64)


def gemv_bf16(w, x):
    """y = W x with W bf16 bits and x fp64 (Eq.3 on a merged matrix)."""
    wv = _arr(w, np.uint16)
    xv = _arr(x, np.float64)
    out, in_ = wv.shape
    y = np.empty(out, np.float64)
    rc = lib().oracle_gemv_bf16(_ptr(wv, C.c_uint16), in_, out, in_, _ptr(xv, C.c_double), _ptr(y, C.c_double))
    _check(rc, "gemv_bf16")
    return y


def ulp_diff(a, b):
    """(max bf16-ULP distance, number of differing elements) between two bit arrays."""
    x = _arr(a, np.uint16)
    y = _arr(b, np.uint16)
    if x.shape != y.shape:
        raise ValueError("oracle.ulp_diff: shape mismatch")
    mx = C.c_int64(0)
    nd = C.c_int64(0)
    rc = lib().oracle_bf16_ulp_diff(_ptr(x, C.c_uint16), _ptr(y, C.c_uint16), x.size, C.byref(mx), C.byref(nd))
    _check(rc, "ulp_diff")
    return int(mx.value), int(nd.value)
