"""numpy-facing wrapper around the C oracle (argument marshalling only).

bf16 matrices are uint16 bit patterns.  Every function allocates and returns its
outputs; names and argument order follow the C functions, which cite the paper.
"""
from __future__ import annotations

import ctypes as C
import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build(force=False))
        _lib.oracle_linear_fwd.restype = C.c_int
        _lib.oracle_linear_bwd_dx.restype = C.c_int
        _lib.oracle_max_threads.restype = C.c_int
        _lib.oracle_select_outliers.restype = C.c_int32
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


i64, i32, f32 = C.c_int64, C.c_int32, C.c_float


def set_threads(n: int):
    lib().oracle_set_threads(C.c_int(n))


def max_threads() -> int:
    return int(lib().oracle_max_threads())


def weight_quantize(W):
    W = _c(W, np.float32)
    K, N = W.shape
    Wq = np.empty((K, N), np.int8)
    dw = np.empty(N, np.float32)
    lib().oracle_weight_quantize(_p(W), i64(K), i64(N), _p(Wq), _p(dw))
    return Wq, dw


def outlier_rows(W, O):
    W = _c(W, np.float32)
    O = _c(O, np.int32)
    K, N = W.shape
    n = O.size
    W_O = np.empty((n, N), np.float32)
    wmax = np.empty(n, np.float32)
    lib().oracle_outlier_rows(_p(W), i64(K), i64(N), _p(O), i32(n), _p(W_O), _p(wmax))
    return W_O, wmax


def scale_update(X, O, W_O, wmax_O, gamma, s_O, colscale):
    """Returns (s_new, colscale_new, what_int [n x c_out], delta_what [c_out], cmax [n]); inputs are not modified."""
    X = _c(X, np.uint16)
    O = _c(O, np.int32)
    W_O = _c(W_O, np.float32)
    wmax_O = _c(wmax_O, np.float32)
    t, K = X.shape
    n = O.size
    N = W_O.shape[1]
    s = np.array(s_O, dtype=np.float32, copy=True)
    cs = np.array(colscale, dtype=np.float32, copy=True)
    assert cs.size == K and s.size == n
    what = np.empty((n, N), np.int8)
    dwh = np.empty(N, np.float32)
    cmax = np.empty(n, np.float32)
    lib().oracle_scale_update(_p(X), i64(t), i64(K), i64(K), _p(O), i32(n), _p(W_O), _p(wmax_O), i64(N), f32(gamma),
                              _p(s), _p(cs), _p(what), _p(dwh), _p(cmax))
    return s, cs, what, dwh, cmax


def quant_act(X, colscale=None, O=None):
    """Returns (Xq [t x c] int8, delta [t], xq_O [t x n] int8)."""
    X = _c(X, np.uint16)
    t, c = X.shape
    cs = None if colscale is None else _c(colscale, np.float32)
    O = np.zeros(0, np.int32) if O is None else _c(O, np.int32)
    n = O.size
    Xq = np.empty((t, c), np.int8)
    d = np.empty(t, np.float32)
    xo = np.empty((t, n), np.int8)
    lib().oracle_quant_act(_p(X), i64(t), i64(c), i64(c), _p(cs), _p(O), i32(n), _p(Xq), _p(d), _p(xo))
    return Xq, d, xo


def linear_fwd(Xq, delta_x, xq_O, Wq, delta_w, what_int, delta_what, X=None, lora_A=None, lora_B=None,
               lora_scale=0.0):
    """Returns (Y fp32 [t x c_out], acc1 int32, acc2 int32)."""
    Xq = _c(Xq, np.int8)
    Wq = _c(Wq, np.int8)
    t, K = Xq.shape
    N = Wq.shape[1]
    xq_O = _c(xq_O, np.int8)
    n = xq_O.shape[1] if xq_O.ndim == 2 else 0
    what_int = _c(what_int, np.int8)
    r = 0 if lora_A is None else lora_A.shape[1]
    Xb = _c(X, np.uint16) if r > 0 else None
    A = _c(lora_A, np.uint16) if r > 0 else None
    B = _c(lora_B, np.uint16) if r > 0 else None
    Y = np.empty((t, N), np.float32)
    acc1 = np.empty((t, N), np.int32)
    acc2 = np.empty((t, N), np.int32)
    ok = lib().oracle_linear_fwd(_p(Xq), _p(_c(delta_x, np.float32)), _p(xq_O), i64(t), _p(Wq),
                                 _p(_c(delta_w, np.float32)), i64(K), i64(N), _p(what_int),
                                 _p(_c(delta_what, np.float32)), i32(n), _p(Xb), i64(K), _p(A), _p(B), i32(r),
                                 f32(lora_scale), _p(Y), i64(N), _p(acc1), _p(acc2))
    assert ok == 1, "int32 accumulator overflow"
    return Y, acc1, acc2


def linear_bwd_dx(dY, Wq, delta_w, lora_A=None, lora_B=None, lora_scale=0.0):
    """Returns (dX fp32 [t x c_in], Gq int8 [t x c_out], delta_g [t], acc int32 [t x c_in])."""
    dY = _c(dY, np.uint16)
    Wq = _c(Wq, np.int8)
    t, N = dY.shape
    K = Wq.shape[0]
    r = 0 if lora_A is None else lora_A.shape[1]
    A = _c(lora_A, np.uint16) if r > 0 else None
    B = _c(lora_B, np.uint16) if r > 0 else None
    dX = np.empty((t, K), np.float32)
    Gq = np.empty((t, N), np.int8)
    dg = np.empty(t, np.float32)
    acc = np.empty((t, K), np.int32)
    ok = lib().oracle_linear_bwd_dx(_p(dY), i64(t), i64(N), _p(Wq), _p(_c(delta_w, np.float32)), i64(K), i64(N),
                                    _p(A), _p(B), i32(r), f32(lora_scale), _p(dX), i64(K), _p(Gq), _p(dg), _p(acc))
    assert ok == 1, "int32 accumulator overflow"
    return dX, Gq, dg, acc


def ref_fwd_fp64(X, W, lora_A=None, lora_B=None, lora_scale=0.0):
    X = _c(X, np.uint16)
    W = _c(W, np.float32)
    t, K = X.shape
    N = W.shape[1]
    r = 0 if lora_A is None else lora_A.shape[1]
    A = _c(lora_A, np.uint16) if r > 0 else None
    B = _c(lora_B, np.uint16) if r > 0 else None
    Y = np.empty((t, N), np.float64)
    lib().oracle_ref_fwd_fp64(_p(X), i64(t), i64(K), i64(K), _p(W), i64(N), _p(A), _p(B), i32(r), f32(lora_scale),
                              _p(Y))
    return Y


def ref_bwd_fp64(dY, W, lora_A=None, lora_B=None, lora_scale=0.0):
    dY = _c(dY, np.uint16)
    W = _c(W, np.float32)
    t, N = dY.shape
    K = W.shape[0]
    r = 0 if lora_A is None else lora_A.shape[1]
    A = _c(lora_A, np.uint16) if r > 0 else None
    B = _c(lora_B, np.uint16) if r > 0 else None
    dX = np.empty((t, K), np.float64)
    lib().oracle_ref_bwd_fp64(_p(dY), i64(t), i64(N), i64(N), _p(W), i64(K), _p(A), _p(B), i32(r), f32(lora_scale),
                              _p(dX))
    return dX


def lora_grads(X, dY, lora_A, lora_B, lora_scale):
    """Returns (dA [c_in x r], dB [r x c_out]) in fp64."""
    X = _c(X, np.uint16)
    dY = _c(dY, np.uint16)
    A = _c(lora_A, np.uint16)
    B = _c(lora_B, np.uint16)
    t, K = X.shape
    N = dY.shape[1]
    r = A.shape[1]
    assert dY.shape[0] == t and A.shape[0] == K and B.shape == (r, N)
    dA = np.empty((K, r), np.float64)
    dB = np.empty((r, N), np.float64)
    lib().oracle_lora_grads(_p(X), _p(dY), i64(t), i64(K), i64(N), i64(K), i64(N), _p(A), _p(B), i32(r),
                            f32(lora_scale), _p(dA), _p(dB))
    return dA, dB


def bwd_dx_outlier_cols(dY, O, W_O, Wq=None, delta_w=None, what_int=None, delta_what=None, colscale=None,
                        lora_A=None, lora_B=None, lora_scale=0.0):
    """Returns (exact [t x n], ste [t x n] or None) in fp64; ste needs Wq, delta_w, what_int, delta_what, colscale."""
    dY = _c(dY, np.uint16)
    O = _c(O, np.int32)
    W_O = _c(W_O, np.float32)
    t, N = dY.shape
    n = O.size
    r = 0 if lora_A is None else lora_A.shape[1]
    A = _c(lora_A, np.uint16) if r > 0 else None
    B = _c(lora_B, np.uint16) if r > 0 else None
    exact = np.empty((t, n), np.float64)
    want_ste = Wq is not None
    ste = np.empty((t, n), np.float64) if want_ste else None
    lib().oracle_bwd_dx_outlier_cols(
        _p(dY), i64(t), i64(N), i64(N), _p(O), i32(n), _p(W_O), _p(_c(Wq, np.int8)) if want_ste else None,
        _p(_c(delta_w, np.float32)) if want_ste else None, _p(_c(what_int, np.int8)) if want_ste else None,
        _p(_c(delta_what, np.float32)) if want_ste else None, _p(_c(colscale, np.float32)) if want_ste else None,
        _p(A), _p(B), i32(r), f32(lora_scale), _p(exact), _p(ste))
    return exact, ste


def outlier_criterion(X, offsets, ratio=100.0):
    """Eq. 6: xi [c_in] int32 for calibration samples stored one after the other (offsets [n_samples + 1])."""
    X = _c(X, np.uint16)
    offsets = _c(offsets, np.int64)
    c_in = X.shape[1]
    xi = np.empty(c_in, np.int32)
    lib().oracle_outlier_criterion(_p(X), i64(c_in), i64(c_in), _p(offsets), i32(offsets.size - 1),
                                   C.c_double(ratio), _p(xi))
    return xi


def select_outliers(xi, budget):
    xi = _c(xi, np.int32)
    O = np.empty(max(budget, 1), np.int32)
    n = lib().oracle_select_outliers(_p(xi), i64(xi.size), i32(budget), _p(O))
    return O[:n].copy()
