"""ctypes front end of the CPU oracle.  TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the bench's cpu_baseline leg may import this
package.  It loads oracle/liboracle.so (plain C, fp64; see dpllm_oracle.c for
the passage of the paper each function follows) and marshals numpy arrays.
Nothing here touches the GPU library.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.orc_half_to_double.restype = C.c_double
        L.orc_half_to_double.argtypes = [C.c_uint16]
        L.orc_threads.restype = C.c_int
        L.orc_unpack.restype = None
        L.orc_unpack.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
        L.orc_index_k.restype = None
        L.orc_index_k.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_int, C.c_void_p]
        L.orc_dequant.restype = None
        L.orc_dequant.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
        L.orc_gemv.restype = None
        L.orc_gemv.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int,
                               C.c_void_p, C.c_int, C.c_void_p]
        L.orc_exact_err.restype = C.c_double
        L.orc_exact_err.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                    C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.orc_estimate.restype = C.c_double
        L.orc_estimate.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.orc_linreg_estimate.restype = C.c_double
        L.orc_linreg_estimate.argtypes = [C.c_void_p, C.c_int, C.c_double, C.c_double]
        L.orc_decide.restype = C.c_int
        L.orc_decide.argtypes = [C.c_double, C.c_float, C.c_int, C.c_int]
        L.orc_effective_bits.restype = C.c_double
        L.orc_effective_bits.argtypes = [C.c_void_p, C.c_void_p, C.c_int]
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _u32(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint32
    return a


def _u16(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16
    return a


def threads() -> int:
    return int(lib().orc_threads())


def half_to_double(bits: int) -> float:
    return float(lib().orc_half_to_double(int(bits)))


def unpack(planes) -> np.ndarray:
    """planes uint32 [p][out][in/32] -> parent codes uint8 [out][in]."""
    planes = _u32(planes)
    p, out, nw = planes.shape
    idx = np.empty((out, nw * 32), dtype=np.uint8)
    lib().orc_unpack(_p(planes), p, out, nw * 32, _p(idx))
    return idx


def index_k(idx_p, p: int, k: int) -> np.ndarray:
    idx_p = np.ascontiguousarray(idx_p, dtype=np.uint8)
    res = np.empty_like(idx_p)
    lib().orc_index_k(_p(idx_p), idx_p.size, p, k, _p(res))
    return res


def dequant(idx_k, lut_k, k: int) -> np.ndarray:
    idx_k = np.ascontiguousarray(idx_k, dtype=np.uint8)
    lut_k = _u16(lut_k)
    out, in_ = idx_k.shape
    assert lut_k.shape == (out, 1 << k)
    W = np.empty((out, in_), dtype=np.float64)
    lib().orc_dequant(_p(idx_k), _p(lut_k), k, out, in_, _p(W))
    return W


def gemv(planes, k: int, lut_k, x) -> np.ndarray:
    """y = W_k x in fp64.  x: fp16 [in] or [B][in]; returns [out] or [B][out]."""
    planes = _u32(planes)
    lut_k = _u16(lut_k)
    x = _u16(x)
    p, out, nw = planes.shape
    in_ = nw * 32
    assert lut_k.shape == (out, 1 << k), (lut_k.shape, out, k)
    squeeze = x.ndim == 1
    xb = x.reshape(1, -1) if squeeze else x
    assert xb.shape[1] == in_
    B = xb.shape[0]
    y = np.empty((B, out), dtype=np.float64)
    lib().orc_gemv(_p(planes), p, k, _p(lut_k), out, in_, _p(np.ascontiguousarray(xb)), B, _p(y))
    return y[0] if squeeze else y


def exact_err(planes, l: int, h: int, lut_l, lut_h, x):
    """(||(W_h - W_l) x||_2, ||W_h x||_2) in fp64."""
    planes = _u32(planes)
    lut_l = _u16(lut_l)
    lut_h = _u16(lut_h)
    x = _u16(x)
    p, out, nw = planes.shape
    norm_h = C.c_double(0.0)
    e = lib().orc_exact_err(_p(planes), p, l, h, _p(lut_l), _p(lut_h), out, nw * 32, _p(x),
                            C.byref(norm_h))
    return float(e), float(norm_h.value)


def estimate(G, x, return_g: bool = False):
    """||G x||_2 in fp64, G fp16 [r][in]."""
    G = _u16(G)
    x = _u16(x)
    r, in_ = G.shape
    assert x.shape == (in_,)
    g = np.empty(r, dtype=np.float64)
    e = float(lib().orc_estimate(_p(G), r, in_, _p(x), _p(g)))
    return (e, g) if return_g else e


def linreg_estimate(x, alpha: float, beta: float) -> float:
    x = _u16(x)
    return float(lib().orc_linreg_estimate(_p(x), x.size, alpha, beta))


def decide(e: float, T: float, l: int, h: int) -> int:
    return int(lib().orc_decide(float(e), float(np.float32(T)), l, h))


def effective_bits(ks, params) -> float:
    ks = np.ascontiguousarray(ks, dtype=np.int32)
    params = np.ascontiguousarray(params, dtype=np.int64)
    return float(lib().orc_effective_bits(_p(ks), _p(params), ks.size))


def decode_step(linears, xs, xs_sel=None):
    """Selector then GEMV for every linear in model order.

    xs_sel: optional list; where an entry is not None the selector of that linear reads it instead of the
            linear's input (paper Sec. 5.2, asynchronous estimation: layers fed by the residual stream may
            estimate on the previous residual vector); the GEMV always reads xs.

    linears: list of dicts with planes, luts {k: lut}, and a selector dict
             {l, h, kind (0 none, 1 projection, 2 linear regression), G, alpha, beta, T}.
    xs:      one fp16 input vector per linear.
    Returns (ys, ks, es).
    """
    ys, ks, es = [], [], []
    for i, (lin, x) in enumerate(zip(linears, xs)):
        sel = lin["selector"]
        l, h = sel["l"], sel["h"]
        xe = x if xs_sel is None or xs_sel[i] is None else xs_sel[i]
        if sel["kind"] == 1:
            e = estimate(sel["G"], xe)
            k = decide(e, sel["T"], l, h)
        elif sel["kind"] == 2:
            e = linreg_estimate(xe, sel["alpha"], sel["beta"])
            k = decide(e, sel["T"], l, h)
        else:
            e, k = 0.0, l
        ys.append(gemv(lin["planes"], k, lin["luts"][k], x))
        ks.append(k)
        es.append(e)
    return ys, np.array(ks, dtype=np.int32), np.array(es, dtype=np.float64)
