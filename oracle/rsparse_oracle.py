"""ctypes binding of oracle/rsparse_oracle.c (argument marshalling only).

TEST INFRASTRUCTURE: see the header of rsparse_oracle.c."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

F16, BF16, F64 = 0, 1, 2

# How close (in units of the local spacing of the 16-bit values) the exact gated input u * silu(g) must be to a
# rounding flip point before an evaluation within 3 fp32 ulp of silu, followed by one fp32 product rounding,
# may round the other way: 3.5 ulp <= 7 * 2^-24 relative, times 2^p spacings per unit of relative error
# (p = 11 significand bits for fp16, 8 for bf16).
RECIPE_BAND = {F16: 7.0 * 2.0 ** -24 * 2.0 ** 11, BF16: 7.0 * 2.0 ** -24 * 2.0 ** 8}

_lib = None


def _load():
    global _lib
    if _lib is None:
        # RSPARSE_ORACLE_LIB: a library built from a (deliberately altered) copy of the source, for the
        # test that plants mistakes in the oracle and expects the pins to catch them
        path = os.environ.get("RSPARSE_ORACLE_LIB") or _build.build(force=False)
        lib = C.CDLL(path)
        lib.orc_rsparse_linear.restype = C.c_int
        lib.orc_rsparse_linear.argtypes = [
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int,
            C.c_int, C.c_int, C.c_int, C.c_int, C.c_float, C.c_int, C.c_int,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int]
        lib.orc_rsparse_linear_ex.restype = C.c_int
        lib.orc_rsparse_linear_ex.argtypes = [
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int,
            C.c_int, C.c_int, C.c_int, C.c_int, C.c_float, C.c_int, C.c_int, C.c_int, C.c_void_p,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int]
        lib.orc_rsparse_linear_masked.restype = C.c_int
        lib.orc_rsparse_linear_masked.argtypes = [
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int,
            C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int]
        lib.orc_topk_mask.restype = C.c_int
        lib.orc_topk_mask.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
        lib.orc_multiphase.restype = C.c_double
        lib.orc_multiphase.argtypes = [C.c_double, C.c_void_p, C.c_int]
        lib.orc_multiphase_residual.restype = C.c_int
        lib.orc_multiphase_residual.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_int,
                                                C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        lib.orc_static_bias.restype = C.c_int
        lib.orc_static_bias.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int,
                                        C.c_void_p, C.c_int, C.c_void_p]
        lib.orc_dense_linear.restype = C.c_int
        lib.orc_dense_linear.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int,
                                         C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int]
        lib.orc_quantile_tau.restype = C.c_double
        lib.orc_quantile_tau.argtypes = [C.c_void_p, C.c_int, C.c_size_t, C.c_double]
        lib.orc_mask.restype = C.c_int
        lib.orc_mask.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_float, C.c_int, C.c_void_p]
        lib.orc_decode16.restype = None
        lib.orc_decode16.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_void_p]
        lib.orc_max_threads.restype = C.c_int
        lib.orc_gated_input.restype = C.c_int
        lib.orc_gated_input.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_size_t, C.c_void_p]
        lib.orc_silu32_array.restype = None
        lib.orc_silu32_array.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p]
        lib.orc_round16_array.restype = None
        lib.orc_round16_array.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_void_p]
        lib.orc_gated_input_plain.restype = C.c_int
        lib.orc_gated_input_plain.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_size_t, C.c_void_p, C.c_void_p]
        lib.orc_round16_from_double.restype = None
        lib.orc_round16_from_double.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_void_p]
        lib.orc_dequant_q4.restype = C.c_int
        lib.orc_dequant_q4.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
        _lib = lib
    return _lib


def _arr(a, kind):
    want = np.float64 if kind == F64 else np.uint16
    a = np.ascontiguousarray(a, dtype=want)
    return a


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def max_threads() -> int:
    return int(_load().orc_max_threads())


def decode16(bits, dtype) -> np.ndarray:
    bits = _arr(bits, dtype)
    out = np.empty(bits.shape, dtype=np.float64)
    _load().orc_decode16(_ptr(bits), bits.size, dtype, _ptr(out))
    return out


def silu32(g) -> np.ndarray:
    """The fp32 SiLU recipe that defines the gated input (see the C source)."""
    g = np.ascontiguousarray(g, dtype=np.float32)
    out = np.empty_like(g)
    _load().orc_silu32_array(_ptr(g), g.size, _ptr(out))
    return out


def gated_input(G16, U16, dtype) -> np.ndarray:
    """h = round16(silu32(g) * u) as uint16 bits (Sec. 3.1, the input of the MLP down projection)."""
    G16 = _arr(G16, dtype)
    U16 = _arr(U16, dtype)
    assert G16.shape == U16.shape
    out = np.empty(G16.shape, dtype=np.uint16)
    rc = _load().orc_gated_input(_ptr(G16), _ptr(U16), dtype, G16.size, _ptr(out))
    assert rc == 0
    return out


def gated_input_plain(G16, U16, dtype):
    """h = round16(u * g / (1 + exp(-g))) from the plain fp64 definition (Sec. 3.1), one rounding.
    Returns (bits, margin): margin = distance of the fp64 value from the nearest rounding flip point, in
    units of the local spacing of the 16-bit values (0 .. 0.5)."""
    G16 = _arr(G16, dtype)
    U16 = _arr(U16, dtype)
    assert G16.shape == U16.shape
    out = np.empty(G16.shape, dtype=np.uint16)
    margin = np.empty(G16.shape, dtype=np.float64)
    rc = _load().orc_gated_input_plain(_ptr(G16), _ptr(U16), dtype, G16.size, _ptr(out), _ptr(margin))
    assert rc == 0
    return out, margin


def round16(f32, dtype) -> np.ndarray:
    """The oracle's fp32 -> fp16 / bf16 rounding (nearest even), as uint16 bits."""
    f = np.ascontiguousarray(f32, dtype=np.float32)
    out = np.empty(f.shape, dtype=np.uint16)
    _load().orc_round16_array(_ptr(f), f.size, dtype, _ptr(out))
    return out


def round16_from_double(v, dtype) -> np.ndarray:
    """One rounding of fp64 values to fp16 / bf16 by the formats' definition, as uint16 bits."""
    v = np.ascontiguousarray(v, dtype=np.float64)
    out = np.empty(v.shape, dtype=np.uint16)
    _load().orc_round16_from_double(_ptr(v), v.size, dtype, _ptr(out))
    return out


def mask(x, x_kind, tau, cmp_mode=0) -> np.ndarray:
    x = _arr(x, x_kind).reshape(-1)
    m = np.empty(x.size, dtype=np.uint8)
    _load().orc_mask(_ptr(x), x_kind, x.size, float(np.float32(tau)), cmp_mode, _ptr(m))
    return m


def rsparse_linear(W, U, SV, X, kind_w, kind_x, tau, *, cmp_mode=0, batch_mask_mode=0,
                   nthreads=1, topk=0, bias=None):
    """Returns dict(Y [B,d_out] float64, act: list of ascending int32 arrays per token,
    union: ascending int32 array).  topk > 0: fixed-count masks instead of the threshold; bias: [d_out] added."""
    W = _arr(W, kind_w)
    d_out, d_in = W.shape
    X = _arr(X, kind_x)
    if X.ndim == 1:
        X = X[None, :]
    B = X.shape[0]
    assert X.shape[1] == d_in
    if U is None:
        r = 0
        U = np.zeros((d_out, 0), dtype=W.dtype)
        SV = np.zeros((0, d_in), dtype=W.dtype)
    U = _arr(U, kind_w)
    SV = _arr(SV, kind_w)
    r = U.shape[1] if U.ndim == 2 else 0
    assert U.shape == (d_out, r) and SV.shape == (r, d_in)
    Y = np.empty((B, d_out), dtype=np.float64)
    act = np.full((B, d_in), -1, dtype=np.int32)
    cnt = np.zeros(B, dtype=np.int32)
    uni = np.full(d_in, -1, dtype=np.int32)
    ucnt = np.zeros(1, dtype=np.int32)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float64)
        assert bias.shape == (d_out,)
    rc = _load().orc_rsparse_linear_ex(_ptr(W), _ptr(U), _ptr(SV), kind_w, _ptr(X), kind_x,
                                       B, d_in, d_out, r, float(np.float32(tau)), cmp_mode, int(topk),
                                       batch_mask_mode, _ptr(bias) if bias is not None else None,
                                       _ptr(Y), _ptr(act), _ptr(cnt), _ptr(uni), _ptr(ucnt), nthreads)
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return {"Y": Y, "act": [act[b, :cnt[b]].copy() for b in range(B)],
            "union": uni[:ucnt[0]].copy()}


def rsparse_linear_masked(W, U, SV, X, kind_w, kind_x, mask, *, bias=None, nthreads=1) -> np.ndarray:
    """Steps 2-4 for given masks [B][d_in] (1 = kept)."""
    W = _arr(W, kind_w)
    d_out, d_in = W.shape
    X = _arr(X, kind_x)
    if X.ndim == 1:
        X = X[None, :]
    B = X.shape[0]
    if U is None:
        U = np.zeros((d_out, 0), dtype=W.dtype)
        SV = np.zeros((0, d_in), dtype=W.dtype)
    U = _arr(U, kind_w)
    SV = _arr(SV, kind_w)
    r = U.shape[1]
    mask = np.ascontiguousarray(mask, dtype=np.uint8).reshape(B, d_in)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float64)
    Y = np.empty((B, d_out), dtype=np.float64)
    rc = _load().orc_rsparse_linear_masked(_ptr(W), _ptr(U), _ptr(SV), kind_w, _ptr(X), kind_x, B, d_in, d_out, r,
                                           _ptr(mask), _ptr(bias) if bias is not None else None, _ptr(Y), nthreads)
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return Y


def topk_mask(x, x_kind, k) -> np.ndarray:
    """uint8 [d_in]: 1 on the k channels of largest magnitude (lower channel first among equals, NaN never)."""
    x = _arr(x, x_kind).reshape(-1)
    m = np.zeros(x.shape[0], dtype=np.uint8)
    if _load().orc_topk_mask(_ptr(x), x_kind, x.shape[0], int(k), _ptr(m)) < 0:
        raise ValueError("oracle rejected its arguments")
    return m


def multiphase(x, T) -> np.ndarray:
    """sigma_T of Sec. 3.2, elementwise, float64 in and out."""
    T = np.ascontiguousarray(T, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    lib = _load()
    return np.array([lib.orc_multiphase(float(v), _ptr(T), len(T)) for v in x.reshape(-1)]).reshape(x.shape)


def multiphase_residual(W, kind_w, h, kind_h, T):
    """(Y_r [d_out], B [l-1][d_out]): the data-dependent residual of one token and its biases (Sec. 3.2)."""
    W = _arr(W, kind_w)
    d_out, d_in = W.shape
    h = _arr(h, kind_h).reshape(-1)
    T = np.ascontiguousarray(T, dtype=np.float64)
    Yr = np.empty(d_out)
    Bj = np.empty((max(len(T) - 1, 0), d_out))
    if _load().orc_multiphase_residual(_ptr(W), kind_w, _ptr(h), kind_h, d_in, d_out, _ptr(T), len(T), _ptr(Yr),
                                       _ptr(Bj) if Bj.size else None) != 0:
        raise ValueError("oracle rejected its arguments")
    return Yr, Bj


def static_bias(W, kind_w, H, kind_h, T) -> np.ndarray:
    """Mean over the calibration tokens H [N][d_in] of the data-dependent residual."""
    W = _arr(W, kind_w)
    d_out, d_in = W.shape
    H = _arr(H, kind_h).reshape(-1, d_in)
    T = np.ascontiguousarray(T, dtype=np.float64)
    b = np.empty(d_out)
    if _load().orc_static_bias(_ptr(W), kind_w, _ptr(H), kind_h, H.shape[0], d_in, d_out, _ptr(T), len(T), _ptr(b)) != 0:
        raise ValueError("oracle rejected its arguments")
    return b


def dense_linear(W, X, kind_w, kind_x, nthreads=1) -> np.ndarray:
    W = _arr(W, kind_w)
    d_out, d_in = W.shape
    X = _arr(X, kind_x)
    if X.ndim == 1:
        X = X[None, :]
    Y = np.empty((X.shape[0], d_out), dtype=np.float64)
    rc = _load().orc_dense_linear(_ptr(W), kind_w, _ptr(X), kind_x, X.shape[0], d_in, d_out,
                                  _ptr(Y), nthreads)
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return Y


def quantile_tau(x, x_kind, s) -> float:
    x = _arr(x, x_kind).reshape(-1)
    return float(_load().orc_quantile_tau(_ptr(x), x_kind, x.size, float(s)))


def dequant_q4(Q, S16, Z, dtype, group=128) -> np.ndarray:
    """W~ = s * (q - z) as float64 [d_out, d_in] (Sec. 4.4, 4-bit weights in GPTQ's group format)."""
    Q = np.ascontiguousarray(Q, dtype=np.uint8)
    d_out, d_in = Q.shape
    S16 = _arr(S16, dtype)
    Z = np.ascontiguousarray(Z, dtype=np.uint8)
    assert S16.shape == Z.shape == (d_out, d_in // group)
    W = np.empty((d_out, d_in), dtype=np.float64)
    if _load().orc_dequant_q4(_ptr(Q), _ptr(S16), dtype, _ptr(Z), d_out, d_in, group, _ptr(W)) != 0:
        raise ValueError("oracle rejected its arguments")
    return W


def rsparse_linear_q4(Q, S16, Z, U16, SV16, X, dtype, tau, *, group=128, **kw):
    """The R-Sparse layer on 4-bit weights: the plain layer with W~ in place of W; factors 16-bit."""
    W = dequant_q4(Q, S16, Z, dtype, group)
    U = None if U16 is None else decode16(U16, dtype)
    SV = None if SV16 is None else decode16(SV16, dtype)
    return rsparse_linear(W, U, SV, X, F64, dtype, tau, **kw)
