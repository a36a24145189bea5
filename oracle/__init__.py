"""ctypes access to the fp64 CPU oracle (oracle/chebykan_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The GPU library never imports or links this.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "chebykan_oracle.c"), os.path.join(_HERE, "chebykan_lut_oracle.c"),
         os.path.join(_HERE, "kan_bases_oracle.c")]
# CHEBYKAN_ORACLE_SANITIZE=1 builds and loads an AddressSanitizer + UndefinedBehaviorSanitizer build instead
# (the interpreter must then run with the sanitizer runtime preloaded; tests/test_sanitizers_host.py does that).
_SANITIZE = os.environ.get("CHEBYKAN_ORACLE_SANITIZE", "0") == "1"
_LIB = os.path.join(_HERE, "liboracle_san.so" if _SANITIZE else "liboracle.so")
_lib: Optional[ctypes.CDLL] = None

MAX_DEGREE = 64


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(s) for s in _SRCS):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
               "-fno-omit-frame-pointer"] if _SANITIZE else ["-O2"]
        cmd = ["gcc", *opt, "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-ffp-contract=off", "-o", tmp, *_SRCS, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int64)
        i64 = ctypes.c_int64
        lib.oracle_cheb_T.argtypes = [ctypes.c_double, ctypes.c_int, dp]
        lib.oracle_cheb_T.restype = None
        lib.oracle_cheb_T_trig.argtypes = [ctypes.c_double, ctypes.c_int, dp]
        lib.oracle_cheb_T_trig.restype = None
        lib.oracle_cheb_dT.argtypes = [ctypes.c_double, ctypes.c_int, dp]
        lib.oracle_cheb_dT.restype = None
        lib.oracle_num_threads.argtypes = []
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_forward.argtypes = [dp, dp, dp, i64, i64, i64, ctypes.c_int]
        lib.oracle_forward.restype = ctypes.c_int
        lib.oracle_backward.argtypes = [dp, dp, dp, dp, dp, i64, i64, i64, ctypes.c_int]
        lib.oracle_backward.restype = ctypes.c_int
        lib.oracle_forward_at.argtypes = [dp, dp, ip, ip, i64, dp, i64, i64, i64, ctypes.c_int]
        lib.oracle_forward_at.restype = ctypes.c_int
        lib.oracle_dx_at.argtypes = [dp, dp, dp, ip, ip, i64, dp, i64, i64, i64, ctypes.c_int]
        lib.oracle_dx_at.restype = ctypes.c_int
        lib.oracle_dC_at.argtypes = [dp, dp, ip, ip, ip, i64, dp, i64, i64, i64, ctypes.c_int]
        lib.oracle_dC_at.restype = ctypes.c_int
        i8p = ctypes.POINTER(ctypes.c_int8)
        lib.oracle_lut_build.argtypes = [dp, ctypes.c_int, i64]
        lib.oracle_lut_build.restype = ctypes.c_int
        lib.oracle_lut_eval.argtypes = [dp, ctypes.c_int, i64, ctypes.c_double, ctypes.c_int, dp, dp,
                                        ctypes.POINTER(ctypes.c_int64), dp]
        lib.oracle_lut_eval.restype = None
        lib.oracle_forward_lut.argtypes = [dp, dp, dp, i64, dp, i64, i64, i64, ctypes.c_int]
        lib.oracle_forward_lut.restype = ctypes.c_int
        lib.oracle_backward_lut.argtypes = [dp, dp, dp, dp, i64, i8p, dp, dp, dp, i64, i64, i64, ctypes.c_int]
        lib.oracle_backward_lut.restype = ctypes.c_int
        lib.oracle_lut_build_derivative.argtypes = [dp, ctypes.c_int, i64]
        lib.oracle_lut_build_derivative.restype = ctypes.c_int
        lib.oracle_lut_eval_derivative.argtypes = [dp, ctypes.c_int, i64, ctypes.c_double, dp]
        lib.oracle_lut_eval_derivative.restype = None
        lib.oracle_dx_lut2.argtypes = [dp, dp, dp, dp, i64, dp, i64, i64, i64, ctypes.c_int]
        lib.oracle_dx_lut2.restype = ctypes.c_int
        lib.oracle_basis_eval.argtypes = [ctypes.c_int, ctypes.c_double, ctypes.c_int, dp, dp]
        lib.oracle_basis_eval.restype = ctypes.c_int
        lib.oracle_forward_basis.argtypes = [ctypes.c_int, dp, dp, dp, i64, i64, i64, ctypes.c_int]
        lib.oracle_forward_basis.restype = ctypes.c_int
        lib.oracle_backward_basis.argtypes = [ctypes.c_int, dp, dp, dp, dp, dp, i64, i64, i64, ctypes.c_int]
        lib.oracle_backward_basis.restype = ctypes.c_int
        lib.oracle_dC_lut_at.argtypes = [dp, dp, dp, i64, ip, ip, ip, i64, dp, i64, i64, i64, ctypes.c_int]
        lib.oracle_dC_lut_at.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.int64)


def _dp(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.POINTER(ctypes.c_double)()
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _ip(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def cheb_T(u: float, degree: int) -> np.ndarray:
    out = np.zeros(degree + 1)
    _load().oracle_cheb_T(float(u), int(degree), _dp(out))
    return out


def cheb_T_trig(u: float, degree: int) -> np.ndarray:
    out = np.zeros(degree + 1)
    _load().oracle_cheb_T_trig(float(u), int(degree), _dp(out))
    return out


def cheb_dT(u: float, degree: int) -> np.ndarray:
    out = np.zeros(degree + 1)
    _load().oracle_cheb_dT(float(u), int(degree), _dp(out))
    return out


def _check_shapes(x, C, dy=None) -> Tuple[int, int, int, int]:
    B, I = x.shape
    I2, O, K = C.shape
    if I2 != I:
        raise ValueError("C.shape[0] must equal x.shape[1]")
    if dy is not None and dy.shape != (B, O):
        raise ValueError("dy must be [batch, out]")
    if K - 1 > MAX_DEGREE:
        raise ValueError("degree above oracle maximum")
    return B, I, O, K - 1


def forward(x, C) -> np.ndarray:
    """y[B,O] in fp64 from x[B,I], C[I,O,d+1] (any float dtype, promoted exactly)."""
    x, C = _f64(x), _f64(C)
    B, I, O, d = _check_shapes(x, C)
    y = np.empty((B, O), dtype=np.float64)
    rc = _load().oracle_forward(_dp(x), _dp(C), _dp(y), B, I, O, d)
    assert rc == 0
    return y


def backward(x, C, dy, need_dx: bool = True, need_dC: bool = True):
    """(dx[B,I], dC[I,O,d+1]) in fp64; an unrequested output is None."""
    x, C, dy = _f64(x), _f64(C), _f64(dy)
    B, I, O, d = _check_shapes(x, C, dy)
    dx = np.empty((B, I), dtype=np.float64) if need_dx else None
    dC = np.empty((I, O, d + 1), dtype=np.float64) if need_dC else None
    rc = _load().oracle_backward(_dp(x), _dp(C), _dp(dy), _dp(dx), _dp(dC), B, I, O, d)
    assert rc == 0
    return dx, dC


def forward_at(x, C, bs, os_) -> np.ndarray:
    x, C = _f64(x), _f64(C)
    B, I, O, d = _check_shapes(x, C)
    bs, os_ = _i64(bs), _i64(os_)
    assert bs.shape == os_.shape and bs.ndim == 1
    assert bs.size == 0 or (bs.min() >= 0 and bs.max() < B and os_.min() >= 0 and os_.max() < O)
    out = np.empty(bs.size, dtype=np.float64)
    rc = _load().oracle_forward_at(_dp(x), _dp(C), _ip(bs), _ip(os_), bs.size, _dp(out), B, I, O, d)
    assert rc == 0
    return out


def dx_at(x, C, dy, bs, is_) -> np.ndarray:
    x, C, dy = _f64(x), _f64(C), _f64(dy)
    B, I, O, d = _check_shapes(x, C, dy)
    bs, is_ = _i64(bs), _i64(is_)
    assert bs.shape == is_.shape and bs.ndim == 1
    assert bs.size == 0 or (bs.min() >= 0 and bs.max() < B and is_.min() >= 0 and is_.max() < I)
    out = np.empty(bs.size, dtype=np.float64)
    rc = _load().oracle_dx_at(_dp(x), _dp(C), _dp(dy), _ip(bs), _ip(is_), bs.size, _dp(out), B, I, O, d)
    assert rc == 0
    return out


def dC_at(x, dy, degree: int, is_, os_, ks) -> np.ndarray:
    x, dy = _f64(x), _f64(dy)
    B, I = x.shape
    O = dy.shape[1]
    assert dy.shape[0] == B
    is_, os_, ks = _i64(is_), _i64(os_), _i64(ks)
    assert is_.shape == os_.shape == ks.shape and is_.ndim == 1
    assert is_.size == 0 or (is_.min() >= 0 and is_.max() < I and os_.min() >= 0 and os_.max() < O
                             and ks.min() >= 0 and ks.max() <= degree)
    out = np.empty(is_.size, dtype=np.float64)
    rc = _load().oracle_dC_at(_dp(x), _dp(dy), _ip(is_), _ip(os_), _ip(ks), is_.size, _dp(out),
                              B, I, O, int(degree))
    assert rc == 0
    return out


def rel_err(got, want) -> float:
    """max |got - want| / RMS(want): the error measure the parity bar is stated in."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if want.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(want * want)))
    diff = float(np.max(np.abs(got - want)))
    if rms == 0.0:
        return 0.0 if diff == 0.0 else float("inf")
    return diff / rms


# ------------------------------------------------- table-interpolated variant

def lut_build(degree: int, n: int) -> np.ndarray:
    """LUT[k, i] = T_k(-1 + i*2/(n-1)) in fp64, shape [degree+1, n] (paper Sec. 4.2.1)."""
    lut = np.empty((degree + 1, n), dtype=np.float64)
    rc = _load().oracle_lut_build(_dp(lut), int(degree), int(n))
    if rc != 0:
        raise ValueError("oracle_lut_build failed")
    return lut


def lut_eval(lut, u: float, shift: int = 0):
    """(T, dT, cell, frac) of the interpolated basis at u (paper Sec. 4.2.2)."""
    lut = _f64(lut)
    K, n = lut.shape
    T = np.empty(K)
    dT = np.empty(K)
    cell = ctypes.c_int64(0)
    frac = ctypes.c_double(0.0)
    _load().oracle_lut_eval(_dp(lut), K - 1, n, float(u), int(shift), _dp(T), _dp(dT), ctypes.byref(cell),
                            ctypes.byref(frac))
    return T, dT, cell.value, frac.value


def lut_build_derivative(degree: int, n: int) -> np.ndarray:
    """dLUT[k, i] = T_k'(-1 + i*2/(n-1)) in fp64, shape [degree+1, n]: the auxiliary derivative table."""
    dlut = np.empty((degree + 1, n), dtype=np.float64)
    rc = _load().oracle_lut_build_derivative(_dp(dlut), int(degree), int(n))
    if rc != 0:
        raise ValueError("oracle_lut_build_derivative failed")
    return dlut


def lut_eval_derivative(dlut, u: float) -> np.ndarray:
    """The interpolated derivative table at u: dT_0..dT_d."""
    dlut = _f64(dlut)
    K, n = dlut.shape
    dT = np.empty(K)
    _load().oracle_lut_eval_derivative(_dp(dlut), K - 1, n, float(u), _dp(dT))
    return dT


def dx_lut2(x, C, dy, dlut) -> np.ndarray:
    """dx of the table variant whose derivative comes from the interpolated auxiliary table."""
    B, I, O, d = _check_shapes(x, C, dy)
    x64, C64, dy64, dlut = _f64(x), _f64(C), _f64(dy), _f64(dlut)
    if dlut.shape[0] != d + 1:
        raise ValueError("table has %d rows, layer needs %d" % (dlut.shape[0], d + 1))
    dx = np.empty((B, I), dtype=np.float64)
    rc = _load().oracle_dx_lut2(_dp(x64), _dp(C64), _dp(dy64), _dp(dlut), dlut.shape[1], _dp(dx), B, I, O, d)
    if rc != 0:
        raise ValueError("oracle_dx_lut2 failed")
    return dx


def forward_lut(x, C, lut) -> np.ndarray:
    B, I, O, d = _check_shapes(x, C)
    x64, C64, lut = _f64(x), _f64(C), _f64(lut)
    if lut.shape[0] != d + 1:
        raise ValueError("table has %d rows, layer needs %d" % (lut.shape[0], d + 1))
    y = np.empty((B, O), dtype=np.float64)
    rc = _load().oracle_forward_lut(_dp(x64), _dp(C64), _dp(lut), lut.shape[1], _dp(y), B, I, O, d)
    if rc != 0:
        raise ValueError("oracle_forward_lut failed")
    return y


def backward_lut(x, C, dy, lut, need_dx: bool = True, need_dC: bool = True, shift=None, want_frac: bool = False):
    """dx, dC (and the in-cell position of every input element when want_frac) of the interpolated layer."""
    B, I, O, d = _check_shapes(x, C, dy)
    x64, C64, dy64, lut = _f64(x), _f64(C), _f64(dy), _f64(lut)
    if lut.shape[0] != d + 1:
        raise ValueError("table has %d rows, layer needs %d" % (lut.shape[0], d + 1))
    dx = np.empty((B, I), dtype=np.float64) if need_dx else None
    dC = np.empty((I, O, d + 1), dtype=np.float64) if need_dC else None
    frac = np.empty((B, I), dtype=np.float64) if want_frac else None
    sh = None
    if shift is not None:
        sh = np.ascontiguousarray(shift, dtype=np.int8)
        if sh.shape != (B, I):
            raise ValueError("shift must be [batch, in]")
    shp = sh.ctypes.data_as(ctypes.POINTER(ctypes.c_int8)) if sh is not None else None
    rc = _load().oracle_backward_lut(_dp(x64), _dp(C64), _dp(dy64), _dp(lut), lut.shape[1], shp, _dp(dx), _dp(dC),
                                     _dp(frac), B, I, O, d)
    if rc != 0:
        raise ValueError("oracle_backward_lut failed")
    return (dx, dC, frac) if want_frac else (dx, dC)


def dC_lut_at(x, dy, lut, is_, os_, ks) -> np.ndarray:
    """Sampled dC[i, o, k] of the interpolated layer, one element at a time."""
    x64, dy64, lut = _f64(x), _f64(dy), _f64(lut)
    B, I = x64.shape
    O = dy64.shape[1]
    is_, os_, ks = _i64(is_), _i64(os_), _i64(ks)
    out = np.empty(len(is_), dtype=np.float64)
    rc = _load().oracle_dC_lut_at(_dp(x64), _dp(dy64), _dp(lut), lut.shape[1], _ip(is_), _ip(os_), _ip(ks), len(is_),
                                  _dp(out), B, I, O, lut.shape[0] - 1)
    if rc != 0:
        raise ValueError("oracle_dC_lut_at failed")
    return out


# ------------------------------------------------------------- other bases
BASIS_CHEBYSHEV, BASIS_LEGENDRE, BASIS_HERMITE, BASIS_FOURIER = 0, 1, 2, 3


def basis_eval(kind: int, x: float, degree: int):
    """(B_0..B_d, dB_0/dx..dB_d/dx) of one basis family at the raw input x."""
    Bv = np.empty(degree + 1)
    dB = np.empty(degree + 1)
    if _load().oracle_basis_eval(int(kind), float(x), int(degree), _dp(Bv), _dp(dB)) != 0:
        raise ValueError("basis kind/degree not supported")
    return Bv, dB


def forward_basis(kind: int, x, C) -> np.ndarray:
    B, I, O, d = _check_shapes(x, C)
    x64, C64 = _f64(x), _f64(C)
    y = np.empty((B, O), dtype=np.float64)
    if _load().oracle_forward_basis(int(kind), _dp(x64), _dp(C64), _dp(y), B, I, O, d) != 0:
        raise ValueError("basis kind/degree not supported")
    return y


def backward_basis(kind: int, x, C, dy, need_dx: bool = True, need_dC: bool = True):
    B, I, O, d = _check_shapes(x, C, dy)
    x64, C64, dy64 = _f64(x), _f64(C), _f64(dy)
    dx = np.empty((B, I), dtype=np.float64) if need_dx else None
    dC = np.empty((I, O, d + 1), dtype=np.float64) if need_dC else None
    if _load().oracle_backward_basis(int(kind), _dp(x64), _dp(C64), _dp(dy64), _dp(dx), _dp(dC), B, I, O, d) != 0:
        raise ValueError("basis kind/degree not supported")
    return dx, dC
