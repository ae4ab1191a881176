"""Python face of the CPU oracle (``xnor_oracle.c``).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the bench's ``cpu_baseline`` leg call this
module; the product package never does, and this module imports nothing from the product package.
All arithmetic lives in the C file; this file only compiles it (gcc, ``-O2 -fopenmp``), loads it
with ctypes and marshals numpy arrays.

Function names follow the paper's pipeline (Sec. III-A step list): ``sign`` / ``pack`` (step 1a),
``dot`` (steps 1b-1d), ``scale_K`` (Eq. 10), ``alpha`` (Eq. 5), ``out`` / ``forward`` (Eq. 11);
``bwn`` is the Binary-Weight-Network layer of Sec. II-A (Eq. 1); ``conv_fp32`` is the real-valued
convolution that Table I (Sec. IV) compares the XNOR convolution with.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "xnor_oracle.c")
_LIB = os.path.join(_HERE, "libxnor_oracle.so")
_lib = None


class _Shape(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int) for k in
                ("N", "C", "H", "W", "F", "kh", "kw", "sh", "sw", "ph", "pw")]


@dataclass(frozen=True)
class Shape:
    N: int
    C: int
    H: int
    W: int
    F: int
    kh: int
    kw: int
    sh: int = 1
    sw: int = 1
    ph: int = 0
    pw: int = 0

    def c(self) -> _Shape:
        return _Shape(self.N, self.C, self.H, self.W, self.F, self.kh, self.kw,
                      self.sh, self.sw, self.ph, self.pw)


def build(force: bool = False) -> str:
    """Compile the oracle with the host C compiler; returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        up = ctypes.POINTER(ctypes.c_uint32)
        sp = ctypes.POINTER(_Shape)
        ci = ctypes.c_int
        lib.oracle_threads.argtypes = []
        lib.oracle_threads.restype = ci
        lib.oracle_out_dims.argtypes = [sp, ctypes.POINTER(ci), ctypes.POINTER(ci)]
        lib.oracle_out_dims.restype = ci
        lib.oracle_sign.argtypes = [fp, ctypes.c_size_t, fp]
        lib.oracle_sign.restype = None
        lib.oracle_pack.argtypes = [fp, ci, ci, ci, ci, up]
        lib.oracle_pack.restype = None
        lib.oracle_dot.argtypes = [fp, fp, sp, ip]
        lib.oracle_dot.restype = ci
        lib.oracle_A.argtypes = [fp, ci, ci, ci, ci, dp]
        lib.oracle_A.restype = None
        lib.oracle_K.argtypes = [fp, sp, dp, fp]
        lib.oracle_K.restype = ci
        lib.oracle_alpha.argtypes = [fp, ci, ci, ci, ci, fp]
        lib.oracle_alpha.restype = None
        lib.oracle_out.argtypes = [ip, fp, fp, ci, ci, ci, ci, fp]
        lib.oracle_out.restype = None
        lib.oracle_bwn.argtypes = [fp, fp, sp, fp, fp, dp]
        lib.oracle_bwn.restype = ci
        lib.oracle_conv_fp32.argtypes = [fp, fp, sp, fp, dp]
        lib.oracle_conv_fp32.restype = ci
        _lib = lib
    return _lib


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _ptr(a: np.ndarray, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def threads() -> int:
    """OpenMP threads the (image, filter) loop of ``dot`` runs on."""
    return _load().oracle_threads()


def out_dims(s: Shape) -> tuple[int, int]:
    oh, ow = ctypes.c_int(), ctypes.c_int()
    if _load().oracle_out_dims(ctypes.byref(s.c()), ctypes.byref(oh), ctypes.byref(ow)):
        raise ValueError(f"bad shape {s}")
    return oh.value, ow.value


def sign(x) -> np.ndarray:
    x = _f32(x)
    s = np.empty_like(x)
    _load().oracle_sign(_ptr(x, ctypes.c_float), x.size, _ptr(s, ctypes.c_float))
    return s


def pack(x) -> np.ndarray:
    """x[N][C][H][W] fp32 -> uint32 [N][H][W][ceil(C/32)], bit j of word w = channel 32w+j >= 0."""
    x = _f32(x)
    N, C, H, W = x.shape
    out = np.empty((N, H, W, (C + 31) // 32), dtype=np.uint32)
    _load().oracle_pack(_ptr(x, ctypes.c_float), N, C, H, W, _ptr(out, ctypes.c_uint32))
    return out


def _check(I: np.ndarray, Wt: np.ndarray, s: Shape):
    if I.shape != (s.N, s.C, s.H, s.W) or Wt.shape != (s.F, s.C, s.kh, s.kw):
        raise ValueError(f"array shapes {I.shape} {Wt.shape} do not match {s}")


def dot(I, Wt, s: Shape) -> np.ndarray:
    I, Wt = _f32(I), _f32(Wt)
    _check(I, Wt, s)
    OH, OW = out_dims(s)
    d = np.empty((s.N, s.F, OH, OW), dtype=np.int32)
    if _load().oracle_dot(_ptr(I, ctypes.c_float), _ptr(Wt, ctypes.c_float),
                          ctypes.byref(s.c()), _ptr(d, ctypes.c_int32)):
        raise ValueError(f"bad shape {s}")
    return d


def channel_mean_abs(I) -> np.ndarray:
    """A of Eq. 10, in double."""
    I = _f32(I)
    N, C, H, W = I.shape
    A = np.empty((N, H, W), dtype=np.float64)
    _load().oracle_A(_ptr(I, ctypes.c_float), N, C, H, W, _ptr(A, ctypes.c_double))
    return A


def scale_K(I, s: Shape) -> np.ndarray:
    I = _f32(I)
    if I.shape != (s.N, s.C, s.H, s.W):
        raise ValueError("input shape mismatch")
    OH, OW = out_dims(s)
    A = np.empty((s.N, s.H, s.W), dtype=np.float64)
    K = np.empty((s.N, OH, OW), dtype=np.float32)
    if _load().oracle_K(_ptr(I, ctypes.c_float), ctypes.byref(s.c()),
                        _ptr(A, ctypes.c_double), _ptr(K, ctypes.c_float)):
        raise ValueError(f"bad shape {s}")
    return K


def alpha(Wt) -> np.ndarray:
    Wt = _f32(Wt)
    F, C, kh, kw = Wt.shape
    a = np.empty((F,), dtype=np.float32)
    _load().oracle_alpha(_ptr(Wt, ctypes.c_float), F, C, kh, kw, _ptr(a, ctypes.c_float))
    return a


def out(d, K, a) -> np.ndarray:
    d = np.ascontiguousarray(d, dtype=np.int32)
    K, a = _f32(K), _f32(a)
    N, F, OH, OW = d.shape
    if K.shape != (N, OH, OW) or a.shape != (F,):
        raise ValueError("shape mismatch")
    O = np.empty((N, F, OH, OW), dtype=np.float32)
    _load().oracle_out(_ptr(d, ctypes.c_int32), _ptr(K, ctypes.c_float), _ptr(a, ctypes.c_float),
                       N, F, OH, OW, _ptr(O, ctypes.c_float))
    return O


def forward(I, Wt, s: Shape):
    """Whole pipeline: returns (dot int32, K fp32, alpha fp32, O fp32)."""
    d = dot(I, Wt, s)
    K = scale_K(I, s)
    a = alpha(Wt)
    return d, K, a, out(d, K, a)


def bwn(I, Wt, s: Shape, want_scale: bool = False):
    """Binary-Weight-Network layer (Eq. 1): O = alpha * (I (+) sign(Wt)), fp32 [N][F][OH][OW].

    With ``want_scale`` also returns S[N][OH][OW] = sum |I| over each output's in-image taps (double)."""
    I, Wt = _f32(I), _f32(Wt)
    _check(I, Wt, s)
    OH, OW = out_dims(s)
    a = alpha(Wt)
    O = np.empty((s.N, s.F, OH, OW), dtype=np.float32)
    S = np.empty((s.N, OH, OW), dtype=np.float64) if want_scale else None
    if _load().oracle_bwn(_ptr(I, ctypes.c_float), _ptr(Wt, ctypes.c_float), ctypes.byref(s.c()),
                          _ptr(a, ctypes.c_float), _ptr(O, ctypes.c_float),
                          _ptr(S, ctypes.c_double) if want_scale else None):
        raise ValueError(f"bad shape {s}")
    return (O, S) if want_scale else O


def conv_fp32(I, Wt, s: Shape, want_scale: bool = False):
    """Real-valued convolution (the float comparison of Table I, Sec. IV): O = sum I * Wt over channels
    and in-image taps, fp32 [N][F][OH][OW], summed in double.

    With ``want_scale`` also returns S[N][F][OH][OW] = sum |I * Wt| over the same terms (double)."""
    I, Wt = _f32(I), _f32(Wt)
    _check(I, Wt, s)
    OH, OW = out_dims(s)
    O = np.empty((s.N, s.F, OH, OW), dtype=np.float32)
    S = np.empty((s.N, s.F, OH, OW), dtype=np.float64) if want_scale else None
    if _load().oracle_conv_fp32(_ptr(I, ctypes.c_float), _ptr(Wt, ctypes.c_float), ctypes.byref(s.c()),
                                _ptr(O, ctypes.c_float), _ptr(S, ctypes.c_double) if want_scale else None):
        raise ValueError(f"bad shape {s}")
    return (O, S) if want_scale else O
