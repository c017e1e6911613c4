"""ctypes front end of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Loads ``oracle/libsga_oracle.so`` (compiled from ``sga_oracle.c`` with gcc; built
on demand when missing or older than its source) and exposes its functions on
numpy arrays.  bf16 tensors travel as ``uint16`` bit patterns.  The product
package never imports this module; only tests, the smoke check and the
benchmark's CPU-baseline leg do.

The operation itself (AVGGT paper, Sec. 4.3) is documented in ``sga_oracle.c``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sga_oracle.c")
_LIB = os.path.join(_HERE, "libsga_oracle.so")

DIAG = 1
MEAN = 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP over query rows)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


class _CShape(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("N", ctypes.c_int32),
        ("n_h", ctypes.c_int32), ("n_w", ctypes.c_int32),
        ("n_special", ctypes.c_int32),
        ("H", ctypes.c_int32), ("D", ctypes.c_int32),
        ("s_h", ctypes.c_int32), ("s_w", ctypes.c_int32),
        ("keep_first_frame", ctypes.c_int32),
        ("flags", ctypes.c_uint32),
        ("scale", ctypes.c_float),
        ("mean_logit_bias", ctypes.c_float),
    ]


@dataclass
class Shape:
    B: int
    N: int
    n_h: int
    n_w: int
    n_special: int
    H: int
    D: int
    s_h: int
    s_w: int
    keep_first_frame: int
    flags: int
    scale: float
    mean_logit_bias: float = 0.0

    @property
    def L(self) -> int:
        return self.n_special + self.n_h * self.n_w

    @property
    def NQ(self) -> int:
        return self.N * self.L

    def c(self) -> _CShape:
        return _CShape(self.B, self.N, self.n_h, self.n_w, self.n_special, self.H, self.D,
                       self.s_h, self.s_w, self.keep_first_frame, self.flags,
                       self.scale, self.mean_logit_bias)


_lib = None


def lib():
    global _lib
    if _lib is None:
        # SGA_ORACLE_LIBRARY_PATH: another build of the same source (the sanitizer run of the tests)
        _lib = ctypes.CDLL(os.environ.get("SGA_ORACLE_LIBRARY_PATH") or build())
        _lib.osga_num_threads.restype = ctypes.c_int
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, "bf16 data must be passed as uint16 bit patterns"
    return a


def num_threads() -> int:
    return int(lib().osga_num_threads())


def sigma_to_strides(sigma: int):
    sh, sw = ctypes.c_int32(0), ctypes.c_int32(0)
    rc = lib().osga_sigma_to_strides(ctypes.c_int(sigma), ctypes.byref(sh), ctypes.byref(sw))
    if rc != 0:
        raise ValueError("sigma %d is not in the paper's table" % sigma)
    return sh.value, sw.value


def is_kept(shape: Shape, tok: int) -> bool:
    cs = shape.c()
    return bool(lib().osga_is_kept(ctypes.byref(cs), ctypes.c_int64(tok)))


def counts(shape: Shape):
    cs = shape.c()
    k, d = ctypes.c_int64(0), ctypes.c_int64(0)
    lib().osga_counts(ctypes.byref(cs), ctypes.byref(k), ctypes.byref(d))
    return k.value, d.value


def kept_indices(shape: Shape) -> np.ndarray:
    m, _ = counts(shape)
    idx = np.empty(m, dtype=np.int32)
    cs = shape.c()
    lib().osga_kept_indices(ctypes.byref(cs), _p(idx))
    return idx


def gather(shape: Shape, K, V, idx: np.ndarray):
    K, V = _u16(K), _u16(V)
    M = int(idx.shape[0])
    Kc = np.empty((shape.B, shape.H, M, shape.D), dtype=np.uint16)
    Vc = np.empty_like(Kc)
    cs = shape.c()
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    lib().osga_gather(ctypes.byref(cs), _p(K), _p(V), _p(idx), ctypes.c_int64(M), _p(Kc), _p(Vc))
    return Kc, Vc


def mean(shape: Shape, K, V):
    K, V = _u16(K), _u16(V)
    km = np.empty((shape.B, shape.H, shape.D), dtype=np.float64)
    vm = np.empty_like(km)
    cs = shape.c()
    lib().osga_mean(ctypes.byref(cs), _p(K), _p(V), _p(km), _p(vm))
    return km, vm


def attn_rows(shape: Shape, Q, K, V, Kc, Vc, kmean, vmean, n_dropped: int, rows,
              want_p: bool = False):
    """SGA output for the query token ids in ``rows``.

    Returns (O [B, nrows, H, D] float64, lse [B, H, nrows] float64, P or None)."""
    Q, K, V, Kc, Vc = _u16(Q), _u16(K), _u16(V), _u16(Kc), _u16(Vc)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    nrows = int(rows.shape[0])
    M = int(Kc.shape[2])
    kmean = np.ascontiguousarray(kmean, dtype=np.float64)
    vmean = np.ascontiguousarray(vmean, dtype=np.float64)
    O = np.empty((shape.B, nrows, shape.H, shape.D), dtype=np.float64)
    lse = np.empty((shape.B, shape.H, nrows), dtype=np.float64)
    P = np.empty((shape.B, shape.H, nrows, M + 2), dtype=np.float64) if want_p else None
    cs = shape.c()
    lib().osga_attn_rows(ctypes.byref(cs), _p(Q), _p(K), _p(V), _p(Kc), _p(Vc), ctypes.c_int64(M),
                         _p(kmean), _p(vmean), ctypes.c_int64(n_dropped), _p(rows),
                         ctypes.c_int64(nrows), _p(O), _p(lse),
                         _p(P) if want_p else ctypes.c_void_p(0))
    return O, lse, P


def dense_rows(shape: Shape, Q, K, V, rows):
    Q, K, V = _u16(Q), _u16(K), _u16(V)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    nrows = int(rows.shape[0])
    O = np.empty((shape.B, nrows, shape.H, shape.D), dtype=np.float64)
    lse = np.empty((shape.B, shape.H, nrows), dtype=np.float64)
    cs = shape.c()
    lib().osga_dense_rows(ctypes.byref(cs), _p(Q), _p(K), _p(V), _p(rows), ctypes.c_int64(nrows),
                          _p(O), _p(lse))
    return O, lse


def sga(shape: Shape, Q, K, V, rows=None, want_p: bool = False):
    """The whole path on the CPU: index list, explicit compacted copy, mean pair,
    then attention for ``rows`` (default: every query).  Returns a dict."""
    idx = kept_indices(shape)
    _, n_dropped = counts(shape)
    Kc, Vc = gather(shape, K, V, idx)
    km, vm = mean(shape, K, V)
    if rows is None:
        rows = np.arange(shape.NQ, dtype=np.int64)
    O, lse, P = attn_rows(shape, Q, K, V, Kc, Vc, km, vm, n_dropped, rows, want_p)
    return dict(idx=idx, n_dropped=n_dropped, Kc=Kc, Vc=Vc, kmean=km, vmean=vm,
                O=O, lse=lse, P=P, rows=np.asarray(rows))


def frame_rows(shape: Shape, Q, K, V, rows):
    """Frame attention (Sec. 4.2): each listed query against the tokens of its own frame."""
    Q, K, V = _u16(Q), _u16(K), _u16(V)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    nrows = int(rows.shape[0])
    O = np.empty((shape.B, nrows, shape.H, shape.D), dtype=np.float64)
    lse = np.empty((shape.B, shape.H, nrows), dtype=np.float64)
    cs = shape.c()
    lib().osga_frame_rows(ctypes.byref(cs), _p(Q), _p(K), _p(V), _p(rows), ctypes.c_int64(nrows),
                          _p(O), _p(lse))
    return O, lse
