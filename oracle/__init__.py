"""ctypes front end of the CPU fp64 oracle (``normtest_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  The GPU library never touches
it and the two share no code.

Arrays are numpy: gradients as a 2-D array of shape (J, n), dtype float32, or
uint16 holding bfloat16 bit patterns; the last axis must be contiguous, the
row stride is free.  State vectors ``w, m, v`` are float32.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "normtest_oracle.c")
_LIB = os.path.join(_HERE, "libnormtest_oracle.so")

F32, BF16 = 0, 1

NONFINITE = 1
ZERO_GRAD_NORM = 2
CLAMPED = 4
T_SATURATED = 16


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no fast-math: the compensated sums rely on IEEE order)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fno-fast-math", "-ffp-contract=off",
             "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"],
            check=True,
        )
        os.replace(tmp, _LIB)
    return _LIB


class _Decision(ctypes.Structure):
    _fields_ = [
        ("gbar_sq", ctypes.c_double),
        ("var_l1", ctypes.c_double),
        ("T", ctypes.c_double),
        ("next_b", ctypes.c_int64),
        ("pass_", ctypes.c_int32),
        ("status", ctypes.c_uint32),
    ]


_lib = None


def _bind(path: str):
    """Load a build of the oracle and declare its prototypes."""
    lib = ctypes.CDLL(path)
    i64, dbl, vp = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
    lib.nto_stats.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp]
    lib.nto_stats.restype = ctypes.c_int
    lib.nto_decide.argtypes = [dbl, dbl, dbl, i64, dbl, i64, i64, i64, ctypes.c_int32,
                               ctypes.POINTER(_Decision)]
    lib.nto_decide.restype = ctypes.c_int
    lib.nto_adamw.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, vp, vp, dbl, dbl, dbl, dbl, dbl,
                              i64, dbl, vp, vp, vp, vp]
    lib.nto_adamw.restype = ctypes.c_int
    lib.nto_coord_test.argtypes = [vp, ctypes.c_int, i64, i64, i64, dbl, i64, ctypes.c_int32, dbl, vp]
    lib.nto_coord_test.restype = ctypes.c_int
    lib.nto_coord_max_ratio.argtypes = [vp, ctypes.c_int, i64, i64, i64, dbl, i64, ctypes.c_int32, vp]
    lib.nto_coord_max_ratio.restype = ctypes.c_int
    lib.nto_resplit.argtypes = [i64, i64, i64, i64, vp, vp, vp]
    lib.nto_resplit.restype = ctypes.c_int
    lib.nto_test_due.argtypes = [i64, i64, i64, i64]
    lib.nto_test_due.restype = ctypes.c_int
    lib.nto_clip_coef.argtypes = [dbl, dbl]
    lib.nto_clip_coef.restype = dbl
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = _bind(build())
    return _lib


def _grad_args(G: np.ndarray):
    if G.ndim != 2:
        raise ValueError("gradients must be a (J, n) array")
    if G.dtype == np.float32:
        dtype = F32
    elif G.dtype == np.uint16:
        dtype = BF16
    else:
        raise ValueError("gradients must be float32 or uint16 (bfloat16 bits), got %s" % G.dtype)
    J, n = G.shape
    isz = G.dtype.itemsize
    if n > 0 and G.strides[1] != isz:
        raise ValueError("last axis must be contiguous")
    if J > 1 and n > 0:
        if G.strides[0] % isz or G.strides[0] < n * isz:
            raise ValueError("bad row stride")
        ld = G.strides[0] // isz
    else:
        ld = max(n, 1)
    return G.ctypes.data, dtype, J, ld, n


class StatsAccumulator:
    """Compensated running sums of A, B, C; feed coordinate ranges in any number of calls."""

    def __init__(self):
        self.acc = np.zeros(6, dtype=np.float64)

    def add(self, G: np.ndarray) -> "StatsAccumulator":
        ptr, dtype, J, ld, n = _grad_args(G)
        if n:
            rc = _load().nto_stats(ptr, dtype, J, ld, n, self.acc.ctypes.data)
            if rc:
                raise ValueError("nto_stats rejected its arguments")
        return self

    @property
    def ABC(self):
        a = self.acc
        return float(a[0] + a[1]), float(a[2] + a[3]), float(a[4] + a[5])


def stats(G: np.ndarray):
    """(A, B, C) = (sum_j ||g_j||^2, ||sum_j g_j||^2, sum_j ||g_j - gbar||^2)."""
    return StatsAccumulator().add(G).ABC


def combine_chunks(parts):
    """Exactly rounded sum of per-chunk (A, B, C) triples (used when chunks were evaluated separately)."""
    return tuple(math.fsum(p[k] for p in parts) for k in range(3))


@dataclass
class Decision:
    gbar_sq: float
    var_l1: float
    T: float
    next_b: int
    passed: bool
    status: int


def decide(A, B, C, J, eta, b_k, b_max=0, round_to=1, ddof=1) -> Decision:
    out = _Decision()
    rc = _load().nto_decide(A, B, C, J, eta, b_k, b_max, round_to, ddof, ctypes.byref(out))
    if rc:
        raise ValueError("nto_decide rejected its arguments")
    return Decision(out.gbar_sq, out.var_l1, out.T, int(out.next_b), bool(out.pass_), int(out.status))


def coord_test(G: np.ndarray, eta: float, b_k: int, ddof: int = 1, band: float = 0.0):
    """Coordinate-wise test: (fail, near, pass) counts over the columns of G; `near` = within the relative
    band of equality (0 when band = 0)."""
    ptr, dtype, J, ld, n = _grad_args(G)
    out = np.zeros(3, dtype=np.int64)
    if n:
        rc = _load().nto_coord_test(ptr, dtype, J, ld, n, eta, b_k, ddof, band, out.ctypes.data)
        if rc:
            raise ValueError("nto_coord_test rejected its arguments")
    else:
        if J - ddof < 1 or not eta > 0 or b_k < 1:
            raise ValueError("nto_coord_test rejected its arguments")
    return int(out[0]), int(out[1]), int(out[2])


def coord_max_ratio(G: np.ndarray, eta: float, b_k: int, ddof: int = 1, start: float = 0.0) -> float:
    """Largest Var_i / (eta^2 b_k gbar_i^2) over the columns of G (0 where a column has no spread, +inf where it
    has spread around a zero mean); `start` carries the maximum of earlier ranges of coordinates."""
    ptr, dtype, J, ld, n = _grad_args(G)
    out = np.array([start], dtype=np.float64)
    if n:
        rc = _load().nto_coord_max_ratio(ptr, dtype, J, ld, n, eta, b_k, ddof, out.ctypes.data)
        if rc:
            raise ValueError("nto_coord_max_ratio rejected its arguments")
    elif J - ddof < 1 or not eta > 0 or b_k < 1:
        raise ValueError("nto_coord_max_ratio rejected its arguments")
    return float(out[0])


def resplit(b: int, J: int, M_base: int, micro_max: int):
    """(micro_batch, accumulation_steps, global_batch) for a target global batch size b."""
    out = (ctypes.c_int64 * 3)()
    rc = _load().nto_resplit(b, J, M_base, micro_max, ctypes.byref(out, 0), ctypes.byref(out, 8), ctypes.byref(out, 16))
    if rc:
        raise ValueError("nto_resplit rejected its arguments")
    return int(out[0]), int(out[1]), int(out[2])


def test_due(step: int, interval: int, b_k: int, b_max: int = 0) -> bool:
    """Does step `step` (counted from 1) run the test, given the test interval and the batch-size maximum?"""
    rc = _load().nto_test_due(step, interval, b_k, b_max)
    if rc < 0:
        raise ValueError("nto_test_due rejected its arguments")
    return bool(rc)


test_due.__test__ = False  # not a pytest test, whatever its name


def clip_coef(gbar_sq: float, max_norm: float) -> float:
    """min(1, max_norm / (||gbar|| + 1e-6)); 1 when max_norm <= 0 (no clipping)."""
    return float(_load().nto_clip_coef(gbar_sq, max_norm))


def adamw(G, w, m, v, lr, beta1, beta2, eps, weight_decay, step, want_gbar=False, grad_scale=1.0):
    """One AdamW step on grad_scale * (mean of the rows of G); returns fp64 (w', m', v'[, gbar])."""
    ptr, dtype, J, ld, n = _grad_args(G)
    for x in (w, m, v):
        if x.dtype != np.float32 or x.ndim != 1 or x.shape[0] != n or not x.flags.c_contiguous:
            raise ValueError("w, m, v must be contiguous float32 vectors of length n")
    wo, mo, vo = (np.empty(n, dtype=np.float64) for _ in range(3))
    go = np.empty(n, dtype=np.float64) if want_gbar else None
    if n:
        rc = _load().nto_adamw(ptr, dtype, J, ld, n, w.ctypes.data, m.ctypes.data, v.ctypes.data,
                               lr, beta1, beta2, eps, weight_decay, step, grad_scale,
                               wo.ctypes.data, mo.ctypes.data, vo.ctypes.data,
                               go.ctypes.data if want_gbar else None)
        if rc:
            raise ValueError("nto_adamw rejected its arguments")
    return (wo, mo, vo, go) if want_gbar else (wo, mo, vo)


def layer_stats(G: np.ndarray, offsets, eta: float, b_k: int, ddof: int = 1, band=None):
    """The estimators of Sec. 3.2 / Alg. 1 restricted to blocks of coordinates: layer l owns columns
    offsets[l] .. offsets[l+1]-1.  Returns one dict per layer with A, B, C, the Decision of the layer's own
    statistic against b_k (no rounding, no cap), n, and, if `band` is given, the coordinate-wise counts."""
    offsets = [int(o) for o in offsets]
    n = G.shape[1]
    if len(offsets) < 2 or offsets[0] < 0 or offsets[-1] > n or any(a > b for a, b in zip(offsets, offsets[1:])):
        raise ValueError("offsets must ascend within [0, n]")
    J = G.shape[0]
    out = []
    for lo, hi in zip(offsets, offsets[1:]):
        A, B, C = stats(G[:, lo:hi])
        row = dict(A=A, B=B, C=C, n=hi - lo, dec=decide(A, B, C, J, eta, b_k, 0, 1, ddof))
        if band is not None:
            row["coord"] = coord_test(G[:, lo:hi], eta, b_k, ddof, band)
            row["coord_max_ratio"] = coord_max_ratio(G[:, lo:hi], eta, b_k, ddof)
        out.append(row)
    return out
