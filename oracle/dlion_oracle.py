"""numpy-facing wrapper around ``dlion_oracle.c`` -- TEST INFRASTRUCTURE.

The C file is the oracle; this module only compiles it with gcc, loads it with
ctypes and turns numpy arrays into pointers.  It holds none of the method's
arithmetic.  Conventions:

* ``x``  : float32 ``[d]``, updated in place.
* ``m``  : float32 ``[N, d]`` (rows may be strided), updated in place.
* ``g``  : float32 ``[N, d]`` or uint16 ``[N, d]`` holding bf16 bit patterns.
* packed : uint64 ``[N, W]``, ``W = ceil(d / 64)``; bit ``j % 64`` of word
  ``j // 64`` is coordinate ``j`` (1 = +1 vote), bits past ``d`` are zero.
* counts : uint16 ``[d]``, number of +1 votes per coordinate.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Sequence

import numpy as np

VOTE = 0
AVG = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(_HERE, "dlion_oracle.c")
_LIB = os.path.join(_HERE, "libdlion_oracle.so")

# -ffp-contract=off: every fp32 operation is rounded on its own (no FMA).
CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-pthread"]


def compile_source(src: str, out: str) -> str:
    """Compile one C source into a shared object with the oracle's flags."""
    tmp = out + f".tmp{os.getpid()}"
    subprocess.run(["gcc", *CFLAGS, "-o", tmp, src], check=True)
    os.replace(tmp, out)
    return out


def build(force: bool = False) -> str:
    """Compile the C oracle (if missing or older than its source) and return the path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(SOURCE)
    if force or stale:
        compile_source(SOURCE, _LIB)
    return _LIB


def words_for(d: int) -> int:
    return (int(d) + 63) // 64


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


def _rows(a: np.ndarray, dtypes: Sequence, name: str):
    """Check a ``[N, d]`` array with contiguous rows; return (N, d, row stride in elements)."""
    if a.ndim != 2:
        raise ValueError(f"{name} must be 2-D [N, d]")
    if a.dtype not in [np.dtype(t) for t in dtypes]:
        raise TypeError(f"{name} has dtype {a.dtype}")
    if a.shape[1] > 1 and a.strides[1] != a.itemsize:
        raise ValueError(f"{name} rows must be contiguous")
    if a.strides[0] % a.itemsize:
        raise ValueError(f"{name} row stride is not a whole number of elements")
    return a.shape[0], a.shape[1], a.strides[0] // a.itemsize


def _gdtype(g: np.ndarray) -> int:
    return 1 if g.dtype == np.uint16 else 0


class Oracle:
    """One loaded copy of the C oracle (the default one, or a variant a test compiled)."""

    def __init__(self, libpath: str | None = None):
        lib = ctypes.CDLL(libpath or build())
        i64, i32, f32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_float, ctypes.c_void_p
        ci = ctypes.c_int
        lib.oracle_worker_step.argtypes = [vp, i64, vp, i64, ci, vp, i64, vp, i64, i32, f32, f32]
        lib.oracle_worker_step.restype = None
        lib.oracle_aggregate_packed.argtypes = [vp, i64, i64, i32, vp]
        lib.oracle_aggregate_packed.restype = None
        lib.oracle_aggregate_signs.argtypes = [vp, i64, i32, vp]
        lib.oracle_aggregate_signs.restype = None
        lib.oracle_apply.argtypes = [vp, vp, i64, i32, ci, f32, f32, vp]
        lib.oracle_apply.restype = None
        lib.oracle_step.argtypes = [vp, vp, i64, vp, i64, ci, i64, i32, ci, f32, f32, f32, f32,
                                    vp, i64, vp]
        lib.oracle_step.restype = None
        lib.oracle_step_threads.argtypes = lib.oracle_step.argtypes + [ci]
        lib.oracle_step_threads.restype = ci
        lib.oracle_delta_planes.argtypes = [i32, ci]
        lib.oracle_delta_planes.restype = ci
        lib.oracle_encode_delta.argtypes = [vp, i64, i32, ci, vp, i64]
        lib.oracle_encode_delta.restype = None
        lib.oracle_apply_encoded.argtypes = [vp, vp, i64, i64, i32, ci, f32, f32, vp]
        lib.oracle_apply_encoded.restype = None
        lib.oracle_worker_step_pw.argtypes = [vp, i64, vp, i64, ci, vp, i64, i64, i32, vp, vp]
        lib.oracle_worker_step_pw.restype = None
        lib.oracle_global_lion_step.argtypes = [vp, vp, i64, vp, i64, ci, i64, i32, f32, f32, f32, f32, vp]
        lib.oracle_global_lion_step.restype = None
        self.lib = lib

    def worker_step(self, m, g, beta1, beta2, want_delta=False):
        """Worker side of one iteration for all N workers; returns ``packed`` (and int8 ``delta``)."""
        N, d, ms = _rows(m, [np.float32], "m")
        Ng, dg, gs = _rows(g, [np.float32, np.uint16], "g")
        if (N, d) != (Ng, dg):
            raise ValueError("m and g shapes differ")
        W = words_for(d)
        packed = np.empty((N, W), dtype=np.uint64)
        delta = np.empty((N, d), dtype=np.int8) if want_delta else None
        self.lib.oracle_worker_step(_ptr(m), ms, _ptr(g), gs, _gdtype(g), _ptr(packed), W,
                                    _ptr(delta) if want_delta else None, d, N, beta1, beta2)
        return (packed, delta) if want_delta else packed

    def aggregate_packed(self, packed, d):
        """Count of +1 votes per coordinate, read from the packed words."""
        N, W, ps = _rows(packed, [np.uint64], "packed")
        if W < words_for(d):
            raise ValueError("packed has too few words for d")
        counts = np.empty(d, dtype=np.uint16)
        self.lib.oracle_aggregate_packed(_ptr(packed), ps, d, N, _ptr(counts))
        return counts

    def aggregate_signs(self, delta):
        """Count of +1 votes per coordinate, from +-1 bytes ``[N, d]``."""
        delta = np.ascontiguousarray(delta, dtype=np.int8)
        N, d = delta.shape
        counts = np.empty(d, dtype=np.uint16)
        self.lib.oracle_aggregate_signs(_ptr(delta), d, N, _ptr(counts))
        return counts

    def apply(self, x, counts, N, mode, lr, lam, want_delta=False):
        """Aggregate (vote or average) and update ``x`` in place; optionally return Delta (fp32)."""
        if x.dtype != np.float32 or x.ndim != 1 or not x.flags.c_contiguous:
            raise TypeError("x must be contiguous float32 [d]")
        if counts.dtype != np.uint16 or counts.shape != x.shape or not counts.flags.c_contiguous:
            raise TypeError("counts must be contiguous uint16 [d]")
        delta = np.empty_like(x) if want_delta else None
        self.lib.oracle_apply(_ptr(x), _ptr(counts), x.shape[0], N, mode, lr, lam,
                              _ptr(delta) if want_delta else None)
        return delta

    def step(self, x, m, g, mode, beta1, beta2, lr, lam, threads=1):
        """One whole iteration; ``x`` and ``m`` updated in place; returns ``(packed, counts)``."""
        N, d, ms = _rows(m, [np.float32], "m")
        Ng, dg, gs = _rows(g, [np.float32, np.uint16], "g")
        if (N, d) != (Ng, dg):
            raise ValueError("m and g shapes differ")
        if x.dtype != np.float32 or x.shape != (d,) or not x.flags.c_contiguous:
            raise TypeError("x must be contiguous float32 [d]")
        W = words_for(d)
        packed = np.empty((N, W), dtype=np.uint64)
        counts = np.empty(d, dtype=np.uint16)
        args = (_ptr(x), _ptr(m), ms, _ptr(g), gs, _gdtype(g), d, N, mode, beta1, beta2, lr, lam,
                _ptr(packed), W, _ptr(counts))
        if threads <= 1:
            self.lib.oracle_step(*args)
        elif self.lib.oracle_step_threads(*args, threads) < 0:
            raise MemoryError("oracle_step_threads")
        return packed, counts

    def delta_planes(self, N, mode):
        """Number of bit-planes of the server -> worker message."""
        return self.lib.oracle_delta_planes(N, mode)

    def encode_delta(self, counts, N, mode):
        """Server -> worker message: ``[planes, W]`` uint64 bit-planes built from the counts."""
        counts = np.ascontiguousarray(counts, dtype=np.uint16)
        d = counts.shape[0]
        W = words_for(d)
        planes = np.empty((self.delta_planes(N, mode), W), dtype=np.uint64)
        self.lib.oracle_encode_delta(_ptr(counts), d, N, mode, _ptr(planes), W)
        return planes

    def apply_encoded(self, x, planes, N, mode, lr, lam, want_delta=False):
        """Worker side of the down-link: decode the planes and update ``x`` in place."""
        if x.dtype != np.float32 or x.ndim != 1 or not x.flags.c_contiguous:
            raise TypeError("x must be contiguous float32 [d]")
        P, W, ps = _rows(planes, [np.uint64], "planes")
        if P != self.delta_planes(N, mode) or W < words_for(x.shape[0]):
            raise ValueError("planes has the wrong shape")
        delta = np.empty_like(x) if want_delta else None
        self.lib.oracle_apply_encoded(_ptr(x), _ptr(planes), ps, x.shape[0], N, mode, lr, lam,
                                      _ptr(delta) if want_delta else None)
        return delta

    def worker_step_pw(self, m, g, beta1, beta2):
        """Worker step with per-worker coefficients (``beta1``, ``beta2`` float32 ``[N]``); returns packed."""
        N, d, ms = _rows(m, [np.float32], "m")
        Ng, dg, gs = _rows(g, [np.float32, np.uint16], "g")
        if (N, d) != (Ng, dg):
            raise ValueError("m and g shapes differ")
        b1 = np.ascontiguousarray(beta1, dtype=np.float32)
        b2 = np.ascontiguousarray(beta2, dtype=np.float32)
        if b1.shape != (N,) or b2.shape != (N,):
            raise ValueError("need one beta1 and one beta2 per worker")
        W = words_for(d)
        packed = np.empty((N, W), dtype=np.uint64)
        self.lib.oracle_worker_step_pw(_ptr(m), ms, _ptr(g), gs, _gdtype(g), _ptr(packed), W, d, N,
                                       _ptr(b1), _ptr(b2))
        return packed

    def global_lion_step(self, x, m, g, beta1, beta2, lr, lam):
        """One Global Lion iteration; ``x``, ``m`` in place; returns the packed sign of the mean blend."""
        N, d, ms = _rows(m, [np.float32], "m")
        Ng, dg, gs = _rows(g, [np.float32, np.uint16], "g")
        if (N, d) != (Ng, dg):
            raise ValueError("m and g shapes differ")
        if x.dtype != np.float32 or x.shape != (d,) or not x.flags.c_contiguous:
            raise TypeError("x must be contiguous float32 [d]")
        bits = np.empty(words_for(d), dtype=np.uint64)
        self.lib.oracle_global_lion_step(_ptr(x), _ptr(m), ms, _ptr(g), gs, _gdtype(g), d, N, beta1, beta2,
                                         lr, lam, _ptr(bits))
        return bits

    def step_mt(self, xs, ms, gs, mode, beta1, beta2, lr, lam, threads: int = 1):
        """Multi-tensor iteration: tensor ``k`` is ``xs[k]`` flat ``[n_k]``, ``ms[k]``/``gs[k]`` ``[N, n_k]``.

        Every tensor is an independent flat problem whose bits start on a fresh
        word; returns the per-tensor packed words concatenated along the word
        axis (``[N, sum_k ceil(n_k/64)]``) and the counts concatenated.
        """
        packed_all, counts_all = [], []
        for xk, mk, gk in zip(xs, ms, gs):
            pk, ck = self.step(xk, mk, gk, mode, beta1, beta2, lr, lam, threads=threads)
            packed_all.append(pk)
            counts_all.append(ck)
        return np.concatenate(packed_all, axis=1), np.concatenate(counts_all)


_default = None


def default() -> Oracle:
    global _default
    if _default is None:
        _default = Oracle()
    return _default


def worker_step(*a, **k):
    return default().worker_step(*a, **k)


def aggregate_packed(*a, **k):
    return default().aggregate_packed(*a, **k)


def aggregate_signs(*a, **k):
    return default().aggregate_signs(*a, **k)


def apply(*a, **k):
    return default().apply(*a, **k)


def step(*a, **k):
    return default().step(*a, **k)


def step_mt(*a, **k):
    return default().step_mt(*a, **k)


def delta_planes(*a, **k):
    return default().delta_planes(*a, **k)


def encode_delta(*a, **k):
    return default().encode_delta(*a, **k)


def apply_encoded(*a, **k):
    return default().apply_encoded(*a, **k)


def worker_step_pw(*a, **k):
    return default().worker_step_pw(*a, **k)


def global_lion_step(*a, **k):
    return default().global_lion_step(*a, **k)
