"""ctypes binding of ``libdlion.so``: argument marshalling only.

Every function here has the name and the meaning of the C entry point it calls
(see ``include/dlion.h``).  Tensors are torch CUDA tensors; the binding passes
their ``data_ptr()``, their row strides and the current HIP stream.  No step of
the method is computed in Python, and nothing falls back to another
implementation: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

VOTE = 0
AVG = 1
F32 = 0
BF16 = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdlion.so")
_lib = None

EXPORTS = (
    "dlion_worker_step", "dlion_aggregate", "dlion_apply", "dlion_aggregate_apply", "dlion_step",
    "dlion_mt_layout", "dlion_worker_step_mt", "dlion_aggregate_mt", "dlion_apply_mt",
    "dlion_aggregate_apply_mt", "dlion_step_mt", "dlion_status_str", "dlion_version",
    "dlion_delta_planes", "dlion_aggregate_encode", "dlion_apply_encoded", "dlion_worker_step_pw",
    "dlion_step_pw", "dlion_step_pw_ws", "dlion_global_lion_step", "dlion_step_ws", "dlion_step_workspace_bytes",
    "dlion_step_mt_ws", "dlion_step_mt_workspace_bytes", "dlion_tuning_defaults", "dlion_set_tuning",
    "dlion_get_tuning", "dlion_membench", "dlion_noalloc_init", "dlion_step_noalloc",
)


class DlionError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: status {status} ({status_str(status)})")


class Seg(ctypes.Structure):
    """Mirror of ``dlion_seg``."""
    _fields_ = [
        ("x", ctypes.c_void_p), ("m", ctypes.c_void_p), ("g", ctypes.c_void_p),
        ("m_stride", ctypes.c_int64), ("g_stride", ctypes.c_int64), ("numel", ctypes.c_int64),
        ("word_begin", ctypes.c_int64), ("tile_begin", ctypes.c_int64),
    ]


class Tuning(ctypes.Structure):
    """Mirror of ``dlion_tuning``: launch-shape overrides, -1 = the library decides."""
    _fields_ = [
        ("unroll", ctypes.c_int32), ("blocks_per_cu", ctypes.c_int32), ("pass_workers", ctypes.c_int32),
        ("step_quads", ctypes.c_int32), ("sliced_waves", ctypes.c_int32), ("sliced_min_workers", ctypes.c_int32),
        ("apply_blocks", ctypes.c_int32), ("blocks_per_cu_pass", ctypes.c_int32), ("block_tiles", ctypes.c_int64),
        ("group_blocks", ctypes.c_int32), ("group_max_workers", ctypes.c_int32),
    ]


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Load ``libdlion.so`` (or the build at ``path``), declare the prototypes and make it the library the
    functions of this module call; raises if the file is missing."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise FileNotFoundError(
            f"{p} is missing: build it first (python -m paper_2404_00438_amd.build); "
            "there is no fallback implementation")
    lib = ctypes.CDLL(p)
    vp, i64, i32, f32, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float, ctypes.c_int
    segp = ctypes.POINTER(Seg)
    protos = {
        "dlion_worker_step": [vp, i64, vp, i64, ci, vp, i64, i64, i32, f32, f32, vp],
        "dlion_aggregate": [vp, i64, i64, i32, vp, vp],
        "dlion_apply": [vp, vp, i64, i32, ci, f32, f32, vp],
        "dlion_aggregate_apply": [vp, vp, i64, i64, i32, ci, f32, f32, vp, vp],
        "dlion_step": [vp, vp, i64, vp, i64, ci, i64, i32, ci, f32, f32, f32, f32, vp, i64, vp, vp],
        "dlion_step_ws": [vp, vp, i64, vp, i64, ci, i64, i32, ci, f32, f32, f32, f32, vp, i64, vp, vp, i64, vp],
        "dlion_step_noalloc": [vp, vp, i64, vp, i64, ci, i64, i32, ci, f32, f32, f32, f32, vp, i64, vp, vp],
        "dlion_noalloc_init": [],
        "dlion_mt_layout": [segp, i32, ctypes.POINTER(i64), ctypes.POINTER(i64)],
        "dlion_worker_step_mt": [segp, vp, i32, ci, vp, i64, i32, f32, f32, vp],
        "dlion_aggregate_mt": [segp, vp, i32, vp, i64, i32, vp, vp],
        "dlion_apply_mt": [segp, vp, i32, vp, i32, ci, f32, f32, vp],
        "dlion_aggregate_apply_mt": [segp, vp, i32, vp, i64, i32, ci, f32, f32, vp, vp],
        "dlion_step_mt": [segp, vp, i32, ci, i32, ci, f32, f32, f32, f32, vp, i64, vp, vp],
        "dlion_step_mt_ws": [segp, vp, i32, ci, i32, ci, f32, f32, f32, f32, vp, i64, vp, vp, i64, vp],
        "dlion_set_tuning": [ctypes.POINTER(Tuning)],
        "dlion_membench": [vp, i64, i32, vp, i64, i32, i32, i32, vp],
        "dlion_delta_planes": [i32, ci],
        "dlion_aggregate_encode": [vp, i64, i64, i32, ci, vp, i64, vp],
        "dlion_apply_encoded": [vp, vp, i64, i64, i32, ci, f32, f32, vp],
        "dlion_worker_step_pw": [vp, i64, vp, i64, ci, vp, i64, i64, i32, vp, vp, vp],
        "dlion_step_pw": [vp, vp, i64, vp, i64, ci, i64, i32, ci, vp, vp, f32, f32, vp, i64, vp, vp],
        "dlion_step_pw_ws": [vp, vp, i64, vp, i64, ci, i64, i32, ci, vp, vp, f32, f32, vp, i64, vp, vp, i64, vp],
        "dlion_global_lion_step": [vp, vp, i64, vp, i64, ci, i64, i32, f32, f32, f32, f32, vp, vp],
    }
    for name, argtypes in protos.items():
        fn = getattr(lib, name)
        fn.argtypes = argtypes
        fn.restype = ci
    lib.dlion_status_str.argtypes = [ci]
    lib.dlion_status_str.restype = ctypes.c_char_p
    lib.dlion_version.argtypes = []
    lib.dlion_version.restype = ci
    lib.dlion_step_workspace_bytes.argtypes = [i64, i32]
    lib.dlion_step_workspace_bytes.restype = i64
    lib.dlion_step_mt_workspace_bytes.argtypes = [i64, i32]
    lib.dlion_step_mt_workspace_bytes.restype = i64
    for name in ("dlion_tuning_defaults", "dlion_get_tuning"):
        getattr(lib, name).argtypes = [ctypes.POINTER(Tuning)]
        getattr(lib, name).restype = None
    _lib = lib                      # every later call goes to the library loaded last
    return lib


def status_str(status: int) -> str:
    return load_library().dlion_status_str(status).decode()


def dlion_version() -> int:
    return load_library().dlion_version()


def words_for(d: int) -> int:
    return (int(d) + 63) // 64


def _check(status: int, what: str) -> None:
    if status != 0:
        raise DlionError(status, what)


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _on_device(t: torch.Tensor) -> bool:
    return t.is_cuda


def _rows(t: torch.Tensor, name: str):
    """``[N, d]`` tensor with unit inner stride -> (pointer, row stride in elements, N, d)."""
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError(f"{name} must be [N, d] with contiguous rows")
    if not _on_device(t):
        raise ValueError(f"{name} must be a device tensor")
    return t.data_ptr(), t.stride(0), t.shape[0], t.shape[1]


def _flat(t: torch.Tensor, name: str, dtype: torch.dtype):
    if t.dtype != dtype or t.dim() != 1 or (t.numel() > 1 and t.stride(0) != 1) or not _on_device(t):
        raise ValueError(f"{name} must be a contiguous 1-D {dtype} device tensor")
    return t.data_ptr()


def _gdtype(g: torch.Tensor) -> int:
    if g.dtype == torch.float32:
        return F32
    if g.dtype == torch.bfloat16:
        return BF16
    raise TypeError("g must be float32 or bfloat16")


def _as_u64(t: torch.Tensor, name: str):
    """packed words are 64-bit; torch carries them as int64 (same bits)."""
    if t.dtype not in (torch.int64, torch.uint64):
        raise TypeError(f"{name} must be int64/uint64 (uint64 words)")
    return t


def _packed(t: torch.Tensor, name: str, words: int, N: Optional[int] = None):
    """``[N, >= words]`` uint64 rows -> (pointer, row stride, N); the C ABI cannot see extents, so they are
    checked here: a short tensor would be a device access out of bounds."""
    pp, ps, Np, width = _rows(_as_u64(t, name), name)
    if width < words:
        raise ValueError(f"{name} rows hold {width} words, {words} are needed")
    if N is not None and Np != N:
        raise ValueError(f"{name} must have {N} rows, has {Np}")
    return pp, ps, Np


def _counts(t: torch.Tensor, name: str, need: int) -> int:
    """contiguous 1-D uint16 device tensor of at least ``need`` entries -> pointer"""
    if t.dtype not in (torch.int16, torch.uint16):
        raise TypeError(f"{name} must be int16/uint16 (uint16 counts)")
    if not _on_device(t) or t.dim() != 1 or (t.numel() > 1 and t.stride(0) != 1):
        raise ValueError(f"{name} must be a contiguous 1-D device tensor")
    if t.numel() < need:
        raise ValueError(f"{name} holds {t.numel()} entries, {need} are needed")
    return t.data_ptr()


def _workspace(t: Optional[torch.Tensor]):
    if t is None:
        return None, 0
    if not _on_device(t) or not t.is_contiguous():
        raise ValueError("workspace must be a contiguous device tensor")
    return t.data_ptr(), t.numel() * t.element_size()


def _workers(m, g):
    """``m``, ``g`` as ``[N, d]`` rows -> (m pointer, m stride, g pointer, g stride, N, d)"""
    mp, ms, N, d = _rows(m, "m")
    gp, gs, Ng, dg = _rows(g, "g")
    if m.dtype != torch.float32 or (N, d) != (Ng, dg):
        raise ValueError("m must be fp32 and m, g must agree on N and d")
    return mp, ms, gp, gs, N, d


def dlion_worker_step(m, g, packed, beta1, beta2, d=None, stream=None):
    mp, ms, gp, gs, N, dd = _workers(m, g)
    d = dd if d is None else int(d)
    if not 0 < d <= dd:
        raise ValueError(f"d = {d} is outside the rows' {dd} elements")
    pp, ps, _ = _packed(packed, "packed", words_for(d), N)
    _check(load_library().dlion_worker_step(mp, ms, gp, gs, _gdtype(g), pp, ps, d, N, beta1, beta2,
                                            _stream(stream)), "dlion_worker_step")


def dlion_aggregate(packed, d, counts, stream=None):
    pp, ps, N = _packed(packed, "packed", words_for(d))
    cp = _counts(counts, "counts", d)
    _check(load_library().dlion_aggregate(pp, ps, d, N, cp, _stream(stream)), "dlion_aggregate")


def dlion_apply(x, counts, N, mode, lr, lam, stream=None):
    xp = _flat(x, "x", torch.float32)
    cp = _counts(counts, "counts", x.numel())
    _check(load_library().dlion_apply(xp, cp, x.numel(), N, mode, lr, lam, _stream(stream)), "dlion_apply")


def dlion_aggregate_apply(x, packed, mode, lr, lam, counts=None, stream=None):
    xp = _flat(x, "x", torch.float32)
    pp, ps, N = _packed(packed, "packed", words_for(x.numel()))
    cp = _counts(counts, "counts", x.numel()) if counts is not None else None
    _check(load_library().dlion_aggregate_apply(xp, pp, ps, x.numel(), N, mode, lr, lam, cp, _stream(stream)),
           "dlion_aggregate_apply")


def _step_args(x, m, g, packed, counts):
    xp = _flat(x, "x", torch.float32)
    mp, ms, gp, gs, N, d = _workers(m, g)
    if x.numel() != d:
        raise ValueError("x, m, g must agree on d")
    pp, ps = (None, 0)
    if packed is not None:
        pp, ps, _ = _packed(packed, "packed", words_for(d), N)
    cp = _counts(counts, "counts", d) if counts is not None else None
    return xp, mp, ms, gp, gs, _gdtype(g), d, N, pp, ps, cp


def dlion_step(x, m, g, mode, beta1, beta2, lr, lam, packed=None, counts=None, stream=None):
    xp, mp, ms, gp, gs, gt, d, N, pp, ps, cp = _step_args(x, m, g, packed, counts)
    _check(load_library().dlion_step(xp, mp, ms, gp, gs, gt, d, N, mode, beta1, beta2, lr, lam,
                                     pp, ps, cp, _stream(stream)), "dlion_step")


def dlion_step_ws(x, m, g, mode, beta1, beta2, lr, lam, workspace, packed=None, counts=None, stream=None):
    """``dlion_step`` with a caller-owned scratch tensor (any dtype; its size in bytes is what counts)."""
    xp, mp, ms, gp, gs, gt, d, N, pp, ps, cp = _step_args(x, m, g, packed, counts)
    wp, wb = _workspace(workspace)
    _check(load_library().dlion_step_ws(xp, mp, ms, gp, gs, gt, d, N, mode, beta1, beta2, lr, lam,
                                        pp, ps, cp, wp, wb, _stream(stream)), "dlion_step_ws")


def dlion_step_noalloc(x, m, g, mode, beta1, beta2, lr, lam, packed=None, counts=None, stream=None):
    """``dlion_step`` whose hand-over workspace is the library's static device array: allocates nothing."""
    xp, mp, ms, gp, gs, gt, d, N, pp, ps, cp = _step_args(x, m, g, packed, counts)
    _check(load_library().dlion_step_noalloc(xp, mp, ms, gp, gs, gt, d, N, mode, beta1, beta2, lr, lam,
                                             pp, ps, cp, _stream(stream)), "dlion_step_noalloc")


def dlion_noalloc_init() -> None:
    _check(load_library().dlion_noalloc_init(), "dlion_noalloc_init")


def dlion_step_workspace_bytes(d: int, N: int) -> int:
    """Size of the workspace with which ``dlion_step_ws`` splits a step over many workers (0: none is used)."""
    return int(load_library().dlion_step_workspace_bytes(d, N))


def dlion_step_mt_workspace_bytes(total_tiles: int, N: int) -> int:
    return int(load_library().dlion_step_mt_workspace_bytes(total_tiles, N))


def dlion_get_tuning() -> Tuning:
    t = Tuning()
    load_library().dlion_get_tuning(ctypes.byref(t))
    return t


def dlion_set_tuning(t: Optional[Tuning] = None, **fields) -> None:
    """Install launch-shape overrides (``None`` and no fields: back to the defaults).  Fields given by
    name override the library's defaults, e.g. ``dlion_set_tuning(pass_workers=3, block_tiles=5)``."""
    if t is None and fields:
        t = Tuning()
        load_library().dlion_tuning_defaults(ctypes.byref(t))
    for k, v in fields.items():
        if k not in dict(Tuning._fields_):
            raise TypeError(f"dlion_tuning has no field {k}")
        setattr(t, k, int(v))
    _check(load_library().dlion_set_tuning(ctypes.byref(t) if t is not None else None), "dlion_set_tuning")


class tuned:
    """``with tuned(pass_workers=3): ...`` -- overrides for the calls inside, the previous ones after."""

    def __init__(self, **fields):
        self.fields = fields

    def __enter__(self):
        self.before = dlion_get_tuning()
        now = dlion_get_tuning()
        dlion_set_tuning(now, **self.fields)
        return self

    def __exit__(self, *exc):
        dlion_set_tuning(self.before)
        return False


class SegTable:
    """Host and device copies of a ``dlion_seg`` table for a list of tensors.

    ``xs[k]`` is the flat fp32 weight tensor ``[n_k]``; ``ms[k]`` / ``gs[k]``
    are ``[N, n_k]`` with contiguous rows.  Any of the three lists may be
    ``None`` when the calls to be made do not touch it (``numels`` then gives
    the sizes).  The object keeps the tensors alive.
    """

    def __init__(self, xs: Optional[Sequence[torch.Tensor]] = None, ms=None, gs=None,
                 numels: Optional[Sequence[int]] = None, device=None):
        lists = [l for l in (xs, ms, gs) if l is not None]
        if numels is None:
            if xs is not None:
                numels = [int(t.numel()) for t in xs]
            elif lists:
                numels = [int(t.shape[1]) for t in lists[0]]
            else:
                raise ValueError("need tensors or numels")
        self.K = len(numels)
        self.numels = list(numels)
        self.keep = (xs, ms, gs)
        self.N = None
        self.g_dtype = F32
        arr = (Seg * self.K)()
        for k in range(self.K):
            s = arr[k]
            s.numel = self.numels[k]
            if xs is not None:
                s.x = _flat(xs[k], "x", torch.float32)
                if xs[k].numel() != s.numel:
                    raise ValueError("x size mismatch")
            if ms is not None:
                s.m, s.m_stride, N, n = _rows(ms[k], "m")
                if ms[k].dtype != torch.float32 or n != s.numel:
                    raise ValueError("m must be fp32 [N, numel]")
                self.N = N if self.N is None else self.N
                if N != self.N:
                    raise ValueError("all tensors must have the same N")
            if gs is not None:
                s.g, s.g_stride, N, n = _rows(gs[k], "g")
                if n != s.numel:
                    raise ValueError("g must be [N, numel]")
                self.N = N if self.N is None else self.N
                if N != self.N:
                    raise ValueError("all tensors must have the same N")
                gd = _gdtype(gs[k])
                if k and gd != self.g_dtype:
                    raise ValueError("all gradients must share one dtype")
                self.g_dtype = gd
        tw, tt = ctypes.c_int64(0), ctypes.c_int64(0)
        _check(load_library().dlion_mt_layout(arr, self.K, ctypes.byref(tw), ctypes.byref(tt)), "dlion_mt_layout")
        self.host = arr
        self.total_words = tw.value
        self.total_tiles = tt.value
        self.word_begin = [arr[k].word_begin for k in range(self.K)]
        if device is None:
            device = lists[0][0].device if lists else torch.device("cuda", torch.cuda.current_device())
        raw = torch.frombuffer(bytearray(bytes(arr)), dtype=torch.uint8)
        self.dev = raw.to(device)

    @property
    def dev_ptr(self) -> int:
        return self.dev.data_ptr()


def _table_workers(table: SegTable, N: int) -> None:
    if table.N is not None and table.N != N:
        raise ValueError(f"the table's tensors have {table.N} worker rows, the call says N = {N}")


def dlion_worker_step_mt(table: SegTable, packed, beta1, beta2, stream=None):
    pp, ps, N = _packed(packed, "packed", table.total_words)
    _table_workers(table, N)
    _check(load_library().dlion_worker_step_mt(table.host, table.dev_ptr, table.K, table.g_dtype, pp, ps, N,
                                               beta1, beta2, _stream(stream)), "dlion_worker_step_mt")


def dlion_aggregate_mt(table: SegTable, packed, counts, stream=None):
    pp, ps, N = _packed(packed, "packed", table.total_words)
    cp = _counts(counts, "counts", 64 * table.total_words)
    _check(load_library().dlion_aggregate_mt(table.host, table.dev_ptr, table.K, pp, ps, N, cp,
                                             _stream(stream)), "dlion_aggregate_mt")


def dlion_apply_mt(table: SegTable, counts, N, mode, lr, lam, stream=None):
    cp = _counts(counts, "counts", 64 * table.total_words)
    _check(load_library().dlion_apply_mt(table.host, table.dev_ptr, table.K, cp, N, mode, lr, lam,
                                         _stream(stream)), "dlion_apply_mt")


def dlion_aggregate_apply_mt(table: SegTable, packed, mode, lr, lam, counts=None, stream=None):
    pp, ps, N = _packed(packed, "packed", table.total_words)
    cp = _counts(counts, "counts", 64 * table.total_words) if counts is not None else None
    _check(load_library().dlion_aggregate_apply_mt(table.host, table.dev_ptr, table.K, pp, ps, N, mode, lr, lam,
                                                   cp, _stream(stream)), "dlion_aggregate_apply_mt")


def dlion_step_mt(table: SegTable, N, mode, beta1, beta2, lr, lam, packed=None, counts=None, workspace=None,
                  stream=None):
    """``dlion_step_mt``; with a ``workspace`` tensor, ``dlion_step_mt_ws``."""
    _table_workers(table, N)
    pp, ps = (None, 0)
    if packed is not None:
        pp, ps, _ = _packed(packed, "packed", table.total_words, N)
    cp = _counts(counts, "counts", 64 * table.total_words) if counts is not None else None
    wp, wb = _workspace(workspace)
    _check(load_library().dlion_step_mt_ws(table.host, table.dev_ptr, table.K, table.g_dtype, N, mode, beta1, beta2,
                                           lr, lam, pp, ps, cp, wp, wb, _stream(stream)), "dlion_step_mt")


def dlion_delta_planes(N: int, mode: int) -> int:
    return load_library().dlion_delta_planes(N, mode)


def dlion_aggregate_encode(packed, d, mode, delta, stream=None):
    pp, ps, N = _packed(packed, "packed", words_for(d))
    dp, ds, _ = _packed(delta, "delta", words_for(d), dlion_delta_planes(N, mode))
    _check(load_library().dlion_aggregate_encode(pp, ps, d, N, mode, dp, ds, _stream(stream)),
           "dlion_aggregate_encode")


def dlion_apply_encoded(x, delta, N, mode, lr, lam, stream=None):
    xp = _flat(x, "x", torch.float32)
    dp, ds, _ = _packed(delta, "delta", words_for(x.numel()), dlion_delta_planes(N, mode))
    _check(load_library().dlion_apply_encoded(xp, dp, ds, x.numel(), N, mode, lr, lam, _stream(stream)),
           "dlion_apply_encoded")


def _betas(beta1, beta2, N):
    for b in (beta1, beta2):
        if b.dtype != torch.float32 or b.dim() != 1 or b.numel() != N or not _on_device(b) or \
                (N > 1 and b.stride(0) != 1):
            raise ValueError("beta1/beta2 must be contiguous float32 device tensors of N elements")
    return beta1.data_ptr(), beta2.data_ptr()


def dlion_worker_step_pw(m, g, packed, beta1, beta2, stream=None):
    mp, ms, gp, gs, N, d = _workers(m, g)
    pp, ps, _ = _packed(packed, "packed", words_for(d), N)
    b1, b2 = _betas(beta1, beta2, N)
    _check(load_library().dlion_worker_step_pw(mp, ms, gp, gs, _gdtype(g), pp, ps, d, N, b1, b2,
                                               _stream(stream)), "dlion_worker_step_pw")


def dlion_step_pw(x, m, g, mode, beta1, beta2, lr, lam, packed=None, counts=None, workspace=None, stream=None):
    """``dlion_step_pw``; with a ``workspace`` tensor, ``dlion_step_pw_ws``."""
    xp, mp, ms, gp, gs, gt, d, N, pp, ps, cp = _step_args(x, m, g, packed, counts)
    b1, b2 = _betas(beta1, beta2, N)
    if workspace is None:
        _check(load_library().dlion_step_pw(xp, mp, ms, gp, gs, gt, d, N, mode, b1, b2, lr, lam,
                                            pp, ps, cp, _stream(stream)), "dlion_step_pw")
        return
    wp, wb = _workspace(workspace)
    _check(load_library().dlion_step_pw_ws(xp, mp, ms, gp, gs, gt, d, N, mode, b1, b2, lr, lam,
                                           pp, ps, cp, wp, wb, _stream(stream)), "dlion_step_pw_ws")


def dlion_global_lion_step(x, m, g, beta1, beta2, lr, lam, sign_bits=None, stream=None):
    xp, mp, ms, gp, gs, gt, d, N, _, _, _ = _step_args(x, m, g, None, None)
    sp = None
    if sign_bits is not None:
        if _as_u64(sign_bits, "sign_bits").dim() != 1 or sign_bits.numel() < words_for(d) or \
                not _on_device(sign_bits) or (sign_bits.numel() > 1 and sign_bits.stride(0) != 1):
            raise ValueError("sign_bits must be a contiguous 1-D device tensor of at least W words")
        sp = sign_bits.data_ptr()
    _check(load_library().dlion_global_lion_step(xp, mp, ms, gp, gs, gt, d, N, beta1, beta2, lr, lam,
                                                 sp, _stream(stream)), "dlion_global_lion_step")


def dlion_membench(src, dst, rows=1, write=True, loads_in_flight=16, waves_per_cu=0, stream=None):
    """Memory-rate probe: ``src`` is ``[rows, n]`` (contiguous rows, any row stride), ``dst`` ``[n]`` of the
    same dtype; bytes per row must be a multiple of 1024.  Returns (bytes read, bytes written)."""
    if src.dim() == 1:
        src = src.unsqueeze(0)
    sp, ss, R, n = _rows(src, "src")
    if R != rows or dst.dim() != 1 or dst.numel() != n or dst.dtype != src.dtype or not _on_device(dst) or \
            (n > 1 and dst.stride(0) != 1):
        raise ValueError("src must be [rows, n] and dst [n] of the same dtype, on the device")
    e = src.element_size()
    _check(load_library().dlion_membench(sp, ss * e, rows, dst.data_ptr(), n * e, 1 if write else 0, loads_in_flight, waves_per_cu,
                                         _stream(stream)), "dlion_membench")
    return rows * n * e, (n * e if write else 0)
