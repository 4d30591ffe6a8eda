"""Thin ctypes binding of libqg.so (declared in include/qg.h).

Argument marshalling only: every step of the path runs in the HIP kernels of the library.
PyTorch supplies device memory and the current stream, nothing else.  There is no fallback:
if the library cannot be loaded or a call returns an error, a RuntimeError is raised.
"""
import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import torch

from . import build as _build

QG_LAYOUT_CANONICAL = 0
QG_LAYOUT_DEVICE = 1
QG_LAYOUT_DEVICE_NARROW = 2
QG_MAX_GROUPED = 16

_LIB = None


class _Desc(ctypes.Structure):
    _fields_ = [("packed", ctypes.c_void_p), ("N", ctypes.c_int64), ("K", ctypes.c_int64),
                ("bits", ctypes.c_int), ("group", ctypes.c_int),
                ("x", ctypes.c_void_p), ("y", ctypes.c_void_p)]


def lib():
    """Load libqg.so, building it first only if no built library is present; a library that
    was built from other sources than the ones in csrc/ is refused (RuntimeError)."""
    global _LIB
    if _LIB is None:
        override = os.environ.get("QG_LIBRARY")             # a library built elsewhere: used as it is
        path = override or _build.OUT
        if not os.path.exists(path):
            path = _build.build(force=True)
        L = ctypes.CDLL(path)
        if not override:
            # a library built from other sources than the ones beside it is not used silently
            L.qg_build_id.restype = ctypes.c_char_p
            built_from = L.qg_build_id().decode() if hasattr(L, "qg_build_id") else "none"
            if built_from != _build.source_id():
                raise RuntimeError(f"{path} is stale (built from {built_from}, sources are "
                                   f"{_build.source_id()}): run `python -m paper_2307_03738_amd.build`")
        i64, i32, vp, sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
        L.qg_cell.restype = i32
        L.qg_cell.argtypes = [i32]
        L.qg_build_id.restype = ctypes.c_char_p
        L.qg_build_id.argtypes = []
        L.qg_status_string.restype = ctypes.c_char_p
        L.qg_status_string.argtypes = [i32]
        L.qg_packed_bytes.restype = sz
        L.qg_packed_bytes.argtypes = [i64, i64, i32, i32, i32]
        L.qg_workspace_bytes.restype = sz
        L.qg_workspace_bytes.argtypes = [i64, i64, i32, i32, i32]
        L.qg_workspace_init.restype = i32
        L.qg_workspace_init.argtypes = [vp, sz, vp]
        L.qg_quantize.restype = i32
        L.qg_quantize.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, vp]
        L.qg_pack.restype = i32
        L.qg_pack.argtypes = [vp, vp, vp, i64, i64, i32, i32, i32, vp, vp]
        L.qg_unpack.restype = i32
        L.qg_unpack.argtypes = [vp, i64, i64, i32, i32, i32, vp, vp, vp, vp]
        L.qg_gemv.restype = i32
        L.qg_gemv.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, sz, vp]
        L.qg_gemv_noalloc.restype = i32
        L.qg_gemv_noalloc.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp]
        L.qg_last_gemv_kernel.restype = ctypes.c_char_p
        L.qg_last_gemv_kernel.argtypes = []
        L.qg_gemv_grouped.restype = i32
        L.qg_gemv_grouped.argtypes = [ctypes.POINTER(_Desc), i32, vp, sz, vp]
        L.qg_gemv_swiglu.restype = i32
        L.qg_gemv_swiglu.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, sz, vp]
        L.qg_gemm_small.restype = i32
        L.qg_gemm_small.argtypes = [vp, i64, i64, i32, i32, vp, i32, vp, vp, sz, vp]
        L.qg_set_gemv_tuning.restype = i32
        L.qg_set_gemv_tuning.argtypes = [i32, i32, i32]
        L.qg_gemv_autotune.restype = i32
        L.qg_gemv_autotune.argtypes = [ctypes.POINTER(_Desc), i32, i32, vp, sz, vp, i32,
                                       ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(i32),
                                       ctypes.POINTER(ctypes.c_float)]
        L.qg_gemv_autotune_report.restype = i32
        L.qg_gemv_autotune_report.argtypes = [ctypes.POINTER(ctypes.c_float), i32, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.qg_set_gemm_tuning.restype = i32
        L.qg_set_gemm_tuning.argtypes = [i32, i32]
        L.qg_to_narrow.restype = i32
        L.qg_to_narrow.argtypes = [vp, i64, i64, i32, i32, vp, vp]
        L.qg_from_narrow.restype = i32
        L.qg_from_narrow.argtypes = [vp, i64, i64, i32, i32, vp, vp]
        L.qg_gemv_narrow.restype = i32
        L.qg_gemv_narrow.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp]
        L.qg_gemv_grouped_narrow.restype = i32
        L.qg_gemv_grouped_narrow.argtypes = [ctypes.POINTER(_Desc), i32, vp]
        L.qg_set_narrow_tuning.restype = i32
        L.qg_set_narrow_tuning.argtypes = [i32]
        L.qg_last_narrow_kernel.restype = ctypes.c_char_p
        L.qg_last_narrow_kernel.argtypes = []
        L.qg_gemv_record_tuning.restype = i32
        L.qg_gemv_record_tuning.argtypes = [ctypes.POINTER(_Desc), i32, i32, i32, i32]
        L.qg_clear_tuning.restype = None
        L.qg_clear_tuning.argtypes = []
        L.qg_gemm_autotune.restype = i32
        L.qg_gemm_autotune.argtypes = [ctypes.POINTER(vp), i32, i64, i64, i32, i32, vp, i32, vp, vp, sz, vp, i32,
                                       ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_float)]
        L.qg_gemm_autotune_report.restype = i32
        L.qg_gemm_autotune_report.argtypes = [ctypes.POINTER(ctypes.c_float), i32, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        _LIB = L
    return _LIB


def _check(rc: int, what: str):
    if rc != 0:
        raise RuntimeError(f"{what}: {lib().qg_status_string(rc).decode()} (status {rc})")


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{name}: expected a contiguous {dtype} tensor on the GPU")
    return t


def qg_cell(bits: int) -> int:
    return int(lib().qg_cell(bits))


def qg_packed_bytes(N: int, K: int, bits: int, group: int, layout: int = QG_LAYOUT_DEVICE) -> int:
    return int(lib().qg_packed_bytes(N, K, bits, group, layout))


def qg_workspace_bytes(N: int, K: int, bits: int, group: int, M: int = 1) -> int:
    return int(lib().qg_workspace_bytes(N, K, bits, group, M))


def qg_workspace_init(workspace: torch.Tensor):
    _check(lib().qg_workspace_init(workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                   _stream()), "qg_workspace_init")


def new_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    """Allocate a workspace of at least nbytes and zero it with the library's own fill."""
    ws = torch.empty(max(256, (nbytes + 255) // 256 * 256), dtype=torch.uint8, device=device)
    qg_workspace_init(ws)
    return ws


def qg_quantize(W: torch.Tensor, bits: int, group: int) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    _dev(W, torch.float32, "W")
    N, K = W.shape
    if group <= 0 or K % group:
        _check(2, "qg_quantize")
    q = torch.empty((N, K), dtype=torch.uint8, device=W.device)
    s = torch.empty((N, K // group), dtype=torch.float32, device=W.device)
    z = torch.empty((N, K // group), dtype=torch.uint8, device=W.device)
    _check(lib().qg_quantize(W.data_ptr(), N, K, bits, group, q.data_ptr(), s.data_ptr(), z.data_ptr(),
                             _stream()), "qg_quantize")
    return q, s, z


def qg_pack(q: torch.Tensor, s: torch.Tensor, z: torch.Tensor, bits: int, group: int,
            layout: int = QG_LAYOUT_DEVICE) -> torch.Tensor:
    _dev(q, torch.uint8, "q"); _dev(s, torch.float32, "s"); _dev(z, torch.uint8, "z")
    N, K = q.shape
    nbytes = qg_packed_bytes(N, K, bits, group, layout)
    if nbytes == 0:
        _check(2, "qg_pack")
    packed = torch.empty(nbytes, dtype=torch.uint8, device=q.device)
    _check(lib().qg_pack(q.data_ptr(), s.data_ptr(), z.data_ptr(), N, K, bits, group, layout,
                         packed.data_ptr(), _stream()), "qg_pack")
    return packed


def qg_unpack(packed: torch.Tensor, N: int, K: int, bits: int, group: int,
              layout: int = QG_LAYOUT_DEVICE) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    _dev(packed, torch.uint8, "packed")
    if packed.numel() < qg_packed_bytes(N, K, bits, group, layout) or group <= 0 or K % group:
        _check(2, "qg_unpack")
    q = torch.empty((N, K), dtype=torch.uint8, device=packed.device)
    s = torch.empty((N, K // group), dtype=torch.float32, device=packed.device)
    z = torch.empty((N, K // group), dtype=torch.uint8, device=packed.device)
    _check(lib().qg_unpack(packed.data_ptr(), N, K, bits, group, layout, q.data_ptr(), s.data_ptr(),
                           z.data_ptr(), _stream()), "qg_unpack")
    return q, s, z


def qg_gemv(packed: torch.Tensor, N: int, K: int, bits: int, group: int, x: torch.Tensor,
            y: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev(packed, torch.uint8, "packed"); _dev(x, torch.float32, "x")
    if x.numel() != K or packed.numel() < qg_packed_bytes(N, K, bits, group, QG_LAYOUT_DEVICE):
        _check(2, "qg_gemv")
    if y is None:
        y = torch.empty(N, dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = new_workspace(qg_workspace_bytes(N, K, bits, group, 1), x.device)
    _check(lib().qg_gemv(packed.data_ptr(), N, K, bits, group, x.data_ptr(), y.data_ptr(),
                         workspace.data_ptr(), workspace.numel(), _stream()), "qg_gemv")
    return y


def qg_gemv_noalloc(packed: torch.Tensor, N: int, K: int, bits: int, group: int, x: torch.Tensor,
                    y: torch.Tensor) -> torch.Tensor:
    """qg_gemv with the library's own scratch array: no workspace argument, nothing allocated
    by the call (y is the caller's)."""
    _dev(packed, torch.uint8, "packed"); _dev(x, torch.float32, "x"); _dev(y, torch.float32, "y")
    if x.numel() != K or y.numel() != N or packed.numel() < qg_packed_bytes(N, K, bits, group, QG_LAYOUT_DEVICE):
        _check(2, "qg_gemv_noalloc")
    _check(lib().qg_gemv_noalloc(packed.data_ptr(), N, K, bits, group, x.data_ptr(), y.data_ptr(), _stream()),
           "qg_gemv_noalloc")
    return y


def qg_to_narrow(packed: torch.Tensor, N: int, K: int, bits: int, group: int) -> torch.Tensor:
    """The narrow-layout copy of a QG_LAYOUT_DEVICE blob."""
    _dev(packed, torch.uint8, "packed")
    nbytes = qg_packed_bytes(N, K, bits, group, QG_LAYOUT_DEVICE_NARROW)
    if nbytes == 0:
        _check(3, "qg_to_narrow")
    if packed.numel() < qg_packed_bytes(N, K, bits, group, QG_LAYOUT_DEVICE):
        _check(2, "qg_to_narrow")
    out = torch.empty(nbytes, dtype=torch.uint8, device=packed.device)
    _check(lib().qg_to_narrow(packed.data_ptr(), N, K, bits, group, out.data_ptr(), _stream()), "qg_to_narrow")
    return out


def qg_from_narrow(narrow: torch.Tensor, N: int, K: int, bits: int, group: int) -> torch.Tensor:
    _dev(narrow, torch.uint8, "narrow")
    if narrow.numel() < qg_packed_bytes(N, K, bits, group, QG_LAYOUT_DEVICE_NARROW) or \
            qg_packed_bytes(N, K, bits, group, QG_LAYOUT_DEVICE_NARROW) == 0:
        _check(2, "qg_from_narrow")
    out = torch.empty(qg_packed_bytes(N, K, bits, group, QG_LAYOUT_DEVICE), dtype=torch.uint8, device=narrow.device)
    _check(lib().qg_from_narrow(narrow.data_ptr(), N, K, bits, group, out.data_ptr(), _stream()), "qg_from_narrow")
    return out


def qg_gemv_narrow(narrow: torch.Tensor, N: int, K: int, bits: int, group: int, x: torch.Tensor,
                   y: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev(narrow, torch.uint8, "narrow"); _dev(x, torch.float32, "x")
    nbytes = qg_packed_bytes(N, K, bits, group, QG_LAYOUT_DEVICE_NARROW)
    if nbytes == 0:
        _check(3, "qg_gemv_narrow")
    if x.numel() != K or narrow.numel() < nbytes:
        _check(2, "qg_gemv_narrow")
    if y is None:
        y = torch.empty(N, dtype=torch.float32, device=x.device)
    _dev(y, torch.float32, "y")
    if y.numel() != N:
        _check(2, "qg_gemv_narrow")
    _check(lib().qg_gemv_narrow(narrow.data_ptr(), N, K, bits, group, x.data_ptr(), y.data_ptr(), _stream()),
           "qg_gemv_narrow")
    return y


class GroupedGemvNarrow:
    """A prepared grouped launch on narrow-layout blobs (dicts with packed, N, K, bits, group, x, y)."""

    def __init__(self, problems: Sequence[dict]):
        self.count = len(problems)
        self.descs = (_Desc * self.count)()
        self._keep = list(problems)
        for i, p in enumerate(problems):
            _dev(p["packed"], torch.uint8, "packed"); _dev(p["x"], torch.float32, "x"); _dev(p["y"], torch.float32, "y")
            nbytes = qg_packed_bytes(p["N"], p["K"], p["bits"], p["group"], QG_LAYOUT_DEVICE_NARROW)
            if nbytes == 0:
                _check(3, "qg_gemv_grouped_narrow")
            if p["x"].numel() != p["K"] or p["y"].numel() != p["N"] or p["packed"].numel() < nbytes:
                _check(2, "qg_gemv_grouped_narrow")
            self.descs[i] = _Desc(p["packed"].data_ptr(), p["N"], p["K"], p["bits"], p["group"],
                                  p["x"].data_ptr(), p["y"].data_ptr())
        self._fn = lib().qg_gemv_grouped_narrow

    def launch(self, stream: Optional[int] = None):
        rc = self._fn(self.descs, self.count, _stream() if stream is None else stream)
        if rc != 0:
            _check(rc, "qg_gemv_grouped_narrow")


def qg_set_narrow_tuning(tiles_per_wave: int = 0):
    _check(lib().qg_set_narrow_tuning(tiles_per_wave), "qg_set_narrow_tuning")


def qg_last_narrow_kernel() -> str:
    return lib().qg_last_narrow_kernel().decode()


def qg_last_gemv_kernel() -> str:
    return lib().qg_last_gemv_kernel().decode()


class GroupedGemv:
    """A prepared grouped launch: the descriptor array is built once, launch() enqueues it."""

    def __init__(self, problems: Sequence[dict], workspace: Optional[torch.Tensor] = None):
        # problems: dicts with packed, N, K, bits, group, x, y
        self.count = len(problems)
        self.descs = (_Desc * self.count)()
        self._keep = list(problems)
        need = 0
        for i, p in enumerate(problems):
            _dev(p["packed"], torch.uint8, "packed"); _dev(p["x"], torch.float32, "x"); _dev(p["y"], torch.float32, "y")
            if p["x"].numel() != p["K"] or p["y"].numel() != p["N"] or \
                    p["packed"].numel() < qg_packed_bytes(p["N"], p["K"], p["bits"], p["group"]):
                _check(2, "qg_gemv_grouped")
            self.descs[i] = _Desc(p["packed"].data_ptr(), p["N"], p["K"], p["bits"], p["group"],
                                  p["x"].data_ptr(), p["y"].data_ptr())
            need += qg_workspace_bytes(p["N"], p["K"], p["bits"], p["group"], 1)
        self.workspace = workspace if workspace is not None else new_workspace(need, problems[0]["x"].device)
        self._fn = lib().qg_gemv_grouped

    def launch(self, stream: Optional[int] = None):
        rc = self._fn(self.descs, self.count, self.workspace.data_ptr(), self.workspace.numel(),
                      _stream() if stream is None else stream)
        if rc != 0:
            _check(rc, "qg_gemv_grouped")


def qg_gemv_grouped(problems: Sequence[dict], workspace: Optional[torch.Tensor] = None):
    GroupedGemv(problems, workspace).launch()
    return [p["y"] for p in problems]


def qg_gemv_swiglu(packed: torch.Tensor, I: int, K: int, bits: int, group: int, x: torch.Tensor,
                   h: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev(packed, torch.uint8, "packed"); _dev(x, torch.float32, "x")
    if x.numel() != K or packed.numel() < qg_packed_bytes(2 * I, K, bits, group, QG_LAYOUT_DEVICE):
        _check(2, "qg_gemv_swiglu")
    if h is None:
        h = torch.empty(I, dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = new_workspace(qg_workspace_bytes(2 * I, K, bits, group, 1), x.device)
    _check(lib().qg_gemv_swiglu(packed.data_ptr(), I, K, bits, group, x.data_ptr(), h.data_ptr(),
                                workspace.data_ptr(), workspace.numel(), _stream()), "qg_gemv_swiglu")
    return h


def qg_gemm_small(packed: torch.Tensor, N: int, K: int, bits: int, group: int, X: torch.Tensor,
                  Y: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev(packed, torch.uint8, "packed"); _dev(X, torch.float32, "X")
    M = X.shape[0]
    if X.dim() != 2 or X.shape[1] != K or packed.numel() < qg_packed_bytes(N, K, bits, group, QG_LAYOUT_DEVICE):
        _check(2, "qg_gemm_small")
    if Y is None:
        Y = torch.empty((M, N), dtype=torch.float32, device=X.device)
    if workspace is None:
        workspace = new_workspace(qg_workspace_bytes(N, K, bits, group, M), X.device)
    _check(lib().qg_gemm_small(packed.data_ptr(), N, K, bits, group, X.data_ptr(), M, Y.data_ptr(),
                               workspace.data_ptr(), workspace.numel(), _stream()), "qg_gemm_small")
    return Y


def qg_set_gemv_tuning(waves_per_block: int = 0, bytes_per_wave: int = 0, kernel: int = 0):
    _check(lib().qg_set_gemv_tuning(waves_per_block, bytes_per_wave, kernel), "qg_set_gemv_tuning")


def qg_gemv_autotune(launches, repeats: int = 20):
    """Times the candidates on the prepared launch(es) -- a GroupedGemv or a list of them with the
    same shapes, rotated -- and leaves the fastest installed; returns (waves_per_block,
    bytes_per_wave, kernel, microseconds per launch)."""
    if isinstance(launches, GroupedGemv):
        launches = [launches]
    count = launches[0].count
    if any(l.count != count for l in launches):
        _check(2, "qg_gemv_autotune")
    descs = (_Desc * (count * len(launches)))()
    for s, l in enumerate(launches):
        for i in range(count):
            descs[s * count + i] = l.descs[i]
    ws = launches[0].workspace
    w, b, k = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    us = ctypes.c_float()
    _check(lib().qg_gemv_autotune(descs, count, len(launches), ws.data_ptr(), ws.numel(), _stream(), repeats,
                                  ctypes.byref(w), ctypes.byref(b), ctypes.byref(k), ctypes.byref(us)),
           "qg_gemv_autotune")
    return w.value, b.value, k.value, us.value


AUTOTUNE_TEAMS = (0, 2, 4, 8, 12, 16)
AUTOTUNE_SIZES = (0, 4096, 8192, 16384, 32768, 49152, 65536)


def qg_gemv_autotune_report():
    """(microseconds per candidate, -1 where the budget dropped it; number timed; number dropped)
    of the last qg_gemv_autotune.  Candidate ((kernel - 1) * 6 + team index) * 7 + size index."""
    us = (ctypes.c_float * 168)()
    timed, dropped = ctypes.c_int(), ctypes.c_int()
    _check(lib().qg_gemv_autotune_report(us, 168, ctypes.byref(timed), ctypes.byref(dropped)), "qg_gemv_autotune_report")
    return list(us), timed.value, dropped.value


def qg_gemv_record_tuning(problems: Sequence[dict], waves_per_block: int, bytes_per_wave: int, kernel: int):
    """Records a launch shape for every later launch whose list of (N, K, bits, group) equals that of
    `problems` (dicts with N, K, bits, group)."""
    descs = (_Desc * len(problems))()
    for i, p in enumerate(problems):
        descs[i] = _Desc(0, p["N"], p["K"], p["bits"], p["group"], 0, 0)
    _check(lib().qg_gemv_record_tuning(descs, len(problems), waves_per_block, bytes_per_wave, kernel),
           "qg_gemv_record_tuning")


def qg_clear_tuning():
    lib().qg_clear_tuning()


def qg_gemm_autotune(packed_sets: Sequence[torch.Tensor], N: int, K: int, bits: int, group: int, X: torch.Tensor,
                     Y: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, repeats: int = 20):
    """Searches the launch shape of qg_gemm_small for this problem, records the fastest and returns
    (K ranges, shape, microseconds per call)."""
    _dev(X, torch.float32, "X")
    M = X.shape[0]
    for b in packed_sets:
        _dev(b, torch.uint8, "packed")
        if b.numel() < qg_packed_bytes(N, K, bits, group, QG_LAYOUT_DEVICE):
            _check(2, "qg_gemm_autotune")
    if X.dim() != 2 or X.shape[1] != K:
        _check(2, "qg_gemm_autotune")
    if Y is None:
        Y = torch.empty((M, N), dtype=torch.float32, device=X.device)
    if workspace is None:
        workspace = new_workspace(qg_workspace_bytes(N, K, bits, group, M), X.device)
    ptrs = (ctypes.c_void_p * len(packed_sets))(*[b.data_ptr() for b in packed_sets])
    sp, sh, us = ctypes.c_int(), ctypes.c_int(), ctypes.c_float()
    _check(lib().qg_gemm_autotune(ptrs, len(packed_sets), N, K, bits, group, X.data_ptr(), M, Y.data_ptr(),
                                  workspace.data_ptr(), workspace.numel(), _stream(), repeats,
                                  ctypes.byref(sp), ctypes.byref(sh), ctypes.byref(us)), "qg_gemm_autotune")
    return sp.value, sh.value, us.value


GEMM_AUTOTUNE_SHAPES = (0, -1) + tuple(range(1, 14))


def qg_gemm_autotune_report():
    """(microseconds per candidate: -1 dropped by the price, -2 not a plan of its own; number timed;
    number dropped) of the last qg_gemm_autotune.  Candidate = GEMM_AUTOTUNE_SHAPES.index(shape) * 8 +
    K ranges - 1."""
    us = (ctypes.c_float * 120)()
    timed, dropped = ctypes.c_int(), ctypes.c_int()
    _check(lib().qg_gemm_autotune_report(us, 120, ctypes.byref(timed), ctypes.byref(dropped)), "qg_gemm_autotune_report")
    return list(us), timed.value, dropped.value


def qg_set_gemm_tuning(splits: int = 0, shape: int = 0):
    _check(lib().qg_set_gemm_tuning(splits, shape), "qg_set_gemm_tuning")
