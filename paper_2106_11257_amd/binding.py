"""ctypes binding of the C ABI in ``include/btard.h``.

Argument marshalling only: every step of the computation runs in the HIP
library.  Device buffers are torch tensors (``data_ptr()``), the stream is
torch's current stream.  There is no CPU fallback: if ``libbtard.so`` is not
built the import of the library fails with an error.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libbtard.so")
_lib = None

BTARD_OK = 0
BTARD_FLAG_NONE = 0
BTARD_FLAG_GRAM = 1
BTARD_FLAG_HOST_SYNC = 2
BTARD_FLAG_GEOMETRIC_MEDIAN = 4
BTARD_FLAG_GRAM_BEGINS = 8


class BtardError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        name = load_library().btard_status_string(status).decode()
        super().__init__(f"{where}: {name} ({status})")


class _Problem(ctypes.Structure):
    _fields_ = [
        ("g", ctypes.c_void_p), ("ldg", ctypes.c_int64), ("n", ctypes.c_int32),
        ("d", ctypes.c_int64), ("offsets_host", ctypes.POINTER(ctypes.c_int64)),
        ("parts", ctypes.c_int32), ("tau", ctypes.c_float), ("eps", ctypes.c_float),
        ("max_iters", ctypes.c_int32), ("v0", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("stream", ctypes.c_void_p), ("flags", ctypes.c_uint32), ("preclip", ctypes.c_float),
        ("tau_schedule", ctypes.POINTER(ctypes.c_float)),
    ]


def status_string(status: int) -> str:
    return load_library().btard_status_string(int(status)).decode()


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """dlopen libbtard.so (built beforehand by ``build.py``); build it if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _build
        _build.build(force=True)
    lib = ctypes.CDLL(_LIB_PATH)
    c = ctypes
    lib.btard_status_string.argtypes = [c.c_int]
    lib.btard_status_string.restype = c.c_char_p
    lib.btard_split_offsets.argtypes = [c.c_int64, c.c_int32, c.POINTER(c.c_int64)]
    lib.btard_split_offsets.restype = c.c_int
    lib.btard_workspace_bytes.argtypes = [c.c_int32, c.c_int32]
    lib.btard_workspace_bytes.restype = c.c_size_t
    lib.btard_centered_clip.argtypes = [
        c.c_void_p, c.c_int64, c.c_int32, c.c_int64, c.POINTER(c.c_int64), c.c_int32,
        c.c_float, c.c_float, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_void_p, c.c_size_t, c.c_void_p, c.c_uint32]
    lib.btard_centered_clip.restype = c.c_int
    lib.btard_cc_begin.argtypes = [c.POINTER(_Problem)]
    lib.btard_cc_begin.restype = c.c_int
    lib.btard_cc_gram.argtypes = [c.POINTER(_Problem)]
    lib.btard_cc_gram.restype = c.c_int
    for name in ("btard_cc_gram_matrix", "btard_cc_gram_iterate"):
        getattr(lib, name).argtypes = [c.POINTER(_Problem)]
        getattr(lib, name).restype = c.c_int
    lib.btard_cc_remaining.argtypes = [c.POINTER(_Problem), c.POINTER(c.c_int32)]
    lib.btard_cc_remaining.restype = c.c_int
    lib.btard_debug_gram.argtypes = [c.POINTER(_Problem), c.c_void_p]
    lib.btard_debug_gram.restype = c.c_int
    lib.btard_debug_last_pass.argtypes = [c.POINTER(_Problem), c.c_int32, c.c_void_p, c.c_uint64]
    lib.btard_debug_last_pass.restype = c.c_int
    lib.btard_debug_plain_stream.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_int64, c.c_void_p,
                                             c.c_int32, c.c_void_p]
    lib.btard_debug_plain_stream.restype = c.c_int
    lib.btard_cc_iterate.argtypes = [c.POINTER(_Problem), c.c_int32, c.c_int32]
    lib.btard_cc_iterate.restype = c.c_int
    lib.btard_cc_finish.argtypes = [c.POINTER(_Problem), c.c_int32, c.c_void_p, c.c_void_p,
                                    c.c_void_p]
    lib.btard_cc_finish.restype = c.c_int
    lib.btard_cc_finish_verify.argtypes = [
        c.POINTER(_Problem), c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_uint64,
        c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p]
    lib.btard_cc_finish_verify.restype = c.c_int
    lib.btard_centered_clip_verify.argtypes = [
        c.c_void_p, c.c_int64, c.c_int32, c.c_int64, c.POINTER(c.c_int64), c.c_int32,
        c.c_float, c.c_float, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_uint64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_size_t,
        c.c_void_p, c.c_uint32]
    lib.btard_centered_clip_verify.restype = c.c_int
    lib.btard_centered_clip_verify_noalloc.argtypes = [
        c.c_void_p, c.c_int64, c.c_int32, c.c_int64, c.POINTER(c.c_int64), c.c_int32,
        c.c_float, c.c_float, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_uint64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_uint32]
    lib.btard_centered_clip_verify_noalloc.restype = c.c_int
    lib.btard_geometric_median.argtypes = [
        c.c_void_p, c.c_int64, c.c_int32, c.c_int64, c.POINTER(c.c_int64), c.c_int32,
        c.c_float, c.c_float, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_void_p, c.c_size_t, c.c_void_p]
    lib.btard_geometric_median.restype = c.c_int
    lib.btard_coordinate_median.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_int64,
                                            c.c_void_p, c.c_void_p]
    lib.btard_coordinate_median.restype = c.c_int
    lib.btard_hash_workspace_bytes.argtypes = [c.c_int32, c.POINTER(c.c_int64), c.c_int32]
    lib.btard_hash_workspace_bytes.restype = c.c_size_t
    lib.btard_partition_hashes.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_int64,
                                           c.POINTER(c.c_int64), c.c_int32, c.c_void_p,
                                           c.c_void_p, c.c_size_t, c.c_void_p]
    lib.btard_partition_hashes.restype = c.c_int
    lib.btard_tau_schedule.argtypes = [c.c_double, c.c_double, c.c_double, c.c_int32,
                                       c.POINTER(c.c_float)]
    lib.btard_tau_schedule.restype = c.c_int
    lib.btard_verification3.argtypes = [c.c_void_p, c.c_int32, c.c_int32, c.c_double, c.c_void_p,
                                        c.c_void_p, c.c_void_p, c.c_void_p]
    lib.btard_verification3.restype = c.c_int
    lib.btard_verification12.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32,
                                         c.c_int32, c.c_double, c.c_double, c.c_void_p,
                                         c.c_void_p, c.c_void_p, c.c_void_p]
    lib.btard_verification12.restype = c.c_int
    lib.btard_cc_preclip_factors.argtypes = [c.POINTER(_Problem), c.c_void_p]
    lib.btard_cc_preclip_factors.restype = c.c_int
    lib.btard_centered_clip_verify_preclipped.argtypes = [
        c.c_void_p, c.c_int64, c.c_int32, c.c_int64, c.POINTER(c.c_int64), c.c_int32,
        c.c_float, c.c_float, c.c_float, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_uint64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_size_t, c.c_void_p, c.c_uint32]
    lib.btard_centered_clip_verify_preclipped.restype = c.c_int
    lib.btard_verify_projections.argtypes = [
        c.c_void_p, c.c_int64, c.c_int32, c.c_int64, c.POINTER(c.c_int64), c.c_int32,
        c.c_void_p, c.c_float, c.c_uint64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_void_p, c.c_int64, c.c_void_p, c.c_size_t, c.c_void_p, c.c_uint32]
    lib.btard_verify_projections.restype = c.c_int
    lib.btard_verify_projections_preclipped.argtypes = [
        c.c_void_p, c.c_int64, c.c_int32, c.c_int64, c.POINTER(c.c_int64), c.c_int32,
        c.c_void_p, c.c_float, c.c_void_p, c.c_float, c.c_uint64, c.c_void_p, c.c_void_p,
        c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_void_p, c.c_void_p, c.c_size_t,
        c.c_void_p, c.c_uint32]
    lib.btard_verify_projections_preclipped.restype = c.c_int
    lib.btard_debug_zhat.argtypes = [c.c_uint64, c.c_int64, c.c_int64, c.c_void_p, c.c_void_p]
    lib.btard_debug_zhat.restype = c.c_int
    _lib = lib
    return lib


def _check(rc: int, where: str) -> None:
    if rc != BTARD_OK:
        raise BtardError(rc, where)


def _stream_ptr(device) -> int:
    return int(torch.cuda.current_stream(device).cuda_stream)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _off_array(offsets: Sequence[int]):
    return (ctypes.c_int64 * len(offsets))(*[int(o) for o in offsets])


def _row_stride(g: torch.Tensor) -> int:
    assert g.dim() == 2 and g.dtype == torch.float32
    assert g.shape[1] == 0 or g.stride(1) == 1, "rows of g must be contiguous"
    return int(g.stride(0)) if g.shape[0] > 1 else int(max(g.shape[1], g.stride(0)))


def split_offsets(d: int, parts: int) -> list:
    """Split(v, parts) of App. D.1 -> parts + 1 offsets."""
    out = (ctypes.c_int64 * (parts + 1))()
    _check(load_library().btard_split_offsets(int(d), int(parts), out), "btard_split_offsets")
    return list(out)


def workspace_bytes(n: int, parts: int) -> int:
    return int(load_library().btard_workspace_bytes(int(n), int(parts)))


def alloc_workspace(n: int, parts: int, device) -> torch.Tensor:
    nbytes = workspace_bytes(n, parts)
    if nbytes == 0:
        raise BtardError(-1, "btard_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def centered_clip(g: torch.Tensor, offsets: Sequence[int], tau: float, eps: float,
                  max_iters: int, v0: Optional[torch.Tensor] = None,
                  v: Optional[torch.Tensor] = None, iters: Optional[torch.Tensor] = None,
                  last_step_norm: Optional[torch.Tensor] = None,
                  workspace: Optional[torch.Tensor] = None, flags: int = BTARD_FLAG_NONE):
    """btard_centered_clip.  Returns (v fp32 [d], iters int32 [P], last_step_norm fp64 [P]).

    Work is enqueued on torch's current stream; the outputs are valid after it
    is synchronised.
    """
    n, d = int(g.shape[0]), int(g.shape[1])
    P = len(offsets) - 1
    dev = g.device
    if v is None:
        v = torch.empty(d, dtype=torch.float32, device=dev)
    if iters is None:
        iters = torch.empty(P, dtype=torch.int32, device=dev)
    if last_step_norm is None:
        last_step_norm = torch.empty(P, dtype=torch.float64, device=dev)
    if workspace is None:
        workspace = alloc_workspace(n, P, dev)
    rc = load_library().btard_centered_clip(
        _ptr(g), _row_stride(g), n, d, _off_array(offsets), P, float(tau), float(eps),
        int(max_iters), _ptr(v0), _ptr(v), _ptr(iters), _ptr(last_step_norm),
        _ptr(workspace), workspace.numel(), _stream_ptr(dev), int(flags))
    _check(rc, "btard_centered_clip")
    return v, iters, last_step_norm


class Problem:
    """Keeps the ctypes problem description (and what it points to) alive."""

    def __init__(self, g, offsets, tau, eps, max_iters, v0, workspace, flags=BTARD_FLAG_NONE,
                 preclip=0.0, tau_schedule=None):
        self.g, self.v0, self.workspace = g, v0, workspace
        self.offsets = _off_array(offsets)
        self.parts = len(offsets) - 1
        self.c = _Problem(
            _ptr(g), _row_stride(g), int(g.shape[0]), int(g.shape[1]), self.offsets,
            self.parts, float(tau), float(eps), int(max_iters), _ptr(v0), _ptr(workspace),
            workspace.numel(), _stream_ptr(g.device), int(flags), float(preclip), None)
        if tau_schedule is not None:
            vals = [float(x) for x in tau_schedule]
            if len(vals) != int(max_iters):
                raise ValueError("tau_schedule needs max_iters entries")
            self.schedule = (ctypes.c_float * max(len(vals), 1))(*vals)
            self.c.tau_schedule = ctypes.cast(self.schedule, ctypes.POINTER(ctypes.c_float))


def make_problem(g: torch.Tensor, offsets: Sequence[int], tau: float, eps: float,
                 max_iters: int, v0: Optional[torch.Tensor] = None,
                 workspace: Optional[torch.Tensor] = None, flags: int = BTARD_FLAG_NONE,
                 preclip: float = 0.0, tau_schedule: Optional[Sequence[float]] = None) -> Problem:
    """preclip: pre-clipping radius lambda of BTARD-Clipped-SGD (0 or inf: none);
    tau_schedule: max_iters clipping radii tau_l (eq. (5)), None: constant tau."""
    if workspace is None:
        workspace = alloc_workspace(int(g.shape[0]), len(offsets) - 1, g.device)
    return Problem(g, offsets, tau, eps, max_iters, v0, workspace, flags, preclip, tau_schedule)


def cc_begin(p: Problem) -> None:
    _check(load_library().btard_cc_begin(ctypes.byref(p.c)), "btard_cc_begin")


def cc_gram(p: Problem) -> None:
    _check(load_library().btard_cc_gram(ctypes.byref(p.c)), "btard_cc_gram")


def cc_gram_matrix(p: Problem) -> None:
    _check(load_library().btard_cc_gram_matrix(ctypes.byref(p.c)), "btard_cc_gram_matrix")


def cc_gram_iterate(p: Problem) -> None:
    _check(load_library().btard_cc_gram_iterate(ctypes.byref(p.c)), "btard_cc_gram_iterate")


def cc_remaining(p: Problem) -> int:
    """Synchronises the stream; upper bound on the iterations still needed."""
    out = ctypes.c_int32(0)
    _check(load_library().btard_cc_remaining(ctypes.byref(p.c), ctypes.byref(out)),
           "btard_cc_remaining")
    return int(out.value)


def debug_gram(p: Problem) -> torch.Tensor:
    N = 16 if int(p.g.shape[0]) <= 16 else 64
    out = torch.empty((p.parts, N, N), dtype=torch.float64, device=p.g.device)
    _check(load_library().btard_debug_gram(ctypes.byref(p.c), _ptr(out)), "btard_debug_gram")
    return out


def cc_iterate(p: Problem, first_iteration: int, count: int) -> None:
    _check(load_library().btard_cc_iterate(ctypes.byref(p.c), int(first_iteration), int(count)),
           "btard_cc_iterate")


def cc_finish(p: Problem, iterations: int, v: Optional[torch.Tensor] = None,
              iters: Optional[torch.Tensor] = None,
              last_step_norm: Optional[torch.Tensor] = None):
    dev = p.g.device
    if v is None:
        v = torch.empty(int(p.g.shape[1]), dtype=torch.float32, device=dev)
    if iters is None:
        iters = torch.empty(p.parts, dtype=torch.int32, device=dev)
    if last_step_norm is None:
        last_step_norm = torch.empty(p.parts, dtype=torch.float64, device=dev)
    _check(load_library().btard_cc_finish(ctypes.byref(p.c), int(iterations), _ptr(v),
                                          _ptr(iters), _ptr(last_step_norm)), "btard_cc_finish")
    return v, iters, last_step_norm


def _verify_outputs(n: int, P: int, dev, out: Optional[dict]) -> dict:
    if out is None:
        out = {}
    for key in ("norms", "weights", "proj"):
        if key not in out:
            out[key] = torch.empty((n, P), dtype=torch.float64, device=dev)
    if "colsum" not in out:
        out["colsum"] = torch.empty(P, dtype=torch.float64, device=dev)
    return out


def debug_last_pass(p: Problem, iterations: int, seed: int, v: torch.Tensor) -> None:
    """btard_debug_last_pass: the fused last pass kernel alone (for timing it)."""
    _check(load_library().btard_debug_last_pass(ctypes.byref(p.c), int(iterations), _ptr(v),
                                                int(seed) & 0xFFFFFFFFFFFFFFFF),
           "btard_debug_last_pass")


def debug_plain_stream(g: torch.Tensor, v: Optional[torch.Tensor], blocks: int) -> None:
    """btard_debug_plain_stream: a plain grid-stride kernel that reads the rows of g and, if v
    is given, writes their fp32 sum to it (a yardstick for the measured kernels)."""
    n, d = g.shape
    if v is not None and (v.dtype != torch.float32 or v.numel() != d or not v.is_contiguous()):
        raise ValueError("v must be a contiguous float32 vector of length d")
    _check(load_library().btard_debug_plain_stream(_ptr(g), _row_stride(g), n, d,
                                                   _ptr(v) if v is not None else None, int(blocks),
                                                   _stream_ptr(g.device)),
           "btard_debug_plain_stream")


def cc_finish_verify(p: Problem, iterations: int, seed: int, v: Optional[torch.Tensor] = None,
                     iters: Optional[torch.Tensor] = None,
                     last_step_norm: Optional[torch.Tensor] = None, out: Optional[dict] = None):
    """btard_cc_finish_verify.  Returns (v, iters, last_step_norm, dict of verification outputs)."""
    dev = p.g.device
    n = int(p.g.shape[0])
    if v is None:
        v = torch.empty(int(p.g.shape[1]), dtype=torch.float32, device=dev)
    if iters is None:
        iters = torch.empty(p.parts, dtype=torch.int32, device=dev)
    if last_step_norm is None:
        last_step_norm = torch.empty(p.parts, dtype=torch.float64, device=dev)
    out = _verify_outputs(n, p.parts, dev, out)
    _check(load_library().btard_cc_finish_verify(
        ctypes.byref(p.c), int(iterations), _ptr(v), _ptr(iters), _ptr(last_step_norm),
        int(seed) & 0xFFFFFFFFFFFFFFFF, _ptr(out["norms"]), _ptr(out["weights"]),
        _ptr(out["proj"]), _ptr(out["colsum"])), "btard_cc_finish_verify")
    return v, iters, last_step_norm, out


def centered_clip_verify(g: torch.Tensor, offsets: Sequence[int], tau: float, eps: float,
                         max_iters: int, seed: int, v0: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None, flags: int = BTARD_FLAG_NONE):
    """btard_centered_clip_verify.  Returns (v, iters, last_step_norm, dict)."""
    n, d = int(g.shape[0]), int(g.shape[1])
    P = len(offsets) - 1
    dev = g.device
    v = torch.empty(d, dtype=torch.float32, device=dev)
    iters = torch.empty(P, dtype=torch.int32, device=dev)
    last_step_norm = torch.empty(P, dtype=torch.float64, device=dev)
    out = _verify_outputs(n, P, dev, None)
    if workspace is None:
        workspace = alloc_workspace(n, P, dev)
    rc = load_library().btard_centered_clip_verify(
        _ptr(g), _row_stride(g), n, d, _off_array(offsets), P, float(tau), float(eps),
        int(max_iters), _ptr(v0), _ptr(v), _ptr(iters), _ptr(last_step_norm),
        int(seed) & 0xFFFFFFFFFFFFFFFF, _ptr(out["norms"]), _ptr(out["weights"]),
        _ptr(out["proj"]), _ptr(out["colsum"]), _ptr(workspace), workspace.numel(),
        _stream_ptr(dev), int(flags))
    _check(rc, "btard_centered_clip_verify")
    return v, iters, last_step_norm, out


def centered_clip_verify_noalloc(g: torch.Tensor, offsets: Sequence[int], tau: float, eps: float,
                                 max_iters: int, seed: int, v: torch.Tensor, iters: torch.Tensor,
                                 last_step_norm: torch.Tensor, out: dict,
                                 v0: Optional[torch.Tensor] = None,
                                 flags: int = BTARD_FLAG_NONE) -> None:
    """btard_centered_clip_verify_noalloc: every buffer is the caller's (v [d] fp32, iters [P]
    int32, last_step_norm [P] fp64, out = dict(norms, weights, proj [n, P], colsum [P]) fp64);
    nothing is allocated here either."""
    n, d = int(g.shape[0]), int(g.shape[1])
    P = len(offsets) - 1
    rc = load_library().btard_centered_clip_verify_noalloc(
        _ptr(g), _row_stride(g), n, d, _off_array(offsets), P, float(tau), float(eps),
        int(max_iters), _ptr(v0), _ptr(v), _ptr(iters), _ptr(last_step_norm),
        int(seed) & 0xFFFFFFFFFFFFFFFF, _ptr(out["norms"]), _ptr(out["weights"]),
        _ptr(out["proj"]), _ptr(out["colsum"]), _stream_ptr(g.device), int(flags))
    _check(rc, "btard_centered_clip_verify_noalloc")


def geometric_median(g: torch.Tensor, offsets: Sequence[int], nu: float, eps: float,
                     max_iters: int, v0: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None):
    """btard_geometric_median.  Returns (v fp32 [d], iters int32 [P], last_step_norm fp64 [P])."""
    n, d = int(g.shape[0]), int(g.shape[1])
    P = len(offsets) - 1
    dev = g.device
    v = torch.empty(d, dtype=torch.float32, device=dev)
    iters = torch.empty(P, dtype=torch.int32, device=dev)
    last_step_norm = torch.empty(P, dtype=torch.float64, device=dev)
    if workspace is None:
        workspace = alloc_workspace(n, P, dev)
    rc = load_library().btard_geometric_median(
        _ptr(g), _row_stride(g), n, d, _off_array(offsets), P, float(nu), float(eps),
        int(max_iters), _ptr(v0), _ptr(v), _ptr(iters), _ptr(last_step_norm),
        _ptr(workspace), workspace.numel(), _stream_ptr(dev))
    _check(rc, "btard_geometric_median")
    return v, iters, last_step_norm


def coordinate_median(g: torch.Tensor, v: Optional[torch.Tensor] = None) -> torch.Tensor:
    """btard_coordinate_median.  Returns v fp32 [d]."""
    n, d = int(g.shape[0]), int(g.shape[1])
    if v is None:
        v = torch.empty(d, dtype=torch.float32, device=g.device)
    rc = load_library().btard_coordinate_median(_ptr(g), _row_stride(g), n, d, _ptr(v),
                                                _stream_ptr(g.device))
    _check(rc, "btard_coordinate_median")
    return v


def hash_workspace_bytes(n: int, offsets: Sequence[int]) -> int:
    return int(load_library().btard_hash_workspace_bytes(int(n), _off_array(offsets),
                                                         len(offsets) - 1))


def partition_hashes(g: torch.Tensor, offsets: Sequence[int],
                     workspace: Optional[torch.Tensor] = None,
                     digests: Optional[torch.Tensor] = None) -> torch.Tensor:
    """btard_partition_hashes.  g: [n, d] fp32 (a 1-D tensor counts as one row).  Returns the
    digests, uint8 [n, parts, 32]."""
    if g.dim() == 1:
        g = g.unsqueeze(0)
    n, d = int(g.shape[0]), int(g.shape[1])
    P = len(offsets) - 1
    dev = g.device
    if workspace is None:
        workspace = torch.empty(max(hash_workspace_bytes(n, offsets), 256), dtype=torch.uint8,
                                device=dev)
    if digests is None:
        digests = torch.empty((n, P, 32), dtype=torch.uint8, device=dev)
    rc = load_library().btard_partition_hashes(
        _ptr(g), _row_stride(g), n, d, _off_array(offsets), P, _ptr(digests), _ptr(workspace),
        workspace.numel(), _stream_ptr(dev))
    _check(rc, "btard_partition_hashes")
    return digests


def tau_schedule(delta: float, sigma: float, b0: float, count: int) -> List[float]:
    """btard_tau_schedule: the radii tau_l of eq. (5), as the fp32 values the library uses."""
    out = (ctypes.c_float * max(count, 1))()
    _check(load_library().btard_tau_schedule(float(delta), float(sigma), float(b0), int(count), out),
           "btard_tau_schedule")
    return [float(out[i]) for i in range(count)]


def verification3(norms: torch.Tensor, delta_max: float):
    """btard_verification3.  norms: [n, parts] fp64 on the device.  Returns (check [n, parts]
    uint8, votes [parts] int32, trigger [parts] uint8)."""
    n, P = int(norms.shape[0]), int(norms.shape[1])
    assert norms.dtype == torch.float64 and norms.is_contiguous()
    dev = norms.device
    check = torch.empty((n, P), dtype=torch.uint8, device=dev)
    votes = torch.empty(P, dtype=torch.int32, device=dev)
    trigger = torch.empty(P, dtype=torch.uint8, device=dev)
    _check(load_library().btard_verification3(_ptr(norms), n, P, float(delta_max), _ptr(check),
                                              _ptr(votes), _ptr(trigger), _stream_ptr(dev)),
           "btard_verification3")
    return check, votes, trigger


def verification12(claimed_norms: torch.Tensor, claimed_proj: torch.Tensor, norms: torch.Tensor,
                   proj: torch.Tensor, rtol: float, atol: float):
    """btard_verification12.  All inputs [n, parts] fp64 on the device.  Returns (bad_norm
    [n, parts] uint8, bad_proj [n, parts] uint8, bad_sum [parts] uint8)."""
    n, P = int(norms.shape[0]), int(norms.shape[1])
    for t in (claimed_norms, claimed_proj, norms, proj):
        assert t.dtype == torch.float64 and t.is_contiguous() and tuple(t.shape) == (n, P)
    dev = norms.device
    bad_norm = torch.empty((n, P), dtype=torch.uint8, device=dev)
    bad_proj = torch.empty((n, P), dtype=torch.uint8, device=dev)
    bad_sum = torch.empty(P, dtype=torch.uint8, device=dev)
    _check(load_library().btard_verification12(
        _ptr(claimed_norms), _ptr(claimed_proj), _ptr(norms), _ptr(proj), n, P, float(rtol),
        float(atol), _ptr(bad_norm), _ptr(bad_proj), _ptr(bad_sum), _stream_ptr(dev)),
        "btard_verification12")
    return bad_norm, bad_proj, bad_sum


def cc_preclip_factors(p: Problem, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """btard_cc_preclip_factors.  Returns the [n, parts] fp64 factors alpha_ij."""
    n = int(p.g.shape[0])
    if out is None:
        out = torch.empty((n, p.parts), dtype=torch.float64, device=p.g.device)
    _check(load_library().btard_cc_preclip_factors(ctypes.byref(p.c), _ptr(out)),
           "btard_cc_preclip_factors")
    return out


def centered_clip_verify_preclipped(g: torch.Tensor, offsets: Sequence[int], lam: float,
                                    tau: float, eps: float, max_iters: int, seed: int,
                                    workspace: Optional[torch.Tensor] = None,
                                    flags: int = BTARD_FLAG_NONE):
    """btard_centered_clip_verify_preclipped.  Returns (v, iters, last_step_norm, dict,
    factors [n, parts])."""
    n, d = int(g.shape[0]), int(g.shape[1])
    P = len(offsets) - 1
    dev = g.device
    v = torch.empty(d, dtype=torch.float32, device=dev)
    iters = torch.empty(P, dtype=torch.int32, device=dev)
    last_step_norm = torch.empty(P, dtype=torch.float64, device=dev)
    factors = torch.empty((n, P), dtype=torch.float64, device=dev)
    out = _verify_outputs(n, P, dev, None)
    if workspace is None:
        workspace = alloc_workspace(n, P, dev)
    rc = load_library().btard_centered_clip_verify_preclipped(
        _ptr(g), _row_stride(g), n, d, _off_array(offsets), P, float(lam), float(tau),
        float(eps), int(max_iters), _ptr(v), _ptr(iters), _ptr(last_step_norm),
        int(seed) & 0xFFFFFFFFFFFFFFFF, _ptr(out["norms"]), _ptr(out["weights"]),
        _ptr(out["proj"]), _ptr(out["colsum"]), _ptr(factors), _ptr(workspace),
        workspace.numel(), _stream_ptr(dev), int(flags))
    _check(rc, "btard_centered_clip_verify_preclipped")
    return v, iters, last_step_norm, out, factors


def verify_projections(g: torch.Tensor, offsets: Sequence[int], v: torch.Tensor, tau: float,
                       seed: int, want_delta: bool = False,
                       workspace: Optional[torch.Tensor] = None,
                       out: Optional[dict] = None) -> dict:
    """btard_verify_projections.  Returns dict(norms, weights, proj [n,P], colsum [P], delta)."""
    n, d = int(g.shape[0]), int(g.shape[1])
    P = len(offsets) - 1
    dev = g.device
    if out is None:
        out = {}
    for key in ("norms", "weights", "proj"):
        if key not in out:
            out[key] = torch.empty((n, P), dtype=torch.float64, device=dev)
    if "colsum" not in out:
        out["colsum"] = torch.empty(P, dtype=torch.float64, device=dev)
    if want_delta and out.get("delta") is None:
        out["delta"] = torch.empty((n, d), dtype=torch.float32, device=dev)
    delta = out.get("delta") if want_delta else None
    if workspace is None:
        workspace = alloc_workspace(n, P, dev)
    rc = load_library().btard_verify_projections(
        _ptr(g), _row_stride(g), n, d, _off_array(offsets), P, _ptr(v), float(tau),
        int(seed) & 0xFFFFFFFFFFFFFFFF, _ptr(out["norms"]), _ptr(out["weights"]),
        _ptr(out["proj"]), _ptr(out["colsum"]), _ptr(delta),
        _row_stride(delta) if delta is not None else 0, _ptr(workspace), workspace.numel(),
        _stream_ptr(dev), BTARD_FLAG_NONE)
    _check(rc, "btard_verify_projections")
    return out


def verify_projections_preclipped(g: torch.Tensor, offsets: Sequence[int], v: torch.Tensor,
                                  tau: float, seed: int, lam: float = 0.0,
                                  factors: Optional[torch.Tensor] = None,
                                  want_delta: bool = False,
                                  workspace: Optional[torch.Tensor] = None,
                                  out: Optional[dict] = None) -> dict:
    """btard_verify_projections_preclipped: the factors are `factors` ([n, P] fp64) if given,
    else those of the radius `lam`.  Returns dict(norms, weights, proj, colsum, delta,
    factors = the factors used)."""
    n, d = int(g.shape[0]), int(g.shape[1])
    P = len(offsets) - 1
    dev = g.device
    if out is None:
        out = {}
    for key in ("norms", "weights", "proj", "factors"):
        if key not in out:
            out[key] = torch.empty((n, P), dtype=torch.float64, device=dev)
    if "colsum" not in out:
        out["colsum"] = torch.empty(P, dtype=torch.float64, device=dev)
    if want_delta and out.get("delta") is None:
        out["delta"] = torch.empty((n, d), dtype=torch.float32, device=dev)
    delta = out.get("delta") if want_delta else None
    if workspace is None:
        workspace = alloc_workspace(n, P, dev)
    if factors is not None:
        assert factors.dtype == torch.float64 and factors.is_contiguous()
        assert tuple(factors.shape) == (n, P)
    rc = load_library().btard_verify_projections_preclipped(
        _ptr(g), _row_stride(g), n, d, _off_array(offsets), P, _ptr(v), float(lam),
        _ptr(factors), float(tau), int(seed) & 0xFFFFFFFFFFFFFFFF, _ptr(out["norms"]),
        _ptr(out["weights"]), _ptr(out["proj"]), _ptr(out["colsum"]), _ptr(delta),
        _row_stride(delta) if delta is not None else 0, _ptr(out["factors"]), _ptr(workspace),
        workspace.numel(), _stream_ptr(dev), BTARD_FLAG_NONE)
    _check(rc, "btard_verify_projections_preclipped")
    return out


def debug_zhat(seed: int, x_begin: int, count: int, device) -> torch.Tensor:
    out = torch.empty(count, dtype=torch.float32, device=device)
    rc = load_library().btard_debug_zhat(int(seed) & 0xFFFFFFFFFFFFFFFF, int(x_begin),
                                         int(count), _ptr(out), _stream_ptr(device))
    _check(rc, "btard_debug_zhat")
    return out


# names as in include/btard.h
btard_status_string = status_string
btard_split_offsets = split_offsets
btard_workspace_bytes = workspace_bytes
btard_centered_clip = centered_clip
btard_cc_begin = cc_begin
btard_cc_gram = cc_gram
btard_cc_gram_matrix = cc_gram_matrix
btard_cc_gram_iterate = cc_gram_iterate
btard_cc_remaining = cc_remaining
btard_debug_gram = debug_gram
btard_debug_last_pass = debug_last_pass
btard_debug_plain_stream = debug_plain_stream
btard_cc_iterate = cc_iterate
btard_cc_finish = cc_finish
btard_verify_projections = verify_projections
btard_verify_projections_preclipped = verify_projections_preclipped
btard_cc_finish_verify = cc_finish_verify
btard_centered_clip_verify = centered_clip_verify
btard_centered_clip_verify_noalloc = centered_clip_verify_noalloc
btard_cc_preclip_factors = cc_preclip_factors
btard_tau_schedule = tau_schedule
btard_hash_workspace_bytes = hash_workspace_bytes
btard_partition_hashes = partition_hashes
btard_geometric_median = geometric_median
btard_coordinate_median = coordinate_median
btard_verification3 = verification3
btard_verification12 = verification12
btard_centered_clip_verify_preclipped = centered_clip_verify_preclipped
btard_debug_zhat = debug_zhat
