"""ctypes/numpy front end of the plain-C fp64 oracle (``btard_oracle.c``).

Test infrastructure only: argument marshalling, no arithmetic of the method.
The shared object is compiled with gcc next to the source on first use.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "btard_oracle.c")
_SO = os.path.join(_HERE, "libbtard_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the .so path."""
    stale = (not os.path.exists(_SO)) or os.path.getmtime(_SO) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
             "-o", _SO, _SRC, "-lm"]
        )
    return _SO


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build())
    c = ctypes
    P = c.POINTER
    lib.oracle_num_threads.restype = c.c_int
    lib.oracle_set_num_threads.argtypes = [c.c_int]
    lib.oracle_set_num_threads.restype = None
    lib.oracle_split.argtypes = [c.c_int64, c.c_int32, P(c.c_int64)]
    lib.oracle_split.restype = c.c_int
    lib.oracle_centered_clip.argtypes = [
        c.c_void_p, c.c_int64, c.c_int32, P(c.c_int64), c.c_int32, c.c_double,
        c.c_double, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_void_p]
    lib.oracle_centered_clip.restype = c.c_int
    lib.oracle_centered_clip_scaled.argtypes = [
        c.c_void_p, c.c_int64, c.c_int32, P(c.c_int64), c.c_int32, c.c_double,
        c.c_double, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_void_p]
    lib.oracle_centered_clip_scaled.restype = c.c_int
    lib.oracle_centered_clip_general.argtypes = [
        c.c_void_p, c.c_int64, c.c_int32, P(c.c_int64), c.c_int32, c.c_double,
        c.c_double, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_void_p, c.c_void_p]
    lib.oracle_centered_clip_general.restype = c.c_int
    lib.oracle_geometric_median.argtypes = [
        c.c_void_p, c.c_int64, c.c_int32, P(c.c_int64), c.c_int32, c.c_double, c.c_double,
        c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p]
    lib.oracle_geometric_median.restype = c.c_int
    lib.oracle_coordinate_median.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_int64,
                                             c.c_void_p]
    lib.oracle_coordinate_median.restype = c.c_int
    lib.oracle_tau_schedule.argtypes = [c.c_double, c.c_double, c.c_double, c.c_int32,
                                        c.c_void_p, c.c_void_p]
    lib.oracle_tau_schedule.restype = c.c_int
    lib.oracle_verification3.argtypes = [c.c_void_p, c.c_int32, c.c_int32, c.c_double,
                                         c.c_void_p, c.c_void_p, c.c_void_p]
    lib.oracle_verification3.restype = c.c_int
    lib.oracle_verification12.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32,
                                          c.c_int32, c.c_double, c.c_double, c.c_void_p,
                                          c.c_void_p, c.c_void_p]
    lib.oracle_verification12.restype = c.c_int
    lib.oracle_preclip_scales.argtypes = [
        c.c_void_p, c.c_int64, c.c_int32, P(c.c_int64), c.c_int32, c.c_double, c.c_void_p,
        c.c_void_p]
    lib.oracle_preclip_scales.restype = c.c_int
    lib.oracle_verify_scaled.argtypes = [
        c.c_void_p, c.c_int64, c.c_int32, P(c.c_int64), c.c_int32, c.c_void_p,
        c.c_double, c.c_uint64, c.c_int64, c.c_double, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64]
    lib.oracle_verify_scaled.restype = c.c_int
    lib.oracle_philox4x32_10.argtypes = [P(c.c_uint32), P(c.c_uint32), P(c.c_uint32)]
    lib.oracle_philox4x32_10.restype = None
    lib.oracle_z_uniforms.argtypes = [c.c_uint64, c.c_int64, c.c_int64, c.c_void_p]
    lib.oracle_z_uniforms.restype = None
    lib.oracle_z_hat.argtypes = [c.c_uint64, c.c_int64, c.c_int64, c.c_void_p]
    lib.oracle_z_hat.restype = None
    lib.oracle_z_norm.argtypes = [c.c_uint64, c.c_int64]
    lib.oracle_z_norm.restype = c.c_double
    lib.oracle_verify.argtypes = [
        c.c_void_p, c.c_int64, c.c_int32, P(c.c_int64), c.c_int32, c.c_void_p,
        c.c_double, c.c_uint64, c.c_int64, c.c_double, c.c_void_p, c.c_void_p,
        c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64]
    lib.oracle_verify.restype = c.c_int
    _lib = lib
    return lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(k: int) -> None:
    """Threads the oracle's coordinate loops use from now on (for timing it on one core)."""
    _load().oracle_set_num_threads(int(k))


def _offsets(off: Sequence[int]):
    arr = (ctypes.c_int64 * len(off))(*[int(o) for o in off])
    return arr


def _as_G(G) -> np.ndarray:
    G = np.asarray(G)
    if G.dtype != np.float32 or G.ndim != 2 or G.strides[1] != 4 or G.strides[0] % 4:
        G = np.ascontiguousarray(G, dtype=np.float32)
    return G


def split(d: int, parts: int) -> np.ndarray:
    off = (ctypes.c_int64 * (parts + 1))()
    if _load().oracle_split(d, parts, off) != 0:
        raise ValueError("oracle_split: bad arguments")
    return np.array(off[:], dtype=np.int64)


def preclip_scales(G, off, lam: float):
    """Pre-clipping factors of BTARD-Clipped-SGD: (alpha [n, P], norms [n, P])."""
    G = _as_G(G)
    n, _ = G.shape
    ld = G.strides[0] // 4 if n > 1 else G.shape[1]
    Pn = len(off) - 1
    alpha = np.zeros((n, Pn)); norms = np.zeros((n, Pn))
    rc = _load().oracle_preclip_scales(G.ctypes.data, ld, n, _offsets(off), Pn, float(lam),
                                       alpha.ctypes.data, norms.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_preclip_scales: bad arguments")
    return alpha, norms


def geometric_median(G, off, nu: float, eps: float, max_iters: int,
                     v0: Optional[np.ndarray] = None):
    """Weiszfeld's iteration per partition: (v [fp64], iters [int32, P], step_norm [fp64, P])."""
    G = _as_G(G)
    n, _ = G.shape
    ld = G.strides[0] // 4 if n > 1 else G.shape[1]
    Pn = len(off) - 1
    width = int(off[-1])
    v = np.zeros(max(width, 1), dtype=np.float64)
    iters = np.zeros(Pn, dtype=np.int32)
    sn = np.zeros(Pn, dtype=np.float64)
    v0p = None
    if v0 is not None:
        v0 = np.ascontiguousarray(v0, dtype=np.float64)
        assert v0.shape[0] >= width
        v0p = v0.ctypes.data
    rc = _load().oracle_geometric_median(G.ctypes.data, ld, n, _offsets(off), Pn, float(nu),
                                         float(eps), int(max_iters), v0p, v.ctypes.data,
                                         iters.ctypes.data, sn.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_geometric_median: bad arguments")
    return v[:width], iters, sn


def coordinate_median(G) -> np.ndarray:
    """Coordinate-wise median of the rows (mean of the two middle values for even n)."""
    G = _as_G(G)
    n, d = G.shape
    ld = G.strides[0] // 4 if n > 1 else d
    v = np.zeros(max(d, 1), dtype=np.float64)
    if _load().oracle_coordinate_median(G.ctypes.data, ld, n, d, v.ctypes.data) != 0:
        raise ValueError("oracle_coordinate_median: bad arguments")
    return v[:d]


def partition_hashes(G, off, chunk_bytes: int = 1024, fanout: int = 32) -> np.ndarray:
    """hash(g_i[j]) of Alg. 2 (lines 2 and 6) with the hash function this build fixes, since
    the paper names none: SHA-256 (the library's) over a tree.  The partition's bytes (fp32,
    little-endian, as stored) are cut into chunks of `chunk_bytes` (an empty partition is one
    empty chunk) and every chunk is hashed; while more than one digest remains, every run of
    `fanout` consecutive digests (the last may be shorter) is replaced by the SHA-256 of
    their concatenation.  Returns uint8 [n, P, 32]."""
    import hashlib
    G = _as_G(G)
    n = G.shape[0]
    Pn = len(off) - 1
    out = np.zeros((n, Pn, 32), dtype=np.uint8)
    for i in range(n):
        for j in range(Pn):
            data = np.ascontiguousarray(G[i, int(off[j]):int(off[j + 1])]).astype("<f4").tobytes()
            nodes = [hashlib.sha256(data[k:k + chunk_bytes]).digest()
                     for k in range(0, max(len(data), 1), chunk_bytes)]
            while len(nodes) > 1:
                nodes = [hashlib.sha256(b"".join(nodes[k:k + fanout])).digest()
                         for k in range(0, len(nodes), fanout)]
            out[i, j] = np.frombuffer(nodes[0], dtype=np.uint8)
    return out


def tau_schedule(delta: float, sigma: float, B0: float, count: int):
    """The clipping radii tau_l of eq. (5): (tau [count], B_l^2 [count])."""
    tau = np.zeros(max(count, 1)); b2 = np.zeros(max(count, 1))
    if _load().oracle_tau_schedule(float(delta), float(sigma), float(B0), int(count),
                                   tau.ctypes.data, b2.ctypes.data) != 0:
        raise ValueError("oracle_tau_schedule: bad arguments")
    return tau[:count], b2[:count]


def verification3(norms, delta_max: float):
    """Verification 3 of Alg. 6: (check [n, P] uint8, votes [P] int32, trigger [P] uint8)."""
    norms = np.ascontiguousarray(norms, dtype=np.float64)
    n, Pn = norms.shape
    check = np.zeros((n, Pn), dtype=np.uint8)
    votes = np.zeros(Pn, dtype=np.int32)
    trigger = np.zeros(Pn, dtype=np.uint8)
    if _load().oracle_verification3(norms.ctypes.data, n, Pn, float(delta_max), check.ctypes.data,
                                    votes.ctypes.data, trigger.ctypes.data) != 0:
        raise ValueError("oracle_verification3: bad arguments")
    return check, votes, trigger


def verification12(claimed_norms, claimed_proj, norms, proj, rtol: float, atol: float):
    """Verifications 1 and 2 of Alg. 6 as comparisons: (bad_norm [n, P], bad_proj [n, P],
    bad_sum [P]), all uint8."""
    arrs = [np.ascontiguousarray(a, dtype=np.float64) for a in (claimed_norms, claimed_proj, norms, proj)]
    n, Pn = arrs[2].shape
    assert all(a.shape == (n, Pn) for a in arrs)
    bad_norm = np.zeros((n, Pn), dtype=np.uint8)
    bad_proj = np.zeros((n, Pn), dtype=np.uint8)
    bad_sum = np.zeros(Pn, dtype=np.uint8)
    if _load().oracle_verification12(arrs[0].ctypes.data, arrs[1].ctypes.data, arrs[2].ctypes.data,
                                     arrs[3].ctypes.data, n, Pn, float(rtol), float(atol),
                                     bad_norm.ctypes.data, bad_proj.ctypes.data,
                                     bad_sum.ctypes.data) != 0:
        raise ValueError("oracle_verification12: bad arguments")
    return bad_norm, bad_proj, bad_sum


def centered_clip(G, off, tau: float, eps: float, max_iters: int,
                  v0: Optional[np.ndarray] = None, want_trace: bool = False,
                  scale: Optional[np.ndarray] = None, tau_l: Optional[Sequence[float]] = None):
    """Returns (v[fp64, ld], iters[int32, P], step_norm[fp64, P], trace|None).
    scale (optional, [n, P]): run on the rows scale[i, j] * G[i, partition j].
    tau_l (optional, max_iters radii): update l uses tau_l[l] instead of tau."""
    G = _as_G(G)
    n, _ = G.shape
    ld = G.strides[0] // 4 if n > 1 else G.shape[1]
    Pn = len(off) - 1
    width = int(off[-1])
    v = np.zeros(max(width, 1), dtype=np.float64)
    iters = np.zeros(Pn, dtype=np.int32)
    sn = np.zeros(Pn, dtype=np.float64)
    trace = np.zeros((Pn, max(max_iters, 1)), dtype=np.float64) if want_trace else None
    v0p = None
    if v0 is not None:
        v0 = np.ascontiguousarray(v0, dtype=np.float64)
        assert v0.shape[0] >= width
        v0p = v0.ctypes.data
    sp = None
    if scale is not None:
        scale = np.ascontiguousarray(scale, dtype=np.float64)
        assert scale.shape == (n, Pn)
        sp = scale.ctypes.data
    tp = None
    if tau_l is not None:
        tau_l = np.ascontiguousarray(tau_l, dtype=np.float64)
        assert tau_l.shape == (max_iters,)
        tp = tau_l.ctypes.data
    rc = _load().oracle_centered_clip_general(
        G.ctypes.data, ld, n, _offsets(off), Pn, float(tau), float(eps),
        int(max_iters), v0p, sp, tp, v.ctypes.data, iters.ctypes.data, sn.ctypes.data,
        trace.ctypes.data if want_trace else None)
    if rc != 0:
        raise ValueError("oracle_centered_clip: bad arguments")
    return v[:width], iters, sn, trace


def philox4x32_10(ctr: Sequence[int], key: Sequence[int]):
    c = (ctypes.c_uint32 * 4)(*ctr)
    k = (ctypes.c_uint32 * 2)(*key)
    o = (ctypes.c_uint32 * 4)()
    _load().oracle_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def z_uniforms(seed: int, x_begin: int, count: int) -> np.ndarray:
    out = np.zeros(count, dtype=np.float64)
    _load().oracle_z_uniforms(seed, x_begin, count, out.ctypes.data)
    return out


def z_hat(seed: int, x_begin: int, count: int) -> np.ndarray:
    out = np.zeros(count, dtype=np.float64)
    _load().oracle_z_hat(seed, x_begin, count, out.ctypes.data)
    return out


def z_norm(seed: int, d: int) -> float:
    return float(_load().oracle_z_norm(seed, d))


def verify(G, off, v, tau: float, seed: int, x_base: int = 0,
           znorm: Optional[float] = None, want_delta: bool = False,
           scale: Optional[np.ndarray] = None):
    """Returns dict(norms, weights, proj [n,P], colsum [P], delta [n,width]|None).
    scale (optional, [n, P]): the quantities of the rows scale[i, j] * G[i, partition j]."""
    G = _as_G(G)
    n, _ = G.shape
    ld = G.strides[0] // 4 if n > 1 else G.shape[1]
    Pn = len(off) - 1
    width = int(off[-1])
    v = np.ascontiguousarray(v, dtype=np.float64)
    assert v.shape[0] >= width
    if znorm is None:
        znorm = z_norm(seed, x_base + width)
    norms = np.zeros((n, Pn)); weights = np.zeros((n, Pn)); proj = np.zeros((n, Pn))
    colsum = np.zeros(Pn)
    delta = np.zeros((n, max(width, 1))) if want_delta else None
    sp = None
    if scale is not None:
        scale = np.ascontiguousarray(scale, dtype=np.float64)
        assert scale.shape == (n, Pn)
        sp = scale.ctypes.data
    rc = _load().oracle_verify_scaled(
        G.ctypes.data, ld, n, _offsets(off), Pn, v.ctypes.data, float(tau),
        int(seed), int(x_base), float(znorm), sp, norms.ctypes.data,
        weights.ctypes.data, proj.ctypes.data, colsum.ctypes.data,
        delta.ctypes.data if want_delta else None, max(width, 1))
    if rc != 0:
        raise ValueError("oracle_verify: bad arguments")
    return dict(norms=norms, weights=weights, proj=proj, colsum=colsum,
                delta=delta[:, :width] if want_delta else None, znorm=znorm)
