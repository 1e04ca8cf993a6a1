"""Thin ctypes binding of libdssync.so: argument marshalling only.

Every function has the name and the argument order of its C entry point in
``include/dssync.h`` and raises :class:`DsError` for a negative status.  Device
buffers are torch tensors (or raw integer addresses); torch is used for device
memory and for the current stream handle, nothing else.  There is no CPU
fallback: if the shared library is missing, the first call raises ImportError.
"""
from __future__ import annotations

import ctypes
import os
from typing import Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdssync.so")

DS_F32, DS_BF16 = 0, 1
DS_MAX_W = 64

DS_MAX_COLUMNS = ((1 << 26) - 1) * 256

EXPORTS = ("ds_status_string", "ds_partition", "ds_pattern", "ds_pattern_period", "ds_pattern_check", "ds_group_sync",
           "ds_ragged_plan_bytes", "ds_ragged_plan", "ds_group_sync_ragged", "ds_group_sync_opt",
           "ds_group_sync_ragged_opt", "ds_consensus_workspace_bytes", "ds_consensus", "ds_consensus_static", "ds_consensus_grouped",
           "ds_group_sync_consensus_workspace_bytes", "ds_group_sync_consensus", "ds_tiled_elements",
           "ds_group_sync_tiled", "ds_consensus_tiled", "ds_consensus_grouped_tiled", "ds_group_sync_consensus_tiled",
           "ds_padded_ld")


class DsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, status_string(status), status))


class ds_local_opt(ctypes.Structure):
    _fields_ = [("V", ctypes.c_void_p), ("ldv", ctypes.c_int64), ("momentum", ctypes.c_float),
                ("weight_decay", ctypes.c_float), ("S", ctypes.c_void_p), ("lds", ctypes.c_int64),
                ("swa_factor", ctypes.c_float)]


class ds_segment(ctypes.Structure):
    _fields_ = [("offset", ctypes.c_int64), ("length", ctypes.c_int64)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError("libdssync.so is not built: run `python -m paper_2007_03298_amd.build` "
                          "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    i32p = ctypes.POINTER(ctypes.c_int32)
    segp = ctypes.POINTER(ds_segment)
    vp, i32, i64, u64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64, ctypes.c_size_t
    lib.ds_status_string.restype = ctypes.c_char_p
    lib.ds_status_string.argtypes = [ctypes.c_int]
    lib.ds_partition.restype = ctypes.c_int
    lib.ds_partition.argtypes = [u64, u64, i32, i32p, i32, i32p, i32p]
    u8p = ctypes.POINTER(ctypes.c_uint8)
    lib.ds_pattern.restype = ctypes.c_int
    lib.ds_pattern.argtypes = [i32, i32p, u8p, i32, u8p, u64, i32p, i32p, i32p]
    lib.ds_pattern_period.restype = ctypes.c_int
    lib.ds_pattern_period.argtypes = [i32, i32p, u8p, i32, u8p, ctypes.POINTER(u64)]
    f64p = ctypes.POINTER(ctypes.c_double)
    lib.ds_pattern_check.restype = ctypes.c_int
    lib.ds_pattern_check.argtypes = [i32, i32, i32p, i32p, i32p, i32p, f64p, f64p]
    lib.ds_group_sync.restype = ctypes.c_int
    lib.ds_group_sync.argtypes = [vp, vp, i32, i64, i64, i64, i32, i32p, i32p, i32, ctypes.c_float, vp]
    lib.ds_ragged_plan_bytes.restype = sz
    lib.ds_ragged_plan_bytes.argtypes = [segp, i32]
    lib.ds_ragged_plan.restype = ctypes.c_int
    lib.ds_ragged_plan.argtypes = [segp, i32, i64, i64, vp, sz, ctypes.POINTER(u64), vp]
    lib.ds_group_sync_ragged.restype = ctypes.c_int
    lib.ds_group_sync_ragged.argtypes = [vp, vp, i32, segp, i32, i64, i64, i32, i32p, i32p, i32,
                                         ctypes.c_float, vp, sz, u64, vp]
    optp = ctypes.POINTER(ds_local_opt)
    lib.ds_group_sync_opt.restype = ctypes.c_int
    lib.ds_group_sync_opt.argtypes = [vp, vp, i32, i64, i64, i64, i32, i32p, i32p, i32, ctypes.c_float, optp, vp]
    lib.ds_group_sync_ragged_opt.restype = ctypes.c_int
    lib.ds_group_sync_ragged_opt.argtypes = [vp, vp, i32, segp, i32, i64, i64, i32, i32p, i32p, i32,
                                             ctypes.c_float, optp, vp, sz, u64, vp]
    lib.ds_consensus_workspace_bytes.restype = sz
    lib.ds_consensus_workspace_bytes.argtypes = [i32, i64]
    lib.ds_consensus.restype = ctypes.c_int
    lib.ds_consensus.argtypes = [vp, i64, i64, i32, vp, vp, sz, vp]
    lib.ds_consensus_static.restype = ctypes.c_int
    lib.ds_consensus_static.argtypes = [vp, i64, i64, i32, vp, vp]
    lib.ds_consensus_grouped.restype = ctypes.c_int
    lib.ds_consensus_grouped.argtypes = [vp, i64, i64, i32, i32p, i32p, i32, vp, vp, sz, vp]
    lib.ds_group_sync_consensus_workspace_bytes.restype = sz
    lib.ds_group_sync_consensus_workspace_bytes.argtypes = [i64, i32]
    lib.ds_group_sync_consensus.restype = ctypes.c_int
    lib.ds_group_sync_consensus.argtypes = [vp, vp, i32, i64, i64, i64, i32, i32p, i32p, i32, ctypes.c_float, vp, vp,
                                            sz, vp]
    lib.ds_tiled_elements.restype = i64
    lib.ds_tiled_elements.argtypes = [i64, i32]
    lib.ds_group_sync_tiled.restype = ctypes.c_int
    lib.ds_group_sync_tiled.argtypes = [vp, vp, i32, i64, i64, i64, i32, i32p, i32p, i32, ctypes.c_float, optp, vp]
    lib.ds_consensus_tiled.restype = ctypes.c_int
    lib.ds_consensus_tiled.argtypes = [vp, i64, i64, i32, vp, vp, sz, vp]
    lib.ds_consensus_grouped_tiled.restype = ctypes.c_int
    lib.ds_consensus_grouped_tiled.argtypes = [vp, i64, i64, i32, i32p, i32p, i32, vp, vp, sz, vp]
    lib.ds_group_sync_consensus_tiled.restype = ctypes.c_int
    lib.ds_group_sync_consensus_tiled.argtypes = [vp, vp, i32, i64, i64, i64, i32, i32p, i32p, i32, ctypes.c_float,
                                                  vp, vp, sz, vp]
    lib.ds_padded_ld.restype = i64
    lib.ds_padded_ld.argtypes = [i64]
    return lib


class _Lazy:
    """Loads the shared library on first use, so that the build module of this
    package can be imported before the library exists.  Any call without a
    built library raises ImportError: there is no fallback path."""

    _lib = None

    def __getattr__(self, name):
        if _Lazy._lib is None:
            _Lazy._lib = _load()
        return getattr(_Lazy._lib, name)


_lib = _Lazy()


def load() -> None:
    """Load the library now (raises ImportError if it is not built)."""
    _lib.ds_status_string


def _addr(buf) -> int:
    """Device (or host) address of a torch tensor, or the integer itself."""
    if buf is None:
        return 0
    if isinstance(buf, int):
        return buf
    return int(buf.data_ptr())


def _stream(stream) -> int:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return stream
    return int(stream.cuda_stream)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _i32p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _segs(segments) -> Tuple[ctypes.Array, int]:
    segments = list(segments)
    arr = (ds_segment * max(len(segments), 1))()
    for s, (o, l) in enumerate(segments):
        arr[s].offset, arr[s].length = int(o), int(l)
    return arr, len(segments)


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise DsError(rc, where)


def status_string(status: int) -> str:
    return _lib.ds_status_string(int(status)).decode()


def ds_partition(seed: int, t: int, W: int, sizes: Sequence[int]) -> Tuple[np.ndarray, np.ndarray]:
    """Groups of iteration ``t``: returns ``(perm[W], off[n_groups+1])`` (host int32)."""
    sz = _i32(sizes)
    perm = np.zeros(max(int(W), 1), dtype=np.int32)
    off = np.zeros(len(sz) + 1, dtype=np.int32)
    _check(_lib.ds_partition(seed & (2**64 - 1), t & (2**64 - 1), int(W), _i32p(sz), len(sz), _i32p(perm),
                             _i32p(off)), "ds_partition")
    return perm[:W], off


def _u8(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.uint8))


def _u8p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))


def ds_pattern(rack_of: Sequence[int], slow_rack: Sequence[int], slow_worker: Sequence[int],
               t: int) -> Tuple[np.ndarray, np.ndarray]:
    """Topology-aware groups of iteration ``t``: ``(perm[W], off[n_groups+1])``."""
    rk, sr, sw = _i32(rack_of), _u8(slow_rack), _u8(slow_worker)
    W = len(rk)
    if len(sw) != W:
        raise ValueError("slow_worker must have one flag per worker")
    perm = np.zeros(max(W, 1), dtype=np.int32)
    off = np.zeros(W + 1, dtype=np.int32)
    n = ctypes.c_int32(0)
    _check(_lib.ds_pattern(W, _i32p(rk), _u8p(sr), len(sr), _u8p(sw), t & (2**64 - 1), _i32p(perm), _i32p(off),
                           ctypes.byref(n)), "ds_pattern")
    return perm[:W], off[:n.value + 1]


def ds_pattern_period(rack_of: Sequence[int], slow_rack: Sequence[int], slow_worker: Sequence[int]) -> int:
    rk, sr, sw = _i32(rack_of), _u8(slow_rack), _u8(slow_worker)
    if len(sw) != len(rk):
        raise ValueError("slow_worker must have one flag per worker")
    B = ctypes.c_uint64(0)
    _check(_lib.ds_pattern_period(len(rk), _i32p(rk), _u8p(sr), len(sr), _u8p(sw), ctypes.byref(B)),
           "ds_pattern_period")
    return int(B.value)


def ds_pattern_check(W: int, divisions) -> Tuple[bool, float, float]:
    """``(connected, rho, sigma)`` of a periodic list of divisions, each a ``(perm, off)`` pair."""
    divisions = list(divisions)
    B = len(divisions)
    perms = np.zeros((max(B, 1), max(W, 1)), dtype=np.int32)
    offs = np.zeros((max(B, 1), max(W, 1) + 1), dtype=np.int32)
    counts = np.zeros(max(B, 1), dtype=np.int32)
    for k, (perm, off) in enumerate(divisions):
        perm, off = _i32(perm), _i32(off)
        if len(perm) != W or not 2 <= len(off) <= W + 1:
            raise ValueError("division %d does not have W workers" % k)
        perms[k, :W] = perm
        offs[k, :len(off)] = off
        counts[k] = len(off) - 1
    connected = ctypes.c_int32(0)
    rho, sigma = ctypes.c_double(0.0), ctypes.c_double(0.0)
    _check(_lib.ds_pattern_check(int(W), B, _i32p(perms), _i32p(offs), _i32p(counts), ctypes.byref(connected),
                                 ctypes.byref(rho), ctypes.byref(sigma)), "ds_pattern_check")
    return bool(connected.value), float(rho.value), float(sigma.value)


def ds_group_sync(X, G, g_dtype: int, P: int, ldx: int, ldg: int, W: int, perm, off, lr: float,
                  stream=None) -> None:
    perm, off = _i32(perm), _i32(off)
    _check(_lib.ds_group_sync(_addr(X), _addr(G), g_dtype, P, ldx, ldg, W, _i32p(perm), _i32p(off),
                              len(off) - 1, lr, _stream(stream)), "ds_group_sync")


def ds_ragged_plan_bytes(segments) -> int:
    arr, S = _segs(segments)
    return int(_lib.ds_ragged_plan_bytes(arr, S))


def ds_ragged_plan(segments, ldx: int, ldg: int, plan, plan_bytes: int, stream=None) -> int:
    """Enqueues the kernels that write the plan; returns ``plan_id`` (what ``*plan_id_out`` received)."""
    arr, S = segments if isinstance(segments, tuple) and isinstance(segments[1], int) else _segs(segments)
    plan_id = ctypes.c_uint64(0)
    _check(_lib.ds_ragged_plan(arr, S, ldx, ldg, _addr(plan), plan_bytes, ctypes.byref(plan_id), _stream(stream)),
           "ds_ragged_plan")
    return int(plan_id.value)


def ds_group_sync_ragged(X, G, g_dtype: int, segments, ldx: int, ldg: int, W: int, perm, off, lr: float,
                         plan, plan_bytes: int, plan_id: int, stream=None) -> None:
    arr, S = segments if isinstance(segments, tuple) and isinstance(segments[1], int) else _segs(segments)
    perm, off = _i32(perm), _i32(off)
    _check(_lib.ds_group_sync_ragged(_addr(X), _addr(G), g_dtype, arr, S, ldx, ldg, W, _i32p(perm), _i32p(off),
                                     len(off) - 1, lr, _addr(plan), plan_bytes, plan_id, _stream(stream)),
           "ds_group_sync_ragged")


def local_opt(V=None, ldv: int = 0, momentum: float = 0.0, weight_decay: float = 0.0, S=None, lds: int = 0,
              swa_factor: float = 0.0) -> ds_local_opt:
    """Fill a ``ds_local_opt`` (momentum buffers ``V``, SWA models ``S``; either may be None)."""
    return ds_local_opt(_addr(V) or None, ldv, momentum, weight_decay, _addr(S) or None, lds, swa_factor)


def ds_group_sync_opt(X, G, g_dtype: int, P: int, ldx: int, ldg: int, W: int, perm, off, lr: float,
                      opt: ds_local_opt | None, stream=None) -> None:
    perm, off = _i32(perm), _i32(off)
    _check(_lib.ds_group_sync_opt(_addr(X), _addr(G), g_dtype, P, ldx, ldg, W, _i32p(perm), _i32p(off),
                                  len(off) - 1, lr, ctypes.byref(opt) if opt is not None else None,
                                  _stream(stream)), "ds_group_sync_opt")


def ds_group_sync_ragged_opt(X, G, g_dtype: int, segments, ldx: int, ldg: int, W: int, perm, off, lr: float,
                             opt: ds_local_opt | None, plan, plan_bytes: int, plan_id: int, stream=None) -> None:
    arr, S = segments if isinstance(segments, tuple) and isinstance(segments[1], int) else _segs(segments)
    perm, off = _i32(perm), _i32(off)
    _check(_lib.ds_group_sync_ragged_opt(_addr(X), _addr(G), g_dtype, arr, S, ldx, ldg, W, _i32p(perm), _i32p(off),
                                         len(off) - 1, lr, ctypes.byref(opt) if opt is not None else None,
                                         _addr(plan), plan_bytes, plan_id, _stream(stream)),
           "ds_group_sync_ragged_opt")


def pack_segments(segments):
    """Marshal a segment list once; the result can be passed as ``segments``."""
    return _segs(segments)


def ds_consensus_workspace_bytes(W: int, P: int) -> int:
    return int(_lib.ds_consensus_workspace_bytes(int(W), int(P)))


def ds_consensus(X, P: int, ld: int, W: int, dev_out, workspace, workspace_bytes: int, stream=None) -> None:
    _check(_lib.ds_consensus(_addr(X), P, ld, W, _addr(dev_out), _addr(workspace), workspace_bytes,
                             _stream(stream)), "ds_consensus")


def ds_consensus_static(X, P: int, ld: int, W: int, dev_out, stream=None) -> None:
    _check(_lib.ds_consensus_static(_addr(X), P, ld, W, _addr(dev_out), _stream(stream)), "ds_consensus_static")


def ds_consensus_grouped(X, P: int, ld: int, W: int, perm, off, dev_out, workspace, workspace_bytes: int,
                         stream=None) -> None:
    perm, off = _i32(perm), _i32(off)
    _check(_lib.ds_consensus_grouped(_addr(X), P, ld, W, _i32p(perm), _i32p(off), len(off) - 1, _addr(dev_out),
                                     _addr(workspace), workspace_bytes, _stream(stream)), "ds_consensus_grouped")


def ds_group_sync_consensus_workspace_bytes(P: int, n_groups: int) -> int:
    return int(_lib.ds_group_sync_consensus_workspace_bytes(int(P), int(n_groups)))


def ds_group_sync_consensus(X, G, g_dtype: int, P: int, ldx: int, ldg: int, W: int, perm, off, lr: float,
                            dev_out, workspace, workspace_bytes: int, stream=None) -> None:
    perm, off = _i32(perm), _i32(off)
    _check(_lib.ds_group_sync_consensus(_addr(X), _addr(G), g_dtype, P, ldx, ldg, W, _i32p(perm), _i32p(off),
                                        len(off) - 1, lr, _addr(dev_out), _addr(workspace), workspace_bytes,
                                        _stream(stream)), "ds_group_sync_consensus")


def ds_tiled_elements(P: int, W: int) -> int:
    return int(_lib.ds_tiled_elements(int(P), int(W)))


def ds_group_sync_tiled(X, G, g_dtype: int, P: int, tile_stride_x: int, tile_stride_g: int, W: int, perm, off,
                        lr: float, opt: ds_local_opt | None = None, stream=None) -> None:
    perm, off = _i32(perm), _i32(off)
    _check(_lib.ds_group_sync_tiled(_addr(X), _addr(G), g_dtype, P, tile_stride_x, tile_stride_g, W, _i32p(perm),
                                    _i32p(off), len(off) - 1, lr, ctypes.byref(opt) if opt is not None else None,
                                    _stream(stream)), "ds_group_sync_tiled")


def ds_consensus_tiled(X, P: int, tile_stride: int, W: int, dev_out, workspace, workspace_bytes: int,
                       stream=None) -> None:
    _check(_lib.ds_consensus_tiled(_addr(X), P, tile_stride, W, _addr(dev_out), _addr(workspace), workspace_bytes,
                                   _stream(stream)), "ds_consensus_tiled")


def ds_consensus_grouped_tiled(X, P: int, tile_stride: int, W: int, perm, off, dev_out, workspace, workspace_bytes: int,
                               stream=None) -> None:
    perm, off = _i32(perm), _i32(off)
    _check(_lib.ds_consensus_grouped_tiled(_addr(X), P, tile_stride, W, _i32p(perm), _i32p(off), len(off) - 1,
                                           _addr(dev_out), _addr(workspace), workspace_bytes, _stream(stream)),
           "ds_consensus_grouped_tiled")


def ds_group_sync_consensus_tiled(X, G, g_dtype: int, P: int, tile_stride_x: int, tile_stride_g: int, W: int, perm,
                                  off, lr: float, dev_out, workspace, workspace_bytes: int, stream=None) -> None:
    perm, off = _i32(perm), _i32(off)
    _check(_lib.ds_group_sync_consensus_tiled(_addr(X), _addr(G), g_dtype, P, tile_stride_x, tile_stride_g, W,
                                              _i32p(perm), _i32p(off), len(off) - 1, lr, _addr(dev_out),
                                              _addr(workspace), workspace_bytes, _stream(stream)),
           "ds_group_sync_consensus_tiled")


def ds_padded_ld(P: int) -> int:
    return int(_lib.ds_padded_ld(int(P)))
