"""CPU oracle for the DS-Sync hot path -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares nothing with the GPU library:
the arithmetic lives in ``ds_oracle.c`` (plain C, fp64) and in ``mixing.py``
(dense mixing matrices, numpy fp64), and this file only marshals numpy arrays
into the C routines.

Paper passages implemented (see ``ds_oracle.c`` for the details):
Listing 1 (local optimizer step, then ``Average(model, group)``), Sec. III-A
step 4, Sec. IV-B2 (``X_{k+1} = W_k X_k``; Lemma 1's left-hand side).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ds_oracle.c")
_LIB = os.path.join(_HERE, "libds_oracle.so")


def build(force: bool = False) -> str:
    """Compile ds_oracle.c with gcc (fp contraction off, OpenMP on)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32p = ctypes.POINTER(ctypes.c_int32)
        lib.orc_mix64.restype = ctypes.c_uint64
        lib.orc_mix64.argtypes = [ctypes.c_uint64]
        lib.orc_key.restype = ctypes.c_uint64
        lib.orc_key.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
        lib.orc_partition.restype = ctypes.c_int
        lib.orc_partition.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int32, i32p,
                                      ctypes.c_int32, i32p, i32p]
        lib.orc_step.restype = ctypes.c_int
        lib.orc_step.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int64,
                                 ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                 i32p, i32p, ctypes.c_int32, ctypes.c_float]
        lib.orc_step_opt.restype = ctypes.c_int
        lib.orc_step_opt.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p,
                                     ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                     ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, i32p, i32p,
                                     ctypes.c_int32, ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                     ctypes.c_float]
        lib.orc_consensus.restype = ctypes.c_int
        lib.orc_consensus.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                      ctypes.c_int32, ctypes.c_void_p]
        lib.orc_scaled_error.restype = ctypes.c_double
        lib.orc_scaled_error.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                         ctypes.c_int64, ctypes.c_int64, ctypes.c_int32]
        lib.orc_num_threads.restype = ctypes.c_int
        lib.orc_num_threads.argtypes = []
        lib.orc_set_num_threads.restype = None
        lib.orc_set_num_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _ptr(a: np.ndarray, ctype=ctypes.c_int32):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def mix64(z: int) -> int:
    """splitmix64 finaliser."""
    return int(_load().orc_mix64(ctypes.c_uint64(z & (2**64 - 1))))


def key(seed: int, t: int) -> int:
    """Per-iteration shuffle key; a pure function of (seed, t)."""
    return int(_load().orc_key(ctypes.c_uint64(seed & (2**64 - 1)), ctypes.c_uint64(t & (2**64 - 1))))


def partition(seed: int, t: int, W: int, sizes: Sequence[int]) -> Tuple[np.ndarray, np.ndarray]:
    """Division of workers 0..W-1 into groups for iteration ``t``.

    Returns ``(perm[W], off[n_groups+1])``; group k is ``perm[off[k]:off[k+1]]``.
    """
    sz = _i32(sizes)
    perm = np.empty(max(W, 1), dtype=np.int32)
    off = np.empty(len(sz) + 1, dtype=np.int32)
    rc = _load().orc_partition(ctypes.c_uint64(seed), ctypes.c_uint64(t), W, _ptr(sz), len(sz),
                               _ptr(perm), _ptr(off))
    if rc != 0:
        raise ValueError("sizes %r do not divide %d workers" % (list(sizes), W))
    return perm[:W], off


def step(X: np.ndarray, G: np.ndarray, perm, off, lr: float,
         col0: int = 0, ncols: int | None = None) -> None:
    """One DS-Sync step in place on ``X`` (fp32 ``[W, ldx]``, C-contiguous).

    ``G`` is fp32 ``[W, ldg]`` or bf16 given as raw ``uint16`` bit patterns.
    Only columns ``col0 .. col0+ncols-1`` are touched.
    """
    if X.dtype != np.float32 or X.ndim != 2 or not X.flags.c_contiguous:
        raise TypeError("X must be a C-contiguous fp32 [W, ld] array")
    if G.ndim != 2 or not G.flags.c_contiguous or G.shape[0] != X.shape[0]:
        raise TypeError("G must be a C-contiguous [W, ld] array")
    if G.dtype == np.float32:
        is_bf16 = 0
    elif G.dtype == np.uint16:
        is_bf16 = 1
    else:
        raise TypeError("G must be float32 or uint16 (bf16 bits)")
    W, ldx = X.shape
    ldg = G.shape[1]
    if ncols is None:
        ncols = min(ldx, ldg) - col0
    if col0 < 0 or ncols < 0 or col0 + ncols > min(ldx, ldg):
        raise ValueError("column range outside the arrays")
    perm = _i32(perm)
    off = _i32(off)
    if sorted(perm.tolist()) != list(range(W)) or off[0] != 0 or off[-1] != W or np.any(np.diff(off) < 1):
        raise ValueError("not a division of the workers into non-empty groups")
    rc = _load().orc_step(X.ctypes.data, G.ctypes.data, is_bf16, col0, ncols, ldx, ldg, W,
                          _ptr(perm), _ptr(off), len(off) - 1, ctypes.c_float(lr))
    if rc != 0:
        raise MemoryError("orc_step failed")


def step_opt(X: np.ndarray, G: np.ndarray, perm, off, lr: float, V: np.ndarray | None = None,
             momentum: float = 0.0, weight_decay: float = 0.0, S: np.ndarray | None = None,
             factor: float = 0.0, col0: int = 0, ncols: int | None = None) -> None:
    """One step with momentum / weight decay on the local update (buffers ``V``,
    fp32 ``[W, ldv]``, local to each worker) and the SWA moving average ``S``
    (fp32 ``[W, lds]``) of Listing 1; in place on ``X``, ``V`` and ``S``."""
    if X.dtype != np.float32 or X.ndim != 2 or not X.flags.c_contiguous:
        raise TypeError("X must be a C-contiguous fp32 [W, ld] array")
    if G.ndim != 2 or not G.flags.c_contiguous or G.shape[0] != X.shape[0] or G.dtype not in (np.float32, np.uint16):
        raise TypeError("G must be a C-contiguous [W, ld] float32 or uint16 (bf16 bits) array")
    W, ldx = X.shape
    width = min(ldx, G.shape[1])
    for A in (V, S):
        if A is not None:
            if A.dtype != np.float32 or A.ndim != 2 or not A.flags.c_contiguous or A.shape[0] != W:
                raise TypeError("V and S must be C-contiguous fp32 [W, ld] arrays")
            width = min(width, A.shape[1])
    if ncols is None:
        ncols = width - col0
    if col0 < 0 or ncols < 0 or col0 + ncols > width:
        raise ValueError("column range outside the arrays")
    perm = _i32(perm)
    off = _i32(off)
    if sorted(perm.tolist()) != list(range(W)) or off[0] != 0 or off[-1] != W or np.any(np.diff(off) < 1):
        raise ValueError("not a division of the workers into non-empty groups")
    rc = _load().orc_step_opt(X.ctypes.data, G.ctypes.data, 1 if G.dtype == np.uint16 else 0,
                              V.ctypes.data if V is not None else None, S.ctypes.data if S is not None else None,
                              col0, ncols, ldx, G.shape[1], V.shape[1] if V is not None else 0,
                              S.shape[1] if S is not None else 0, W, _ptr(perm), _ptr(off), len(off) - 1,
                              ctypes.c_float(lr), ctypes.c_float(momentum), ctypes.c_float(weight_decay),
                              ctypes.c_float(factor))
    if rc != 0:
        raise MemoryError("orc_step_opt failed")


def consensus(X: np.ndarray, P: int | None = None) -> np.ndarray:
    """``d_i = || X[i,:P] - mean_j X[j,:P] ||_2`` for every worker i, fp64."""
    if X.dtype != np.float32 or X.ndim != 2 or not X.flags.c_contiguous:
        raise TypeError("X must be a C-contiguous fp32 [W, ld] array")
    W, ld = X.shape
    if P is None:
        P = ld
    out = np.empty(W, dtype=np.float64)
    rc = _load().orc_consensus(X.ctypes.data, P, ld, W, out.ctypes.data)
    if rc != 0:
        raise MemoryError("orc_consensus failed")
    return out


def scaled_error(got: np.ndarray, want: np.ndarray, col0: int = 0, ncols: int | None = None) -> float:
    """Yardstick of the parity tests: ``max |got - want| / max(|want|, rms(want row))`` over a
    column window of two fp32 ``[W, ld]`` blocks (the rms over that window)."""
    for A in (got, want):
        if A.dtype != np.float32 or A.ndim != 2 or not A.flags.c_contiguous:
            raise TypeError("fp32 C-contiguous [W, ld] arrays expected")
    if got.shape[0] != want.shape[0]:
        raise ValueError("row counts differ")
    width = min(got.shape[1], want.shape[1])
    if ncols is None:
        ncols = width - col0
    if col0 < 0 or ncols < 0 or col0 + ncols > width:
        raise ValueError("column range outside the arrays")
    return float(_load().orc_scaled_error(got.ctypes.data, want.ctypes.data, col0, ncols, got.shape[1],
                                          want.shape[1], got.shape[0]))


def num_threads() -> int:
    return int(_load().orc_num_threads())


def set_num_threads(n: int) -> None:
    _load().orc_set_num_threads(int(n))
