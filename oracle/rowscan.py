"""ctypes front end of oracle/rowscan.c -- TEST INFRASTRUCTURE, not product code.

Builds liborc_rowscan.so with gcc (-O2 -fopenmp) on demand and exposes the
row-sampled oracle: neighbour lists and degrees by scanning the mask predicate
over every key, and masked attention (two-pass softmax, float64) for sampled
query rows.  Nothing here touches the GPU or the HIP library.
"""
import ctypes
import os
import subprocess

import numpy as np

from sga_inputs.masks import MaskSpec

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rowscan.c")
_LIB = os.path.join(_HERE, "liborc_rowscan.so")
_lib = None


class _OrcMask(ctypes.Structure):
    _fields_ = [
        ("kind", ctypes.c_int32), ("window", ctypes.c_int32),
        ("stride", ctypes.c_int32), ("n_global", ctypes.c_int32),
        ("block", ctypes.c_int32), ("window_blocks", ctypes.c_int32),
        ("n_global_blocks", ctypes.c_int32), ("n_random_blocks", ctypes.c_int32),
        ("L", ctypes.c_int64), ("seed", ctypes.c_uint64),
    ]


def build(force=False):
    """Compile the C oracle (gcc, OpenMP)."""
    if force or not os.path.exists(_LIB) or \
            os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-std=c11", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        P = ctypes.POINTER
        lib.orc_row_neighbors.restype = ctypes.c_int64
        lib.orc_row_neighbors.argtypes = [P(_OrcMask), ctypes.c_int64,
                                          ctypes.c_void_p, ctypes.c_int64]
        lib.orc_degrees.restype = None
        lib.orc_degrees.argtypes = [P(_OrcMask), ctypes.c_void_p, ctypes.c_int64,
                                    ctypes.c_void_p]
        lib.orc_count_edges.restype = ctypes.c_int64
        lib.orc_count_edges.argtypes = [P(_OrcMask)]
        lib.orc_attend_gathered.restype = None
        lib.orc_attend_gathered.argtypes = [ctypes.c_void_p, ctypes.c_void_p,
                                            ctypes.c_void_p, ctypes.c_int64,
                                            ctypes.c_int32, ctypes.c_double,
                                            ctypes.c_void_p, ctypes.c_void_p]
        lib.orc_attend_rows.restype = ctypes.c_int64
        lib.orc_attend_rows.argtypes = [P(_OrcMask), ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_void_p, ctypes.c_int32,
                                        ctypes.c_double, ctypes.c_void_p,
                                        ctypes.c_int64, ctypes.c_void_p,
                                        ctypes.c_void_p]
        lib.orc_num_threads.restype = ctypes.c_int
        lib.orc_num_threads.argtypes = []
        _lib = lib
    return _lib


def _mk(spec: MaskSpec) -> _OrcMask:
    if spec.kind == 3 and spec.L % spec.block != 0:
        raise ValueError("block mask needs L divisible by the block size")
    return _OrcMask(spec.kind, spec.window, spec.stride, spec.n_global, spec.block,
                    spec.window_blocks, spec.n_global_blocks, spec.n_random_blocks,
                    spec.L, spec.seed & ((1 << 64) - 1))


def num_threads() -> int:
    return int(_load().orc_num_threads())


def row_neighbors(spec: MaskSpec, i: int) -> np.ndarray:
    lib = _load()
    mk = _mk(spec)
    n = lib.orc_row_neighbors(ctypes.byref(mk), i, None, 0)
    out = np.empty(max(n, 1), dtype=np.int64)
    lib.orc_row_neighbors(ctypes.byref(mk), i, out.ctypes.data, n)
    return out[:n]


def degrees(spec: MaskSpec, rows) -> np.ndarray:
    lib = _load()
    mk = _mk(spec)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    deg = np.empty(len(rows), dtype=np.int64)
    lib.orc_degrees(ctypes.byref(mk), rows.ctypes.data, len(rows), deg.ctypes.data)
    return deg


def count_edges(spec: MaskSpec) -> int:
    mk = _mk(spec)
    return int(_load().orc_count_edges(ctypes.byref(mk)))


def attend_gathered(q, Kg, Vg, scale):
    """q [d], Kg/Vg [n, d] -> (O [d] float64, lse float)."""
    lib = _load()
    q = np.ascontiguousarray(q, dtype=np.float32)
    Kg = np.ascontiguousarray(Kg, dtype=np.float32)
    Vg = np.ascontiguousarray(Vg, dtype=np.float32)
    n, d = Kg.shape if Kg.ndim == 2 else (0, len(q))
    out = np.empty(d, dtype=np.float64)
    lse = np.empty(1, dtype=np.float64)
    lib.orc_attend_gathered(q.ctypes.data, Kg.ctypes.data, Vg.ctypes.data, n, d,
                            float(scale), out.ctypes.data, lse.ctypes.data)
    return out, float(lse[0])


def attend_rows(spec: MaskSpec, Q, K, V, scale, rows):
    """One head, whole Q/K/V [L, d] on the host (any float dtype; widened to
    fp32 exactly).  Returns (O [n, d] float64, lse [n] float64, edges)."""
    lib = _load()
    mk = _mk(spec)
    Q = np.ascontiguousarray(Q, dtype=np.float32)
    K = np.ascontiguousarray(K, dtype=np.float32)
    V = np.ascontiguousarray(V, dtype=np.float32)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    d = Q.shape[1]
    out = np.empty((len(rows), d), dtype=np.float64)
    lse = np.empty(len(rows), dtype=np.float64)
    edges = lib.orc_attend_rows(ctypes.byref(mk), Q.ctypes.data, K.ctypes.data,
                                V.ctypes.data, d, float(scale), rows.ctypes.data,
                                len(rows), out.ctypes.data, lse.ctypes.data)
    return out, lse, int(edges)
