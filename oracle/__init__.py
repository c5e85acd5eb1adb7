"""CPU oracle for ASNN levels and full activation -- test infrastructure.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg
may import this package.  It never imports the GPU package, and the GPU
package never imports it.

``levels`` / ``activate`` call the plain-C implementation in
``asnn_oracle.c`` (compiled on first use with gcc); ``segment_network`` is the
paper's set-based segmentation algorithm written out in Python for small
networks.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

from .segment_network import segment_network  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "asnn_oracle.c")
_LIB = os.path.join(_HERE, "libasnn_oracle.so")
_lock = threading.Lock()
_lib = None

F64 = 0   # accumulate + sigmoid in double, round once to float on store
F32 = 1   # the same steps serially in float (sensitivity probe, not the reference)

ERRORS = {-1: "index out of range", -2: "cycle", -3: "edge into an input node",
          -4: "duplicate input id", -5: "allocation failed"}


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"asnn oracle error {code}: {ERRORS.get(code, '?')}")
        self.code = code


def build(force: bool = False) -> str:
    """Compile asnn_oracle.c into a shared library next to it (gcc -O2, no
    fast-math, no contraction)."""
    with _lock:
        stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
        if force or stale:
            tmp = _LIB + f".tmp{os.getpid()}"
            subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
                                   "-Wall", "-o", tmp, _SRC, "-lm"])
            os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i32p = ctypes.POINTER(ctypes.c_int32)
        f32p = ctypes.POINTER(ctypes.c_float)
        lib.asnn_oracle_levels.restype = ctypes.c_int
        lib.asnn_oracle_levels.argtypes = [ctypes.c_int32, ctypes.c_int64, i32p, i32p, i32p, i32p]
        lib.asnn_oracle_activate.restype = ctypes.c_int
        lib.asnn_oracle_activate.argtypes = [ctypes.c_int32, ctypes.c_int64, i32p, i32p, f32p,
                                             ctypes.c_int32, i32p, f32p, ctypes.c_int32,
                                             ctypes.c_int, ctypes.c_int, f32p, ctypes.POINTER(ctypes.c_double)]
        lib.asnn_oracle_required.restype = ctypes.c_int
        lib.asnn_oracle_required.argtypes = [ctypes.c_int32, ctypes.c_int64, i32p, i32p, ctypes.c_int32, i32p, i32p]
        _lib = lib
    return _lib


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def levels(n_nodes, src, dst):
    """-> (level[int32 N], n_levels).  Raises OracleError on a cycle / bad id."""
    lib = _load()
    src, dst = _i32(src), _i32(dst)
    assert src.shape == dst.shape and src.ndim == 1
    level = np.zeros(max(n_nodes, 1), dtype=np.int32)
    nl = ctypes.c_int32(0)
    rc = lib.asnn_oracle_levels(n_nodes, src.shape[0], _p(src, ctypes.c_int32), _p(dst, ctypes.c_int32),
                                _p(level, ctypes.c_int32), ctypes.byref(nl))
    if rc:
        raise OracleError(rc)
    return level[:n_nodes], int(nl.value)


def activate(n_nodes, src, dst, w, input_ids, X, mode=F64, raw_inputs=False, timing=None):
    """-> val[float32 N, B] in ORIGINAL node ids: every node's activation.
    timing: optional dict; receives {"activation_seconds": wall time of the node loop without the adjacency build}."""
    lib = _load()
    src, dst, w, input_ids = _i32(src), _i32(dst), _f32(w), _i32(input_ids)
    X = _f32(X)
    if X.ndim == 1:
        X = X.reshape(-1, 1)
    assert X.shape[0] == input_ids.shape[0]
    B = X.shape[1]
    val = np.full((max(n_nodes, 1), max(B, 1)), np.nan, dtype=np.float32)
    seconds = ctypes.c_double(0.0)
    rc = lib.asnn_oracle_activate(n_nodes, src.shape[0], _p(src, ctypes.c_int32), _p(dst, ctypes.c_int32),
                                  _p(w, ctypes.c_float), input_ids.shape[0], _p(input_ids, ctypes.c_int32),
                                  _p(X, ctypes.c_float), B, int(mode), int(bool(raw_inputs)),
                                  _p(val, ctypes.c_float), ctypes.byref(seconds))
    if timing is not None:
        timing["activation_seconds"] = float(seconds.value)
    if rc:
        raise OracleError(rc)
    return val[:n_nodes, :B]


def required(n_nodes, src, dst, output_ids):
    """-> bool[N]: the segmentation algorithm's set R (nodes from which an output is reachable, outputs included)."""
    lib = _load()
    src, dst, output_ids = _i32(src), _i32(dst), _i32(output_ids)
    mask = np.zeros(max(n_nodes, 1), dtype=np.int32)
    rc = lib.asnn_oracle_required(n_nodes, src.shape[0], _p(src, ctypes.c_int32), _p(dst, ctypes.c_int32),
                                  output_ids.shape[0], _p(output_ids, ctypes.c_int32), _p(mask, ctypes.c_int32))
    if rc:
        raise OracleError(rc)
    return mask[:n_nodes].astype(bool)
