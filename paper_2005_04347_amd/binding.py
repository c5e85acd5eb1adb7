"""ctypes binding for libasnn (see include/asnn.h).

Argument marshalling only: torch tensors provide device memory and the
current stream; every step of the path runs inside the library's HIP kernels.
There is no CPU fallback: loading fails loudly when libasnn.so is missing.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libasnn.so")

FLAG_RAW_INPUTS = 1
FLAG_ACC_F32 = 2
FLAG_LEVEL_LAUNCHES = 4
FLAG_DATAFLOW = 8
FLAG_WORKGROUP = 16
HEAVY_INDEGREE = 256
MEDIUM_INDEGREE = 32
CLASSES = 3

ERR_NAMES = {
    -1: "ASNN_ERR_NULL", -2: "ASNN_ERR_SIZE", -3: "ASNN_ERR_INDEX", -4: "ASNN_ERR_INPUT_HAS_INEDGE",
    -5: "ASNN_ERR_DUP_INPUT", -6: "ASNN_ERR_CYCLE", -7: "ASNN_ERR_WORKSPACE", -8: "ASNN_ERR_HIP",
    -9: "ASNN_ERR_LEVEL_ORDER", -10: "ASNN_ERR_NO_DEVICE", -11: "ASNN_ERR_TIMEOUT", -12: "ASNN_ERR_SCRATCH",
}
STATIC_SCRATCH_BYTES = 32 << 20
STATIC_SCRATCH = 1          # ASNN_STATIC_SCRATCH: names the library's own scratch in asnn_activate_status

EXPORTS = [
    "asnn_strerror", "asnn_last_hip_error", "asnn_version",
    "asnn_levels_workspace_bytes", "asnn_build_levels",
    "asnn_required_workspace_bytes", "asnn_required_set", "asnn_filter_workspace_bytes", "asnn_filter_required",
    "asnn_compact_workspace_bytes", "asnn_compact_required", "asnn_relabel_ids",
    "asnn_pack_workspace_bytes", "asnn_pack_csr", "asnn_activate_workspace_bytes", "asnn_activate",
    "asnn_activate_status", "asnn_activate_schedule", "asnn_activate_static", "asnn_device_copy",
    "asnn_device_read", "asnn_device_gather", "asnn_device_gather_store",
]


class AsnnError(RuntimeError):
    def __init__(self, code: int, where: str):
        lib = load()
        msg = lib.asnn_strerror(code).decode()
        extra = f" (hipError {lib.asnn_last_hip_error()})" if code == -8 else ""
        super().__init__(f"{where}: {ERR_NAMES.get(code, code)}: {msg}{extra}")
        self.code = code


_lib = None


def load() -> ctypes.CDLL:
    """Loads libasnn.so built in-tree (python -m paper_2005_04347_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} not found: build it with `python -m paper_2005_04347_amd.build` "
                          "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, u32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32, ctypes.c_size_t
    lib.asnn_strerror.restype = ctypes.c_char_p
    lib.asnn_strerror.argtypes = [ctypes.c_int]
    lib.asnn_last_hip_error.restype = ctypes.c_int
    lib.asnn_last_hip_error.argtypes = []
    lib.asnn_version.restype = ctypes.c_int
    lib.asnn_version.argtypes = []
    lib.asnn_levels_workspace_bytes.restype = sz
    lib.asnn_levels_workspace_bytes.argtypes = [i32, i64]
    lib.asnn_build_levels.restype = ctypes.c_int
    lib.asnn_build_levels.argtypes = [i32, i64, vp, vp, vp, i32, vp, ctypes.POINTER(i32), vp, sz, vp]
    lib.asnn_required_workspace_bytes.restype = sz
    lib.asnn_required_workspace_bytes.argtypes = [i32, i64]
    lib.asnn_required_set.restype = ctypes.c_int
    lib.asnn_required_set.argtypes = [i32, i64, vp, vp, vp, i32, vp, ctypes.POINTER(i32), vp, sz, vp]
    lib.asnn_filter_workspace_bytes.restype = sz
    lib.asnn_filter_workspace_bytes.argtypes = [i64]
    lib.asnn_filter_required.restype = ctypes.c_int
    lib.asnn_filter_required.argtypes = [i32, i64, vp, vp, vp, vp, vp, vp, vp, ctypes.POINTER(i64), vp, sz, vp]
    lib.asnn_compact_workspace_bytes.restype = sz
    lib.asnn_compact_workspace_bytes.argtypes = [i32]
    lib.asnn_compact_required.restype = ctypes.c_int
    lib.asnn_compact_required.argtypes = [i32, vp, vp, ctypes.POINTER(i32), vp, sz, vp]
    lib.asnn_relabel_ids.restype = ctypes.c_int
    lib.asnn_relabel_ids.argtypes = [vp, i64, vp, i32, vp, vp]
    lib.asnn_pack_workspace_bytes.restype = sz
    lib.asnn_pack_workspace_bytes.argtypes = [i32, i64]
    lib.asnn_pack_csr.restype = ctypes.c_int
    lib.asnn_pack_csr.argtypes = [vp, vp, vp, vp, ctypes.POINTER(AsnnPacked), vp, sz, vp]
    lib.asnn_activate_workspace_bytes.restype = sz
    lib.asnn_activate_workspace_bytes.argtypes = [ctypes.POINTER(AsnnPacked), i32]
    lib.asnn_activate.restype = ctypes.c_int
    lib.asnn_activate.argtypes = [ctypes.POINTER(AsnnPacked), vp, i32, vp, i32, vp, i32, vp, vp, vp, sz, u32, vp]
    lib.asnn_activate_static.restype = ctypes.c_int
    lib.asnn_activate_static.argtypes = [ctypes.POINTER(AsnnPacked), vp, i32, vp, i32, vp, i32, vp, vp, u32, vp]
    lib.asnn_activate_schedule.restype = ctypes.c_int
    lib.asnn_activate_schedule.argtypes = [ctypes.POINTER(AsnnPacked), i32, ctypes.c_int, u32]
    lib.asnn_activate_status.restype = ctypes.c_int
    lib.asnn_activate_status.argtypes = [vp, vp]
    lib.asnn_device_copy.restype = ctypes.c_int
    lib.asnn_device_copy.argtypes = [vp, vp, sz, vp]
    lib.asnn_device_read.restype = ctypes.c_int
    lib.asnn_device_read.argtypes = [vp, sz, vp, vp]
    lib.asnn_device_gather.restype = ctypes.c_int
    lib.asnn_device_gather.argtypes = [vp, i32, i32, i32, i32, u32, vp, vp]
    lib.asnn_device_gather_store.restype = ctypes.c_int
    lib.asnn_device_gather_store.argtypes = [vp, i32, i32, i32, i32, u32, vp, vp]
    _lib = lib
    return lib


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None or t.numel() == 0 else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev_i32(a, device):
    if isinstance(a, torch.Tensor):
        return a.to(device=device, dtype=torch.int32).contiguous()
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(device)


def _dev_f32(a, device):
    if isinstance(a, torch.Tensor):
        return a.to(device=device, dtype=torch.float32).contiguous()
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)


def _workspace(nbytes: int, device):
    # torch's caching allocator returns 512-byte aligned blocks
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def asnn_build_levels(n_nodes: int, src: torch.Tensor, dst: torch.Tensor, input_ids: torch.Tensor):
    """-> (level: int32 device tensor [n_nodes], n_levels: int)."""
    lib = load()
    device = src.device
    n_edges = int(src.numel())
    level = torch.empty(max(n_nodes, 1), dtype=torch.int32, device=device)
    nbytes = lib.asnn_levels_workspace_bytes(n_nodes, n_edges)
    ws = _workspace(nbytes, device)
    n_levels = ctypes.c_int32(-1)
    rc = lib.asnn_build_levels(n_nodes, n_edges, _ptr(src), _ptr(dst), _ptr(input_ids), int(input_ids.numel()),
                               ctypes.c_void_p(level.data_ptr()), ctypes.byref(n_levels),
                               ctypes.c_void_p(ws.data_ptr()), ws.numel(), _stream())
    if rc != 0:
        raise AsnnError(rc, "asnn_build_levels")
    return level[:n_nodes], int(n_levels.value)


def asnn_required_set(n_nodes: int, src: torch.Tensor, dst: torch.Tensor, output_ids: torch.Tensor):
    """-> (required: int32 device tensor [n_nodes] of 0/1, n_required: int)."""
    lib = load()
    device = src.device
    n_edges = int(src.numel())
    required = torch.empty(max(n_nodes, 1), dtype=torch.int32, device=device)
    ws = _workspace(lib.asnn_required_workspace_bytes(n_nodes, n_edges), device)
    count = ctypes.c_int32(-1)
    rc = lib.asnn_required_set(n_nodes, n_edges, _ptr(src), _ptr(dst), _ptr(output_ids), int(output_ids.numel()),
                               ctypes.c_void_p(required.data_ptr()), ctypes.byref(count),
                               ctypes.c_void_p(ws.data_ptr()), ws.numel(), _stream())
    if rc != 0:
        raise AsnnError(rc, "asnn_required_set")
    return required[:n_nodes], int(count.value)


def asnn_filter_required(n_nodes: int, src, dst, w, required):
    """-> (src, dst, w) of the connections that end in a required node, order kept."""
    lib = load()
    device = src.device
    n_edges = int(src.numel())
    so = torch.empty(max(n_edges, 1), dtype=torch.int32, device=device)
    do = torch.empty(max(n_edges, 1), dtype=torch.int32, device=device)
    wo = torch.empty(max(n_edges, 1), dtype=torch.float32, device=device)
    ws = _workspace(lib.asnn_filter_workspace_bytes(n_edges), device)
    kept = ctypes.c_int64(-1)
    rc = lib.asnn_filter_required(n_nodes, n_edges, _ptr(src), _ptr(dst), _ptr(w), _ptr(required),
                                  ctypes.c_void_p(so.data_ptr()), ctypes.c_void_p(do.data_ptr()),
                                  ctypes.c_void_p(wo.data_ptr()), ctypes.byref(kept),
                                  ctypes.c_void_p(ws.data_ptr()), ws.numel(), _stream())
    if rc != 0:
        raise AsnnError(rc, "asnn_filter_required")
    k = int(kept.value)
    return so[:k], do[:k], wo[:k]


def asnn_compact_required(n_nodes: int, required: torch.Tensor):
    """-> (new_id: int32 device tensor [n_nodes], dense id of every node of R or -1; n_required: int)."""
    lib = load()
    device = required.device
    new_id = torch.empty(max(n_nodes, 1), dtype=torch.int32, device=device)
    ws = _workspace(lib.asnn_compact_workspace_bytes(n_nodes), device)
    count = ctypes.c_int32(-1)
    rc = lib.asnn_compact_required(n_nodes, _ptr(required), ctypes.c_void_p(new_id.data_ptr()), ctypes.byref(count),
                                   ctypes.c_void_p(ws.data_ptr()), ws.numel(), _stream())
    if rc != 0:
        raise AsnnError(rc, "asnn_compact_required")
    return new_id[:n_nodes], int(count.value)


def asnn_relabel_ids(ids: torch.Tensor, new_id: torch.Tensor) -> torch.Tensor:
    """ids carried over to the numbering new_id (from asnn_compact_required); -1 where an id is outside R."""
    lib = load()
    out = torch.empty_like(ids)
    rc = lib.asnn_relabel_ids(_ptr(ids), int(ids.numel()), _ptr(new_id), int(new_id.numel()), _ptr(out), _stream())
    if rc != 0:
        raise AsnnError(rc, "asnn_relabel_ids")
    return out


class AsnnPacked(ctypes.Structure):
    """Mirror of `asnn_packed` in include/asnn.h."""
    _fields_ = [
        ("n_nodes", ctypes.c_int32), ("n_levels", ctypes.c_int32), ("n_edges", ctypes.c_int64),
        ("n_units", ctypes.c_int32), ("first_unit", ctypes.c_int32),
        ("max_heavy_indegree", ctypes.c_int32), ("reserved", ctypes.c_int32),
        ("level_ptr_host", ctypes.c_void_p), ("level_ptr", ctypes.c_void_p), ("perm", ctypes.c_void_p),
        ("inv_perm", ctypes.c_void_p), ("row_ptr", ctypes.c_void_p), ("col", ctypes.c_void_p),
        ("w", ctypes.c_void_p), ("unit_ptr", ctypes.c_void_p),
    ]


@dataclass
class PackedGraph:
    n_nodes: int
    n_edges: int
    n_levels: int
    level_ptr: torch.Tensor          # device int32 [3*n_levels+1]
    level_ptr_host: np.ndarray       # host int32 [3*n_levels+1]
    perm: torch.Tensor               # device int32 [n_nodes]  packed row -> original id
    inv_perm: torch.Tensor           # device int32 [n_nodes]  original id -> packed row
    row_ptr: torch.Tensor            # device int32 [n_nodes+1]
    col: torch.Tensor                # device int32 [n_edges]
    w: torch.Tensor                  # device float32 [n_edges]
    unit_ptr: torch.Tensor           # device int32 [n_nodes + n_edges//512 + 2], n_units+1 entries used
    n_units: int = 0
    first_unit: int = 0
    record: Optional[AsnnPacked] = None   # the C record (points into the tensors above)


def asnn_pack_csr(n_nodes: int, n_levels: int, src, dst, w, level) -> PackedGraph:
    lib = load()
    device = src.device
    n_edges = int(src.numel())
    nk = CLASSES * n_levels + 1
    level_ptr = torch.empty(nk, dtype=torch.int32, device=device)
    level_ptr_host = np.zeros(nk, dtype=np.int32)
    perm = torch.empty(n_nodes, dtype=torch.int32, device=device)
    inv_perm = torch.empty(n_nodes, dtype=torch.int32, device=device)
    row_ptr = torch.empty(n_nodes + 1, dtype=torch.int32, device=device)
    col = torch.empty(max(n_edges, 1), dtype=torch.int32, device=device)
    wp = torch.empty(max(n_edges, 1), dtype=torch.float32, device=device)
    unit_ptr = torch.empty(n_nodes + n_edges // 512 + 2, dtype=torch.int32, device=device)
    ws = _workspace(lib.asnn_pack_workspace_bytes(n_nodes, n_edges), device)
    rec = AsnnPacked(n_nodes=n_nodes, n_levels=n_levels, n_edges=n_edges, n_units=0, first_unit=0,
                     level_ptr_host=level_ptr_host.ctypes.data, level_ptr=level_ptr.data_ptr(), perm=perm.data_ptr(),
                     inv_perm=inv_perm.data_ptr(), row_ptr=row_ptr.data_ptr(), col=col.data_ptr(), w=wp.data_ptr(),
                     unit_ptr=unit_ptr.data_ptr())
    rc = lib.asnn_pack_csr(_ptr(src), _ptr(dst), _ptr(w), _ptr(level), ctypes.byref(rec),
                           ctypes.c_void_p(ws.data_ptr()), ws.numel(), _stream())
    if rc != 0:
        raise AsnnError(rc, "asnn_pack_csr")
    return PackedGraph(n_nodes, n_edges, n_levels, level_ptr, level_ptr_host, perm, inv_perm, row_ptr,
                       col[:n_edges], wp[:n_edges], unit_ptr, int(rec.n_units), int(rec.first_unit), rec)


def asnn_activate_workspace(g: PackedGraph, B: int, device) -> torch.Tensor:
    """Device scratch for the dataflow schedule of asnn_activate (contents need not be preserved)."""
    lib = load()
    return _workspace(lib.asnn_activate_workspace_bytes(ctypes.byref(g.record), B), device)


def asnn_activate(g: PackedGraph, input_ids: torch.Tensor, X: torch.Tensor,
                  output_ids: Optional[torch.Tensor] = None, V: Optional[torch.Tensor] = None,
                  Y: Optional[torch.Tensor] = None, flags: int = 0, workspace: Optional[torch.Tensor] = None):
    """Enqueues one full activation on the current stream.
    X: float32 [n_inputs, B].  Returns (V [n_nodes, B] in packed row order, Y [n_outputs, B] or None)."""
    lib = load()
    assert X.dim() == 2 and X.dtype == torch.float32 and X.is_contiguous()
    B = int(X.shape[1])
    n_in = int(input_ids.numel())
    assert X.shape[0] == n_in
    device = X.device
    if V is None:
        V = torch.empty((g.n_nodes, B), dtype=torch.float32, device=device)
    assert V.shape == (g.n_nodes, B) and V.is_contiguous() and V.dtype == torch.float32
    n_out = 0 if output_ids is None else int(output_ids.numel())
    if output_ids is not None and Y is None:
        Y = torch.empty((n_out, B), dtype=torch.float32, device=device)
    ws_ptr = None if workspace is None else ctypes.c_void_p(workspace.data_ptr())
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib.asnn_activate(ctypes.byref(g.record), _ptr(input_ids), n_in, _ptr(output_ids), n_out, _ptr(X), B,
                           ctypes.c_void_p(V.data_ptr()), _ptr(Y), ws_ptr, ws_bytes, flags, _stream())
    if rc != 0:
        raise AsnnError(rc, "asnn_activate")
    return V, Y


class BoundActivation:
    """One asnn_activate call with every argument marshalled once: launch() only makes the foreign
    call.  For loops that activate the same network on the same buffers again and again (one input
    vector per activation: there the marshalling of thirteen arguments and the look-up of the
    current stream cost more than the kernel).  The stream is the one that was current when the
    object was made; X, V, Y and the workspace are kept alive by it."""

    def __init__(self, g: PackedGraph, input_ids, X, output_ids, V, Y, flags, workspace):
        lib = load()
        assert X.dim() == 2 and X.dtype == torch.float32 and X.is_contiguous()
        B = int(X.shape[1])
        n_in = int(input_ids.numel())
        assert X.shape[0] == n_in
        assert V.shape == (g.n_nodes, B) and V.is_contiguous() and V.dtype == torch.float32
        n_out = 0 if output_ids is None else int(output_ids.numel())
        assert n_out == 0 or (Y is not None and Y.shape == (n_out, B) and Y.is_contiguous())
        self._keep = (g, input_ids, X, output_ids, V, Y, workspace)
        self._fn = lib.asnn_activate
        self._args = (ctypes.byref(g.record), _ptr(input_ids), ctypes.c_int32(n_in), _ptr(output_ids), ctypes.c_int32(n_out),
                      _ptr(X), ctypes.c_int32(B), ctypes.c_void_p(V.data_ptr()), _ptr(Y),
                      None if workspace is None else ctypes.c_void_p(workspace.data_ptr()),
                      ctypes.c_size_t(0 if workspace is None else workspace.numel() * workspace.element_size()),
                      ctypes.c_uint32(flags), _stream())
        self.V, self.Y = V, Y

    def launch(self) -> None:
        rc = self._fn(*self._args)
        if rc != 0:
            raise AsnnError(rc, "asnn_activate")


def asnn_activate_static(g: PackedGraph, input_ids: torch.Tensor, X: torch.Tensor, V: torch.Tensor,
                         output_ids: Optional[torch.Tensor] = None, Y: Optional[torch.Tensor] = None, flags: int = 0):
    """asnn_activate with the library's own scratch in the place of a workspace.  The binding allocates
    nothing either: the caller brings V (and Y when output_ids is given).  Returns (V, Y)."""
    lib = load()
    assert X.dim() == 2 and X.dtype == torch.float32 and X.is_contiguous()
    B = int(X.shape[1])
    n_in = int(input_ids.numel())
    assert X.shape[0] == n_in
    assert V.shape == (g.n_nodes, B) and V.is_contiguous() and V.dtype == torch.float32
    n_out = 0 if output_ids is None else int(output_ids.numel())
    assert n_out == 0 or (Y is not None and Y.shape == (n_out, B) and Y.is_contiguous() and Y.dtype == torch.float32)
    rc = lib.asnn_activate_static(ctypes.byref(g.record), _ptr(input_ids), n_in, _ptr(output_ids), n_out, _ptr(X), B,
                                  ctypes.c_void_p(V.data_ptr()), _ptr(Y), flags, _stream())
    if rc != 0:
        raise AsnnError(rc, "asnn_activate_static")
    return V, Y


def asnn_activate_schedule(g: PackedGraph, B: int, has_workspace: bool = True, flags: int = 0) -> str:
    """'levels', 'dataflow' or 'workgroup': the schedule asnn_activate would take."""
    lib = load()
    rc = lib.asnn_activate_schedule(ctypes.byref(g.record), B, int(has_workspace), flags)
    if rc < 0:
        raise AsnnError(rc, "asnn_activate_schedule")
    return ("levels", "dataflow", "workgroup")[rc]


def asnn_activate_status(workspace: Optional[torch.Tensor]) -> None:
    """Synchronises the current stream; raises if a dataflow wait of the last activation gave up."""
    lib = load()
    if isinstance(workspace, int):       # STATIC_SCRATCH
        ws = ctypes.c_void_p(workspace)
    else:
        ws = None if workspace is None else ctypes.c_void_p(workspace.data_ptr())
    rc = lib.asnn_activate_status(ws, _stream())
    if rc != 0:
        raise AsnnError(rc, "asnn_activate_status")


def asnn_device_copy(dst: torch.Tensor, src: torch.Tensor):
    """Streaming copy src -> dst on the current stream (bandwidth yardstick)."""
    lib = load()
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    rc = lib.asnn_device_copy(ctypes.c_void_p(dst.data_ptr()), ctypes.c_void_p(src.data_ptr()), nbytes, _stream())
    if rc != 0:
        raise AsnnError(rc, "asnn_device_copy")


def asnn_device_read(src: torch.Tensor, sink: torch.Tensor):
    """Streaming read of src on the current stream (bandwidth yardstick); sink: a device float."""
    lib = load()
    rc = lib.asnn_device_read(ctypes.c_void_p(src.data_ptr()), src.numel() * src.element_size(),
                              ctypes.c_void_p(sink.data_ptr()), _stream())
    if rc != 0:
        raise AsnnError(rc, "asnn_device_read")


def asnn_device_gather(buf: torch.Tensor, rows_per_launch: int, gathers: int, seed: int, sink: torch.Tensor):
    """Random row gather over the float32 matrix buf in the launch shape of one level (bandwidth yardstick)."""
    lib = load()
    assert buf.dim() == 2 and buf.dtype == torch.float32 and buf.is_contiguous()
    rc = lib.asnn_device_gather(ctypes.c_void_p(buf.data_ptr()), int(buf.shape[0]), int(buf.shape[1]), rows_per_launch,
                                gathers, seed, ctypes.c_void_p(sink.data_ptr()), _stream())
    if rc != 0:
        raise AsnnError(rc, "asnn_device_gather")


def asnn_device_gather_store(buf: torch.Tensor, gathers: int, seed: int, out: torch.Tensor):
    """The same gather, every wavefront storing its tile of one row of out (out.shape[0] rows per launch)."""
    lib = load()
    assert buf.dim() == 2 and buf.dtype == torch.float32 and buf.is_contiguous()
    assert out.dim() == 2 and out.dtype == torch.float32 and out.is_contiguous() and out.shape[1] == buf.shape[1]
    rc = lib.asnn_device_gather_store(ctypes.c_void_p(buf.data_ptr()), int(buf.shape[0]), int(buf.shape[1]),
                                      int(out.shape[0]), gathers, seed, ctypes.c_void_p(out.data_ptr()), _stream())
    if rc != 0:
        raise AsnnError(rc, "asnn_device_gather_store")


class Network:
    """Convenience wrapper: build levels + pack once, activate many times."""

    def __init__(self, n_nodes, src, dst, w, input_ids, output_ids, device="cuda:0", required_only=False, compact=False):
        """required_only: drop the connections no output depends on (same rows of V, bit-identical on R).
        compact: also drop the nodes no output depends on: the network is renumbered (self.new_id), V has
        |R| rows and nothing outside R is allocated or written."""
        self.device = torch.device(device)
        self.n_nodes = int(n_nodes)
        self.src = _dev_i32(src, self.device)
        self.dst = _dev_i32(dst, self.device)
        self.w_edges = _dev_f32(w, self.device)
        self.input_ids = _dev_i32(input_ids, self.device)
        self.output_ids = _dev_i32(output_ids, self.device)
        self.required = None
        self.new_id = None           # compact=True: original id -> id in the compacted network, -1 outside R
        with torch.cuda.device(self.device):
            if required_only or compact:       # keep only the connections the outputs depend on
                self.required, self.n_required = asnn_required_set(self.n_nodes, self.src, self.dst, self.output_ids)
                self.src, self.dst, self.w_edges = asnn_filter_required(self.n_nodes, self.src, self.dst, self.w_edges,
                                                                        self.required)
            if compact:                        # and number the required nodes densely: V has |R| rows
                self.new_id, count = asnn_compact_required(self.n_nodes, self.required)
                self.src = asnn_relabel_ids(self.src, self.new_id)
                self.dst = asnn_relabel_ids(self.dst, self.new_id)
                self.input_ids = asnn_relabel_ids(self.input_ids, self.new_id)     # -1: a sensor no output depends on (skipped)
                self.output_ids = asnn_relabel_ids(self.output_ids, self.new_id)
                self.n_nodes_original, self.n_nodes = self.n_nodes, count
                self.sensor_ids = self.input_ids[self.input_ids >= 0]              # what the level builder may be told
            self.level, self.n_levels = asnn_build_levels(self.n_nodes, self.src, self.dst,
                                                          self.sensor_ids if compact else self.input_ids)
            self.graph = asnn_pack_csr(self.n_nodes, self.n_levels, self.src, self.dst, self.w_edges, self.level)

        self._workspaces = {}

    def workspace(self, B: int) -> torch.Tensor:
        if B not in self._workspaces:
            self._workspaces[B] = asnn_activate_workspace(self.graph, B, self.device)
        return self._workspaces[B]

    def activate(self, X, V=None, Y=None, flags: int = 0, use_workspace: bool = True, check: bool = False):
        """check=True synchronises after the call and raises if a dataflow wait gave up (see
        asnn_activate_status): for callers that share the device with other processes."""
        X = _dev_f32(X, self.device)
        with torch.cuda.device(self.device):
            ws = self.workspace(int(X.shape[1])) if use_workspace else None
            out = asnn_activate(self.graph, self.input_ids, X, self.output_ids, V=V, Y=Y, flags=flags, workspace=ws)
            if check:
                asnn_activate_status(ws)
            return out

    def bind(self, X: torch.Tensor, V: Optional[torch.Tensor] = None, Y: Optional[torch.Tensor] = None,
             flags: int = 0, use_workspace: bool = True) -> BoundActivation:
        """Marshals one activation of this network once; the returned object's launch() enqueues it on the
        stream that is current now, reading X and writing V and Y in place every time."""
        assert X.is_cuda or X.is_pinned()
        B = int(X.shape[1])
        with torch.cuda.device(self.device):
            if V is None:
                V = torch.empty((self.n_nodes, B), dtype=torch.float32, device=self.device)
            if Y is None:
                Y = torch.empty((int(self.output_ids.numel()), B), dtype=torch.float32, device=self.device)
            ws = self.workspace(B) if use_workspace else None
            return BoundActivation(self.graph, self.input_ids, X, self.output_ids, V, Y, flags, ws)

    def check(self, B: int) -> None:
        """Synchronises and raises if the last dataflow activation at batch B timed out."""
        with torch.cuda.device(self.device):
            asnn_activate_status(self._workspaces.get(B))

    def values_original_order(self, V: torch.Tensor) -> torch.Tensor:
        """V (packed rows) -> [n_nodes, B] indexed by original node id (plain torch indexing, for tests)."""
        return V[self.graph.inv_perm.long()]
