"""ctypes binding of libgnnagg.so: argument marshalling only.

Each function mirrors the C entry point of the same name in ``include/gnnagg.h``
and takes torch tensors that already live on the GPU.  Output tensors and
workspaces are allocated here with torch (device memory is all torch is used
for); no arithmetic of the method happens in Python.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

SUM, WSUM, MEAN, MAX, SUM_SCALED = 0, 1, 2, 3, 4
F32, BF16 = 0, 1
SELF_LOOPS, NORM_SYM = 1, 2
PLAN_CLASSES = 33
F_CHUNK_AUTO = -1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libgnnagg.so")
_lib = None


class GnnaggError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__("%s failed: %d (%s)" % (fn, status, gnnagg_strerror(status)))


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libgnnagg.so built in-tree; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                "%s is missing: build it with `python -m paper_2104_03058_amd.build`" % _LIB_PATH)
        lib = ctypes.CDLL(_LIB_PATH)
        i64, i32, u32, ci, vp, f32 = (ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32, ctypes.c_int,
                                      ctypes.c_void_p, ctypes.c_float)
        szp = ctypes.POINTER(ctypes.c_size_t)
        lib.gnnagg_version.restype = ci
        lib.gnnagg_version.argtypes = []
        lib.gnnagg_strerror.restype = ctypes.c_char_p
        lib.gnnagg_strerror.argtypes = [ci]
        lib.gnnagg_build_csr.restype = ci
        lib.gnnagg_build_csr.argtypes = [i64, i64, vp, vp, u32, vp, vp, vp, vp, vp, szp, vp]
        lib.gnnagg_plan_rows.restype = ci
        lib.gnnagg_plan_rows.argtypes = [i64, vp, vp, vp, vp, szp, vp]
        lib.gnnagg_aggregate.restype = ci
        lib.gnnagg_aggregate.argtypes = [ci, i64, vp, vp, vp, vp, ci, vp, ci, i32, i32, vp, vp, vp]
        lib.gnnagg_aggregate_ws.restype = ci
        lib.gnnagg_aggregate_ws.argtypes = [ci, i64, vp, vp, vp, vp, ci, i64, vp, ci, i64, i32, i32, vp, vp, vp, szp,
                                            vp]
        lib.gnnagg_aggregate_update.restype = ci
        lib.gnnagg_aggregate_update.argtypes = [ci, i64, vp, vp, vp, vp, ci, i64, i32, i32, vp, i32, vp, ci, vp, ci,
                                                i64, vp, vp, vp, szp, vp]
        lib.gnnagg_aggregate_noalloc.restype = ci
        lib.gnnagg_aggregate_noalloc.argtypes = [ci, i64, vp, vp, vp, vp, ci, i64, vp, ci, i64, i32, i32, vp, vp, vp]
        lib.gnnagg_row_pitch.restype = i64
        lib.gnnagg_plan_source_blocks.argtypes = [i64, vp, vp, i32, vp, vp, vp, vp, szp, vp]
        lib.gnnagg_plan_source_blocks.restype = ci
        lib.gnnagg_aggregate_blocked.argtypes = [ci, i64, vp, vp, vp, vp, ci, i64, vp, ci, i64, i32, i32, i32, vp, vp,
                                                 vp, vp, szp, vp]
        lib.gnnagg_aggregate_blocked.restype = ci
        lib.gnnagg_tune_blocked.argtypes = [ci, i64, vp, vp, vp, vp, ci, i64, vp, ci, i64, i32, i32, vp, vp, vp, vp, szp,
                                            vp, vp, vp]
        lib.gnnagg_tune_blocked.restype = ci
        lib.gnnagg_auto_source_blocks.argtypes = [ci, i64, i32, ci, i64, vp]
        lib.gnnagg_auto_source_blocks.restype = i32
        lib.gnnagg_row_pitch.argtypes = [i32, ci]
        lib.gnnagg_gat_attention.restype = ci
        lib.gnnagg_gat_attention.argtypes = [i64, vp, vp, vp, vp, vp, i32, i32, f32, vp, vp, i32, vp, vp, vp, szp,
                                             vp]
        lib.gnnagg_auto_f_chunk.restype = i32
        lib.gnnagg_auto_f_chunk.argtypes = [i64, i32, ci, i64, vp]
        lib.gnnagg_combine.restype = ci
        lib.gnnagg_combine.argtypes = [i64, vp, ci, i32, vp, vp, i32, ci, vp, vp, vp]
        lib.gnnagg_check_csr.restype = ci
        lib.gnnagg_check_csr.argtypes = [i64, i64, vp, vp, vp, szp, vp]
        lib.gnnagg_rank_sources.restype = ci
        lib.gnnagg_rank_sources.argtypes = [i64, i64, vp, vp, vp, vp, szp, vp]
        lib.gnnagg_tune_f_chunk.restype = ci
        lib.gnnagg_tune_f_chunk.argtypes = [ci, i64, vp, vp, vp, vp, ci, i64, vp, ci, i64, i32, vp, vp, vp, szp, vp,
                                            ctypes.POINTER(i32), ctypes.POINTER(f32)]
        lib.gnnagg_set_workgroup_cap.restype = ci
        lib.gnnagg_combine_scaled.argtypes = [i64, vp, ci, i32, vp, vp, i32, ci, vp, vp, vp, vp]
        lib.gnnagg_combine_scaled.restype = ci
        lib.gnnagg_gcn_factors.argtypes = [i64, vp, vp, vp]
        lib.gnnagg_gcn_factors.restype = ci
        lib.gnnagg_scale_rows.argtypes = [i64, i32, vp, ci, i64, vp, vp, i64, vp]
        lib.gnnagg_scale_rows.restype = ci
        lib.gnnagg_set_workgroup_cap.argtypes = [ci]
        lib.gnnagg_mfma_f64_probe.restype = ci
        lib.gnnagg_mfma_f64_probe.argtypes = [vp, i64, i32, vp]
        lib.gnnagg_copy_probe.restype = ci
        lib.gnnagg_line_gather_probe.argtypes = [vp, ctypes.c_size_t, vp, i32, i32, vp, vp]
        lib.gnnagg_line_gather_probe.restype = ci
        lib.gnnagg_copy_probe.argtypes = [vp, vp, ctypes.c_size_t, vp]
        _lib = lib
    return _lib


def gnnagg_version() -> int:
    return load_library().gnnagg_version()


def gnnagg_strerror(status: int) -> str:
    return load_library().gnnagg_strerror(status).decode()


def _dev(t: Optional[torch.Tensor], dtype=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("%s must be a GPU tensor" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    return ctypes.c_void_p(t.data_ptr())


_TOKENS = {}


def _token(device) -> torch.Tensor:
    """A 256-byte device buffer per device, handed over where a call wants a workspace pointer but needs
    no workspace."""
    key = (device.type, device.index if device.index is not None else torch.cuda.current_device())
    if key not in _TOKENS:
        _TOKENS[key] = torch.empty(256, dtype=torch.uint8, device=device)
    return _TOKENS[key]


def _rows(t: torch.Tensor, name: str):
    """A 2-D GPU tensor whose rows are contiguous; the rows themselves may be a pitch apart."""
    if not t.is_cuda:
        raise ValueError("%s must be a GPU tensor" % name)
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1) or (t.shape[0] > 1 and t.stride(0) < t.shape[1]):
        raise ValueError("%s must be [N, F] with contiguous rows" % name)
    return ctypes.c_void_p(t.data_ptr())


def _weights(op: int, edge_w: Optional[torch.Tensor], rowptr: torch.Tensor, colidx: torch.Tensor):
    """The edge_w argument of an aggregation call: one weight per edge for WSUM, one factor per destination
    for SUM_SCALED (the library cannot see the length of the array it is handed)."""
    if edge_w is not None and op in (WSUM, SUM_SCALED):
        need = int(colidx.numel()) if op == WSUM else int(rowptr.numel()) - 1
        if edge_w.dim() != 1 or int(edge_w.numel()) < need:
            raise ValueError("edge_w must hold %d values for this operator" % need)
    return _dev(edge_w, torch.float32, "edge_w")


def gnnagg_row_pitch(F: int, dtype: torch.dtype = torch.float32) -> int:
    """Elements per row that put every row of an [N, F] matrix on 128-byte line boundaries."""
    return int(load_library().gnnagg_row_pitch(F, F32 if dtype == torch.float32 else BF16))


def pitched_empty(N: int, F: int, dtype: torch.dtype = torch.float32, device="cuda") -> torch.Tensor:
    """An uninitialised [N, F] view into an [N, gnnagg_row_pitch] allocation (memory only, no arithmetic)."""
    return torch.empty((N, gnnagg_row_pitch(F, dtype)), dtype=dtype, device=device)[:, :F]


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _workspace(nbytes: int, device) -> torch.Tensor:
    # torch's caching allocator hands out 512-byte aligned blocks
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _check(fn: str, rc: int):
    if rc != 0:
        raise GnnaggError(fn, rc)


def gnnagg_build_csr(N: int, src: torch.Tensor, dst: torch.Tensor, flags: int = 0, want_w: bool = False,
                     want_perm: bool = False, stream=None):
    """COO -> destination-indexed CSR on the GPU.
    Returns (rowptr int64 [N+1], colidx int32 [nnz], edge_w float32 [nnz] | None, perm int64 [nnz] | None)."""
    lib = load_library()
    E = int(src.shape[0])
    if dst.shape[0] != E:
        raise ValueError("src and dst differ in length")
    dev = src.device
    nnz = E + (N if flags & SELF_LOOPS else 0)
    need = ctypes.c_size_t(0)
    _check("gnnagg_build_csr", lib.gnnagg_build_csr(N, E, None, None, flags, None, None, None, None, None,
                                                     ctypes.byref(need), None))
    ws = _workspace(need.value, dev)
    rowptr = torch.empty(N + 1, dtype=torch.int64, device=dev)
    colidx = torch.empty(nnz, dtype=torch.int32, device=dev)
    w = torch.empty(nnz, dtype=torch.float32, device=dev) if want_w else None
    perm = torch.empty(nnz, dtype=torch.int64, device=dev) if want_perm else None
    have = ctypes.c_size_t(ws.numel())
    rc = lib.gnnagg_build_csr(N, E, _dev(src, torch.int32, "src"), _dev(dst, torch.int32, "dst"), flags,
                              _dev(rowptr), _dev(colidx), _dev(w), _dev(perm), _dev(ws), ctypes.byref(have),
                              _stream(stream))
    _check("gnnagg_build_csr", rc)
    return rowptr, colidx, w, perm


def gnnagg_check_csr(rowptr: torch.Tensor, colidx: torch.Tensor, stream=None) -> bool:
    """True if (rowptr, colidx) is a well-formed CSR of N = len(rowptr) - 1 vertices (the aggregation calls trust
    their CSR; check one that did not come from gnnagg_build_csr)."""
    lib = load_library()
    N, nnz = int(rowptr.shape[0]) - 1, int(colidx.shape[0])
    need = ctypes.c_size_t(0)
    _check("gnnagg_check_csr", lib.gnnagg_check_csr(N, nnz, None, None, None, ctypes.byref(need), None))
    ws = _workspace(need.value, rowptr.device)
    have = ctypes.c_size_t(ws.numel())
    rc = lib.gnnagg_check_csr(N, nnz, _dev(rowptr, torch.int64, "rowptr"), _dev(colidx, torch.int32, "colidx"), _dev(ws),
                              ctypes.byref(have), _stream(stream))
    if rc == -1:
        return False
    _check("gnnagg_check_csr", rc)
    return True


@dataclass
class RowPlan:
    """Degree-sorted row schedule: device row order plus host class offsets."""
    row_order: torch.Tensor
    class_off: "ctypes.Array"

    def class_offsets(self):
        return list(self.class_off)


def gnnagg_plan_rows(rowptr: torch.Tensor, stream=None) -> RowPlan:
    lib = load_library()
    N = int(rowptr.shape[0]) - 1
    dev = rowptr.device
    need = ctypes.c_size_t(0)
    _check("gnnagg_plan_rows", lib.gnnagg_plan_rows(N, None, None, None, None, ctypes.byref(need), None))
    ws = _workspace(need.value, dev)
    order = torch.empty(max(N, 1), dtype=torch.int32, device=dev)
    class_off = (ctypes.c_int64 * (PLAN_CLASSES + 1))()
    have = ctypes.c_size_t(ws.numel())
    rc = lib.gnnagg_plan_rows(N, _dev(rowptr, torch.int64, "rowptr"), _dev(order),
                              ctypes.cast(class_off, ctypes.c_void_p), _dev(ws), ctypes.byref(have),
                              _stream(stream))
    _check("gnnagg_plan_rows", rc)
    return RowPlan(order[:N] if N > 0 else order[:0], class_off)


def _x_dtype(X: torch.Tensor) -> int:
    if X.dtype == torch.float32:
        return F32
    if X.dtype == torch.bfloat16:
        return BF16
    raise TypeError("X must be float32 or bfloat16")


def gnnagg_aggregate_workspace_bytes(N: int, F: int, plan: Optional["RowPlan"]) -> int:
    """Size of the workspace with which gnnagg_aggregate_ws splits very long rows (the size query of the C call);
    0 when the plan holds no such row."""
    if plan is None or N == 0:
        return 0
    need = ctypes.c_size_t(0)
    _check("gnnagg_aggregate_ws",
           load_library().gnnagg_aggregate_ws(0, N, None, None, None, None, F32, 0, None, F32, 0, F, 0,
                                              _dev(plan.row_order, torch.int32, "row_order"),
                                              ctypes.cast(plan.class_off, ctypes.c_void_p), None,
                                              ctypes.byref(need), None))
    return int(need.value)


def gnnagg_aggregate(op: int, rowptr: torch.Tensor, colidx: torch.Tensor, edge_w: Optional[torch.Tensor],
                     X: torch.Tensor, out: Optional[torch.Tensor] = None, f_chunk: int = 0,
                     plan: Optional[RowPlan] = None, stream=None,
                     workspace: Optional[torch.Tensor] = None, split_long_rows: bool = True) -> torch.Tensor:
    """out[N,F] (fp32, or bf16 if a bf16 tensor is passed) = aggregation of X[N,F] over the CSR; enqueued on the
    current stream.  X and out may be row-pitched views (contiguous rows, stride(0) >= F; see pitched_empty).
    With pitched rows, or a plan that holds very long rows, the call goes through gnnagg_aggregate_ws (the
    workspace is allocated here unless one of at least gnnagg_aggregate_workspace_bytes is passed in);
    split_long_rows=False keeps every row with one workgroup."""
    lib = load_library()
    if X.dim() != 2:
        raise ValueError("X must be [N, F]")
    N, F = int(X.shape[0]), int(X.shape[1])
    if rowptr.shape[0] != N + 1:
        raise ValueError("rowptr must have N+1 entries")
    if out is None:
        out = torch.empty((N, F), dtype=torch.float32, device=X.device)
    elif tuple(out.shape) != (N, F):
        raise ValueError("out must be [N, F]")
    if out.dtype not in (torch.float32, torch.bfloat16):
        raise TypeError("out must be float32 or bfloat16")
    order, class_off = _plan_args(plan, N)
    x_pitch, out_pitch = int(X.stride(0)) if N > 1 else F, int(out.stride(0)) if N > 1 else F
    pitched = x_pitch != F or out_pitch != F
    need = gnnagg_aggregate_workspace_bytes(N, F, plan) if split_long_rows else 0
    if need > 0 or pitched:
        own = workspace is None and need > 0
        if workspace is None:  # nothing to hold: any aligned pointer serves, kept per device
            workspace = torch.empty(need, dtype=torch.uint8, device=X.device) if need > 0 else _token(X.device)
        have = ctypes.c_size_t(workspace.numel() * workspace.element_size())
        rc = lib.gnnagg_aggregate_ws(op, N, _dev(rowptr, torch.int64, "rowptr"), _dev(colidx, torch.int32, "colidx"),
                                     _weights(op, edge_w, rowptr, colidx), _rows(X, "X"), _x_dtype(X), x_pitch,
                                     _rows(out, "out"), F32 if out.dtype == torch.float32 else BF16, out_pitch, F,
                                     f_chunk, order, class_off, _dev(workspace), ctypes.byref(have), _stream(stream))
        _check("gnnagg_aggregate_ws", rc)
        if own:  # read and written by the kernels just enqueued: keep it alive until they ran
            workspace.record_stream(torch.cuda.current_stream() if stream is None else stream)
    else:
        rc = lib.gnnagg_aggregate(op, N, _dev(rowptr, torch.int64, "rowptr"), _dev(colidx, torch.int32, "colidx"),
                                  _weights(op, edge_w, rowptr, colidx), _dev(X, None, "X"), _x_dtype(X),
                                  _dev(out, None, "out"), F32 if out.dtype == torch.float32 else BF16, F, f_chunk,
                                  order, class_off, _stream(stream))
        _check("gnnagg_aggregate", rc)
    return out


def gnnagg_aggregate_update(op: int, rowptr: torch.Tensor, colidx: torch.Tensor, edge_w: Optional[torch.Tensor],
                            X: torch.Tensor, W2: Optional[torch.Tensor] = None, bias: Optional[torch.Tensor] = None,
                            relu: bool = False, out: Optional[torch.Tensor] = None, f_chunk: int = 0,
                            plan: Optional[RowPlan] = None, stream=None,
                            workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """out = act(aggregate(X) + bias) ([N,F]) or, with W2 [F,H2], act(aggregate(X) @ W2 + bias) ([N,H2]) in the
    aggregation kernels themselves; X and out may be row-pitched views."""
    lib = load_library()
    if X.dim() != 2:
        raise ValueError("X must be [N, F]")
    N, F = int(X.shape[0]), int(X.shape[1])
    if rowptr.shape[0] != N + 1:
        raise ValueError("rowptr must have N+1 entries")
    H2 = 0
    if W2 is not None:
        if W2.dim() != 2 or W2.shape[0] != F:
            raise ValueError("W2 must be [F, H2]")
        H2 = int(W2.shape[1])
    cols = H2 if W2 is not None else F
    if bias is not None and tuple(bias.shape) != (cols,):
        raise ValueError("bias must have one entry per output column")
    if out is None:
        out = torch.empty((N, cols), dtype=torch.float32, device=X.device)
    elif tuple(out.shape) != (N, cols):
        raise ValueError("out must be [N, %d]" % cols)
    order, class_off = _plan_args(plan, N)
    x_pitch, out_pitch = int(X.stride(0)) if N > 1 else F, int(out.stride(0)) if N > 1 else cols
    need = gnnagg_aggregate_workspace_bytes(N, F, plan)
    own = workspace is None and need > 0
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device) if need > 0 else _token(X.device)
    have = ctypes.c_size_t(workspace.numel() * workspace.element_size())
    rc = lib.gnnagg_aggregate_update(op, N, _dev(rowptr, torch.int64, "rowptr"), _dev(colidx, torch.int32, "colidx"),
                                     _weights(op, edge_w, rowptr, colidx), _rows(X, "X"), _x_dtype(X), x_pitch, F,
                                     f_chunk, _dev(W2, torch.float32, "W2"), H2, _dev(bias, torch.float32, "bias"),
                                     int(bool(relu)), _rows(out, "out"),
                                     F32 if out.dtype == torch.float32 else BF16, out_pitch, order, class_off,
                                     _dev(workspace), ctypes.byref(have), _stream(stream))
    _check("gnnagg_aggregate_update", rc)
    if own:
        workspace.record_stream(torch.cuda.current_stream() if stream is None else stream)
    return out


def gnnagg_aggregate_noalloc(op: int, rowptr: torch.Tensor, colidx: torch.Tensor, edge_w: Optional[torch.Tensor],
                             X: torch.Tensor, out: torch.Tensor, f_chunk: int = 0, plan: Optional[RowPlan] = None,
                             stream=None) -> torch.Tensor:
    """gnnagg_aggregate into a caller's `out` with no allocation anywhere: split rows use the library's fixed
    scratch array (raises GnnaggError with status -4 when the plan needs more than that array holds)."""
    lib = load_library()
    if X.dim() != 2:
        raise ValueError("X must be [N, F]")
    N, F = int(X.shape[0]), int(X.shape[1])
    if rowptr.shape[0] != N + 1:
        raise ValueError("rowptr must have N+1 entries")
    if tuple(out.shape) != (N, F):
        raise ValueError("out must be [N, F]")
    order, class_off = _plan_args(plan, N)
    x_pitch, out_pitch = int(X.stride(0)) if N > 1 else F, int(out.stride(0)) if N > 1 else F
    rc = lib.gnnagg_aggregate_noalloc(op, N, _dev(rowptr, torch.int64, "rowptr"),
                                      _dev(colidx, torch.int32, "colidx"), _weights(op, edge_w, rowptr, colidx),
                                      _rows(X, "X"), _x_dtype(X), x_pitch, _rows(out, "out"),
                                      F32 if out.dtype == torch.float32 else BF16, out_pitch, F, f_chunk, order,
                                      class_off, _stream(stream))
    _check("gnnagg_aggregate_noalloc", rc)
    return out


@dataclass
class SourceBlocks:
    """Per-graph tables of a blocked aggregation: where each row's edges into each block of sources begin, and a
    row order with its host class offsets per block."""
    B: int
    block_ptr: torch.Tensor   # [(B+1) * N] int64
    row_order: torch.Tensor   # [B * N] int32
    class_off: "ctypes.Array"  # [B * (PLAN_CLASSES + 1)] int64, host


def gnnagg_plan_source_blocks(rowptr: torch.Tensor, colidx: torch.Tensor, B: int, stream=None) -> SourceBlocks:
    lib = load_library()
    N = int(rowptr.shape[0]) - 1
    dev = rowptr.device
    need = ctypes.c_size_t(0)
    _check("gnnagg_plan_source_blocks",
           lib.gnnagg_plan_source_blocks(N, None, None, B, None, None, None, None, ctypes.byref(need), None))
    ws = _workspace(need.value, dev)
    block_ptr = torch.empty(max((B + 1) * N, 1), dtype=torch.int64, device=dev)
    order = torch.empty(max(B * N, 1), dtype=torch.int32, device=dev)
    class_off = (ctypes.c_int64 * (B * (PLAN_CLASSES + 1)))()
    have = ctypes.c_size_t(ws.numel())
    rc = lib.gnnagg_plan_source_blocks(N, _dev(rowptr, torch.int64, "rowptr"), _dev(colidx, torch.int32, "colidx"), B,
                                       _dev(block_ptr), _dev(order), ctypes.cast(class_off, ctypes.c_void_p),
                                       _dev(ws), ctypes.byref(have), _stream(stream))
    _check("gnnagg_plan_source_blocks", rc)
    return SourceBlocks(B, block_ptr, order, class_off)


def gnnagg_aggregate_blocked(op: int, rowptr: torch.Tensor, colidx: torch.Tensor, edge_w: Optional[torch.Tensor],
                             X: torch.Tensor, blocks: SourceBlocks, out: Optional[torch.Tensor] = None,
                             f_chunk: int = 0, stream=None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """gnnagg_aggregate over the source blocks of `blocks` (gnnagg_plan_source_blocks of the same CSR); X and out may
    be row-pitched views.  The workspace (states in transit between blocks) is allocated here unless passed in."""
    lib = load_library()
    if X.dim() != 2:
        raise ValueError("X must be [N, F]")
    N, F = int(X.shape[0]), int(X.shape[1])
    if rowptr.shape[0] != N + 1:
        raise ValueError("rowptr must have N+1 entries")
    if blocks.row_order.numel() < blocks.B * N or blocks.block_ptr.numel() < (blocks.B + 1) * N:
        raise ValueError("blocks were planned for another graph")
    if out is None:
        out = torch.empty((N, F), dtype=torch.float32, device=X.device)
    elif tuple(out.shape) != (N, F):
        raise ValueError("out must be [N, F]")
    x_pitch, out_pitch = int(X.stride(0)) if N > 1 else F, int(out.stride(0)) if N > 1 else F
    args = lambda ws, have: lib.gnnagg_aggregate_blocked(  # noqa: E731
        op, N, _dev(rowptr, torch.int64, "rowptr"), _dev(colidx, torch.int32, "colidx"),
        _weights(op, edge_w, rowptr, colidx), _rows(X, "X"), _x_dtype(X), x_pitch, _rows(out, "out"),
        F32 if out.dtype == torch.float32 else BF16, out_pitch, F, f_chunk, blocks.B,
        _dev(blocks.block_ptr, torch.int64, "block_ptr"), _dev(blocks.row_order, torch.int32, "row_order"),
        ctypes.cast(blocks.class_off, ctypes.c_void_p), ws, ctypes.byref(have), _stream(stream))
    own = workspace is None
    if workspace is None:
        need = ctypes.c_size_t(0)
        _check("gnnagg_aggregate_blocked", args(None, need))
        workspace = torch.empty(need.value, dtype=torch.uint8, device=X.device) if need.value > 0 else _token(X.device)
    have = ctypes.c_size_t(workspace.numel() * workspace.element_size())
    _check("gnnagg_aggregate_blocked", args(_dev(workspace), have))
    if own and workspace.numel() > 256:
        workspace.record_stream(torch.cuda.current_stream() if stream is None else stream)
    return out


def gnnagg_aggregate_blocked_workspace_bytes(N: int, F: int, blocks: SourceBlocks) -> int:
    need = ctypes.c_size_t(0)
    _check("gnnagg_aggregate_blocked",
           load_library().gnnagg_aggregate_blocked(0, N, None, None, None, None, F32, 0, None, F32, 0, F, 0, blocks.B,
                                                   _dev(blocks.block_ptr, torch.int64, "block_ptr"),
                                                   _dev(blocks.row_order, torch.int32, "row_order"),
                                                   ctypes.cast(blocks.class_off, ctypes.c_void_p), None,
                                                   ctypes.byref(need), None))
    return int(need.value)


def _plan_args(plan: Optional["RowPlan"], N: int):
    if plan is None or N == 0:
        return None, None
    return _dev(plan.row_order, torch.int32, "row_order"), ctypes.cast(plan.class_off, ctypes.c_void_p)


def gnnagg_gat_workspace_bytes(N: int, heads: int, C: int, plan: Optional["RowPlan"] = None) -> int:
    """Size of the workspace gnnagg_gat_attention needs (the size query of the C call).  It depends on the
    plan when the plan holds rows long enough to be split: query with the plan the call will use."""
    need = ctypes.c_size_t(0)
    order, class_off = _plan_args(plan, N)
    _check("gnnagg_gat_attention",
           load_library().gnnagg_gat_attention(N, None, None, None, None, None, heads, C, 0.2, None, None, 0, order,
                                               class_off, None, ctypes.byref(need), None))
    return int(need.value)


def gnnagg_gat_attention(rowptr: torch.Tensor, colidx: torch.Tensor, H: torch.Tensor, a_src: torch.Tensor,
                         a_dst: torch.Tensor, negative_slope: float = 0.2, want_alpha: bool = False,
                         want_out: bool = True, f_chunk: int = 0, plan: Optional[RowPlan] = None, stream=None,
                         out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None):
    """H [N,heads,C] fp32 -> (alpha [nnz,heads] | None, out [N,heads,C] | None).  `out` and `workspace`
    (at least gnnagg_gat_workspace_bytes) may be passed in to avoid allocating per call."""
    lib = load_library()
    if H.dim() != 3:
        raise ValueError("H must be [N, heads, C]")
    N, heads, C = (int(v) for v in H.shape)
    if tuple(a_src.shape) != (heads, C) or tuple(a_dst.shape) != (heads, C):
        raise ValueError("a_src and a_dst must be [heads, C]")
    dev = H.device
    nnz = int(colidx.shape[0])
    order, class_off = _plan_args(plan, N)
    need = ctypes.c_size_t(0)
    _check("gnnagg_gat_attention",
           lib.gnnagg_gat_attention(N, None, None, None, None, None, heads, C, negative_slope, None, None, f_chunk,
                                    order, class_off, None, ctypes.byref(need), None))
    ws = workspace if workspace is not None else _workspace(need.value, dev)
    alpha = torch.empty((nnz, heads), dtype=torch.float32, device=dev) if want_alpha else None
    if want_out and out is None:
        out = torch.empty((N, heads, C), dtype=torch.float32, device=dev)
    elif not want_out:
        out = None
    have = ctypes.c_size_t(ws.numel())
    rc = lib.gnnagg_gat_attention(N, _dev(rowptr, torch.int64, "rowptr"), _dev(colidx, torch.int32, "colidx"),
                                  _dev(H, torch.float32, "H"), _dev(a_src, torch.float32, "a_src"),
                                  _dev(a_dst, torch.float32, "a_dst"), heads, C, negative_slope, _dev(alpha),
                                  _dev(out), f_chunk, order, class_off,
                                  _dev(ws), ctypes.byref(have), _stream(stream))
    _check("gnnagg_gat_attention", rc)
    # the score arrays in ws are read by the kernels just enqueued: keep ws alive until they ran
    if workspace is None:
        ws.record_stream(torch.cuda.current_stream() if stream is None else stream)
    return alpha, out


def gnnagg_copy_probe(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    """Plain streaming copy of src into dst (same byte size): the measurement aid of the library."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("dst and src differ in size")
    _check("gnnagg_copy_probe", load_library().gnnagg_copy_probe(_dev(dst), _dev(src), nbytes, _stream(stream)))


def gnnagg_tune_f_chunk(op: int, rowptr: torch.Tensor, colidx: torch.Tensor, edge_w: Optional[torch.Tensor],
                        X: torch.Tensor, out: torch.Tensor, plan: Optional[RowPlan] = None, stream=None):
    """(best chunk width, its milliseconds per call) for this graph, X layout and operator, by measurement."""
    lib = load_library()
    N, F = int(X.shape[0]), int(X.shape[1])
    order, class_off = _plan_args(plan, N)
    need = gnnagg_aggregate_workspace_bytes(N, F, plan)
    ws = torch.empty(need, dtype=torch.uint8, device=X.device) if need > 0 else _token(X.device)
    have = ctypes.c_size_t(ws.numel())
    best, ms = ctypes.c_int32(0), ctypes.c_float(0.0)
    rc = lib.gnnagg_tune_f_chunk(op, N, _dev(rowptr, torch.int64, "rowptr"), _dev(colidx, torch.int32, "colidx"),
                                 _weights(op, edge_w, rowptr, colidx), _rows(X, "X"), _x_dtype(X),
                                 int(X.stride(0)) if N > 1 else F, _rows(out, "out"),
                                 F32 if out.dtype == torch.float32 else BF16, int(out.stride(0)) if N > 1 else F, F,
                                 order, class_off, _dev(ws), ctypes.byref(have), _stream(stream), ctypes.byref(best),
                                 ctypes.byref(ms))
    _check("gnnagg_tune_f_chunk", rc)
    return int(best.value), float(ms.value)


def gnnagg_tune_blocked(op: int, rowptr: torch.Tensor, colidx: torch.Tensor, edge_w: Optional[torch.Tensor],
                        X: torch.Tensor, out: torch.Tensor, blocks: "SourceBlocks", stream=None,
                        workspace: Optional[torch.Tensor] = None):
    """(best chunk width, its milliseconds per call) of the blocked call with these block tables, by measurement."""
    lib = load_library()
    N, F = int(X.shape[0]), int(X.shape[1])
    if workspace is None:
        need = gnnagg_aggregate_blocked_workspace_bytes(N, F, blocks)
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device) if need > 0 else _token(X.device)
    have = ctypes.c_size_t(workspace.numel())
    best, ms = ctypes.c_int32(0), ctypes.c_float(0.0)
    rc = lib.gnnagg_tune_blocked(op, N, _dev(rowptr, torch.int64, "rowptr"), _dev(colidx, torch.int32, "colidx"),
                                 _weights(op, edge_w, rowptr, colidx), _rows(X, "X"), _x_dtype(X),
                                 int(X.stride(0)) if N > 1 else F, _rows(out, "out"),
                                 F32 if out.dtype == torch.float32 else BF16, int(out.stride(0)) if N > 1 else F, F,
                                 blocks.B, _dev(blocks.block_ptr, torch.int64, "block_ptr"),
                                 _dev(blocks.row_order, torch.int32, "row_order"),
                                 ctypes.cast(blocks.class_off, ctypes.c_void_p), _dev(workspace), ctypes.byref(have),
                                 _stream(stream), ctypes.byref(best), ctypes.byref(ms))
    _check("gnnagg_tune_blocked", rc)
    return int(best.value), float(ms.value)


def gnnagg_line_gather_probe(buf: torch.Tensor, rounds: int, workgroups: int, sink: torch.Tensor,
                             idx: Optional[torch.Tensor] = None, stream=None) -> int:
    """Enqueues the one-line gather probe over `buf` (uint8, 128-byte aligned): the pattern alone, or with `idx`
    (int32, workgroups * 256 * rounds line numbers) the index stream and fp64 sums as well; returns the lines it
    reads."""
    lines = workgroups * 32 * 8 * rounds
    if idx is not None and idx.numel() < lines:
        raise ValueError("idx must hold one line number per line read")
    rc = load_library().gnnagg_line_gather_probe(_dev(buf), buf.numel() * buf.element_size(),
                                                 _dev(idx, torch.int32, "idx"), rounds, workgroups, _dev(sink),
                                                 _stream(stream))
    _check("gnnagg_line_gather_probe", rc)
    return lines


def gnnagg_mfma_f64_probe(sink: torch.Tensor, iters: int, workgroups: int, stream=None) -> float:
    """Measurement aid: enqueues the fp64 matrix-instruction loop; returns the flop it performs."""
    _check("gnnagg_mfma_f64_probe",
           load_library().gnnagg_mfma_f64_probe(_dev(sink, torch.float64, "sink"), iters, workgroups, _stream(stream)))
    return float(workgroups) * 4 * iters * 8 * 2048.0


def gnnagg_set_workgroup_cap(cap: int) -> None:
    """Measurement aid: force the number of aggregation workgroups per compute unit (-1: the library's rule)."""
    _check("gnnagg_set_workgroup_cap", load_library().gnnagg_set_workgroup_cap(cap))


def gnnagg_auto_f_chunk(N: int, F: int, x_dtype: int = F32, x_pitch: int = 0,
                        plan: Optional[RowPlan] = None) -> int:
    """Chunk width the library uses for f_chunk = F_CHUNK_AUTO on an X of that row pitch (0 = F) and plan."""
    class_off = ctypes.cast(plan.class_off, ctypes.c_void_p) if plan is not None else None
    return int(load_library().gnnagg_auto_f_chunk(N, F, x_dtype, x_pitch, class_off))


def gnnagg_auto_source_blocks(op: int, N: int, F: int, x_dtype: int = F32, x_pitch: int = 0,
                              plan: Optional[RowPlan] = None) -> int:
    """Number of source blocks the library recommends for this operator, graph and width (1: use the plain calls)."""
    return int(load_library().gnnagg_auto_source_blocks(
        op, N, F, x_dtype, x_pitch, ctypes.cast(plan.class_off, ctypes.c_void_p) if plan is not None else None))


def gnnagg_combine(X: torch.Tensor, W: torch.Tensor, bias: Optional[torch.Tensor] = None, relu: bool = False,
                   out: Optional[torch.Tensor] = None, stream=None,
                   out_rows: Optional[torch.Tensor] = None, row_scale: Optional[torch.Tensor] = None) -> torch.Tensor:
    """out[N,H] fp32 = act(X[N,F] @ W[F,H] + bias); X fp32 or bf16, W and bias fp32.  With out_rows (int32 [N], a
    permutation) row i of the result is stored as row out_rows[i]; with row_scale (fp32 [N]) it is multiplied by
    row_scale[i] on its way out (gnnagg_combine_scaled)."""
    if X.dim() != 2 or W.dim() != 2 or W.shape[0] != X.shape[1]:
        raise ValueError("X must be [N,F] and W [F,H]")
    N, F, H = int(X.shape[0]), int(X.shape[1]), int(W.shape[1])
    if bias is not None and tuple(bias.shape) != (H,):
        raise ValueError("bias must be [H]")
    if out_rows is not None and tuple(out_rows.shape) != (N,):
        raise ValueError("out_rows must be [N]")
    if out is None:
        out = torch.empty((N, H), dtype=torch.float32, device=X.device)
    elif tuple(out.shape) != (N, H):
        raise ValueError("out must be [N, H]")
    if row_scale is not None:
        if row_scale.dim() != 1 or int(row_scale.numel()) < N:
            raise ValueError("row_scale must be [N]")
        rc = load_library().gnnagg_combine_scaled(N, _dev(X, None, "X"), _x_dtype(X), F, _dev(W, torch.float32, "W"),
                                                  _dev(bias, torch.float32, "bias"), H, int(bool(relu)),
                                                  _dev(row_scale, torch.float32, "row_scale"),
                                                  _dev(out, torch.float32, "out"),
                                                  _dev(out_rows, torch.int32, "out_rows"), _stream(stream))
        _check("gnnagg_combine_scaled", rc)
        return out
    rc = load_library().gnnagg_combine(N, _dev(X, None, "X"), _x_dtype(X), F, _dev(W, torch.float32, "W"),
                                       _dev(bias, torch.float32, "bias"), H, int(bool(relu)),
                                       _dev(out, torch.float32, "out"), _dev(out_rows, torch.int32, "out_rows"),
                                       _stream(stream))
    _check("gnnagg_combine", rc)
    return out


def gnnagg_gcn_factors(rowptr: torch.Tensor, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """s[i] = 1/sqrt(deg(i)) as fp32 (0 for an empty row): GCN's edge weight 1/sqrt(d_i d_j) is s[i] * s[j]."""
    N = int(rowptr.numel()) - 1
    if out is None:
        out = torch.empty(max(N, 1), dtype=torch.float32, device=rowptr.device)[:N]
    elif out.dim() != 1 or int(out.numel()) != N:
        raise ValueError("out must be [N]")
    _check("gnnagg_gcn_factors",
           load_library().gnnagg_gcn_factors(N, _dev(rowptr, torch.int64, "rowptr"), _dev(out, torch.float32, "out"),
                                             _stream(stream)))
    return out


def gnnagg_scale_rows(X: torch.Tensor, scale: torch.Tensor, out: Optional[torch.Tensor] = None,
                      stream=None) -> torch.Tensor:
    """out[j, :] = scale[j] * X[j, :] in fp32 (X fp32 or bf16, rows may be a pitch apart).  out=None: a new matrix
    with its rows on 128-byte lines; out=X (fp32) scales in place."""
    if X.dim() != 2:
        raise ValueError("X must be [N, F]")
    N, F = int(X.shape[0]), int(X.shape[1])
    if scale.dim() != 1 or int(scale.numel()) < N:
        raise ValueError("scale must be [N]")
    if out is None:
        out = pitched_empty(N, F, torch.float32, X.device)
    elif tuple(out.shape) != (N, F) or out.dtype != torch.float32:
        raise ValueError("out must be fp32 [N, F]")
    x_pitch = int(X.stride(0)) if N > 1 else F
    out_pitch = int(out.stride(0)) if N > 1 else F
    rc = load_library().gnnagg_scale_rows(N, F, _rows(X, "X"), _x_dtype(X), x_pitch, _dev(scale, torch.float32, "scale"),
                                          _rows(out, "out"), out_pitch, _stream(stream))
    _check("gnnagg_scale_rows", rc)
    return out


def gnnagg_rank_sources(N: int, colidx: torch.Tensor, stream=None):
    """(rank int32 [N], colidx_ranked int32 [nnz]): vertices ordered by how often they occur in colidx."""
    lib = load_library()
    nnz = int(colidx.shape[0])
    dev = colidx.device
    need = ctypes.c_size_t(0)
    _check("gnnagg_rank_sources", lib.gnnagg_rank_sources(N, nnz, None, None, None, None, ctypes.byref(need), None))
    ws = _workspace(need.value, dev)
    rank = torch.empty(max(N, 1), dtype=torch.int32, device=dev)
    ranked = torch.empty(max(nnz, 1), dtype=torch.int32, device=dev)
    have = ctypes.c_size_t(ws.numel())
    _check("gnnagg_rank_sources",
           lib.gnnagg_rank_sources(N, nnz, _dev(colidx, torch.int32, "colidx"), _dev(rank), _dev(ranked), _dev(ws),
                                   ctypes.byref(have), _stream(stream)))
    ws.record_stream(torch.cuda.current_stream() if stream is None else stream)
    return rank[:N], ranked[:nnz]
