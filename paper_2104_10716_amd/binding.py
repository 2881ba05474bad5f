"""ctypes binding of libes_spmm.so: same names as the C ABI, tensors in, status
checked.  No arithmetic happens here."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

ES_FULL, ES_BUCKET, ES_FASTRAND = 0, 1, 2
MODES = {"full": ES_FULL, "bucket": ES_BUCKET, "fastrand": ES_FASTRAND}
ES_NORM_NONE, ES_NORM_MEAN, ES_NORM_RSQRT, ES_NORM_RESCALE, ES_NORM_INV_DEGREE = 0, 1, 2, 3, 4
NORMS = {"none": ES_NORM_NONE, "mean": ES_NORM_MEAN, "rsqrt": ES_NORM_RSQRT, "rescale": ES_NORM_RESCALE,
         "inv_degree": ES_NORM_INV_DEGREE}


class es_launch_opts_t(ctypes.Structure):
    _fields_ = [("rows_per_wave", ctypes.c_int32), ("lanes_per_row", ctypes.c_int32),
                ("long_row_threshold", ctypes.c_int32), ("column_partition", ctypes.c_int32),
                ("kernel", ctypes.c_int32)]


class es_launch_info_t(ctypes.Structure):
    _fields_ = [("vector_width", ctypes.c_int32), ("aligned", ctypes.c_int32),
                ("lanes_per_row", ctypes.c_int32), ("chunks_per_lane", ctypes.c_int32),
                ("rows_per_wave", ctypes.c_int32), ("edge_slots", ctypes.c_int32),
                ("loads_in_flight", ctypes.c_int32), ("tile_slots_per_row", ctypes.c_int32),
                ("long_row_threshold", ctypes.c_int32), ("long_row_workgroups", ctypes.c_int64),
                ("grid_x", ctypes.c_int64), ("grid_y", ctypes.c_int64), ("flattened", ctypes.c_int32),
                ("column_ranges", ctypes.c_int32)]


_PKG = os.path.dirname(os.path.abspath(__file__))
# ES_SPMM_LIBRARY: load another build of the same sources (an instrumented one, say)
_LIB_PATH = os.environ.get("ES_SPMM_LIBRARY") or os.path.join(_PKG, "libes_spmm.so")
_lib = None


class EsSpmmError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {es_spmm_status_string(status)} ({status})")


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the HIP library; raises if it has not been built (there is no
    fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2104_10716_amd.build` "
            "(or __graft_entry__.build()); there is no CPU fallback")
    lib = ctypes.CDLL(_LIB_PATH)
    vp = ctypes.c_void_p
    lib.es_spmm.restype = ctypes.c_int
    lib.es_spmm.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                            ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                            ctypes.c_uint64, vp]
    lib.es_spmm_norm.restype = ctypes.c_int
    lib.es_spmm_norm.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                 ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                 ctypes.c_uint64, ctypes.c_int32, vp]
    lib.es_spmm_backward.restype = ctypes.c_int
    lib.es_spmm_backward.argtypes = lib.es_spmm_norm.argtypes
    optp = ctypes.POINTER(es_launch_opts_t)
    lib.es_spmm_ex.restype = ctypes.c_int
    lib.es_spmm_ex.argtypes = lib.es_spmm_norm.argtypes[:-1] + [optp, vp]
    lib.es_spmm_backward_ex.restype = ctypes.c_int
    lib.es_spmm_backward_ex.argtypes = lib.es_spmm_ex.argtypes
    lib.es_spmm_ws.restype = ctypes.c_int
    lib.es_spmm_ws.argtypes = lib.es_spmm_ex.argtypes[:-1] + [vp, ctypes.c_size_t, vp]
    lib.es_spmm_static_ws.restype = ctypes.c_int
    lib.es_spmm_static_ws.argtypes = lib.es_spmm_ex.argtypes
    lib.es_spmm_workspace_bytes.restype = ctypes.c_size_t
    lib.es_spmm_workspace_bytes.argtypes = [ctypes.c_int64]
    lib.es_spmm_sample_edges.restype = ctypes.c_int
    lib.es_spmm_sample_edges.argtypes = [vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                         ctypes.c_uint64, ctypes.c_int32, vp, vp, vp]
    lib.es_spmm_materialize.restype = ctypes.c_int
    lib.es_spmm_materialize.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                        ctypes.c_int32, ctypes.c_uint64, vp, vp, vp, vp]
    lib.es_spmm_materialize_transposed.restype = ctypes.c_int
    lib.es_spmm_materialize_transposed.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int64,
                                                   ctypes.c_int32, ctypes.c_int32, ctypes.c_uint64,
                                                   ctypes.c_int32, vp, vp, vp, vp, vp]
    lib.es_spmm_transpose_graph.restype = ctypes.c_int
    lib.es_spmm_transpose_graph.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int64, vp, vp, vp, vp, vp, vp, vp,
                                            vp]
    lib.es_spmm_backward_pull.restype = ctypes.c_int
    lib.es_spmm_backward_pull.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int64,
                                          ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                          ctypes.c_int32, ctypes.c_uint64, ctypes.c_int32, vp]
    lib.es_spmm_validate_csr.restype = ctypes.c_int
    lib.es_spmm_validate_csr.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int64, vp, vp]
    lib.es_spmm_launch_info.restype = ctypes.c_int
    lib.es_spmm_launch_info.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                        ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                        ctypes.c_int32, optp, ctypes.POINTER(es_launch_info_t)]
    lib.es_spmm_status_string.restype = ctypes.c_char_p
    lib.es_spmm_status_string.argtypes = [ctypes.c_int]
    lib.es_spmm_max_W.restype = ctypes.c_int32
    lib.es_spmm_max_W.argtypes = [ctypes.c_int32]
    lib.es_spmm_tile_slots.restype = ctypes.c_int32
    lib.es_spmm_tile_slots.argtypes = [ctypes.c_int32]
    _lib = lib
    return lib


def _mode(mode) -> int:
    return MODES[mode] if isinstance(mode, str) else int(mode)


def _stream_ptr(stream) -> Optional[int]:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _dev_ptr(t, dtype, name):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr() or None


def es_spmm_status_string(status: int) -> str:
    return load_library().es_spmm_status_string(int(status)).decode()


def es_spmm_max_W(F: int) -> int:
    return int(load_library().es_spmm_max_W(int(F)))


def es_spmm_tile_slots(rows_per_wave: int = 0) -> int:
    return int(load_library().es_spmm_tile_slots(int(rows_per_wave)))


def _opts_ptr(opts):
    """None, an es_launch_opts_t, or a dict with its field names -> ctypes pointer (or None)."""
    if opts is None:
        return None
    if isinstance(opts, dict):
        unknown = set(opts) - {name for name, _ in es_launch_opts_t._fields_}
        if unknown:
            raise ValueError(f"unknown launch option(s): {sorted(unknown)}")
        opts = es_launch_opts_t(**{k: int(v) for k, v in opts.items()})
    return ctypes.byref(opts)


def _spmm_args(rowptr, colidx, vals, X, Y, F, nnz):
    import torch
    if X.dim() != 2 or Y.dim() != 2 or X.stride(1) != 1 or Y.stride(1) != 1:
        raise ValueError("X and Y must be 2-D with contiguous columns")
    N = rowptr.numel() - 1
    if X.shape[0] != N or Y.shape[0] != N:
        raise ValueError("X and Y need one row per CSR row")
    if F is None:
        F = X.shape[1]
    if F > X.shape[1] or F > Y.shape[1]:
        raise ValueError("F exceeds the width of X or Y")
    ldx = X.stride(0) if N > 1 else max(X.shape[1], 1)
    ldy = Y.stride(0) if N > 1 else max(Y.shape[1], 1)
    if vals is not None and vals.numel() != colidx.numel():
        raise ValueError("vals and colidx differ in length")
    if nnz is None:
        nnz = colidx.numel()
    return (_dev_ptr(rowptr, torch.int32, "rowptr"), _dev_ptr(colidx, torch.int32, "colidx"),
            _dev_ptr(vals, torch.float32, "vals"), _dev_ptr(X, torch.float32, "X"),
            _dev_ptr(Y, torch.float32, "Y"), N, nnz, int(F), int(ldx), int(ldy))


def es_spmm(rowptr, colidx, vals, X, Y, W: int, mode, seed: int = 0, F: Optional[int] = None,
            stream=None, nnz: Optional[int] = None):
    """Y[:, :F] = sample_W(A) @ X[:, :F] on the tensors' device; returns Y.
    rowptr/colidx int32, vals float32 or None, X/Y 2-D float32 with unit column
    stride (row stride = leading dimension).  Enqueued on `stream` (default:
    torch's current stream); not synchronised.  `nnz` (default: len(colidx)) is
    only the launch-shape hint of the C ABI."""
    lib = load_library()
    args = _spmm_args(rowptr, colidx, vals, X, Y, F, nnz)
    rc = lib.es_spmm(*args, int(W), _mode(mode), int(seed) & 0xFFFFFFFFFFFFFFFF, _stream_ptr(stream))
    if rc != 0:
        raise EsSpmmError(rc, "es_spmm")
    return Y


def es_spmm_norm(rowptr, colidx, vals, X, Y, W: int, mode, seed: int = 0, norm="none",
                 F: Optional[int] = None, stream=None, nnz: Optional[int] = None):
    """es_spmm with a row factor ("none", "mean", "rsqrt", "rescale") applied in the kernel."""
    lib = load_library()
    args = _spmm_args(rowptr, colidx, vals, X, Y, F, nnz)
    nm = NORMS[norm] if isinstance(norm, str) else int(norm)
    rc = lib.es_spmm_norm(*args, int(W), _mode(mode), int(seed) & 0xFFFFFFFFFFFFFFFF, nm,
                          _stream_ptr(stream))
    if rc != 0:
        raise EsSpmmError(rc, "es_spmm_norm")
    return Y


def es_spmm_ex(rowptr, colidx, vals, X, Y, W: int, mode, seed: int = 0, norm="none", opts=None,
               F: Optional[int] = None, stream=None, nnz: Optional[int] = None):
    """es_spmm_norm with per-call launch options (None, a dict of es_launch_opts_t fields, or the struct)."""
    lib = load_library()
    args = _spmm_args(rowptr, colidx, vals, X, Y, F, nnz)
    nm = NORMS[norm] if isinstance(norm, str) else int(norm)
    rc = lib.es_spmm_ex(*args, int(W), _mode(mode), int(seed) & 0xFFFFFFFFFFFFFFFF, nm, _opts_ptr(opts),
                        _stream_ptr(stream))
    if rc != 0:
        raise EsSpmmError(rc, "es_spmm_ex")
    return Y


def es_spmm_workspace_bytes(N: int) -> int:
    return int(load_library().es_spmm_workspace_bytes(int(N)))


def es_spmm_ws(rowptr, colidx, vals, X, Y, W: int, mode, seed: int = 0, norm="none", opts=None,
               workspace=None, F: Optional[int] = None, stream=None, nnz: Optional[int] = None):
    """es_spmm_ex with a caller-owned workspace (a device tensor of at least
    es_spmm_workspace_bytes(N) bytes, any dtype), which enables the column-partitioned product."""
    lib = load_library()
    args = _spmm_args(rowptr, colidx, vals, X, Y, F, nnz)
    nm = NORMS[norm] if isinstance(norm, str) else int(norm)
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        if not workspace.is_cuda or not workspace.is_contiguous():
            raise ValueError("workspace must be a contiguous device tensor")
        ws_ptr, ws_bytes = workspace.data_ptr() or None, workspace.numel() * workspace.element_size()
    rc = lib.es_spmm_ws(*args, int(W), _mode(mode), int(seed) & 0xFFFFFFFFFFFFFFFF, nm, _opts_ptr(opts),
                        ws_ptr, ws_bytes, _stream_ptr(stream))
    if rc != 0:
        raise EsSpmmError(rc, "es_spmm_ws")
    return Y


ES_SPMM_STATIC_WS_MAX_ROWS = 1048576


def es_spmm_static_ws(rowptr, colidx, vals, X, Y, W: int, mode, seed: int = 0, norm="none", opts=None,
                      F: Optional[int] = None, stream=None, nnz: Optional[int] = None):
    """es_spmm_ws on the library's own static workspace (allocates nothing; at most
    ES_SPMM_STATIC_WS_MAX_ROWS rows; calls on one GPU must not overlap in time)."""
    lib = load_library()
    args = _spmm_args(rowptr, colidx, vals, X, Y, F, nnz)
    nm = NORMS[norm] if isinstance(norm, str) else int(norm)
    rc = lib.es_spmm_static_ws(*args, int(W), _mode(mode), int(seed) & 0xFFFFFFFFFFFFFFFF, nm,
                               _opts_ptr(opts), _stream_ptr(stream))
    if rc != 0:
        raise EsSpmmError(rc, "es_spmm_static_ws")
    return Y


def es_spmm_backward_ex(rowptr, colidx, vals, dY, dX, W: int, mode, seed: int = 0, norm="none", opts=None,
                        F: Optional[int] = None, stream=None, nnz: Optional[int] = None):
    """es_spmm_backward with per-call launch options."""
    lib = load_library()
    args = _spmm_args(rowptr, colidx, vals, dY, dX, F, nnz)
    nm = NORMS[norm] if isinstance(norm, str) else int(norm)
    rc = lib.es_spmm_backward_ex(*args, int(W), _mode(mode), int(seed) & 0xFFFFFFFFFFFFFFFF, nm,
                                 _opts_ptr(opts), _stream_ptr(stream))
    if rc != 0:
        raise EsSpmmError(rc, "es_spmm_backward_ex")
    return dX


def es_spmm_backward(rowptr, colidx, vals, dY, dX, W: int, mode, seed: int = 0, norm="none",
                     F: Optional[int] = None, stream=None, nnz: Optional[int] = None):
    """dX[:, :F] = sample_W(A)^T @ dY[:, :F] (dX is overwritten); returns dX."""
    lib = load_library()
    args = _spmm_args(rowptr, colidx, vals, dY, dX, F, nnz)
    nm = NORMS[norm] if isinstance(norm, str) else int(norm)
    rc = lib.es_spmm_backward(*args, int(W), _mode(mode), int(seed) & 0xFFFFFFFFFFFFFFFF, nm,
                              _stream_ptr(stream))
    if rc != 0:
        raise EsSpmmError(rc, "es_spmm_backward")
    return dX


def es_spmm_sample_edges(rowptr, W: int, mode, seed: int = 0, rows_per_wave: int = 0,
                         pos=None, cnt=None, stream=None):
    """(pos [N, W] int32, cnt [N] int32) on the device of rowptr."""
    import torch
    lib = load_library()
    N = rowptr.numel() - 1
    if pos is None:
        pos = torch.empty((N, int(W)), dtype=torch.int32, device=rowptr.device)
    if cnt is None:
        cnt = torch.empty((N,), dtype=torch.int32, device=rowptr.device)
    if pos.numel() != N * int(W) or cnt.numel() != N or not pos.is_contiguous():
        raise ValueError("pos must be a contiguous [N, W] tensor and cnt [N]")
    rc = lib.es_spmm_sample_edges(_dev_ptr(rowptr, torch.int32, "rowptr"), N, int(W), _mode(mode),
                                  int(seed) & 0xFFFFFFFFFFFFFFFF, int(rows_per_wave),
                                  _dev_ptr(pos, torch.int32, "pos"), _dev_ptr(cnt, torch.int32, "cnt"),
                                  _stream_ptr(stream))
    if rc != 0:
        raise EsSpmmError(rc, "es_spmm_sample_edges")
    return pos, cnt


def es_spmm_materialize(rowptr, colidx, vals, W: int, mode, seed: int = 0, out_rowptr=None,
                        out_colidx=None, out_vals=None, stream=None):
    """Sampled graph as CSR tensors (out_rowptr [N+1], out_colidx, out_vals).
    The value arrays are allocated at the capacity bound min(nnz, N*W); the
    entries in use are the first out_rowptr[-1]."""
    import torch
    lib = load_library()
    N = rowptr.numel() - 1
    nnz = colidx.numel()
    m = _mode(mode)
    cap = nnz if m == ES_FULL else min(nnz, N * int(W))
    dev = rowptr.device
    if out_rowptr is None:
        out_rowptr = torch.empty((N + 1,), dtype=torch.int32, device=dev)
    if out_colidx is None:
        out_colidx = torch.empty((cap,), dtype=torch.int32, device=dev)
    if out_vals is None:
        out_vals = torch.empty((cap,), dtype=torch.float32, device=dev)
    if out_rowptr.numel() != N + 1 or out_colidx.numel() < cap or out_vals.numel() < cap:
        raise ValueError("output tensors are too small")
    rc = lib.es_spmm_materialize(_dev_ptr(rowptr, torch.int32, "rowptr"), _dev_ptr(colidx, torch.int32, "colidx"),
                                 _dev_ptr(vals, torch.float32, "vals"), N, nnz, int(W), m,
                                 int(seed) & 0xFFFFFFFFFFFFFFFF,
                                 _dev_ptr(out_rowptr, torch.int32, "out_rowptr"),
                                 _dev_ptr(out_colidx, torch.int32, "out_colidx"),
                                 _dev_ptr(out_vals, torch.float32, "out_vals"), _stream_ptr(stream))
    if rc != 0:
        raise EsSpmmError(rc, "es_spmm_materialize")
    return out_rowptr, out_colidx, out_vals


def es_spmm_launch_info(N: int, nnz: int, F: int, W: int, mode, ldx: Optional[int] = None,
                        ldy: Optional[int] = None, aligned16: bool = True, backward: bool = False,
                        opts=None) -> dict:
    """Launch shape the library would pick (host-only; needs no GPU)."""
    info = es_launch_info_t()
    rc = load_library().es_spmm_launch_info(int(N), int(nnz), int(F), int(F if ldx is None else ldx),
                                            int(F if ldy is None else ldy), int(W), _mode(mode),
                                            int(bool(aligned16)), int(bool(backward)), _opts_ptr(opts),
                                            ctypes.byref(info))
    if rc != 0:
        raise EsSpmmError(rc, "es_spmm_launch_info")
    return {name: int(getattr(info, name)) for name, _ in es_launch_info_t._fields_}


def es_spmm_materialize_transposed(rowptr, colidx, vals, W: int, mode, seed: int = 0, norm="none",
                                   out_ptr=None, out_end=None, out_idx=None, out_vals=None, stream=None):
    """Transposed sampled graph as CSR tensors (out_ptr [N+1], out_end [N], out_idx, out_vals);
    index / value arrays are allocated at the capacity bound min(nnz, N*W)."""
    import torch
    lib = load_library()
    N = rowptr.numel() - 1
    nnz = colidx.numel()
    m = _mode(mode)
    cap = nnz if m == ES_FULL else min(nnz, N * int(W))
    dev = rowptr.device
    if out_ptr is None:
        out_ptr = torch.empty((N + 1,), dtype=torch.int32, device=dev)
    if out_end is None:
        out_end = torch.empty((N,), dtype=torch.int32, device=dev)
    if out_idx is None:
        out_idx = torch.empty((cap,), dtype=torch.int32, device=dev)
    if out_vals is None:
        out_vals = torch.empty((cap,), dtype=torch.float32, device=dev)
    if (out_ptr.numel() != N + 1 or out_end.numel() != N or out_idx.numel() < cap
            or out_vals.numel() < cap):
        raise ValueError("output tensors are too small")
    nm = NORMS[norm] if isinstance(norm, str) else int(norm)
    rc = lib.es_spmm_materialize_transposed(
        _dev_ptr(rowptr, torch.int32, "rowptr"), _dev_ptr(colidx, torch.int32, "colidx"),
        _dev_ptr(vals, torch.float32, "vals"), N, nnz, int(W), m, int(seed) & 0xFFFFFFFFFFFFFFFF, nm,
        _dev_ptr(out_ptr, torch.int32, "out_ptr"), _dev_ptr(out_end, torch.int32, "out_end"),
        _dev_ptr(out_idx, torch.int32, "out_idx"), _dev_ptr(out_vals, torch.float32, "out_vals"),
        _stream_ptr(stream))
    if rc != 0:
        raise EsSpmmError(rc, "es_spmm_materialize_transposed")
    return out_ptr, out_end, out_idx, out_vals


def es_spmm_transpose_graph(rowptr, colidx, vals, stream=None):
    """Transposed graph for es_spmm_backward_pull, built once per graph: a dict of device
    tensors t_ptr [N+1], t_end [N], t_row, t_idx, t_slot, t_vals [nnz], t_pinv [N], plus
    t_rows [2N], the per-call scratch of es_spmm_backward_pull."""
    import torch
    lib = load_library()
    N = rowptr.numel() - 1
    nnz = colidx.numel()
    dev = rowptr.device
    t = {"t_ptr": torch.empty((N + 1,), dtype=torch.int32, device=dev),
         "t_end": torch.empty((N,), dtype=torch.int32, device=dev),
         "t_row": torch.empty((nnz,), dtype=torch.int32, device=dev),
         "t_idx": torch.empty((nnz,), dtype=torch.int32, device=dev),
         "t_slot": torch.empty((nnz,), dtype=torch.int32, device=dev),
         "t_rows": torch.empty((2 * N,), dtype=torch.int32, device=dev),
         "t_vals": torch.empty((nnz,), dtype=torch.float32, device=dev),
         "t_pinv": torch.empty((N,), dtype=torch.int32, device=dev)}
    rc = lib.es_spmm_transpose_graph(
        _dev_ptr(rowptr, torch.int32, "rowptr"), _dev_ptr(colidx, torch.int32, "colidx"),
        _dev_ptr(vals, torch.float32, "vals"), N, nnz, t["t_ptr"].data_ptr() or None,
        t["t_end"].data_ptr() or None, t["t_row"].data_ptr() or None, t["t_idx"].data_ptr() or None,
        t["t_slot"].data_ptr() or None, t["t_vals"].data_ptr() or None, t["t_pinv"].data_ptr() or None,
        _stream_ptr(stream))
    if rc != 0:
        raise EsSpmmError(rc, "es_spmm_transpose_graph")
    return t


def es_spmm_backward_pull(rowptr, t, dY, dX, W: int, mode, seed: int = 0, norm="none",
                          F: Optional[int] = None, stream=None):
    """dX[:, :F] = sample_W(A)^T @ dY[:, :F] as a gather over `t`, the dict
    es_spmm_transpose_graph returned for the same graph; returns dX."""
    import torch
    lib = load_library()
    if dY.dim() != 2 or dX.dim() != 2 or dY.stride(1) != 1 or dX.stride(1) != 1:
        raise ValueError("dY and dX must be 2-D with contiguous columns")
    N = rowptr.numel() - 1
    if dY.shape[0] != N or dX.shape[0] != N:
        raise ValueError("dY and dX need one row per CSR row")
    if F is None:
        F = dY.shape[1]
    ldy = dY.stride(0) if N > 1 else max(dY.shape[1], 1)
    ldx = dX.stride(0) if N > 1 else max(dX.shape[1], 1)
    nm = NORMS[norm] if isinstance(norm, str) else int(norm)
    rc = lib.es_spmm_backward_pull(
        _dev_ptr(rowptr, torch.int32, "rowptr"), _dev_ptr(t["t_ptr"], torch.int32, "t_ptr"),
        _dev_ptr(t["t_row"], torch.int32, "t_row"), _dev_ptr(t["t_idx"], torch.int32, "t_idx"),
        _dev_ptr(t["t_slot"], torch.int32, "t_slot"), _dev_ptr(t["t_vals"], torch.float32, "t_vals"),
        _dev_ptr(t["t_pinv"], torch.int32, "t_pinv"), _dev_ptr(t["t_rows"], torch.int32, "t_rows"),
        _dev_ptr(dY, torch.float32, "dY"), _dev_ptr(dX, torch.float32, "dX"), N, t["t_row"].numel(),
        int(F), int(ldy), int(ldx), int(W), _mode(mode), int(seed) & 0xFFFFFFFFFFFFFFFF, nm,
        _stream_ptr(stream))
    if rc != 0:
        raise EsSpmmError(rc, "es_spmm_backward_pull")
    return dX


def es_spmm_validate_csr(rowptr, colidx, report=None, stream=None):
    """Device-side CSR check; returns the int32[4] report tensor (row-pointer faults,
    column ids out of range, rows with unsorted columns, longest row)."""
    import torch
    lib = load_library()
    N = rowptr.numel() - 1
    if report is None:
        report = torch.empty((4,), dtype=torch.int32, device=rowptr.device)
    rc = lib.es_spmm_validate_csr(_dev_ptr(rowptr, torch.int32, "rowptr"), _dev_ptr(colidx, torch.int32, "colidx"),
                                  N, colidx.numel(), _dev_ptr(report, torch.int32, "report"),
                                  _stream_ptr(stream))
    if rc != 0:
        raise EsSpmmError(rc, "es_spmm_validate_csr")
    return report
