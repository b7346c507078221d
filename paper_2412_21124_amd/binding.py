"""ctypes binding of ``libnormtest.so`` (``include/normtest.h``): argument marshalling only.

Every step of the path runs in the library's HIP kernels.  torch supplies device memory and the
current stream, nothing else.  There is no CPU fallback: if the library cannot be loaded or a call
fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass
from typing import Optional

import torch

from . import build as _build

NT_F32, NT_BF16 = 0, 1
NT_DO_STATS, NT_DO_ADAMW, NT_PARTIAL, NT_WRITE_GBAR, NT_COORD_TEST, NT_ONE_PASS = 1, 2, 4, 8, 16, 32
NT_STATUS_NONFINITE = 1
NT_STATUS_ZERO_GRAD_NORM = 2
NT_STATUS_CLAMPED = 4
NT_STATUS_PARTIAL_ONLY = 8
NT_STATUS_T_SATURATED = 16
NT_STATUS_NO_STATS = 32
NT_STATUS_BAD_RANGE = 64
NT_OK, NT_ERR_BAD_ARG, NT_ERR_UNSUPPORTED, NT_ERR_WORKSPACE_TOO_SMALL, NT_ERR_TOO_LARGE, NT_ERR_HIP_BASE = 0, -1, -2, -3, -4, -1000


class nt_hyper(ctypes.Structure):
    _fields_ = [
        ("lr", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
        ("eps", ctypes.c_double), ("weight_decay", ctypes.c_double), ("eta", ctypes.c_double),
        ("step", ctypes.c_int64), ("b_k", ctypes.c_int64), ("b_max", ctypes.c_int64),
        ("round_to", ctypes.c_int64), ("ddof", ctypes.c_int32), ("flags", ctypes.c_uint32),
    ]


class nt_shard_info(ctypes.Structure):
    _fields_ = [
        ("shard_id", ctypes.c_int32), ("num_shards", ctypes.c_int32),
        ("shard_offset", ctypes.c_int64), ("d_global", ctypes.c_int64),
    ]


class nt_result(ctypes.Structure):
    _fields_ = [
        ("A", ctypes.c_double), ("B", ctypes.c_double), ("C", ctypes.c_double),
        ("A_lo", ctypes.c_double), ("B_lo", ctypes.c_double), ("C_lo", ctypes.c_double),
        ("gbar_sq", ctypes.c_double), ("var_l1", ctypes.c_double), ("T", ctypes.c_double),
        ("clip_coef", ctypes.c_double), ("next_b", ctypes.c_int64), ("coord_fail", ctypes.c_int64),
        ("pass_", ctypes.c_int32), ("status", ctypes.c_uint32), ("coord_max_ratio", ctypes.c_double),
    ]

    def as_dict(self) -> dict:
        d = {k: getattr(self, k) for k, _ in self._fields_}
        d["pass"] = d.pop("pass_")
        return d


RESULT_BYTES = ctypes.sizeof(nt_result)


class nt_layer_stats(ctypes.Structure):
    _fields_ = [
        ("A", ctypes.c_double), ("B", ctypes.c_double), ("C", ctypes.c_double),
        ("gbar_sq", ctypes.c_double), ("var_l1", ctypes.c_double), ("T", ctypes.c_double),
        ("n", ctypes.c_int64), ("coord_fail", ctypes.c_int64), ("pass_", ctypes.c_int32), ("status", ctypes.c_uint32),
        ("coord_max_ratio", ctypes.c_double),
    ]

    def as_dict(self) -> dict:
        d = {k: getattr(self, k) for k, _ in self._fields_}
        d["pass"] = d.pop("pass_")
        return d


LAYER_BYTES = ctypes.sizeof(nt_layer_stats)


class NormtestError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s failed with code %d: %s" % (where, code, normtest_strerror(code)))


_lib = None


def lib(path: Optional[str] = None):
    """The loaded C-ABI library (built on first use if missing).  `path` loads another build of it."""
    global _lib
    if _lib is None or path is not None:
        L = ctypes.CDLL(path if path is not None else _build.ensure_built())
        vp, i64 = ctypes.c_void_p, ctypes.c_int64
        L.normtest_tile_coords.argtypes = [i64]
        L.normtest_tile_coords.restype = i64
        L.normtest_workspace_bytes.argtypes = [i64, i64]
        L.normtest_workspace_bytes.restype = ctypes.c_size_t
        L.normtest_workspace_bytes_for.argtypes = [ctypes.c_int, i64, i64, ctypes.c_uint32]
        L.normtest_workspace_bytes_for.restype = ctypes.c_size_t
        L.normtest_step.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, vp, vp, vp,
                                    ctypes.POINTER(nt_hyper), ctypes.POINTER(nt_shard_info),
                                    vp, ctypes.c_size_t, vp, vp]
        L.normtest_step.restype = ctypes.c_int
        L.normtest_step_static.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, vp, vp, vp,
                                           ctypes.POINTER(nt_hyper), ctypes.POINTER(nt_shard_info), vp, vp]
        L.normtest_step_static.restype = ctypes.c_int
        L.normtest_static_max_coords.argtypes = [i64]
        L.normtest_static_max_coords.restype = i64
        L.normtest_step_rows.argtypes = [vp, ctypes.c_int, i64, i64, vp, vp, vp, vp,
                                         ctypes.POINTER(nt_hyper), ctypes.POINTER(nt_shard_info),
                                         vp, ctypes.c_size_t, vp, vp]
        L.normtest_step_rows.restype = ctypes.c_int
        L.normtest_combine.argtypes = [ctypes.POINTER(nt_result), ctypes.c_int32, i64,
                                       ctypes.POINTER(nt_hyper), ctypes.POINTER(nt_result)]
        L.normtest_combine.restype = ctypes.c_int
        L.normtest_step_clipped.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, vp, vp, vp, ctypes.c_double,
                                            ctypes.POINTER(nt_hyper), ctypes.POINTER(nt_shard_info),
                                            vp, ctypes.c_size_t, vp, vp]
        L.normtest_step_clipped.restype = ctypes.c_int
        L.normtest_layer_stats.argtypes = [vp, ctypes.c_int, ctypes.c_int, i64, i64, i64, vp, ctypes.c_int32, vp, vp, vp]
        L.normtest_layer_stats.restype = ctypes.c_int
        L.normtest_adamw_gbar.argtypes = [vp, i64, vp, vp, vp, ctypes.POINTER(nt_hyper), ctypes.c_double, vp, vp]
        L.normtest_adamw_gbar.restype = ctypes.c_int
        L.normtest_clip_coef.argtypes = [ctypes.c_double, ctypes.c_double]
        L.normtest_clip_coef.restype = ctypes.c_double
        L.normtest_resplit.argtypes = [i64, i64, i64, i64, ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(i64)]
        L.normtest_resplit.restype = ctypes.c_int
        L.normtest_schedule_flags.argtypes = [i64, i64, i64, i64, ctypes.c_uint32]
        L.normtest_schedule_flags.restype = ctypes.c_uint32
        L.normtest_calib_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.normtest_calib_copy.restype = ctypes.c_int
        L.normtest_calib_streams.argtypes = [vp, ctypes.c_size_t, i64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                             ctypes.c_int, i64, vp]
        L.normtest_calib_streams.restype = ctypes.c_int
        L.normtest_strerror.argtypes = [ctypes.c_int]
        L.normtest_strerror.restype = ctypes.c_char_p
        _lib = L
    return _lib


def normtest_strerror(code: int) -> str:
    return lib().normtest_strerror(code).decode()


def normtest_tile_coords(J: int) -> int:
    return int(lib().normtest_tile_coords(J))


def normtest_workspace_bytes(J: int, d: int) -> int:
    return int(lib().normtest_workspace_bytes(J, d))


def normtest_workspace_bytes_for(gdtype: int, J: int, d: int, flags: int) -> int:
    return int(lib().normtest_workspace_bytes_for(gdtype, J, d, flags))


def make_hyper(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, eta=0.1, step=1, b_k=1,
               b_max=0, round_to=1, ddof=1, flags=NT_DO_STATS | NT_DO_ADAMW) -> nt_hyper:
    return nt_hyper(lr, beta1, beta2, eps, weight_decay, eta, step, b_k, b_max, round_to, ddof, flags)


def _gdtype(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return NT_F32
    if t.dtype == torch.bfloat16:
        return NT_BF16
    raise TypeError("gradients must be float32 or bfloat16, got %s" % t.dtype)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _matrix_layout(grads: torch.Tensor, d: Optional[int], where: str):
    """(J, d, ld, device) of a (J, ld) gradient tensor whose rows are the gradient vectors."""
    if grads.dim() != 2 or (grads.shape[1] > 1 and grads.stride(1) != 1):
        raise ValueError("grads must be (J, ld) with a contiguous last axis")
    J = grads.shape[0]
    ld = grads.stride(0) if J > 1 else grads.shape[1]
    d = grads.shape[1] if d is None else d
    if grads.device.type != "cuda":
        raise ValueError("%s needs device tensors; there is no CPU path" % where)
    return J, d, ld, grads.device


def _check_vectors(dev, d: int, required: bool = False, **tensors):
    """w, m, v, gbar: contiguous float32 vectors of at least d elements on the gradients' device."""
    for name, t in tensors.items():
        if t is None and not required:
            continue
        if t is None or t.dtype != torch.float32 or t.device != dev or not t.is_contiguous() or t.numel() < d:
            raise ValueError("%s must be a contiguous float32 tensor of >= d elements on %s" % (name, dev))


def _nbytes(t: torch.Tensor) -> int:
    return t.numel() * t.element_size()


def normtest_step(grads: torch.Tensor, w: Optional[torch.Tensor], m: Optional[torch.Tensor],
                  v: Optional[torch.Tensor], hyper: nt_hyper, *, d: Optional[int] = None,
                  shard: Optional[nt_shard_info] = None, gbar_out: Optional[torch.Tensor] = None,
                  workspace: Optional[torch.Tensor] = None, result: Optional[torch.Tensor] = None,
                  stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Enqueue one step on `stream` (default: torch's current stream) and return the device tensor
    (uint8[sizeof(nt_result)]) that will hold the nt_result; read it with `read_result` after a sync.

    grads: (J, ld) device tensor whose rows are the gradient vectors (last axis contiguous); the first
    d columns are used (default: all).  w, m, v: float32 device vectors of length >= d, updated in place.
    """
    J, d, ld, dev = _matrix_layout(grads, d, "normtest_step")
    _check_vectors(dev, d, w=w, m=m, v=v, gbar_out=gbar_out)
    need = normtest_workspace_bytes_for(_gdtype(grads), J, d, hyper.flags)
    own_workspace = workspace is None
    if own_workspace:
        workspace = torch.empty(max(need, 8), dtype=torch.uint8, device=dev)
    if result is None:
        result = torch.empty(RESULT_BYTES, dtype=torch.uint8, device=dev)
    if stream is None:
        stream = torch.cuda.current_stream(dev)
    with torch.cuda.device(dev):
        rc = lib().normtest_step(_ptr(grads), _gdtype(grads), J, d, ld, _ptr(w), _ptr(m), _ptr(v),
                                 _ptr(gbar_out), ctypes.byref(hyper),
                                 ctypes.byref(shard) if shard is not None else None,
                                 _ptr(workspace), _nbytes(workspace),
                                 _ptr(result), ctypes.c_void_p(stream.cuda_stream))
    if rc != NT_OK:
        raise NormtestError(rc, "normtest_step")
    if own_workspace:
        workspace.record_stream(stream)   # keep the scratch alive until the stream has consumed it
    return result


def normtest_static_max_coords(J: int) -> int:
    return int(lib().normtest_static_max_coords(J))


def normtest_step_static(grads: torch.Tensor, w: Optional[torch.Tensor], m: Optional[torch.Tensor],
                         v: Optional[torch.Tensor], hyper: nt_hyper, result: torch.Tensor, *, d: Optional[int] = None,
                         shard: Optional[nt_shard_info] = None, gbar_out: Optional[torch.Tensor] = None,
                         stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """normtest_step without a workspace (the library's built-in scratch) and without any allocation here:
    the caller passes the device tensor for the nt_result."""
    J, d, ld, dev = _matrix_layout(grads, d, "normtest_step_static")
    _check_vectors(dev, d, w=w, m=m, v=v, gbar_out=gbar_out)
    if result is None or result.device != dev or _nbytes(result) < RESULT_BYTES:
        raise ValueError("result must be a device tensor of at least RESULT_BYTES bytes")
    if stream is None:
        stream = torch.cuda.current_stream(dev)
    with torch.cuda.device(dev):
        rc = lib().normtest_step_static(_ptr(grads), _gdtype(grads), J, d, ld, _ptr(w), _ptr(m), _ptr(v),
                                        _ptr(gbar_out), ctypes.byref(hyper),
                                        ctypes.byref(shard) if shard is not None else None,
                                        _ptr(result), ctypes.c_void_p(stream.cuda_stream))
    if rc != NT_OK:
        raise NormtestError(rc, "normtest_step_static")
    return result


def make_row_table(rows) -> torch.Tensor:
    """Device-resident table of the rows' addresses (int64[J]) for normtest_step_rows.  The caller keeps
    the rows and the table alive until the step has run."""
    dev = rows[0].device
    return torch.tensor([r.data_ptr() for r in rows], dtype=torch.int64, device=dev)


def normtest_step_rows(rows, w: Optional[torch.Tensor], m: Optional[torch.Tensor], v: Optional[torch.Tensor],
                       hyper: nt_hyper, *, d: Optional[int] = None, table: Optional[torch.Tensor] = None,
                       shard: Optional[nt_shard_info] = None, gbar_out: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None, result: Optional[torch.Tensor] = None,
                       stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """normtest_step for J separately allocated gradient rows (a sequence of 1-D device tensors of one dtype)."""
    J = len(rows)
    dev = rows[0].device
    if dev.type != "cuda":
        raise ValueError("normtest_step_rows needs device tensors; there is no CPU path")
    d = min(r.numel() for r in rows) if d is None else d
    for r in rows:
        if r.dtype != rows[0].dtype or r.device != dev or r.dim() != 1 or not r.is_contiguous() or r.numel() < d:
            raise ValueError("rows must be contiguous 1-D tensors of one dtype and >= d elements on %s" % dev)
    _check_vectors(dev, d, w=w, m=m, v=v, gbar_out=gbar_out)
    if table is None:
        table = make_row_table(rows)
    own_workspace = workspace is None
    if own_workspace:
        need = normtest_workspace_bytes_for(_gdtype(rows[0]), J, d, hyper.flags)
        workspace = torch.empty(max(need, 8), dtype=torch.uint8, device=dev)
    if result is None:
        result = torch.empty(RESULT_BYTES, dtype=torch.uint8, device=dev)
    if stream is None:
        stream = torch.cuda.current_stream(dev)
    with torch.cuda.device(dev):
        rc = lib().normtest_step_rows(_ptr(table), _gdtype(rows[0]), J, d, _ptr(w), _ptr(m), _ptr(v), _ptr(gbar_out),
                                      ctypes.byref(hyper), ctypes.byref(shard) if shard is not None else None,
                                      _ptr(workspace), _nbytes(workspace),
                                      _ptr(result), ctypes.c_void_p(stream.cuda_stream))
    if rc != NT_OK:
        raise NormtestError(rc, "normtest_step_rows")
    table.record_stream(stream)
    if own_workspace:
        workspace.record_stream(stream)
    return result


def normtest_step_clipped(grads: torch.Tensor, w: torch.Tensor, m: torch.Tensor, v: torch.Tensor,
                          gbar_buf: torch.Tensor, max_norm: float, hyper: nt_hyper, *, d: Optional[int] = None,
                          shard: Optional[nt_shard_info] = None, workspace: Optional[torch.Tensor] = None,
                          result: Optional[torch.Tensor] = None,
                          stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Two-phase gradient-clipped step (statistics + gbar, then AdamW on the clipped gbar); see normtest_step."""
    J, d, ld, dev = _matrix_layout(grads, d, "normtest_step_clipped")
    _check_vectors(dev, d, required=True, w=w, m=m, v=v, gbar_buf=gbar_buf)
    own_workspace = workspace is None
    if own_workspace:
        need = normtest_workspace_bytes_for(_gdtype(grads), J, d, hyper.flags | NT_WRITE_GBAR)
        workspace = torch.empty(max(need, 8), dtype=torch.uint8, device=dev)
    if result is None:
        result = torch.empty(RESULT_BYTES, dtype=torch.uint8, device=dev)
    if stream is None:
        stream = torch.cuda.current_stream(dev)
    with torch.cuda.device(dev):
        rc = lib().normtest_step_clipped(_ptr(grads), _gdtype(grads), J, d, ld, _ptr(w), _ptr(m), _ptr(v),
                                         _ptr(gbar_buf), float(max_norm), ctypes.byref(hyper),
                                         ctypes.byref(shard) if shard is not None else None,
                                         _ptr(workspace), _nbytes(workspace),
                                         _ptr(result), ctypes.c_void_p(stream.cuda_stream))
    if rc != NT_OK:
        raise NormtestError(rc, "normtest_step_clipped")
    if own_workspace:
        workspace.record_stream(stream)
    return result


def normtest_adamw_gbar(gbar: torch.Tensor, w: torch.Tensor, m: torch.Tensor, v: torch.Tensor, hyper: nt_hyper,
                        grad_scale: float = 1.0, *, d: Optional[int] = None, result: Optional[torch.Tensor] = None,
                        stream: Optional[torch.cuda.Stream] = None) -> None:
    """AdamW on grad_scale (* result.clip_coef) * gbar for a mean gradient already in device memory."""
    d = gbar.numel() if d is None else d
    dev = gbar.device
    if dev.type != "cuda":
        raise ValueError("normtest_adamw_gbar needs device tensors; there is no CPU path")
    _check_vectors(dev, d, required=True, gbar=gbar, w=w, m=m, v=v)
    if stream is None:
        stream = torch.cuda.current_stream(dev)
    with torch.cuda.device(dev):
        rc = lib().normtest_adamw_gbar(_ptr(gbar), d, _ptr(w), _ptr(m), _ptr(v), ctypes.byref(hyper),
                                       float(grad_scale), _ptr(result), ctypes.c_void_p(stream.cuda_stream))
    if rc != NT_OK:
        raise NormtestError(rc, "normtest_adamw_gbar")


def normtest_layer_stats(grads, layer_offsets: torch.Tensor, workspace: torch.Tensor, *, d: Optional[int] = None,
                         table: Optional[torch.Tensor] = None, layers: Optional[torch.Tensor] = None,
                         stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Enqueue the per-layer table after a step that used `workspace` on the same stream.  grads: the (J, ld)
    tensor of that step, or the sequence of rows given to normtest_step_rows (then `table` may carry the
    address table already made).  layer_offsets: int64 device tensor of L+1 ascending offsets.  Returns the
    device tensor (uint8[L * sizeof(nt_layer_stats)]); read it with `read_layers` after a sync."""
    rows = None if isinstance(grads, torch.Tensor) else list(grads)
    first = grads if rows is None else rows[0]
    dev = first.device
    if dev.type != "cuda":
        raise ValueError("normtest_layer_stats needs device tensors; there is no CPU path")
    if rows is None:
        J, d, ld, _ = _matrix_layout(grads, d, "normtest_layer_stats")
        gptr = _ptr(grads)
    else:
        J = len(rows)
        d = min(r.numel() for r in rows) if d is None else d
        ld = d
        if table is None:
            table = make_row_table(rows)
        gptr = _ptr(table)
    if (layer_offsets.dtype != torch.int64 or layer_offsets.device != dev or layer_offsets.dim() != 1
            or not layer_offsets.is_contiguous() or layer_offsets.numel() < 2):
        raise ValueError("layer_offsets must be a contiguous int64 device vector of L+1 >= 2 entries")
    L = layer_offsets.numel() - 1
    if workspace.device != dev or _nbytes(workspace) < normtest_workspace_bytes_for(_gdtype(first), J, d, NT_DO_STATS):
        raise ValueError("workspace must be the device workspace of the preceding step")
    if layers is None:
        layers = torch.empty(L * LAYER_BYTES, dtype=torch.uint8, device=dev)
    elif _nbytes(layers) < L * LAYER_BYTES:
        raise ValueError("layers must hold L * sizeof(nt_layer_stats) bytes")
    if stream is None:
        stream = torch.cuda.current_stream(dev)
    with torch.cuda.device(dev):
        rc = lib().normtest_layer_stats(gptr, 0 if rows is None else 1, _gdtype(first), J, d, ld, _ptr(layer_offsets), L,
                                        _ptr(workspace), _ptr(layers), ctypes.c_void_p(stream.cuda_stream))
    if rc != NT_OK:
        raise NormtestError(rc, "normtest_layer_stats")
    if table is not None:
        table.record_stream(stream)
    return layers


def read_layers(layers: torch.Tensor, L: Optional[int] = None):
    """Synchronising read of a device nt_layer_stats array: a list of nt_layer_stats."""
    host = layers.cpu().numpy().tobytes()
    L = len(host) // LAYER_BYTES if L is None else L
    return [nt_layer_stats.from_buffer_copy(host, l * LAYER_BYTES) for l in range(L)]


def normtest_clip_coef(gbar_sq: float, max_norm: float) -> float:
    return float(lib().normtest_clip_coef(gbar_sq, max_norm))


def normtest_resplit(b: int, J: int, accum_base: int, micro_max: int):
    """(micro_batch, accumulation_steps, global_batch) for a target global batch size b."""
    micro, accum, glob = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    rc = lib().normtest_resplit(b, J, accum_base, micro_max, ctypes.byref(micro), ctypes.byref(accum), ctypes.byref(glob))
    if rc != NT_OK:
        raise NormtestError(rc, "normtest_resplit")
    return micro.value, accum.value, glob.value


def normtest_schedule_flags(step: int, test_interval: int, b_k: int, b_max: int, flags: int) -> int:
    return int(lib().normtest_schedule_flags(step, test_interval, b_k, b_max, flags))


def read_result(result: torch.Tensor) -> nt_result:
    """Synchronising read of the device nt_result."""
    host = result.cpu().numpy().tobytes()
    return nt_result.from_buffer_copy(host)


def normtest_combine(partials, J: int, hyper: nt_hyper) -> nt_result:
    arr = (nt_result * len(partials))(*partials)
    out = nt_result()
    rc = lib().normtest_combine(arr, len(partials), J, ctypes.byref(hyper), ctypes.byref(out))
    if rc != NT_OK:
        raise NormtestError(rc, "normtest_combine")
    return out


def normtest_calib_copy(dst: torch.Tensor, src: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() < nbytes:
        raise ValueError("dst smaller than src")
    if stream is None:
        stream = torch.cuda.current_stream(src.device)
    with torch.cuda.device(src.device):
        rc = lib().normtest_calib_copy(_ptr(dst), _ptr(src), nbytes, ctypes.c_void_p(stream.cuda_stream))
    if rc != NT_OK:
        raise NormtestError(rc, "normtest_calib_copy")


def calib_streams_bytes(coords: int, row_reads: int, reads: int, writes: int) -> int:
    """Scratch bytes normtest_calib_streams needs (the rule stated in the header)."""
    r2 = (coords * 2 + 255) // 256 * 256
    r4 = (coords * 4 + 255) // 256 * 256
    return row_reads * r2 + (reads + writes) * r4 + 16


def normtest_calib_streams(buf: torch.Tensor, coords: int, row_reads: int, reads: int, writes: int, rmw: bool = False,
                           launch_coords: int = 0, stream: Optional[torch.cuda.Stream] = None) -> None:
    if stream is None:
        stream = torch.cuda.current_stream(buf.device)
    with torch.cuda.device(buf.device):
        rc = lib().normtest_calib_streams(_ptr(buf), buf.numel() * buf.element_size(), coords, row_reads, reads, writes,
                                          1 if rmw else 0, launch_coords, ctypes.c_void_p(stream.cuda_stream))
    if rc != NT_OK:
        raise NormtestError(rc, "normtest_calib_streams")
