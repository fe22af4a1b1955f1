"""ctypes marshalling for libgta.so: argument packing only, no arithmetic."""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, c_char, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None
NUM_CLASSES = 33
GTA_F32, GTA_BF16 = 0, 1


class GtaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"gta status {status}: {message}")
        self.status = status


class _PlanOpts(Structure):
    _fields_ = [("pack_max_deg", c_int32), ("wave_max_deg", c_int32), ("hub_chunk", c_int32),
                ("validate", c_int32), ("keep_dz_min_nnz", c_int32)]


class _PlanInfo(Structure):
    _fields_ = [("n_dst", c_int64), ("n_src", c_int64), ("nnz", c_int64),
                ("pack_max_deg", c_int32), ("wave_max_deg", c_int32), ("hub_chunk", c_int32),
                ("n_chunked", c_int64 * 2), ("n_hub", c_int64 * 2), ("n_chunks", c_int64 * 2)]


class _AgpSample(Structure):
    _fields_ = [("strategy", c_int32), ("gpus", c_int32), ("beta", ctypes.c_double)]


class _LaunchRecord(Structure):
    _fields_ = [("name", c_char * 40), ("ms", c_float), ("rows", c_int64), ("entries", c_int64)]


def lib_path() -> str:
    return os.path.join(_HERE, "libgta.so")


def load_library():
    """Loads libgta.so; builds it first only when no built library exists.  Never falls back."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(path)
    vp = c_void_p
    lib.gta_plan_workspace_bytes.restype = c_size_t
    lib.gta_plan_workspace_bytes.argtypes = [c_int64, c_int64, c_int64, POINTER(_PlanOpts)]
    lib.gta_plan_create.restype = c_int
    lib.gta_plan_create.argtypes = [POINTER(vp), vp, vp, c_int64, c_int64, c_int64, POINTER(_PlanOpts),
                                    vp, c_size_t, vp]
    lib.gta_plan_retained_bytes.restype = c_size_t
    lib.gta_plan_retained_bytes.argtypes = [c_int64, c_int64, c_int64, POINTER(_PlanOpts)]
    lib.gta_plan_compact.restype = c_int
    lib.gta_plan_compact.argtypes = [vp, vp, c_size_t, vp]
    lib.gta_plan_destroy.restype = None
    lib.gta_plan_destroy.argtypes = [vp]
    lib.gta_plan_get_info.restype = c_int
    lib.gta_plan_get_info.argtypes = [vp, POINTER(_PlanInfo)]
    lib.gta_plan_export_bins.restype = c_int
    lib.gta_plan_export_bins.argtypes = [vp, c_int, vp, vp, vp, vp]
    lib.gta_plan_export_transpose.restype = c_int
    lib.gta_plan_export_transpose.argtypes = [vp, vp, vp, vp]
    lib.gta_attn_scratch_bytes.restype = c_size_t
    lib.gta_attn_scratch_bytes.argtypes = [vp, c_int, c_int, c_int]
    lib.gta_attn_scratch_bytes_min.restype = c_size_t
    lib.gta_attn_scratch_bytes_min.argtypes = [vp, c_int, c_int, c_int]
    lib.gta_attn_fwd.restype = c_int
    lib.gta_attn_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, c_int64, c_int64, c_int, c_int, c_int,
                                 c_float, vp, c_size_t, vp]
    lib.gta_attn_fwd_noalloc.restype = c_int
    lib.gta_attn_fwd_noalloc.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, c_int64, c_int64, c_int, c_int, c_int,
                                         c_float, vp]
    lib.gta_attn_bwd.restype = c_int
    lib.gta_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, c_int64, c_int64, c_int,
                                 c_int, c_int, c_float, vp, c_size_t, vp]
    lib.gta_attn_fwd_halo.restype = c_int
    lib.gta_attn_fwd_halo.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, c_int64, vp, vp, c_int64, c_int64, c_int,
                                      c_int, c_int, c_float, vp, c_size_t, vp]
    lib.gta_attn_bwd_halo.restype = c_int
    lib.gta_attn_bwd_halo.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, c_int64, vp, vp, vp, vp, vp, vp, vp, vp,
                                      c_int64, c_int64, c_int, c_int, c_int, c_float, vp, c_size_t, vp]
    lib.gta_attn_merge.restype = c_int
    lib.gta_attn_merge.argtypes = [vp, vp, vp, vp, vp, vp, c_int64, c_int, c_int, c_int, vp]
    lib.gta_sddmm.restype = c_int
    lib.gta_sddmm.argtypes = [vp, vp, vp, vp, vp, vp, c_int64, c_int64, c_int, c_int, c_int, vp, c_size_t, vp]
    lib.gta_edge_softmax.restype = c_int
    lib.gta_edge_softmax.argtypes = [vp, vp, vp, vp, vp, c_int64, c_int, c_float, vp]
    lib.gta_edge_softmax_bwd.restype = c_int
    lib.gta_edge_softmax_bwd.argtypes = [vp, vp, vp, vp, vp, c_int64, c_int, c_float, vp]
    lib.gta_spmm.restype = c_int
    lib.gta_spmm.argtypes = [vp, vp, vp, vp, vp, vp, c_int64, c_int64, c_int, c_int, c_int, c_int, vp,
                             c_size_t, vp]
    for fn in (lib.gta_head_split, lib.gta_head_merge):
        fn.restype = c_int
        fn.argtypes = [vp, vp, c_int64, c_int, c_int, c_int, c_int, vp]
    lib.gta_linear.restype = c_int
    lib.gta_linear.argtypes = [vp, vp, vp, vp, c_int64, c_int, c_int, c_int, c_int, vp]
    lib.gta_linear_dw_scratch_bytes.restype = c_size_t
    lib.gta_linear_dw_scratch_bytes.argtypes = [c_int64, c_int, c_int]
    lib.gta_linear_dw.restype = c_int
    lib.gta_linear_dw.argtypes = [vp, vp, vp, c_int64, c_int, c_int, c_int, vp, c_size_t, vp]
    lib.gta_linear_dw_group_scratch_bytes.restype = c_size_t
    lib.gta_linear_dw_group_scratch_bytes.argtypes = [c_int64, c_int, c_int, c_int]
    lib.gta_linear_dw_group.restype = c_int
    lib.gta_linear_dw_group.argtypes = [vp, vp, vp, c_int, c_int64, c_int, c_int, c_int, vp, c_size_t, vp]
    lib.gta_linear_group_scratch_bytes.restype = c_size_t
    lib.gta_linear_group_scratch_bytes.argtypes = [c_int, c_int, c_int]
    lib.gta_linear_group.restype = c_int
    lib.gta_linear_group.argtypes = [vp, c_int, vp, c_int, vp, vp, c_int64, c_int, c_int, c_int, vp, c_size_t, vp]
    lib.gta_sga_layer_scratch_bytes.restype = c_size_t
    lib.gta_sga_layer_scratch_bytes.argtypes = [vp, c_int, c_int, c_int]
    lib.gta_sga_layer_fwd.restype = c_int
    lib.gta_sga_layer_fwd.argtypes = [vp] * 14 + [c_int64, c_int, c_int, c_int, c_float, vp, c_size_t, vp]
    lib.gta_sga_layer_bwd.restype = c_int
    lib.gta_sga_layer_bwd.argtypes = [vp] * 22 + [c_int64, c_int, c_int, c_int, c_float, vp, c_size_t, vp]
    lib.gta_agp_select.restype = c_int
    lib.gta_agp_select.argtypes = [ctypes.c_double, c_int64, POINTER(_AgpSample), c_int, c_int, POINTER(c_int),
                                   POINTER(c_int), POINTER(ctypes.c_double)]
    lib.gta_stream_probe.restype = c_int
    lib.gta_stream_probe.argtypes = [c_int, vp, vp, vp, c_size_t, vp]
    lib.gta_profile_enable.restype = c_int
    lib.gta_profile_enable.argtypes = [c_int]
    lib.gta_profile_read.restype = c_int
    lib.gta_profile_read.argtypes = [POINTER(_LaunchRecord), c_int, c_int]
    lib.gta_last_error.restype = c_char_p
    lib.gta_version.restype = c_char_p
    _LIB = lib
    return lib


def _check(status: int):
    if status != 0:
        raise GtaError(status, load_library().gta_last_error().decode())


def _ptr(t):
    return None if t is None else c_void_p(t.data_ptr())


def _stream():
    return c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return GTA_F32
    if t.dtype == torch.bfloat16:
        return GTA_BF16
    raise GtaError(2, f"unsupported tensor dtype {t.dtype}")


def _need(name: str, t, shape, dtype, device):
    """Raises GtaError unless t is a contiguous tensor of exactly this shape, dtype and device.  The C
    ABI takes raw pointers and cannot see a mismatch, so every tensor is checked before a call."""
    if not isinstance(t, torch.Tensor):
        raise GtaError(1, f"{name}: expected a tensor, got {type(t).__name__}")
    if t.device != device:
        raise GtaError(1, f"{name}: on {t.device}, expected {device}")
    if t.dtype != dtype:
        raise GtaError(1, f"{name}: dtype {t.dtype}, expected {dtype}")
    if tuple(t.shape) != tuple(shape):
        raise GtaError(1, f"{name}: shape {tuple(t.shape)}, expected {tuple(shape)}")
    if not t.is_contiguous():
        raise GtaError(1, f"{name}: must be contiguous")


def _need3(name: str, t):
    if not isinstance(t, torch.Tensor) or t.dim() != 3:
        raise GtaError(1, f"{name}: expected a tensor [rows, heads, head_dim]")
    return tuple(t.shape)


def _need_all(device, dtype, **named):
    """named: name=(tensor, shape); every tensor must have the given dtype, shape and device."""
    for name, (t, shape) in named.items():
        _need(name, t, shape, dtype, device)


def gta_version() -> str:
    return load_library().gta_version().decode()


class Plan:
    """Owns the device workspace of a gta_plan and keeps the graph tensors alive."""

    def __init__(self, handle, workspace, indptr, indices, n_dst, n_src):
        self.handle, self.workspace = handle, workspace
        self.indptr, self.indices, self.n_dst, self.n_src = indptr, indices, n_dst, n_src
        self._scratch = {}

    def __del__(self):
        if getattr(self, "handle", None):
            load_library().gta_plan_destroy(self.handle)
            self.handle = None

    @property
    def nnz(self) -> int:
        return int(self.info().nnz)

    def info(self) -> _PlanInfo:
        info = _PlanInfo()
        _check(load_library().gta_plan_get_info(self.handle, ctypes.byref(info)))
        return info

    def export_bins(self, side: int) -> dict:
        info = self.info()
        n_rows = self.n_dst if side == 0 else self.n_src
        bin_rows = np.empty(n_rows, dtype=np.int32)
        bin_off = np.empty(NUM_CLASSES + 1, dtype=np.int64)
        chunk_ptr = np.empty(info.n_chunked[side] + 1, dtype=np.int32)
        chunks = np.empty((info.n_chunks[side], 4), dtype=np.int32)
        _check(load_library().gta_plan_export_bins(self.handle, side, bin_rows.ctypes.data, bin_off.ctypes.data,
                                                   chunk_ptr.ctypes.data, chunks.ctypes.data))
        return dict(bin_rows=bin_rows, bin_off=bin_off, chunk_ptr=chunk_ptr, chunks=chunks,
                    n_chunked=int(info.n_chunked[side]), n_hub=int(info.n_hub[side]))

    def export_transpose(self) -> dict:
        info = self.info()
        t_indptr = np.empty(self.n_src + 1, dtype=np.int64)
        t_indices = np.empty(info.nnz, dtype=np.int32)
        t_eid = np.empty(info.nnz, dtype=np.int32)
        _check(load_library().gta_plan_export_transpose(self.handle, t_indptr.ctypes.data,
                                                        t_indices.ctypes.data, t_eid.ctypes.data))
        return dict(t_indptr=t_indptr, t_indices=t_indices, t_eid=t_eid)

    def scratch(self, heads: int, head_dim: int, dtype_code: int, lean: bool = False) -> torch.Tensor:
        key = (heads, head_dim, dtype_code, lean)
        if key not in self._scratch:
            nbytes = gta_attn_scratch_bytes(self, heads, head_dim, dtype_code, lean)
            if nbytes == 0:
                raise GtaError(2, "unsupported shape for scratch query")
            self._scratch[key] = torch.empty(nbytes, dtype=torch.uint8, device=self.indptr.device)
        return self._scratch[key]


def gta_plan_create(indptr: torch.Tensor, indices: torch.Tensor, n_src: int, pack_max_deg=0,
                    wave_max_deg=0, hub_chunk=0, validate=True, keep_dz_min_nnz=0, compact=True) -> Plan:
    """The plan is built once per graph, so the CSR arrays are checked on the device by default
    (validate=True): the kernels that use the plan do not bounds-check the indices.  compact=True
    moves the plan into a buffer of just the size it keeps using and drops the build workspace."""
    lib = load_library()
    if not isinstance(indptr, torch.Tensor) or not isinstance(indices, torch.Tensor):
        raise GtaError(1, "indptr and indices must be tensors")
    if indptr.dtype != torch.int64 or indices.dtype != torch.int32:
        raise GtaError(1, "indptr must be int64 and indices int32")
    if indptr.dim() != 1 or indices.dim() != 1 or indptr.numel() < 1:
        raise GtaError(1, "indptr [n_dst + 1] and indices [nnz] must be one-dimensional")
    if not (indptr.is_cuda and indices.is_cuda and indptr.is_contiguous() and indices.is_contiguous()):
        raise GtaError(1, "graph tensors must be contiguous device tensors")
    if indptr.device != indices.device:
        raise GtaError(1, "indptr and indices are on different devices")
    n_dst = indptr.numel() - 1
    nnz = indices.numel()
    opts = _PlanOpts(pack_max_deg, wave_max_deg, hub_chunk, int(bool(validate)), keep_dz_min_nnz)
    nbytes = lib.gta_plan_workspace_bytes(n_dst, n_src, nnz, ctypes.byref(opts))
    if nbytes == 0:
        raise GtaError(1, "bad sizes or plan options")
    workspace = torch.empty(nbytes, dtype=torch.uint8, device=indptr.device)
    handle = c_void_p()
    _check(lib.gta_plan_create(ctypes.byref(handle), _ptr(indptr), _ptr(indices), n_dst, n_src, nnz,
                               ctypes.byref(opts), _ptr(workspace), nbytes, _stream()))
    if compact:
        keep = lib.gta_plan_retained_bytes(n_dst, n_src, nnz, ctypes.byref(opts))
        small = torch.empty(max(keep, 256), dtype=torch.uint8, device=indptr.device)
        status = lib.gta_plan_compact(handle, _ptr(small), small.numel(), _stream())
        if status != 0:
            lib.gta_plan_destroy(handle)
            _check(status)
        workspace = small
    return Plan(handle, workspace, indptr, indices, n_dst, n_src)


def gta_attn_scratch_bytes(plan: Plan, heads: int, head_dim: int, dtype_code: int, lean: bool = False) -> int:
    """Recommended scratch size, or with lean=True the smallest accepted one."""
    lib = load_library()
    fn = lib.gta_attn_scratch_bytes_min if lean else lib.gta_attn_scratch_bytes
    return int(fn(plan.handle, heads, head_dim, dtype_code))


def _attn_shapes(plan: Plan, Q, n_src=None):
    """(n_dst, heads, head_dim), dtype code, device and the [n_src, H, D] shape, checked against the plan."""
    n_dst, heads, head_dim = _need3("Q", Q)
    if n_dst != plan.n_dst:
        raise GtaError(1, f"Q has {n_dst} rows, the plan {plan.n_dst}")
    n_src = plan.n_src if n_src is None else n_src
    if n_src != plan.n_src:
        raise GtaError(1, f"K / V have {n_src} rows in total, the plan {plan.n_src}")
    return (n_dst, heads, head_dim), _dtype_code(Q), plan.indptr.device, (n_src, heads, head_dim)


def gta_attn_fwd(plan: Plan, Q, K, V, scale: float = 0.0, out=None, lse=None):
    """out [n_dst,H,D] (dtype of Q) and lse [n_dst,H] float32."""
    qs, code, dev, ks = _attn_shapes(plan, Q)
    n_dst, heads, head_dim = qs
    if out is None:
        out = torch.empty(qs, dtype=Q.dtype, device=dev)
    if lse is None:
        lse = torch.empty((n_dst, heads), dtype=torch.float32, device=dev)
    _need_all(dev, Q.dtype, Q=(Q, qs), K=(K, ks), V=(V, ks), out=(out, qs))
    _need("lse", lse, (n_dst, heads), torch.float32, dev)
    scratch = plan.scratch(heads, head_dim, code)
    _check(load_library().gta_attn_fwd(plan.handle, _ptr(plan.indptr), _ptr(plan.indices), _ptr(Q), _ptr(K),
                                       _ptr(V), _ptr(out), _ptr(lse), n_dst, plan.n_src, heads, head_dim,
                                       code, scale, _ptr(scratch), scratch.numel(), _stream()))
    return out, lse


def gta_attn_fwd_noalloc(plan: Plan, Q, K, V, out, lse, scale: float = 0.0):
    """gta_attn_fwd without any allocation: out [n_dst,H,D] and lse [n_dst,H] must be given, and the
    partial results of split rows go to the library's built-in device array."""
    qs, code, dev, ks = _attn_shapes(plan, Q)
    n_dst, heads, head_dim = qs
    _need_all(dev, Q.dtype, Q=(Q, qs), K=(K, ks), V=(V, ks), out=(out, qs))
    _need("lse", lse, (n_dst, heads), torch.float32, dev)
    _check(load_library().gta_attn_fwd_noalloc(plan.handle, _ptr(plan.indptr), _ptr(plan.indices), _ptr(Q),
                                               _ptr(K), _ptr(V), _ptr(out), _ptr(lse), n_dst, plan.n_src, heads,
                                               head_dim, code, scale, _stream()))
    return out, lse


def gta_attn_bwd(plan: Plan, Q, K, V, out, lse, dOut, scale: float = 0.0, dQ=None, dK=None, dV=None,
                 lean_scratch: bool = False):
    """lean_scratch=True passes the minimum scratch, which selects the backward form that keeps
    nothing per stored entry."""
    qs, code, dev, ks = _attn_shapes(plan, Q)
    n_dst, heads, head_dim = qs
    dQ = torch.empty(qs, dtype=Q.dtype, device=dev) if dQ is None else dQ
    dK = torch.empty(ks, dtype=Q.dtype, device=dev) if dK is None else dK
    dV = torch.empty(ks, dtype=Q.dtype, device=dev) if dV is None else dV
    _need_all(dev, Q.dtype, Q=(Q, qs), K=(K, ks), V=(V, ks), out=(out, qs), dOut=(dOut, qs), dQ=(dQ, qs),
              dK=(dK, ks), dV=(dV, ks))
    _need("lse", lse, (n_dst, heads), torch.float32, dev)
    scratch = plan.scratch(heads, head_dim, code, lean_scratch)
    _check(load_library().gta_attn_bwd(plan.handle, _ptr(plan.indptr), _ptr(plan.indices), _ptr(Q), _ptr(K),
                                       _ptr(V), _ptr(out), _ptr(lse), _ptr(dOut), _ptr(dQ), _ptr(dK), _ptr(dV),
                                       n_dst, plan.n_src, heads, head_dim, code, scale, _ptr(scratch),
                                       scratch.numel(), _stream()))
    return dQ, dK, dV


def _halo_rows(K_local, K_halo):
    n_local = _need3("K_local", K_local)[0]
    return n_local, n_local + (0 if K_halo is None else _need3("K_halo", K_halo)[0])


def gta_attn_fwd_halo(plan: Plan, Q, K_local, V_local, K_halo, V_halo, scale: float = 0.0, out=None, lse=None):
    """gta_attn_fwd with K / V given as the owned rows and a separate tensor of halo rows."""
    n_local, n_src = _halo_rows(K_local, K_halo)
    qs, code, dev, _ = _attn_shapes(plan, Q, n_src)
    n_dst, heads, head_dim = qs
    if out is None:
        out = torch.empty(qs, dtype=Q.dtype, device=dev)
    if lse is None:
        lse = torch.empty((n_dst, heads), dtype=torch.float32, device=dev)
    ls, hs = (n_local, heads, head_dim), (n_src - n_local, heads, head_dim)
    _need_all(dev, Q.dtype, Q=(Q, qs), K_local=(K_local, ls), V_local=(V_local, ls), out=(out, qs))
    if n_src > n_local:
        _need_all(dev, Q.dtype, K_halo=(K_halo, hs), V_halo=(V_halo, hs))
    _need("lse", lse, (n_dst, heads), torch.float32, dev)
    scratch = plan.scratch(heads, head_dim, code)
    _check(load_library().gta_attn_fwd_halo(plan.handle, _ptr(plan.indptr), _ptr(plan.indices), _ptr(Q),
                                            _ptr(K_local), _ptr(V_local), _ptr(K_halo), _ptr(V_halo), n_local,
                                            _ptr(out), _ptr(lse), n_dst, n_src, heads, head_dim, code, scale,
                                            _ptr(scratch), scratch.numel(), _stream()))
    return out, lse


def gta_attn_bwd_halo(plan: Plan, Q, K_local, V_local, K_halo, V_halo, out, lse, dOut, scale: float = 0.0,
                      lean_scratch: bool = False):
    """gta_attn_bwd with K / V, dK / dV as owned rows plus halo rows; returns dQ, dK_local, dV_local,
    dK_halo, dV_halo."""
    n_local, n_src = _halo_rows(K_local, K_halo)
    qs, code, dev, _ = _attn_shapes(plan, Q, n_src)
    n_dst, heads, head_dim = qs
    ls, hs = (n_local, heads, head_dim), (n_src - n_local, heads, head_dim)
    _need_all(dev, Q.dtype, Q=(Q, qs), K_local=(K_local, ls), V_local=(V_local, ls), out=(out, qs),
              dOut=(dOut, qs))
    if n_src > n_local:
        _need_all(dev, Q.dtype, K_halo=(K_halo, hs), V_halo=(V_halo, hs))
    _need("lse", lse, (n_dst, heads), torch.float32, dev)
    dQ = torch.empty(qs, dtype=Q.dtype, device=dev)
    dK_local, dV_local = torch.empty_like(K_local), torch.empty_like(V_local)
    dK_halo = None if n_src == n_local else torch.empty_like(K_halo)
    dV_halo = None if n_src == n_local else torch.empty_like(V_halo)
    scratch = plan.scratch(heads, head_dim, code, lean_scratch)
    _check(load_library().gta_attn_bwd_halo(plan.handle, _ptr(plan.indptr), _ptr(plan.indices), _ptr(Q),
                                            _ptr(K_local), _ptr(V_local), _ptr(K_halo), _ptr(V_halo), n_local,
                                            _ptr(out), _ptr(lse), _ptr(dOut), _ptr(dQ), _ptr(dK_local),
                                            _ptr(dV_local), _ptr(dK_halo), _ptr(dV_halo), n_dst, n_src, heads,
                                            head_dim, code, scale, _ptr(scratch), scratch.numel(), _stream()))
    return dQ, dK_local, dV_local, dK_halo, dV_halo


def gta_attn_merge(out_a, lse_a, out_b, lse_b, out=None, lse=None):
    """Attention over the union of two disjoint entry sets from the two partial (out, lse) results."""
    shape = _need3("out_a", out_a)
    n_rows, heads, head_dim = shape
    dev = out_a.device
    if out is None:
        out = torch.empty_like(out_a)
    if lse is None:
        lse = torch.empty((n_rows, heads), dtype=torch.float32, device=dev)
    _need_all(dev, out_a.dtype, out_a=(out_a, shape), out_b=(out_b, shape), out=(out, shape))
    _need_all(dev, torch.float32, lse_a=(lse_a, (n_rows, heads)), lse_b=(lse_b, (n_rows, heads)),
              lse=(lse, (n_rows, heads)))
    _check(load_library().gta_attn_merge(_ptr(out_a), _ptr(lse_a), _ptr(out_b), _ptr(lse_b), _ptr(out), _ptr(lse),
                                         n_rows, heads, head_dim, _dtype_code(out_a), _stream()))
    return out, lse


def gta_sddmm(plan: Plan, X, Y, Z=None):
    """Z [nnz,H] float32 = per-entry, per-head dot products of X[dst] and Y[src]."""
    qs, code, dev, ks = _attn_shapes(plan, X)
    n_dst, heads, head_dim = qs
    nnz = plan.indices.numel()
    if Z is None:
        Z = torch.empty((nnz, heads), dtype=torch.float32, device=dev)
    _need_all(dev, X.dtype, X=(X, qs), Y=(Y, ks))
    _need("Z", Z, (nnz, heads), torch.float32, dev)
    scratch = plan.scratch(heads, head_dim, code)
    _check(load_library().gta_sddmm(plan.handle, _ptr(plan.indptr), _ptr(plan.indices), _ptr(X), _ptr(Y), _ptr(Z),
                                    n_dst, plan.n_src, heads, head_dim, code, _ptr(scratch), scratch.numel(),
                                    _stream()))
    return Z


def _entry_matrix(plan: Plan, name: str, t):
    """A float32 [nnz, heads] matrix of per-entry values; returns heads."""
    if not isinstance(t, torch.Tensor) or t.dim() != 2:
        raise GtaError(1, f"{name}: expected a tensor [nnz, heads]")
    _need(name, t, (plan.indices.numel(), t.shape[1]), torch.float32, plan.indptr.device)
    return t.shape[1]


def gta_edge_softmax(plan: Plan, Z, scale: float, U=None, lse=None):
    heads = _entry_matrix(plan, "Z", Z)
    U = torch.empty_like(Z) if U is None else U
    if lse is None:
        lse = torch.empty((plan.n_dst, heads), dtype=torch.float32, device=Z.device)
    _need("U", U, Z.shape, torch.float32, Z.device)
    _need("lse", lse, (plan.n_dst, heads), torch.float32, Z.device)
    _check(load_library().gta_edge_softmax(plan.handle, _ptr(plan.indptr), _ptr(Z), _ptr(U), _ptr(lse),
                                           plan.n_dst, heads, scale, _stream()))
    return U, lse


def gta_edge_softmax_bwd(plan: Plan, U, dU, scale: float, dZ=None):
    heads = _entry_matrix(plan, "U", U)
    dZ = torch.empty_like(U) if dZ is None else dZ
    _need("dU", dU, U.shape, torch.float32, U.device)
    _need("dZ", dZ, U.shape, torch.float32, U.device)
    _check(load_library().gta_edge_softmax_bwd(plan.handle, _ptr(plan.indptr), _ptr(U), _ptr(dU), _ptr(dZ),
                                               plan.n_dst, heads, scale, _stream()))
    return dZ


def gta_spmm(plan: Plan, W, X, transposed: bool = False, Y=None):
    """transposed=False: Y[dst] = sum W[e] X[src];  transposed=True: Y[src] = sum W[e] X[dst]."""
    _, heads, head_dim = _need3("X", X)
    code = _dtype_code(X)
    dev = plan.indptr.device
    rows_in = plan.n_dst if transposed else plan.n_src
    rows_out = plan.n_src if transposed else plan.n_dst
    if Y is None:
        Y = torch.empty((rows_out, heads, head_dim), dtype=X.dtype, device=dev)
    _need_all(dev, X.dtype, X=(X, (rows_in, heads, head_dim)), Y=(Y, (rows_out, heads, head_dim)))
    _need("W", W, (plan.indices.numel(), heads), torch.float32, dev)
    scratch = plan.scratch(heads, head_dim, code)
    _check(load_library().gta_spmm(plan.handle, _ptr(plan.indptr), _ptr(plan.indices), _ptr(W), _ptr(X), _ptr(Y),
                                   plan.n_dst, plan.n_src, heads, head_dim, code, int(bool(transposed)),
                                   _ptr(scratch), scratch.numel(), _stream()))
    return Y


def _need2(name: str, t):
    if not isinstance(t, torch.Tensor) or t.dim() != 2:
        raise GtaError(1, f"{name}: expected a two-dimensional tensor")
    return tuple(t.shape)


def gta_linear(X, W, C=None, trans_w: bool = False, Y=None):
    """Y = X @ W (+ C) with W [d_in, d_out], or Y = X @ W.T (+ C) with W [d_out, d_in] when trans_w."""
    n, d_in = _need2("X", X)
    ws = _need2("W", W)
    d_out = ws[0] if trans_w else ws[1]
    dev = X.device
    if Y is None:
        Y = torch.empty((n, d_out), dtype=X.dtype, device=dev)
    _need_all(dev, X.dtype, X=(X, (n, d_in)), W=(W, (d_out, d_in) if trans_w else (d_in, d_out)), Y=(Y, (n, d_out)))
    if C is not None:
        _need("C", C, (n, d_out), X.dtype, dev)
    _check(load_library().gta_linear(_ptr(X), _ptr(W), _ptr(C), _ptr(Y), n, d_in, d_out, _dtype_code(X),
                                     int(bool(trans_w)), _stream()))
    return Y


def gta_linear_dw(X, dY, dW=None):
    """dW [d_in, d_out] float32 = X.T @ dY."""
    n, d_in = _need2("X", X)
    d_out = _need2("dY", dY)[1]
    dev = X.device
    lib = load_library()
    if dW is None:
        dW = torch.empty((d_in, d_out), dtype=torch.float32, device=dev)
    _need_all(dev, X.dtype, X=(X, (n, d_in)), dY=(dY, (n, d_out)))
    _need("dW", dW, (d_in, d_out), torch.float32, dev)
    nbytes = lib.gta_linear_dw_scratch_bytes(n, d_in, d_out)
    scratch = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
    _check(lib.gta_linear_dw(_ptr(X), _ptr(dY), _ptr(dW), n, d_in, d_out, _dtype_code(X), _ptr(scratch),
                             scratch.numel(), _stream()))
    return dW


def gta_linear_dw_group(Xs, dYs, dWs=None):
    """dWs[k] [d_in, d_out] float32 = Xs[k].T @ dYs[k] for 1 to 4 products of one shape (one launch for bfloat16)."""
    Xs, dYs = list(Xs), list(dYs)
    p = len(Xs)
    if not 1 <= p <= 4 or len(dYs) != p:
        raise GtaError(1, "1 to 4 products, one dY per X")
    n, d_in = _need2("X[0]", Xs[0])
    d_out = _need2("dY[0]", dYs[0])[1]
    dev, dt = Xs[0].device, Xs[0].dtype
    if dWs is None:
        dWs = [torch.empty((d_in, d_out), dtype=torch.float32, device=dev) for _ in range(p)]
    dWs = list(dWs)
    if len(dWs) != p:
        raise GtaError(1, "one dW per product")
    for k in range(p):
        _need(f"X[{k}]", Xs[k], (n, d_in), dt, dev)
        _need(f"dY[{k}]", dYs[k], (n, d_out), dt, dev)
        _need(f"dW[{k}]", dWs[k], (d_in, d_out), torch.float32, dev)
    if len({t.data_ptr() for t in dWs}) != p:
        raise GtaError(1, "the dW tensors must be distinct")
    lib = load_library()
    arr = lambda ts: (c_void_p * len(ts))(*[t.data_ptr() for t in ts])
    nbytes = lib.gta_linear_dw_group_scratch_bytes(n, d_in, d_out, p)
    scratch = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
    _check(lib.gta_linear_dw_group(arr(Xs), arr(dYs), arr(dWs), p, n, d_in, d_out, _dtype_code(Xs[0]),
                                   _ptr(scratch), scratch.numel(), _stream()))
    return dWs


def gta_linear_group(Xs, Ws, Cs=None, trans_w: bool = False, Ys=None):
    """Ys[po] = sum_pi Xs[pi] @ op(Ws[po * len(Xs) + pi]) (+ Cs[po]); bfloat16 [n, d] tensors, d in {64, 128, 256}."""
    Xs, Ws = list(Xs), list(Ws)
    p_in = len(Xs)
    if p_in == 0 or len(Ws) % p_in:
        raise GtaError(1, "the number of weights must be a multiple of the number of inputs")
    p_out = len(Ws) // p_in
    n, d = _need2("X[0]", Xs[0])
    dev, dt = Xs[0].device, Xs[0].dtype
    if Ys is None:
        Ys = [torch.empty((n, d), dtype=dt, device=dev) for _ in range(p_out)]
    Ys = list(Ys)
    if len(Ys) != p_out or (Cs is not None and len(Cs) != p_out):
        raise GtaError(1, "one output (and addend) per group of weights")
    for i, t in enumerate(Xs):
        _need(f"X[{i}]", t, (n, d), dt, dev)
    for i, t in enumerate(Ws):
        _need(f"W[{i}]", t, (d, d), dt, dev)
    for i, t in enumerate(Ys):
        _need(f"Y[{i}]", t, (n, d), dt, dev)
    for i, t in enumerate(Cs or []):
        _need(f"C[{i}]", t, (n, d), dt, dev)
    inputs = {t.data_ptr() for t in Xs + list(Cs or [])}
    if any(y.data_ptr() in inputs for y in Ys):
        raise GtaError(1, "an output aliases an input or addend")
    lib = load_library()
    arr = lambda ts: (c_void_p * len(ts))(*[t.data_ptr() for t in ts])
    nbytes = lib.gta_linear_group_scratch_bytes(d, p_in, p_out)
    scratch = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
    _check(lib.gta_linear_group(arr(Xs), p_in, arr(Ws), p_out, arr(list(Cs)) if Cs is not None else None, arr(Ys),
                                n, d, _dtype_code(Xs[0]), int(bool(trans_w)), _ptr(scratch), scratch.numel(),
                                _stream()))
    return Ys


def _layer_scratch(plan: Plan, heads, head_dim, code):
    key = ("layer", heads, head_dim, code)
    if key not in plan._scratch:
        nbytes = load_library().gta_sga_layer_scratch_bytes(plan.handle, heads, head_dim, code)
        if nbytes == 0:
            raise GtaError(2, "unsupported shape for the layer form")
        plan._scratch[key] = torch.empty(nbytes, dtype=torch.uint8, device=plan.indptr.device)
    return plan._scratch[key]


def _layer_shapes(plan: Plan, X, heads: int, weights):
    n, d = _need2("X", X)
    if n != plan.n_dst or plan.n_src != plan.n_dst:
        raise GtaError(1, "the layer form needs n_src == n_dst == rows of X")
    if heads <= 0 or d % heads:
        raise GtaError(1, f"hidden size {d} is not divisible by heads = {heads}")
    dev = plan.indptr.device
    _need("X", X, (n, d), X.dtype, dev)
    for name, w in weights.items():
        _need(name, w, (d, d), X.dtype, dev)
    return n, d, d // heads, _dtype_code(X), dev


def gta_sga_layer_fwd(plan: Plan, X, Wq, Wk, Wv, Wo, heads: int, scale: float = 0.0, saved=None):
    """X [n, d] -> (X' [n, d], saved) with saved = dict(Q, K, V, Y, lse) for the backward."""
    n, d, head_dim, code, dev = _layer_shapes(plan, X, heads, dict(Wq=Wq, Wk=Wk, Wv=Wv, Wo=Wo))
    if saved is None:
        saved = dict(Q=torch.empty_like(X), K=torch.empty_like(X), V=torch.empty_like(X), Y=torch.empty_like(X),
                     lse=torch.empty((n, heads), dtype=torch.float32, device=dev))
    _need_all(dev, X.dtype, **{k: (saved[k], (n, d)) for k in ("Q", "K", "V", "Y")})
    _need("lse", saved["lse"], (n, heads), torch.float32, dev)
    Xout = torch.empty_like(X)
    scratch = _layer_scratch(plan, heads, head_dim, code)
    _check(load_library().gta_sga_layer_fwd(
        plan.handle, _ptr(plan.indptr), _ptr(plan.indices), _ptr(X), _ptr(Wq), _ptr(Wk), _ptr(Wv), _ptr(Wo),
        _ptr(saved["Q"]), _ptr(saved["K"]), _ptr(saved["V"]), _ptr(saved["Y"]), _ptr(saved["lse"]), _ptr(Xout),
        n, heads, head_dim, code, scale, _ptr(scratch), scratch.numel(), _stream()))
    return Xout, saved


def gta_sga_layer_bwd(plan: Plan, X, Wq, Wk, Wv, Wo, saved, dXout, heads: int, scale: float = 0.0):
    """Returns dX [n, d] and float32 dWq, dWk, dWv, dWo [d, d]."""
    n, d, head_dim, code, dev = _layer_shapes(plan, X, heads, dict(Wq=Wq, Wk=Wk, Wv=Wv, Wo=Wo))
    _need_all(dev, X.dtype, dXout=(dXout, (n, d)), **{k: (saved[k], (n, d)) for k in ("Q", "K", "V", "Y")})
    _need("lse", saved["lse"], (n, heads), torch.float32, dev)
    work = [torch.empty_like(X) for _ in range(3)]
    dX = torch.empty_like(X)
    dW = [torch.empty((d, d), dtype=torch.float32, device=dev) for _ in range(4)]
    scratch = _layer_scratch(plan, heads, head_dim, code)
    _check(load_library().gta_sga_layer_bwd(
        plan.handle, _ptr(plan.indptr), _ptr(plan.indices), _ptr(X), _ptr(Wq), _ptr(Wk), _ptr(Wv), _ptr(Wo),
        _ptr(saved["Q"]), _ptr(saved["K"]), _ptr(saved["V"]), _ptr(saved["Y"]), _ptr(saved["lse"]), _ptr(dXout),
        _ptr(work[0]), _ptr(work[1]), _ptr(work[2]), _ptr(dX), _ptr(dW[0]), _ptr(dW[1]), _ptr(dW[2]), _ptr(dW[3]),
        n, heads, head_dim, code, scale, _ptr(scratch), scratch.numel(), _stream()))
    return dX, dW[0], dW[1], dW[2], dW[3]


def gta_head_split(X, parts: int, S=None):
    """X [n, H, D] -> S [parts, n, H/parts, D] (block r = heads r*H/parts .. (r+1)*H/parts)."""
    n, heads, head_dim = _need3("X", X)
    ss = (parts, n, max(heads // max(parts, 1), 1), head_dim)
    if S is None:
        S = torch.empty(ss, dtype=X.dtype, device=X.device)
    _need("X", X, (n, heads, head_dim), X.dtype, X.device)
    _need("S", S, ss, X.dtype, X.device)
    _check(load_library().gta_head_split(_ptr(X), _ptr(S), n, heads, head_dim, _dtype_code(X), parts, _stream()))
    return S


def gta_head_merge(S, X=None):
    """Inverse of gta_head_split: S [parts, n, H/parts, D] -> X [n, H, D]."""
    if not isinstance(S, torch.Tensor) or S.dim() != 4:
        raise GtaError(1, "S: expected a tensor [parts, rows, heads/parts, head_dim]")
    parts, n, hp, head_dim = S.shape
    if X is None:
        X = torch.empty((n, hp * parts, head_dim), dtype=S.dtype, device=S.device)
    _need("S", S, tuple(S.shape), S.dtype, S.device)
    _need("X", X, (n, hp * parts, head_dim), S.dtype, S.device)
    _check(load_library().gta_head_merge(_ptr(S), _ptr(X), n, hp * parts, head_dim, _dtype_code(S), parts, _stream()))
    return X


def gta_agp_select(t_iter1: float, n_nodes: int, samples, max_gpus: int):
    """samples: iterable of (strategy id, gpus, beta).  Returns (strategy, gpus, estimated t_iter)."""
    samples = list(samples)
    arr = (_AgpSample * max(1, len(samples)))(*[_AgpSample(int(c), int(i), float(b)) for c, i, b in samples])
    strategy, gpus, est = c_int(), c_int(), ctypes.c_double()
    _check(load_library().gta_agp_select(t_iter1, n_nodes, arr, len(samples), max_gpus, ctypes.byref(strategy),
                                         ctypes.byref(gpus), ctypes.byref(est)))
    return strategy.value, gpus.value, est.value


def gta_stream_probe(mode: int, dst, a, b=None):
    """mode 0: read a; 1: dst = a; 2: dst = a + b (float32 tensors of equal size, multiples of 16 bytes)."""
    n = a.numel()
    for name, t in (("dst", dst), ("a", a)) + ((("b", b),) if mode == 2 else ()):
        _need(name, t, (n,) if mode or name != "dst" else tuple(t.shape), torch.float32, a.device)
    if mode == 0 and dst.numel() < 4:
        raise GtaError(1, "dst needs at least 16 bytes")
    _check(load_library().gta_stream_probe(int(mode), _ptr(dst), _ptr(a), _ptr(b), n * 4, _stream()))


def gta_profile_enable(on):
    """0 = off, 1 = time every launch, 2 = also launch the row schedules of a pass separately."""
    _check(load_library().gta_profile_enable(int(on)))


def gta_profile_read(reset: bool = True):
    lib = load_library()
    n = lib.gta_profile_read(None, 0, 0)
    buf = (_LaunchRecord * max(n, 1))()
    lib.gta_profile_read(buf, n, int(bool(reset)))
    return [dict(name=buf[i].name.decode(), ms=float(buf[i].ms), rows=int(buf[i].rows),
                 entries=int(buf[i].entries)) for i in range(n)]
