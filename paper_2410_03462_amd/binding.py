"""ctypes binding of ``libgrf_hip.so`` (the C ABI declared in ``include/grf.h``).

Argument marshalling only: every step of the method runs in the library's HIP kernels.
PyTorch provides device memory and the current stream.  There is no CPU path: if the
library has not been built, or no GPU is present, calls raise.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch  # noqa: F401  (imported first so that the HIP runtime already loaded by torch is shared)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgrf_hip.so")

GRF_OK, GRF_EINVAL, GRF_ECAPACITY, GRF_EUNSUPPORTED, GRF_EHIP, GRF_EWORKSPACE = 0, -1, -2, -3, -4, -5
GRF_DTYPE_F32, GRF_DTYPE_BF16 = 0, 1
GRF_PHI_RELU, GRF_PHI_IDENTITY, GRF_PHI_ELU1 = 0, 1, 2
_FEATURE_MAPS = {"relu": GRF_PHI_RELU, "identity": GRF_PHI_IDENTITY, "elu1": GRF_PHI_ELU1}
_STATUS_NAMES = {GRF_EINVAL: "GRF_EINVAL", GRF_ECAPACITY: "GRF_ECAPACITY", GRF_EUNSUPPORTED: "GRF_EUNSUPPORTED",
                 GRF_EHIP: "GRF_EHIP", GRF_EWORKSPACE: "GRF_EWORKSPACE"}


class GrfError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


class _Graph(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int64), ("nnz", ctypes.c_int64), ("row_ptr", ctypes.c_void_p),
                ("col", ctypes.c_void_p), ("w", ctypes.c_void_p)]


class _Phi(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int64), ("capacity", ctypes.c_int64), ("row_ptr", ctypes.c_void_p),
                ("col", ctypes.c_void_p), ("val", ctypes.c_void_p)]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library.  Raises if it has not been built (``python -m paper_2410_03462_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2410_03462_amd.build`; "
                               "there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        L.grf_last_error.restype = ctypes.c_char_p
        L.grf_sample_nnz_bound.restype = ctypes.c_int64
        L.grf_sample_nnz_bound.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32]
        L.grf_sample_workspace_bytes.restype = ctypes.c_size_t
        L.grf_sample_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
        L.grf_sample.restype = ctypes.c_int32
        L.grf_sample.argtypes = [ctypes.POINTER(_Graph), ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                 ctypes.c_double, ctypes.c_int32, ctypes.c_uint64,
                                 ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                 ctypes.POINTER(_Phi), ctypes.POINTER(ctypes.c_int64)]
        L.grf_sample_async.restype = ctypes.c_int32
        L.grf_sample_async.argtypes = [ctypes.POINTER(_Graph), ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                       ctypes.c_double, ctypes.c_int32, ctypes.c_uint64,
                                       ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.POINTER(_Phi)]
        L.grf_sample_walks.restype = ctypes.c_int32
        L.grf_sample_walks.argtypes = [ctypes.POINTER(_Graph), ctypes.c_double, ctypes.c_int32, ctypes.c_int32,
                                       ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p]
        L.grf_debug_force_wide_offsets.restype = None
        L.grf_debug_force_wide_offsets.argtypes = [ctypes.c_int32]
        L.grf_debug_force_row_kernel.restype = None
        L.grf_debug_force_row_kernel.argtypes = [ctypes.c_int32]
        L.grf_bucket_record_floats.restype = ctypes.c_int64
        L.grf_bucket_record_floats.argtypes = [ctypes.c_int32]
        L.grf_attention_workspace_bytes.restype = ctypes.c_size_t
        L.grf_attention_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                                    ctypes.c_int64, ctypes.c_int32, ctypes.c_int32]
        L.grf_buckets_workspace_bytes.restype = ctypes.c_size_t
        L.grf_buckets_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int32]
        common = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                  ctypes.POINTER(_Phi), ctypes.c_int64, ctypes.c_int32, ctypes.c_int32]
        L.grf_form_buckets.restype = ctypes.c_int32
        L.grf_form_buckets.argtypes = [ctypes.c_void_p, ctypes.c_void_p, *common,
                                       ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
        L.grf_gather_buckets.restype = ctypes.c_int32
        L.grf_gather_buckets.argtypes = [ctypes.c_void_p, *common, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.grf_masked_linear_attention.restype = ctypes.c_int32
        L.grf_masked_linear_attention.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, *common,
                                                  ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                                  ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.grf_fused_attention_workspace_bytes.restype = ctypes.c_size_t
        L.grf_fused_attention_workspace_bytes.argtypes = L.grf_attention_workspace_bytes.argtypes
        L.grf_masked_linear_attention_fused.restype = ctypes.c_int32
        L.grf_masked_linear_attention_fused.argtypes = L.grf_masked_linear_attention.argtypes
        L.grf_phi_prepare_bytes.restype = ctypes.c_size_t
        L.grf_phi_prepare_bytes.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int32]
        for name in ("grf_phi_prepare", "grf_phi_prepare_values"):
            getattr(L, name).restype = ctypes.c_int32
            getattr(L, name).argtypes = [ctypes.POINTER(_Phi), ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.grf_form_buckets_prepared.restype = ctypes.c_int32
        L.grf_form_buckets_prepared.argtypes = [ctypes.c_void_p, ctypes.c_void_p, *common,
                                                ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
        for name in ("grf_masked_linear_attention_prepared", "grf_masked_linear_attention_fused_prepared"):
            getattr(L, name).restype = ctypes.c_int32
            getattr(L, name).argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, *common,
                                         ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.grf_masked_linear_attention_fused_static.restype = ctypes.c_int32
        L.grf_masked_linear_attention_fused_static.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, *common,
                                                               ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.grf_asymmetric_masked_attention.restype = ctypes.c_int32
        L.grf_asymmetric_masked_attention.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, *common,
                                                      ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.grf_attention_backward_workspace_bytes.restype = ctypes.c_size_t
        L.grf_attention_backward_workspace_bytes.argtypes = L.grf_attention_workspace_bytes.argtypes
        L.grf_masked_linear_attention_backward.restype = ctypes.c_int32
        L.grf_masked_linear_attention_backward.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, *common,
                                                           ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                                           ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                                           ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.grf_masked_linear_attention_backward_prepared.restype = ctypes.c_int32
        L.grf_masked_linear_attention_backward_prepared.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, *common,
                                                                    ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                                                    ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t,
                                                                    ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                                                    ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.grf_knn_graph_nnz_bound.restype = ctypes.c_int64
        L.grf_knn_graph_nnz_bound.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32]
        L.grf_knn_graph_workspace_bytes.restype = ctypes.c_size_t
        L.grf_knn_graph_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32]
        L.grf_knn_graph.restype = ctypes.c_int32
        L.grf_knn_graph.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_float,
                                    ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                    ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.POINTER(ctypes.c_int64)]
        L.grf_asymmetric_backward_workspace_bytes.restype = ctypes.c_size_t
        L.grf_asymmetric_backward_workspace_bytes.argtypes = L.grf_attention_workspace_bytes.argtypes
        L.grf_asymmetric_masked_attention_backward.restype = ctypes.c_int32
        L.grf_asymmetric_masked_attention_backward.argtypes = L.grf_masked_linear_attention_backward.argtypes
        L.grf_sample_backward_workspace_bytes.restype = ctypes.c_size_t
        L.grf_sample_backward_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
        L.grf_sample_backward.restype = ctypes.c_int32
        L.grf_sample_backward.argtypes = [ctypes.POINTER(_Graph), ctypes.c_int32, ctypes.c_int32, ctypes.c_double,
                                          ctypes.c_int32, ctypes.c_uint64, ctypes.POINTER(_Phi), ctypes.c_int64,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
        _lib = L
    return _lib


def _check(status: int):
    if status != GRF_OK:
        raise GrfError(status, lib().grf_last_error().decode())


def _require_gpu():
    if not torch.cuda.is_available():
        raise RuntimeError("no GPU visible: this library has no CPU path")


def _stream_ptr(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None or t.numel() == 0 else int(t.data_ptr())


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


# --------------------------------------------------------------------------- containers

@dataclass
class DeviceGraph:
    """Weighted adjacency matrix in CSR on the GPU."""
    n: int
    row_ptr: torch.Tensor   # int32 [n+1]
    col: torch.Tensor       # int32 [nnz]
    w: torch.Tensor         # float32 [nnz]

    @property
    def nnz(self) -> int:
        return int(self.col.numel())

    @staticmethod
    def from_host(g, device="cuda:0") -> "DeviceGraph":
        _require_gpu()
        return DeviceGraph(int(g.n),
                           torch.from_numpy(np.ascontiguousarray(g.row_ptr, dtype=np.int32)).to(device),
                           torch.from_numpy(np.ascontiguousarray(g.col, dtype=np.int32)).to(device),
                           torch.from_numpy(np.ascontiguousarray(g.w, dtype=np.float32)).to(device))

    def _struct(self) -> _Graph:
        return _Graph(self.n, self.nnz, _ptr(self.row_ptr), _ptr(self.col), _ptr(self.w))


@dataclass
class Phi:
    """GRF matrix in CSR on the GPU; ``val`` is [n_f, capacity], the first ``nnz`` entries of each plane are live."""
    n: int
    nnz: int
    row_ptr: torch.Tensor   # int32 [n+1]
    col: torch.Tensor       # int32 [capacity]
    val: torch.Tensor       # float32 [n_f, capacity]

    @property
    def capacity(self) -> int:
        return int(self.col.numel())

    @property
    def n_f(self) -> int:
        return int(self.val.shape[0])

    @staticmethod
    def empty(n: int, capacity: int, n_f: int, device="cuda:0") -> "Phi":
        return Phi(n, 0, torch.empty(n + 1, dtype=torch.int32, device=device),
                   torch.empty(capacity, dtype=torch.int32, device=device),
                   torch.empty((n_f, capacity), dtype=torch.float32, device=device))

    @staticmethod
    def from_host(n: int, row_ptr, col, val, device="cuda:0") -> "Phi":
        val = np.atleast_2d(np.ascontiguousarray(val, dtype=np.float32))
        return Phi(int(n), int(col.shape[0]),
                   torch.from_numpy(np.ascontiguousarray(row_ptr, dtype=np.int32)).to(device),
                   torch.from_numpy(np.ascontiguousarray(col, dtype=np.int32)).to(device),
                   torch.from_numpy(val).to(device))

    def to_host(self):
        return (self.row_ptr.cpu().numpy(), self.col[: self.nnz].cpu().numpy(), self.val[:, : self.nnz].cpu().numpy())

    def _struct(self) -> _Phi:
        return _Phi(self.n, self.capacity, _ptr(self.row_ptr), _ptr(self.col), _ptr(self.val))


# --------------------------------------------------------------------------- entry points (same names as the C ABI)

GRF_WEIGHT_INV_DEGREE, GRF_WEIGHT_EXP, GRF_WEIGHT_GAUSS = 0, 1, 2
_WEIGHT_KINDS = {"inv_degree": GRF_WEIGHT_INV_DEGREE, "exp": GRF_WEIGHT_EXP, "gauss": GRF_WEIGHT_GAUSS}


def grf_knn_graph_nnz_bound(n: int, k: int, symmetrise: bool = True) -> int:
    return int(lib().grf_knn_graph_nnz_bound(n, k, 1 if symmetrise else 0))


def grf_knn_graph_workspace_bytes(n: int, k: int) -> int:
    return int(lib().grf_knn_graph_workspace_bytes(n, k))


def grf_knn_graph(points: torch.Tensor, k: int, symmetrise: bool = True, weights: str = "gauss", sigma: float = 1.0,
                  workspace: Optional[torch.Tensor] = None, stream=None, out: Optional[DeviceGraph] = None,
                  sync: bool = True) -> DeviceGraph:
    """Exact k-nearest-neighbour graph of ``points`` (CUDA fp32 [n, 3]) as a DeviceGraph.

    ``sync=False``: no host synchronisation (capturable into a HIP graph); the result's ``col`` / ``w`` keep their full
    bound-sized length and the entry count stays on the device in ``row_ptr[n]``.  ``out`` reuses a previous result's
    buffers (they must have the bound's size)."""
    _require_gpu()
    L = lib()
    if points.dim() != 2 or points.shape[1] != 3 or points.dtype != torch.float32 or not points.is_cuda or not points.is_contiguous():
        raise ValueError("points must be a contiguous CUDA fp32 tensor [n, 3]")
    n = int(points.shape[0])
    bound = L.grf_knn_graph_nnz_bound(n, k, 1 if symmetrise else 0)
    if bound < 0:
        raise GrfError(GRF_EUNSUPPORTED, f"unsupported k={k}")
    dev = points.device
    if workspace is None:
        workspace = _workspace(L.grf_knn_graph_workspace_bytes(n, k), dev)
    if out is not None:
        if out.n != n or out.col.numel() < bound:
            raise ValueError("out does not match the point count or is smaller than the bound")
        row_ptr, col, w = out.row_ptr, out.col, out.w
    else:
        row_ptr = torch.empty(n + 1, dtype=torch.int32, device=dev)
        col = torch.empty(max(bound, 1), dtype=torch.int32, device=dev)
        w = torch.empty(max(bound, 1), dtype=torch.float32, device=dev)
    nnz = ctypes.c_int64(0)
    _check(L.grf_knn_graph(_ptr(points), n, int(k), 1 if symmetrise else 0, _WEIGHT_KINDS[weights], float(sigma),
                           _ptr(workspace), workspace.numel(), _stream_ptr(stream),
                           _ptr(row_ptr), _ptr(col), _ptr(w), int(col.numel()), ctypes.byref(nnz) if sync else None))
    if not sync:
        return DeviceGraph(n, row_ptr, col, w)
    return DeviceGraph(n, row_ptr, col[: nnz.value], w[: nnz.value])


def grf_sample_nnz_bound(n: int, n_walks: int, f_len: int) -> int:
    return int(lib().grf_sample_nnz_bound(n, n_walks, f_len))


def grf_sample(graph: DeviceGraph, f, p_halt: float, n_walks: int, seed: int,
               out: Optional[Phi] = None, capacity: Optional[int] = None, stream=None,
               workspace: Optional[torch.Tensor] = None) -> Phi:
    """Sample Phi_hat.  ``f`` is a host array [n_f, f_len] (or [f_len]).

    With ``out`` the caller's buffers are reused (GrfError(GRF_ECAPACITY) if too small).  Otherwise the
    buffers are sized by ``capacity``, or, if None, by a first call that only counts.
    """
    _require_gpu()
    L = lib()
    f = np.ascontiguousarray(np.atleast_2d(np.asarray(f, dtype=np.float32)))
    n_f, f_len = f.shape
    dev = graph.row_ptr.device
    ws = workspace if workspace is not None else _workspace(L.grf_sample_workspace_bytes(graph.n, n_walks, f_len, n_f), dev)
    gs = graph._struct()
    nnz = ctypes.c_int64(0)

    def call(phi: Phi) -> int:
        ps = phi._struct()
        return L.grf_sample(ctypes.byref(gs), f.ctypes.data_as(ctypes.c_void_p), f_len, n_f, float(p_halt),
                            int(n_walks), int(seed) & 0xFFFFFFFFFFFFFFFF, _ptr(ws), ws.numel(), _stream_ptr(stream),
                            ctypes.byref(ps), ctypes.byref(nnz))

    if out is None:
        if capacity is None:
            probe = Phi.empty(graph.n, 0, n_f, dev)
            st = call(probe)
            if st not in (GRF_OK, GRF_ECAPACITY):
                _check(st)
            capacity = int(nnz.value)
        out = Phi.empty(graph.n, int(capacity), n_f, dev)
    elif out.n_f != n_f or out.n != graph.n:
        raise ValueError("out does not match the graph / number of f sets")
    _check(call(out))
    out.nnz = int(nnz.value)
    return out


def grf_sample_async(graph: DeviceGraph, f: torch.Tensor, p_halt: float, n_walks: int, seed: int,
                     out: Optional[Phi] = None, workspace: Optional[torch.Tensor] = None, stream=None) -> Phi:
    """grf_sample without touching the host: ``f`` is a CUDA fp32 tensor [n_f, f_len] (or [f_len]) read on the stream,
    nothing is synchronised, and the result's ``nnz`` is its capacity (grf_sample_nnz_bound), an upper bound that the
    attention calls accept; the count stays on the device in ``row_ptr[n]``.  Capturable into a HIP graph when ``out``
    and ``workspace`` are passed (no allocation inside the capture)."""
    _require_gpu()
    L = lib()
    f2 = f.reshape(-1, f.shape[-1])
    if not f2.is_cuda or f2.dtype != torch.float32 or not f2.is_contiguous():
        raise ValueError("f must be a contiguous CUDA fp32 tensor")
    n_f, f_len = int(f2.shape[0]), int(f2.shape[1])
    dev = graph.row_ptr.device
    if out is None:
        out = Phi.empty(graph.n, int(L.grf_sample_nnz_bound(graph.n, n_walks, f_len)), n_f, dev)
    elif out.n_f != n_f or out.n != graph.n:
        raise ValueError("out does not match the graph / number of f sets")
    ws = workspace if workspace is not None else _workspace(L.grf_sample_workspace_bytes(graph.n, n_walks, f_len, n_f), dev)
    gs, ps = graph._struct(), out._struct()
    _check(L.grf_sample_async(ctypes.byref(gs), _ptr(f2), f_len, n_f, float(p_halt), int(n_walks),
                              int(seed) & 0xFFFFFFFFFFFFFFFF, _ptr(ws), ws.numel(), _stream_ptr(stream), ctypes.byref(ps)))
    out.nnz = out.capacity
    return out


def grf_sample_walks(graph: DeviceGraph, p_halt: float, n_walks: int, max_nodes: int, seed: int, stream=None) -> torch.Tensor:
    """Trajectories [n, n_walks, max_nodes] int32 on the GPU, -1 past the end of a walk."""
    _require_gpu()
    traj = torch.empty((graph.n, n_walks, max_nodes), dtype=torch.int32, device=graph.row_ptr.device)
    gs = graph._struct()
    _check(lib().grf_sample_walks(ctypes.byref(gs), float(p_halt), int(n_walks), int(max_nodes),
                                  int(seed) & 0xFFFFFFFFFFFFFFFF, _stream_ptr(stream), _ptr(traj)))
    return traj


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return GRF_DTYPE_F32
    if t.dtype == torch.bfloat16:
        return GRF_DTYPE_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _check_qkv(*ts):
    shape, dtype = ts[0].shape, ts[0].dtype
    for t in ts:
        if not t.is_cuda or not t.is_contiguous() or t.shape != shape or t.dtype != dtype or t.dim() != 4:
            raise ValueError("Q, K, V must be contiguous CUDA tensors of one shape [B,H,n,d] and dtype")
    return shape


def grf_debug_force_wide_offsets(on: bool) -> None:
    lib().grf_debug_force_wide_offsets(1 if on else 0)


def grf_debug_force_row_kernel(which: int) -> None:
    """0: the library chooses; 1 / 2: the sampler's wavefront / workgroup kernel wherever both can serve."""
    lib().grf_debug_force_row_kernel(int(which))


def grf_bucket_record_floats(d: int) -> int:
    return int(lib().grf_bucket_record_floats(d))


def grf_attention_workspace_bytes(B: int, H: int, n: int, d: int, nnz: int, n_f: int = 1, bh_chunk: int = 0) -> int:
    return int(lib().grf_attention_workspace_bytes(B, H, n, d, nnz, n_f, bh_chunk))


def grf_buckets_workspace_bytes(n: int, nnz: int, n_f: int = 1) -> int:
    return int(lib().grf_buckets_workspace_bytes(n, nnz, n_f))


def grf_phi_prepare_bytes(n: int, nnz: int, n_f: int = 1) -> int:
    return int(lib().grf_phi_prepare_bytes(n, nnz, n_f))


def grf_phi_prepare(phi: Phi, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Column lists of ``phi`` built once, as an opaque uint8 buffer to pass as ``prepared=`` to the attention calls."""
    _require_gpu()
    L = lib()
    need = L.grf_phi_prepare_bytes(phi.n, phi.nnz, phi.n_f)
    buf = out if out is not None else _workspace(need, phi.row_ptr.device)
    ps = phi._struct()
    _check(L.grf_phi_prepare(ctypes.byref(ps), phi.nnz, phi.n_f, _ptr(buf), buf.numel(), _stream_ptr(stream)))
    return buf


def grf_phi_prepare_values(phi: Phi, prepared: torch.Tensor, stream=None) -> torch.Tensor:
    """Refresh the value planes inside ``prepared`` from ``phi.val`` (same pattern, new modulation f)."""
    _require_gpu()
    ps = phi._struct()
    _check(lib().grf_phi_prepare_values(ctypes.byref(ps), phi.nnz, phi.n_f, _ptr(prepared), prepared.numel(), _stream_ptr(stream)))
    return prepared


def grf_form_buckets_prepared(K, V, phi: Phi, prepared: torch.Tensor, feature_map: str = "relu", out: Optional[torch.Tensor] = None, stream=None):
    return grf_form_buckets(K, V, phi, feature_map, out=out, stream=stream, prepared=prepared)


def grf_masked_linear_attention_prepared(Q, K, V, phi: Phi, prepared: torch.Tensor, **kw):
    return grf_masked_linear_attention(Q, K, V, phi, prepared=prepared, **kw)


def grf_masked_linear_attention_fused_prepared(Q, K, V, phi: Phi, prepared: torch.Tensor, **kw):
    return grf_masked_linear_attention_fused(Q, K, V, phi, prepared=prepared, **kw)


def grf_masked_linear_attention_backward_prepared(Q, K, V, phi: Phi, prepared: torch.Tensor, out, den, d_out, **kw):
    return grf_masked_linear_attention_backward(Q, K, V, phi, out, den, d_out, prepared=prepared, **kw)


def grf_form_buckets(K: torch.Tensor, V: torch.Tensor, phi: Phi, feature_map: str = "relu",
                     out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None,
                     prepared: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Bucket records [B*H, n, d*d + d] fp32: S_l (d x d, feature index major) then z_l."""
    _require_gpu()
    L = lib()
    B, H, n, d = _check_qkv(K, V)
    rec = L.grf_bucket_record_floats(d)
    if rec < 0:
        raise GrfError(GRF_EUNSUPPORTED, f"head dimension d={d} is not supported")
    buckets = out if out is not None else torch.empty((B * H, n, rec), dtype=torch.float32, device=K.device)
    if buckets.numel() != B * H * n * rec or buckets.dtype != torch.float32 or not buckets.is_contiguous():
        raise ValueError("bucket buffer has the wrong size, dtype or layout")
    ps = phi._struct()
    if prepared is not None:
        _check(L.grf_form_buckets_prepared(_ptr(K), _ptr(V), _dtype_code(K), B, H, n, d, ctypes.byref(ps), phi.nnz, phi.n_f,
                                           _FEATURE_MAPS[feature_map], _ptr(prepared), prepared.numel(), _stream_ptr(stream), _ptr(buckets)))
        return buckets
    ws = workspace if workspace is not None else _workspace(L.grf_buckets_workspace_bytes(n, phi.nnz, phi.n_f), K.device)
    _check(L.grf_form_buckets(_ptr(K), _ptr(V), _dtype_code(K), B, H, n, d, ctypes.byref(ps), phi.nnz, phi.n_f,
                              _FEATURE_MAPS[feature_map], _ptr(ws), ws.numel(), _stream_ptr(stream), _ptr(buckets)))
    return buckets


def grf_gather_buckets(Q: torch.Tensor, phi: Phi, buckets: torch.Tensor, feature_map: str = "relu",
                       return_num_den: bool = False, out: Optional[torch.Tensor] = None, stream=None):
    """out [B,H,n,d] fp32 (and num, den if asked) from records written by grf_form_buckets."""
    _require_gpu()
    L = lib()
    B, H, n, d = _check_qkv(Q)
    rec = L.grf_bucket_record_floats(d)
    if rec < 0:
        raise GrfError(GRF_EUNSUPPORTED, f"head dimension d={d} is not supported")
    if buckets.numel() != B * H * n * rec or buckets.dtype != torch.float32 or not buckets.is_contiguous():
        raise ValueError("bucket buffer has the wrong size, dtype or layout")
    if out is None:
        out = torch.empty((B, H, n, d), dtype=torch.float32, device=Q.device)
    num = torch.empty((B, H, n, d), dtype=torch.float32, device=Q.device) if return_num_den else None
    den = torch.empty((B, H, n), dtype=torch.float32, device=Q.device) if return_num_den else None
    ps = phi._struct()
    _check(L.grf_gather_buckets(_ptr(Q), _dtype_code(Q), B, H, n, d, ctypes.byref(ps), phi.nnz, phi.n_f,
                                _FEATURE_MAPS[feature_map], _ptr(buckets), _stream_ptr(stream),
                                _ptr(out), _ptr(num), _ptr(den)))
    return (out, num, den) if return_num_den else out


def grf_fused_attention_workspace_bytes(B: int, H: int, n: int, d: int, nnz: int, n_f: int = 1, bh_chunk: int = 0) -> int:
    return int(lib().grf_fused_attention_workspace_bytes(B, H, n, d, nnz, n_f, bh_chunk))


def grf_masked_linear_attention_fused(Q, K, V, phi: Phi, feature_map: str = "relu", bh_chunk: Optional[int] = None,
                                      return_num_den: bool = False, workspace: Optional[torch.Tensor] = None,
                                      out: Optional[torch.Tensor] = None, stream=None, prepared: Optional[torch.Tensor] = None):
    """Bucket-fused variant: same results as grf_masked_linear_attention without bucket records in HBM.
    ``prepared``: the buffer of grf_phi_prepare(phi), which saves rebuilding the column lists."""
    return _attention_call("grf_masked_linear_attention_fused", "grf_fused_attention_workspace_bytes",
                           Q, K, V, phi, feature_map, bh_chunk, return_num_den, workspace, out, stream, prepared)


def grf_masked_linear_attention_fused_static(Q, K, V, phi: Phi, feature_map: str = "relu", return_num_den: bool = False,
                                             out: Optional[torch.Tensor] = None, num: Optional[torch.Tensor] = None,
                                             den: Optional[torch.Tensor] = None, stream=None):
    """The bucket-fused call on the library's own static scratch array: no workspace, and the library allocates
    nothing (pass ``out`` / ``num`` / ``den`` and this binding allocates nothing either)."""
    _require_gpu()
    L = lib()
    B, H, n, d = _check_qkv(Q, K, V)
    if out is None:
        out = torch.empty((B, H, n, d), dtype=torch.float32, device=Q.device)
    if return_num_den and num is None:
        num = torch.empty((B, H, n, d), dtype=torch.float32, device=Q.device)
    if return_num_den and den is None:
        den = torch.empty((B, H, n), dtype=torch.float32, device=Q.device)
    ps = phi._struct()
    _check(L.grf_masked_linear_attention_fused_static(_ptr(Q), _ptr(K), _ptr(V), _dtype_code(Q), B, H, n, d, ctypes.byref(ps),
                                                      phi.nnz, phi.n_f, _FEATURE_MAPS[feature_map], _stream_ptr(stream),
                                                      _ptr(out), _ptr(num), _ptr(den)))
    return (out, num, den) if return_num_den else out


def grf_masked_linear_attention(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, phi: Phi,
                                feature_map: str = "relu", bh_chunk: Optional[int] = None, return_num_den: bool = False,
                                workspace: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                                stream=None, prepared: Optional[torch.Tensor] = None):
    """out [B,H,n,d] fp32 (and num, den if asked).

    ``bh_chunk``: (batch, head) slices whose buckets are resident at once; 0 = all; None = all when a workspace is
    passed, else as many as fit WORKSPACE_BUDGET_BYTES."""
    return _attention_call("grf_masked_linear_attention", "grf_attention_workspace_bytes",
                           Q, K, V, phi, feature_map, bh_chunk, return_num_den, workspace, out, stream, prepared)


WORKSPACE_BUDGET_BYTES = 4 << 30


def _auto_chunk(L, ws_query: str, B: int, H: int, n: int, d: int, nnz: int, n_f: int) -> int:
    """Slices per chunk when the caller names none and brings no workspace: as many as keep the per-slice part of
    the workspace within WORKSPACE_BUDGET_BYTES (at least one).  Beyond a few GB more resident slices buy nothing,
    and at the largest workload fewer are measurably faster (the scattered reads stay within fewer pages)."""
    slices = B * H
    if slices <= 1:
        return 0
    one, two = getattr(L, ws_query)(B, H, n, d, nnz, n_f, 1), getattr(L, ws_query)(B, H, n, d, nnz, n_f, 2)
    per_slice = max(two - one, 1)
    fit = max(1, min(slices, (WORKSPACE_BUDGET_BYTES - min(one - per_slice, WORKSPACE_BUDGET_BYTES)) // per_slice))
    n_chunks = -(-slices // fit)
    return int(-(-slices // n_chunks))          # equal chunks


def _attention_call(entry: str, ws_query: str, Q, K, V, phi, feature_map, bh_chunk, return_num_den, workspace, out, stream,
                    prepared=None):
    _require_gpu()
    L = lib()
    B, H, n, d = _check_qkv(Q, K, V)
    if bh_chunk is None:
        bh_chunk = _auto_chunk(L, ws_query, B, H, n, d, phi.nnz, phi.n_f) if workspace is None else 0
    need = getattr(L, ws_query)(B, H, n, d, phi.nnz, phi.n_f, bh_chunk)
    if need == 0:
        raise GrfError(GRF_EUNSUPPORTED, f"unsupported problem (d={d})")
    if prepared is not None:
        need -= L.grf_phi_prepare_bytes(n, phi.nnz, phi.n_f)
    if workspace is None:
        workspace = _workspace(need, Q.device)
    if out is None:
        out = torch.empty((B, H, n, d), dtype=torch.float32, device=Q.device)
    num = torch.empty((B, H, n, d), dtype=torch.float32, device=Q.device) if return_num_den else None
    den = torch.empty((B, H, n), dtype=torch.float32, device=Q.device) if return_num_den else None
    ps = phi._struct()
    if prepared is not None:
        _check(getattr(L, entry + "_prepared")(_ptr(Q), _ptr(K), _ptr(V), _dtype_code(Q), B, H, n, d, ctypes.byref(ps),
                                               phi.nnz, phi.n_f, _FEATURE_MAPS[feature_map], int(bh_chunk),
                                               _ptr(prepared), prepared.numel(), _ptr(workspace), workspace.numel(),
                                               _stream_ptr(stream), _ptr(out), _ptr(num), _ptr(den)))
        return (out, num, den) if return_num_den else out
    _check(getattr(L, entry)(_ptr(Q), _ptr(K), _ptr(V), _dtype_code(Q), B, H, n, d, ctypes.byref(ps),
                             phi.nnz, phi.n_f, _FEATURE_MAPS[feature_map], int(bh_chunk),
                             _ptr(workspace), workspace.numel(), _stream_ptr(stream),
                             _ptr(out), _ptr(num), _ptr(den)))
    return (out, num, den) if return_num_den else out


def grf_asymmetric_masked_attention(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, phi: Phi, feature_map: str = "relu",
                                    return_num_den: bool = False, out: Optional[torch.Tensor] = None, stream=None):
    """Asymmetric-GRF masked attention (mask estimate = phi itself, sampled with f = alpha)."""
    _require_gpu()
    L = lib()
    B, H, n, d = _check_qkv(Q, K, V)
    if out is None:
        out = torch.empty((B, H, n, d), dtype=torch.float32, device=Q.device)
    num = torch.empty((B, H, n, d), dtype=torch.float32, device=Q.device) if return_num_den else None
    den = torch.empty((B, H, n), dtype=torch.float32, device=Q.device) if return_num_den else None
    ps = phi._struct()
    _check(L.grf_asymmetric_masked_attention(_ptr(Q), _ptr(K), _ptr(V), _dtype_code(Q), B, H, n, d, ctypes.byref(ps),
                                             phi.nnz, phi.n_f, _FEATURE_MAPS[feature_map], _stream_ptr(stream),
                                             _ptr(out), _ptr(num), _ptr(den)))
    return (out, num, den) if return_num_den else out


# --------------------------------------------------------------------------- gradients

def grf_attention_backward_workspace_bytes(B: int, H: int, n: int, d: int, nnz: int, n_f: int = 1, bh_chunk: int = 0) -> int:
    return int(lib().grf_attention_backward_workspace_bytes(B, H, n, d, nnz, n_f, bh_chunk))


def grf_asymmetric_backward_workspace_bytes(B: int, H: int, n: int, d: int, nnz: int, n_f: int = 1, bh_chunk: int = 0) -> int:
    return int(lib().grf_asymmetric_backward_workspace_bytes(B, H, n, d, nnz, n_f, bh_chunk))


def grf_asymmetric_masked_attention_backward(Q, K, V, phi: Phi, out, den, d_out, feature_map: str = "relu", bh_chunk: Optional[int] = None,
                                             want_dphi: bool = True, workspace: Optional[torch.Tensor] = None, stream=None):
    """Backward of grf_asymmetric_masked_attention: (dQ, dK, dV, dphi_val), arguments as the symmetric backward."""
    return _backward_call("grf_asymmetric_masked_attention_backward", "grf_asymmetric_backward_workspace_bytes",
                          Q, K, V, phi, out, den, d_out, feature_map, bh_chunk, want_dphi, workspace, stream)


def grf_masked_linear_attention_backward(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, phi: Phi,
                                         out: torch.Tensor, den: torch.Tensor, d_out: torch.Tensor,
                                         feature_map: str = "relu", bh_chunk: Optional[int] = None, want_dphi: bool = True,
                                         workspace: Optional[torch.Tensor] = None, stream=None,
                                         prepared: Optional[torch.Tensor] = None):
    """(dQ, dK, dV, dphi_val) for d_out = dL/dout; ``out`` and ``den`` are the saved forward results (fp32).

    dphi_val is [n_f, capacity] fp32 (entries beyond nnz untouched), or None when ``want_dphi`` is False."""
    return _backward_call("grf_masked_linear_attention_backward", "grf_attention_backward_workspace_bytes",
                          Q, K, V, phi, out, den, d_out, feature_map, bh_chunk, want_dphi, workspace, stream, prepared)


def _backward_call(entry, ws_query, Q, K, V, phi, out, den, d_out, feature_map, bh_chunk, want_dphi, workspace, stream, prepared=None):
    _require_gpu()
    L = lib()
    B, H, n, d = _check_qkv(Q, K, V)
    if bh_chunk is None:
        bh_chunk = _auto_chunk(L, ws_query, B, H, n, d, phi.nnz, phi.n_f) if workspace is None else 0
    for t, shape in ((out, (B, H, n, d)), (d_out, (B, H, n, d)), (den, (B, H, n))):
        if tuple(t.shape) != shape or t.dtype != torch.float32 or not t.is_contiguous() or not t.is_cuda:
            raise ValueError("out, den, d_out must be contiguous fp32 CUDA tensors of shapes [B,H,n,d], [B,H,n], [B,H,n,d]")
    need = getattr(L, ws_query)(B, H, n, d, phi.nnz, phi.n_f, bh_chunk)
    if need == 0:
        raise GrfError(GRF_EUNSUPPORTED, f"unsupported problem (d={d})")
    if prepared is not None:
        need -= L.grf_phi_prepare_bytes(n, phi.nnz, phi.n_f)
    if workspace is None:
        workspace = _workspace(need, Q.device)
    dQ, dK, dV = (torch.empty((B, H, n, d), dtype=torch.float32, device=Q.device) for _ in range(3))
    dphi = torch.empty((phi.n_f, phi.capacity), dtype=torch.float32, device=Q.device) if want_dphi else None
    ps = phi._struct()
    if prepared is not None:
        _check(getattr(L, entry + "_prepared")(
            _ptr(Q), _ptr(K), _ptr(V), _dtype_code(Q), B, H, n, d, ctypes.byref(ps), phi.nnz, phi.n_f,
            _FEATURE_MAPS[feature_map], _ptr(out), _ptr(den), _ptr(d_out), int(bh_chunk), _ptr(prepared), prepared.numel(),
            _ptr(workspace), workspace.numel(), _stream_ptr(stream), _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(dphi)))
        return dQ, dK, dV, dphi
    _check(getattr(L, entry)(
        _ptr(Q), _ptr(K), _ptr(V), _dtype_code(Q), B, H, n, d, ctypes.byref(ps), phi.nnz, phi.n_f,
        _FEATURE_MAPS[feature_map], _ptr(out), _ptr(den), _ptr(d_out), int(bh_chunk),
        _ptr(workspace), workspace.numel(), _stream_ptr(stream), _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(dphi)))
    return dQ, dK, dV, dphi


def grf_sample_backward(graph: DeviceGraph, f_len: int, p_halt: float, n_walks: int, seed: int, phi: Phi,
                        dphi_val: torch.Tensor, stream=None) -> torch.Tensor:
    """df [n_f, f_len] fp32 on the GPU from dphi_val [n_f, capacity]; same walk arguments as the grf_sample call."""
    _require_gpu()
    L = lib()
    if tuple(dphi_val.shape) != (phi.n_f, phi.capacity) or dphi_val.dtype != torch.float32 or not dphi_val.is_contiguous():
        raise ValueError("dphi_val must be a contiguous fp32 tensor [n_f, capacity]")
    dev = graph.row_ptr.device
    ws = _workspace(L.grf_sample_backward_workspace_bytes(graph.n, int(n_walks), int(f_len), phi.n_f), dev)
    df = torch.empty((phi.n_f, f_len), dtype=torch.float32, device=dev)
    gs, ps = graph._struct(), phi._struct()
    _check(L.grf_sample_backward(ctypes.byref(gs), int(f_len), phi.n_f, float(p_halt), int(n_walks),
                                 int(seed) & 0xFFFFFFFFFFFFFFFF, ctypes.byref(ps), phi.nnz, _ptr(dphi_val),
                                 _ptr(ws), ws.numel(), _stream_ptr(stream), _ptr(df)))
    return df
