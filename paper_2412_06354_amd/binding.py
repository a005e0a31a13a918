"""Thin ctypes binding of libgnn_mi355x.so (argument marshalling only).

PyTorch-ROCm supplies device memory (``tensor.data_ptr()``) and the HIP stream
(``torch.cuda.current_stream().cuda_stream``); every step of the path runs in the
library's kernels.  There is no CPU or eager fallback: if the library is missing
or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgnn_mi355x.so")

MSG_COPY_XJ, MSG_E_MUL_XJ, MSG_XJ_SUB_XI, MSG_XI_DOT_XJ = 0, 1, 2, 3
AGGR_SUM, AGGR_MEAN, AGGR_MAX, AGGR_MIN, AGGR_PROD = 0, 1, 2, 3, 4
EDGE_ORDER_COO, EDGE_ORDER_CSR = 0, 1

_c = ctypes
_vp, _i32, _i64, _f32, _sz = _c.c_void_p, _c.c_int32, _c.c_int64, _c.c_float, _c.c_size_t

# name -> (restype, argtypes); every symbol declared in include/gnn.h
SIGNATURES = {
    "gnn_status_string": (_c.c_char_p, [_c.c_int]),
    "gnn_build_csr": (_c.c_int, [_vp, _vp, _i64, _i32, _vp, _c.POINTER(_vp)]),
    "gnn_build_csr_ex": (_c.c_int, [_vp, _vp, _i64, _i32, _i32, _i32, _vp, _c.POINTER(_vp)]),
    "gnn_build_csr_batch": (_c.c_int, [_i32, _vp, _vp, _vp, _i32, _vp, _vp]),
    "gnn_graph_reserve": (_c.c_int, [_vp, _i32, _i32]),
    "gnn_check_graph_indicator": (_c.c_int, [_vp, _i32, _i32, _vp]),
    "gnn_graph_destroy": (_c.c_int, [_vp]),
    "gnn_graph_rowptr": (_vp, [_vp]),
    "gnn_graph_colidx": (_vp, [_vp]),
    "gnn_graph_perm": (_vp, [_vp]),
    "gnn_graph_indegree": (_vp, [_vp]),
    "gnn_graph_num_nodes": (_i32, [_vp]),
    "gnn_graph_num_edges": (_i64, [_vp]),
    "gnn_graph_work_sizes": (None, [_vp, _c.POINTER(_i32), _c.POINTER(_i32), _c.POINTER(_i32)]),
    "gnn_graph_work_lists": (None, [_vp] + [_c.POINTER(_vp)] * 6),
    "gnn_edge_data_to_csr": (_c.c_int, [_vp, _vp, _i32, _vp, _vp]),
    "gnn_edge_data_to_coo": (_c.c_int, [_vp, _vp, _i32, _vp, _vp]),
    "gnn_graph_build_edge_route": (_c.c_int, [_vp, _vp]),
    "gnn_propagate": (_c.c_int, [_vp, _vp, _i32, _vp, _i32, _c.c_int, _c.c_int, _c.c_int, _vp, _vp]),
    "gnn_propagate_noalloc": (_c.c_int, [_vp, _vp, _i32, _vp, _i32, _c.c_int, _c.c_int, _c.c_int, _vp, _vp]),
    "gnn_build_csr_bipartite": (_c.c_int, [_vp, _vp, _i64, _i32, _i32, _vp, _c.POINTER(_vp)]),
    "gnn_graph_num_src_nodes": (_i32, [_vp]),
    "gnn_hetero_propagate": (_c.c_int, [_i32, _vp, _vp, _vp, _i32, _i32, _c.c_int, _c.c_int, _c.c_int, _vp, _vp]),
    "gnn_release_cached_memory": (_c.c_int, []),
    "gnn_propagate_bf16": (_c.c_int, [_vp, _vp, _i32, _vp, _c.c_int, _c.c_int, _c.c_int, _vp, _vp]),
    "gnn_f32_to_bf16": (_c.c_int, [_vp, _i64, _vp, _vp]),
    "gnn_propagate_f16": (_c.c_int, [_vp, _vp, _i32, _vp, _c.c_int, _c.c_int, _c.c_int, _vp, _vp]),
    "gnn_f32_to_f16": (_c.c_int, [_vp, _i64, _vp, _vp]),
    "gnn_apply_edges": (_c.c_int, [_vp, _vp, _i32, _vp, _i32, _c.c_int, _c.c_int, _vp, _c.c_int, _vp]),
    "gnn_aggregate_neighbors": (_c.c_int, [_vp, _vp, _i32, _c.c_int, _c.c_int, _vp, _vp]),
    "gnn_propagate_backward_workspace_bytes": (_sz, [_i32, _i32, _c.c_int]),
    "gnn_propagate_argmax": (_c.c_int, [_vp, _vp, _i32, _vp, _i32, _c.c_int, _c.c_int, _vp, _vp, _vp]),
    "gnn_propagate_backward": (_c.c_int, [_vp, _vp, _vp, _i32, _vp, _i32, _c.c_int, _c.c_int, _vp, _vp, _vp, _vp, _vp,
                                          _sz, _vp]),
    "gnn_gcnconv_workspace_bytes": (_sz, [_i32, _i32]),
    "gnn_gcnconv": (_c.c_int, [_vp, _vp, _i32, _vp, _vp, _i32, _i32, _c.c_int, _vp, _vp, _sz, _vp]),
    "gnn_gcnconv_backward_workspace_bytes": (_sz, [_i32, _i32, _i32]),
    "gnn_gcnconv_backward": (_c.c_int, [_vp, _vp, _vp, _i32, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "gnn_segment_softmax": (_c.c_int, [_vp, _vp, _i32, _c.c_int, _vp, _vp]),
    "gnn_segment_softmax_backward": (_c.c_int, [_vp, _vp, _vp, _i32, _c.c_int, _vp, _vp]),
    "gnn_gatconv_workspace_bytes": (_sz, [_i32, _i32, _i32]),
    "gnn_gatconv": (_c.c_int, [_vp, _vp, _i32, _vp, _vp, _vp, _i32, _i32, _f32, _vp, _vp, _vp, _sz, _vp]),
    "gnn_gatconv_backward_workspace_bytes": (_sz, [_i32, _i32, _i32, _i32]),
    "gnn_gatconv_backward": (_c.c_int, [_vp, _vp, _vp, _i32, _vp, _vp, _vp, _i32, _i32, _f32, _vp, _vp, _vp, _vp, _vp,
                                        _vp, _vp, _vp, _sz, _vp]),
    "gnn_graph_pool": (_c.c_int, [_vp, _i32, _i32, _vp, _i32, _c.c_int, _vp, _vp]),
    "gnn_graph_pool_workspace_bytes": (_c.c_size_t, [_i32, _i32, _i32]),
    "gnn_graph_pool_ws": (_c.c_int, [_vp, _i32, _i32, _vp, _i32, _c.c_int, _vp, _vp, _c.c_size_t, _vp]),
    "gnn_gin_update": (_c.c_int, [_vp, _vp, _i32, _f32, _vp, _vp]),
    "gnn_batchnorm_workspace_bytes": (_sz, [_i32, _i32]),
    "gnn_batchnorm": (_c.c_int, [_vp, _i32, _i32, _vp, _vp, _f32, _c.c_int, _i32, _vp, _vp, _vp, _vp, _sz, _vp]),
    "gnn_dense": (_c.c_int, [_vp, _i64, _i32, _vp, _i32, _vp, _c.c_int, _vp, _vp]),
    "gnn_example_model_workspace_bytes": (_sz, [_i32, _i32, _i32, _i32]),
    "gnn_example_model_forward": (_c.c_int, [_vp, _vp, _i32, _vp, _i32, _vp, _vp, _i32, _vp, _vp, _f32, _vp, _vp, _i32,
                                             _vp, _vp, _i32, _vp, _vp, _sz, _vp]),
    "gnn_mse_loss": (_c.c_int, [_vp, _vp, _i64, _vp, _vp, _vp]),
    "gnn_relu_backward": (_c.c_int, [_vp, _vp, _i64, _vp, _vp]),
    "gnn_graph_pool_backward": (_c.c_int, [_vp, _i32, _i32, _vp, _i32, _c.c_int, _vp, _vp]),
    "gnn_dense_backward_workspace_bytes": (_sz, [_i64, _i32, _i32]),
    "gnn_dense_backward": (_c.c_int, [_vp, _i64, _i32, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "gnn_batchnorm_backward_workspace_bytes": (_sz, [_i32, _i32]),
    "gnn_batchnorm_backward": (_c.c_int, [_vp, _i32, _i32, _vp, _vp, _vp, _f32, _vp, _vp, _vp, _vp, _vp, _vp, _sz,
                                          _vp]),
    "gnn_adam_step": (_c.c_int, [_vp, _vp, _vp, _vp, _i64, _f32, _f32, _f32, _f32, _i32, _vp]),
    "gnn_example_model_train_workspace_bytes": (_sz, [_i32, _i32, _i32, _i32, _i32, _i32]),
    "gnn_example_model_train_step": (_c.c_int, [_vp, _vp, _vp, _i32, _vp, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp,
                                                _f32, _f32, _f32, _f32, _f32, _i32, _vp, _vp, _sz, _vp]),
    "gnn_dense_xw": (_c.c_int, [_vp, _i64, _i32, _vp, _i32, _vp, _vp, _vp]),
}

_lib = None


class GnnError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        msg = lib().gnn_status_string(code).decode() if _lib is not None else "?"
        super().__init__(f"{what}: {msg} (gnn_status {code})")


def lib():
    """Loads the shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2412_06354_amd.build`")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def _check(code: int, what: str):
    if code != 0:
        raise GnnError(code, what)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: Optional[torch.Tensor], dtype, name: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise TypeError(f"{name} must live in device memory")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _edge_rows(t: torch.Tensor, num_edges: int) -> torch.Tensor:
    """[E, width] view of per-edge data given as [E] or [E, width] (also when E == 0)."""
    if num_edges == 0:
        return t.reshape(0, int(t.shape[1]) if t.dim() == 2 else 1)
    return t.reshape(num_edges, -1)


class Graph:
    """Owner of a ``gnn_graph`` handle (CSR by destination + work lists, all in device memory)."""

    def __init__(self, handle: int, device: torch.device):
        self._h = handle
        self.device = device
        self.num_nodes = int(lib().gnn_graph_num_nodes(handle))
        self.num_src_nodes = int(lib().gnn_graph_num_src_nodes(handle))
        self.num_edges = int(lib().gnn_graph_num_edges(handle))
        self._reserved_heads = 0

    def reserve(self, max_feat_dim: int = 0, max_heads: int = 0) -> None:
        """gnn_graph_reserve: sizes the handle's scratch memory (may allocate and synchronise the device)."""
        _check(lib().gnn_graph_reserve(self._h, int(max_feat_dim), int(max_heads)), "gnn_graph_reserve")
        self._reserved_heads = max(self._reserved_heads, int(max_heads))

    def build_edge_route(self) -> None:
        """gnn_graph_build_edge_route: one float per edge then moves between COO and CSR order in streams."""
        _check(lib().gnn_graph_build_edge_route(self._h, _stream()), "gnn_graph_build_edge_route")

    def _view(self, ptr: int, count: int) -> torch.Tensor:
        """Copy of a library-owned int32 device array as a tensor."""
        out = torch.empty(count, dtype=torch.int32, device=self.device)
        if count:   # ordered on the caller's stream, like the work that fills and later reads the arrays
            _hip_memcpy_d2d(out.data_ptr(), ptr, 4 * count, _stream())
        return out

    @property
    def rowptr(self):
        return self._view(lib().gnn_graph_rowptr(self._h), self.num_nodes + 1)

    @property
    def colidx(self):
        return self._view(lib().gnn_graph_colidx(self._h), self.num_edges)

    @property
    def perm(self):
        return self._view(lib().gnn_graph_perm(self._h), self.num_edges)

    @property
    def indegree(self):
        return self._view(lib().gnn_graph_indegree(self._h), self.num_nodes)

    def work_sizes(self):
        a, b, c = _i32(), _i32(), _i32()
        lib().gnn_graph_work_sizes(self._h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c))
        return {"small_rows": a.value, "items": b.value, "split_rows": c.value}

    def work_lists(self):
        """Copies of the work lists as int32 tensors (see gnn_graph_work_lists)."""
        sizes = self.work_sizes()
        ptrs = [_vp() for _ in range(6)]
        lib().gnn_graph_work_lists(self._h, *[ctypes.byref(p) for p in ptrs])
        names = ("small_rows", "item_row", "item_start", "item_slot", "split_rows", "split_slot0")
        counts = (sizes["small_rows"],) + (sizes["items"],) * 3 + (sizes["split_rows"],) * 2
        return {k: self._view(p.value or 0, c) for k, p, c in zip(names, ptrs, counts)}

    def close(self):
        if self._h:
            torch.cuda.synchronize()
            lib().gnn_graph_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


_hip = None


def _hip_memcpy_d2d(dst: int, src: int, nbytes: int, stream: int):
    """Device-to-device copy enqueued on `stream` (a plain hipMemcpy between device buffers is ordered with the
    null stream only, which the non-blocking streams PyTorch creates do not wait for)."""
    global _hip
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")
        _hip.hipMemcpyAsync.restype = ctypes.c_int
        _hip.hipMemcpyAsync.argtypes = [_vp, _vp, _sz, ctypes.c_int, _vp]
    rc = _hip.hipMemcpyAsync(dst, src, nbytes, 3, stream)  # hipMemcpyDeviceToDevice
    if rc != 0:
        raise RuntimeError(f"hipMemcpyAsync failed ({rc})")


def build_csr(src: torch.Tensor, dst: torch.Tensor, num_nodes: int, small_max_degree: int = 0,
              chunk_edges: int = 0) -> Graph:
    e = int(src.shape[0])
    if int(dst.shape[0]) != e:
        raise ValueError("src and dst must have the same length")
    out = _vp()
    if small_max_degree == 0 and chunk_edges == 0:
        rc = lib().gnn_build_csr(_dev(src, torch.int32, "src"), _dev(dst, torch.int32, "dst"), e, num_nodes,
                                 _stream(), ctypes.byref(out))
    else:
        rc = lib().gnn_build_csr_ex(_dev(src, torch.int32, "src"), _dev(dst, torch.int32, "dst"), e, num_nodes,
                                    small_max_degree, chunk_edges, _stream(), ctypes.byref(out))
    _check(rc, "gnn_build_csr")
    return Graph(out.value, src.device)


def build_csr_batch(srcs, dsts, num_nodes: int):
    """Temporal snapshots over one node set -> one Graph per snapshot (one allocation, one synchronisation)."""
    t = len(srcs)
    if t == 0 or len(dsts) != t:
        raise ValueError("one src and one dst array per snapshot")
    for a, b in zip(srcs, dsts):
        if int(a.shape[0]) != int(b.shape[0]):
            raise ValueError("src and dst must have the same length")
    arr = _vp * t
    sp = arr(*[_dev(a, torch.int32, "src") if a.numel() else None for a in srcs])
    dp = arr(*[_dev(a, torch.int32, "dst") if a.numel() else None for a in dsts])
    ne = (_i64 * t)(*[int(a.shape[0]) for a in srcs])
    out = arr()
    rc = lib().gnn_build_csr_batch(t, sp, dp, ne, num_nodes, _stream(), out)
    _check(rc, "gnn_build_csr_batch")
    return [Graph(out[i], srcs[0].device) for i in range(t)]


def check_graph_indicator(graph_indicator: torch.Tensor, num_graphs: int) -> None:
    """Raises GnnError (index range / not sorted) unless the indicator is what gnn_graph_pool expects."""
    rc = lib().gnn_check_graph_indicator(_dev(graph_indicator, torch.int32, "graph_indicator"),
                                         int(graph_indicator.shape[0]), num_graphs, _stream())
    _check(rc, "gnn_check_graph_indicator")


def release_cached_memory() -> None:
    _check(lib().gnn_release_cached_memory(), "gnn_release_cached_memory")


def build_csr_bipartite(src: torch.Tensor, dst: torch.Tensor, num_src_nodes: int, num_dst_nodes: int) -> Graph:
    """One relation of a heterogeneous graph: rows are the destination type's nodes."""
    e = int(src.shape[0])
    if int(dst.shape[0]) != e:
        raise ValueError("src and dst must have the same length")
    out = _vp()
    rc = lib().gnn_build_csr_bipartite(_dev(src, torch.int32, "src"), _dev(dst, torch.int32, "dst"), e, num_src_nodes,
                                       num_dst_nodes, _stream(), ctypes.byref(out))
    _check(rc, "gnn_build_csr_bipartite")
    return Graph(out.value, src.device)


def hetero_propagate(graphs, xs, es=None, msg: int = MSG_COPY_XJ, aggr: int = AGGR_SUM,
                     e_order: int = EDGE_ORDER_COO, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Sum over relations (graphs[r], xs[r], es[r]) that end in one destination node type."""
    r = len(graphs)
    if r == 0 or len(xs) != r or (es is not None and len(es) != r):
        raise ValueError("one feature matrix (and one edge-data array) per relation")
    f = int(xs[0].shape[1])
    e_dim = 1
    e2 = None
    if es is not None:
        e2 = [_edge_rows(e, g.num_edges) for g, e in zip(graphs, es)]
        e_dim = int(e2[0].shape[1])
    for g, x in zip(graphs, xs):
        if tuple(x.shape) != (g.num_src_nodes, f):
            raise ValueError("x[r] must be [num_src_nodes of relation r, F]")
    if out is None:
        out = torch.empty((graphs[0].num_nodes, f), dtype=torch.float32, device=xs[0].device)
    arr = _vp * r
    gh = arr(*[g._h for g in graphs])
    xp = arr(*[_dev(x, torch.float32, "x") for x in xs])
    ep = arr(*[_dev(e, torch.float32, "e") for e in e2]) if e2 is not None else None
    rc = lib().gnn_hetero_propagate(r, gh, xp, ep, f, e_dim, e_order, msg, aggr, _dev(out, torch.float32, "out"),
                                    _stream())
    _check(rc, "gnn_hetero_propagate")
    return out


def edge_data_to_csr(g: Graph, e: torch.Tensor) -> torch.Tensor:
    e2 = _edge_rows(e, g.num_edges)
    out = torch.empty_like(e2)
    _check(lib().gnn_edge_data_to_csr(g._h, _dev(e2, torch.float32, "e"), e2.shape[1],
                                      out.data_ptr(), _stream()), "gnn_edge_data_to_csr")
    return out.reshape(e.shape)


def edge_data_to_coo(g: Graph, e_csr: torch.Tensor) -> torch.Tensor:
    e2 = _edge_rows(e_csr, g.num_edges)
    out = torch.empty_like(e2)
    _check(lib().gnn_edge_data_to_coo(g._h, _dev(e2, torch.float32, "e_csr"), e2.shape[1],
                                      out.data_ptr(), _stream()), "gnn_edge_data_to_coo")
    return out.reshape(e_csr.shape)


def propagate(g: Graph, x: torch.Tensor, e: Optional[torch.Tensor] = None, msg: int = MSG_COPY_XJ,
              aggr: int = AGGR_SUM, e_order: int = EDGE_ORDER_COO,
              out: Optional[torch.Tensor] = None) -> torch.Tensor:
    n, f = x.shape
    if n != g.num_src_nodes:
        raise ValueError("x must have one row per (source) node")
    e_dim = 1
    if e is not None:
        e = _edge_rows(e, g.num_edges)
        e_dim = int(e.shape[1])
    if out is None:
        out = torch.empty((g.num_nodes, f), dtype=torch.float32, device=x.device)
    rc = lib().gnn_propagate(g._h, _dev(x, torch.float32, "x"), f, _dev(e, torch.float32, "e"), e_dim,
                             e_order, msg, aggr, _dev(out, torch.float32, "out"), _stream())
    _check(rc, "gnn_propagate")
    return out


def propagate_noalloc(g: Graph, x: torch.Tensor, e: Optional[torch.Tensor], msg: int, aggr: int, e_order: int,
                      out: torch.Tensor) -> torch.Tensor:
    """gnn_propagate_noalloc: the caller passes every buffer, the partial rows go to the library's fixed array."""
    n, f = x.shape
    e_dim = 1
    if e is not None:
        e = _edge_rows(e, g.num_edges)
        e_dim = int(e.shape[1])
    rc = lib().gnn_propagate_noalloc(g._h, _dev(x, torch.float32, "x"), f, _dev(e, torch.float32, "e"), e_dim,
                                     e_order, msg, aggr, _dev(out, torch.float32, "out"), _stream())
    _check(rc, "gnn_propagate_noalloc")
    return out


def f32_to_bf16(x: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """float32 -> bfloat16 codes (an int16 tensor holding the 16-bit patterns), round to nearest even."""
    if out is None:
        out = torch.empty(x.shape, dtype=torch.int16, device=x.device)
    rc = lib().gnn_f32_to_bf16(_dev(x, torch.float32, "x"), x.numel(), _dev(out, torch.int16, "out"), _stream())
    _check(rc, "gnn_f32_to_bf16")
    return out


def propagate_bf16(g: Graph, x_bf16: torch.Tensor, e: Optional[torch.Tensor] = None, msg: int = MSG_COPY_XJ,
                   aggr: int = AGGR_SUM, e_order: int = EDGE_ORDER_COO,
                   out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """x_bf16: [N, F] int16 tensor of bfloat16 codes (from f32_to_bf16, or a torch.bfloat16 tensor viewed as int16)."""
    n, f = x_bf16.shape
    if n != g.num_nodes:
        raise ValueError("x must have one row per node")
    if e is not None and e.numel() != g.num_edges:
        raise ValueError("one weight per edge")
    if out is None:
        out = torch.empty((n, f), dtype=torch.float32, device=x_bf16.device)
    rc = lib().gnn_propagate_bf16(g._h, _dev(x_bf16, torch.int16, "x_bf16"), f, _dev(e, torch.float32, "e"), e_order,
                                  msg, aggr, _dev(out, torch.float32, "out"), _stream())
    _check(rc, "gnn_propagate_bf16")
    return out


def f32_to_f16(x: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """float32 -> IEEE binary16 codes (an int16 tensor holding the 16-bit patterns), round to nearest even."""
    if out is None:
        out = torch.empty(x.shape, dtype=torch.int16, device=x.device)
    rc = lib().gnn_f32_to_f16(_dev(x, torch.float32, "x"), x.numel(), _dev(out, torch.int16, "out"), _stream())
    _check(rc, "gnn_f32_to_f16")
    return out


def propagate_f16(g: Graph, x_f16: torch.Tensor, e: Optional[torch.Tensor] = None, msg: int = MSG_COPY_XJ,
                  aggr: int = AGGR_SUM, e_order: int = EDGE_ORDER_COO,
                  out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """x_f16: [N, F] int16 tensor of binary16 codes (from f32_to_f16, or a torch.float16 tensor viewed as int16)."""
    n, f = x_f16.shape
    if n != g.num_nodes:
        raise ValueError("x must have one row per node")
    if e is not None and e.numel() != g.num_edges:
        raise ValueError("one weight per edge")
    if out is None:
        out = torch.empty((n, f), dtype=torch.float32, device=x_f16.device)
    rc = lib().gnn_propagate_f16(g._h, _dev(x_f16, torch.int16, "x_f16"), f, _dev(e, torch.float32, "e"), e_order,
                                 msg, aggr, _dev(out, torch.float32, "out"), _stream())
    _check(rc, "gnn_propagate_f16")
    return out


def apply_edges(g: Graph, x: torch.Tensor, e: Optional[torch.Tensor] = None, msg: int = MSG_COPY_XJ,
                e_order: int = EDGE_ORDER_COO, m_order: int = EDGE_ORDER_COO,
                out: Optional[torch.Tensor] = None) -> torch.Tensor:
    n, f = x.shape
    if n != g.num_src_nodes:
        raise ValueError("x must have one row per (source) node")
    e_dim = 1
    if e is not None:
        e = _edge_rows(e, g.num_edges)
        e_dim = int(e.shape[1])
    if out is None:
        out = torch.empty((g.num_edges, 1 if msg == MSG_XI_DOT_XJ else f), dtype=torch.float32, device=x.device)
    rc = lib().gnn_apply_edges(g._h, _dev(x, torch.float32, "x"), f, _dev(e, torch.float32, "e"), e_dim, e_order, msg,
                               _dev(out, torch.float32, "out"), m_order, _stream())
    _check(rc, "gnn_apply_edges")
    return out


def aggregate_neighbors(g: Graph, m: torch.Tensor, aggr: int = AGGR_SUM, m_order: int = EDGE_ORDER_COO,
                        out: Optional[torch.Tensor] = None) -> torch.Tensor:
    ne, f = m.shape
    if ne != g.num_edges:
        raise ValueError("m must have one row per edge")
    if out is None:
        out = torch.empty((g.num_nodes, f), dtype=torch.float32, device=m.device)
    rc = lib().gnn_aggregate_neighbors(g._h, _dev(m, torch.float32, "m"), f, m_order, aggr,
                                       _dev(out, torch.float32, "out"), _stream())
    _check(rc, "gnn_aggregate_neighbors")
    return out


def propagate_argmax(g: Graph, x: torch.Tensor, out_max: torch.Tensor, e: Optional[torch.Tensor] = None,
                     msg: int = MSG_COPY_XJ, e_order: int = EDGE_ORDER_COO) -> torch.Tensor:
    n, f = x.shape
    e_dim = 1
    if e is not None:
        e = _edge_rows(e, g.num_edges)
        e_dim = int(e.shape[1])
    am = torch.empty((n, f), dtype=torch.int32, device=x.device)
    rc = lib().gnn_propagate_argmax(g._h, _dev(x, torch.float32, "x"), f, _dev(e, torch.float32, "e"), e_dim, e_order,
                                    msg, _dev(out_max, torch.float32, "out_max"), am.data_ptr(), _stream())
    _check(rc, "gnn_propagate_argmax")
    return am


def propagate_backward(g: Graph, g_by_source: Optional[Graph], x: torch.Tensor, grad_out: torch.Tensor,
                       e: Optional[torch.Tensor] = None, msg: int = MSG_COPY_XJ, aggr: int = AGGR_SUM,
                       want_grad_x: bool = True, want_grad_e: bool = True,
                       argmax: Optional[torch.Tensor] = None):
    """-> (grad_x or None, grad_e or None); edge data and grad_e are in the caller's edge order."""
    n, f = grad_out.shape
    e_dim = 1
    e2 = None
    if e is not None:
        e2 = _edge_rows(e, g.num_edges)
        e_dim = int(e2.shape[1])
    grad_x = torch.empty_like(grad_out) if want_grad_x else None
    grad_e = torch.empty_like(e2) if (want_grad_e and e2 is not None and msg == MSG_E_MUL_XJ) else None
    need = int(lib().gnn_propagate_backward_workspace_bytes(n, f, aggr))
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=grad_out.device)
    rc = lib().gnn_propagate_backward(g._h, g_by_source._h if g_by_source is not None else None,
                                      _dev(x, torch.float32, "x"), f, _dev(e2, torch.float32, "e"), e_dim, msg, aggr,
                                      _dev(grad_out, torch.float32, "grad_out"), _dev(argmax, torch.int32, "argmax"),
                                      _dev(grad_x, torch.float32, "grad_x"),
                                      _dev(grad_e, torch.float32, "grad_e"), ws.data_ptr(), ws.numel(), _stream())
    _check(rc, "gnn_propagate_backward")
    if grad_e is not None and e is not None:
        grad_e = grad_e.reshape(e.shape)
    return grad_x, grad_e


ACT_NONE, ACT_RELU = 0, 1


def gcnconv(g: Graph, x: torch.Tensor, w: torch.Tensor, bias: Optional[torch.Tensor] = None,
            add_self_loops: bool = True, out: Optional[torch.Tensor] = None,
            workspace: Optional[torch.Tensor] = None, relu: bool = False) -> torch.Tensor:
    n, f_in = x.shape
    f_out = int(w.shape[1])
    if n != g.num_nodes or w.shape[0] != f_in:
        raise ValueError("shape mismatch")
    need = int(lib().gnn_gcnconv_workspace_bytes(n, f_out))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    if out is None:
        out = torch.empty((n, f_out), dtype=torch.float32, device=x.device)
    rc = lib().gnn_gcnconv(g._h, _dev(x, torch.float32, "x"), f_in, _dev(w, torch.float32, "w"),
                           _dev(bias, torch.float32, "bias"), f_out, 1 if add_self_loops else 0,
                           ACT_RELU if relu else ACT_NONE, _dev(out, torch.float32, "out"), workspace.data_ptr(),
                           workspace.numel(), _stream())
    _check(rc, "gnn_gcnconv")
    return out


def gcnconv_backward(g: Graph, g_by_source: Graph, x: torch.Tensor, w: torch.Tensor, grad_out: torch.Tensor,
                     add_self_loops: bool = True, workspace: Optional[torch.Tensor] = None):
    """-> (grad_x [N, f_in], grad_w [f_in, f_out], grad_b [f_out])."""
    n, f_in = x.shape
    f_out = int(w.shape[1])
    if tuple(grad_out.shape) != (n, f_out) or w.shape[0] != f_in:
        raise ValueError("shape mismatch")
    need = int(lib().gnn_gcnconv_backward_workspace_bytes(n, f_in, f_out))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    gx = torch.empty_like(x)
    gw = torch.empty_like(w)
    gb = torch.empty(f_out, dtype=torch.float32, device=x.device)
    rc = lib().gnn_gcnconv_backward(g._h, g_by_source._h, _dev(x, torch.float32, "x"), f_in, _dev(w, torch.float32, "w"),
                                    f_out, 1 if add_self_loops else 0, _dev(grad_out, torch.float32, "grad_out"),
                                    gx.data_ptr(), gw.data_ptr(), gb.data_ptr(), workspace.data_ptr(),
                                    workspace.numel(), _stream())
    _check(rc, "gnn_gcnconv_backward")
    return gx, gw, gb


def segment_softmax(g: Graph, scores: torch.Tensor, order: int = EDGE_ORDER_COO,
                    out: Optional[torch.Tensor] = None) -> torch.Tensor:
    s2 = _edge_rows(scores, g.num_edges)
    if out is None:
        out = torch.empty_like(scores)
    if g.num_edges and g._reserved_heads < int(s2.shape[1]):
        g.reserve(0, int(s2.shape[1]))
    rc = lib().gnn_segment_softmax(g._h, _dev(s2, torch.float32, "scores"), int(s2.shape[1]) if g.num_edges else 1,
                                   order, _dev(out, torch.float32, "out"), _stream())
    _check(rc, "gnn_segment_softmax")
    return out


def segment_softmax_backward(g: Graph, alpha: torch.Tensor, grad_alpha: torch.Tensor, order: int = EDGE_ORDER_COO,
                             out: Optional[torch.Tensor] = None) -> torch.Tensor:
    if alpha.shape != grad_alpha.shape:
        raise ValueError("shape mismatch")
    a2, g2 = _edge_rows(alpha, g.num_edges), _edge_rows(grad_alpha, g.num_edges)
    if out is None:
        out = torch.empty_like(alpha)
    if g.num_edges and g._reserved_heads < int(a2.shape[1]):
        g.reserve(0, int(a2.shape[1]))
    rc = lib().gnn_segment_softmax_backward(g._h, _dev(a2, torch.float32, "alpha"),
                                            _dev(g2, torch.float32, "grad_alpha"),
                                            int(a2.shape[1]) if g.num_edges else 1, order,
                                            _dev(out, torch.float32, "out"), _stream())
    _check(rc, "gnn_segment_softmax_backward")
    return out


def gatconv(g: Graph, x: torch.Tensor, w: torch.Tensor, a_src: torch.Tensor, a_dst: torch.Tensor,
            negative_slope: float = 0.2, out: Optional[torch.Tensor] = None,
            workspace: Optional[torch.Tensor] = None, softmax_stats: Optional[torch.Tensor] = None) -> torch.Tensor:
    """softmax_stats: optional [N, heads, 2] float32 tensor that receives what gatconv_backward needs."""
    n, f_in = x.shape
    heads, ch = a_src.shape
    if n != g.num_nodes or tuple(w.shape) != (f_in, heads * ch) or tuple(a_dst.shape) != (heads, ch):
        raise ValueError("shape mismatch")
    if softmax_stats is not None and tuple(softmax_stats.shape) != (n, heads, 2):
        raise ValueError("softmax_stats must be [N, heads, 2]")
    need = int(lib().gnn_gatconv_workspace_bytes(n, heads, ch))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    if out is None:
        out = torch.empty((n, heads * ch), dtype=torch.float32, device=x.device)
    rc = lib().gnn_gatconv(g._h, _dev(x, torch.float32, "x"), f_in, _dev(w, torch.float32, "w"),
                           _dev(a_src, torch.float32, "a_src"), _dev(a_dst, torch.float32, "a_dst"), heads, ch,
                           float(negative_slope), _dev(out, torch.float32, "out"),
                           _dev(softmax_stats, torch.float32, "softmax_stats"), workspace.data_ptr(),
                           workspace.numel(), _stream())
    _check(rc, "gnn_gatconv")
    return out


def gatconv_backward(g: Graph, g_by_source: Graph, x: torch.Tensor, w: torch.Tensor, a_src: torch.Tensor,
                     a_dst: torch.Tensor, out: torch.Tensor, softmax_stats: torch.Tensor, grad_out: torch.Tensor,
                     negative_slope: float = 0.2, workspace: Optional[torch.Tensor] = None):
    """-> (grad_x, grad_w, grad_a_src, grad_a_dst); `out` and `softmax_stats` come from gatconv."""
    n, f_in = x.shape
    heads, ch = a_src.shape
    hc = heads * ch
    if (n != g.num_nodes or tuple(w.shape) != (f_in, hc) or tuple(a_dst.shape) != (heads, ch) or
            tuple(out.shape) != (n, hc) or tuple(grad_out.shape) != (n, hc) or
            tuple(softmax_stats.shape) != (n, heads, 2)):
        raise ValueError("shape mismatch")
    need = int(lib().gnn_gatconv_backward_workspace_bytes(n, f_in, heads, ch))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    gx = torch.empty((n, f_in), dtype=torch.float32, device=x.device)
    gw = torch.empty((f_in, hc), dtype=torch.float32, device=x.device)
    gas = torch.empty((heads, ch), dtype=torch.float32, device=x.device)
    gad = torch.empty((heads, ch), dtype=torch.float32, device=x.device)
    rc = lib().gnn_gatconv_backward(g._h, g_by_source._h, _dev(x, torch.float32, "x"), f_in,
                                    _dev(w, torch.float32, "w"), _dev(a_src, torch.float32, "a_src"),
                                    _dev(a_dst, torch.float32, "a_dst"), heads, ch, float(negative_slope),
                                    _dev(out, torch.float32, "out"), _dev(softmax_stats, torch.float32, "softmax_stats"),
                                    _dev(grad_out, torch.float32, "grad_out"), gx.data_ptr(), gw.data_ptr(),
                                    gas.data_ptr(), gad.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream())
    _check(rc, "gnn_gatconv_backward")
    return gx, gw, gas, gad


def batchnorm(x: torch.Tensor, gamma: Optional[torch.Tensor] = None, beta: Optional[torch.Tensor] = None,
              eps: float = 1e-5, relu: bool = False, mean: Optional[torch.Tensor] = None,
              var: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None):
    """-> (out, mean, var); batch statistics unless both mean and var are given."""
    n, f = x.shape
    given = mean is not None and var is not None
    if not given:
        mean = torch.empty(f, dtype=torch.float32, device=x.device)
        var = torch.empty(f, dtype=torch.float32, device=x.device)
    if out is None:
        out = torch.empty_like(x)
    ws = torch.empty(max(int(lib().gnn_batchnorm_workspace_bytes(n, f)), 256), dtype=torch.uint8, device=x.device)
    rc = lib().gnn_batchnorm(_dev(x, torch.float32, "x"), n, f, _dev(gamma, torch.float32, "gamma"),
                             _dev(beta, torch.float32, "beta"), float(eps), ACT_RELU if relu else ACT_NONE,
                             1 if given else 0, _dev(mean, torch.float32, "mean"), _dev(var, torch.float32, "var"),
                             _dev(out, torch.float32, "out"), ws.data_ptr(), ws.numel(), _stream())
    _check(rc, "gnn_batchnorm")
    return out, mean, var


def dense(x: torch.Tensor, w: torch.Tensor, bias: Optional[torch.Tensor] = None, relu: bool = False,
          out: Optional[torch.Tensor] = None) -> torch.Tensor:
    rows, k = x.shape
    if int(w.shape[0]) != k:
        raise ValueError("shape mismatch")
    n = int(w.shape[1])
    if out is None:
        out = torch.empty((rows, n), dtype=torch.float32, device=x.device)
    rc = lib().gnn_dense(_dev(x, torch.float32, "x"), rows, k, _dev(w, torch.float32, "w"), n,
                         _dev(bias, torch.float32, "bias"), ACT_RELU if relu else ACT_NONE,
                         _dev(out, torch.float32, "out"), _stream())
    _check(rc, "gnn_dense")
    return out


def example_model_forward(g: Graph, graph_indicator: torch.Tensor, num_graphs: int, x: torch.Tensor, params: dict,
                          eps: float = 1e-5, out: Optional[torch.Tensor] = None,
                          workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """params: device tensors w1 [f0,f1], b1, gamma, beta, w2 [f1,f2], b2, w3 [f2,f3], b3."""
    n, f0 = x.shape
    f1, f2, f3 = int(params["w1"].shape[1]), int(params["w2"].shape[1]), int(params["w3"].shape[1])
    if (n != g.num_nodes or int(params["w1"].shape[0]) != f0 or int(params["w2"].shape[0]) != f1 or
            int(params["w3"].shape[0]) != f2 or int(graph_indicator.shape[0]) != n):
        raise ValueError("shape mismatch")
    need = int(lib().gnn_example_model_workspace_bytes(n, num_graphs, f1, f2))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    if out is None:
        out = torch.empty((num_graphs, f3), dtype=torch.float32, device=x.device)
    t = lambda k: _dev(params.get(k), torch.float32, k)
    rc = lib().gnn_example_model_forward(g._h, _dev(graph_indicator, torch.int32, "graph_indicator"), num_graphs,
                                         _dev(x, torch.float32, "x"), f0, t("w1"), t("b1"), f1, t("gamma"), t("beta"),
                                         float(eps), t("w2"), t("b2"), f2, t("w3"), t("b3"), f3,
                                         _dev(out, torch.float32, "out"), workspace.data_ptr(), workspace.numel(),
                                         _stream())
    _check(rc, "gnn_example_model_forward")
    return out


PARAM_ORDER = ("w1", "b1", "gamma", "beta", "w2", "b2", "w3", "b3")


def mse_loss(pred: torch.Tensor, target: torch.Tensor):
    """-> (loss as a 1-element device tensor, grad with respect to pred)."""
    if pred.shape != target.shape:
        raise ValueError("shape mismatch")
    loss = torch.empty(1, dtype=torch.float32, device=pred.device)
    grad = torch.empty_like(pred)
    rc = lib().gnn_mse_loss(_dev(pred, torch.float32, "pred"), _dev(target, torch.float32, "target"), pred.numel(),
                            loss.data_ptr(), grad.data_ptr(), _stream())
    _check(rc, "gnn_mse_loss")
    return loss, grad


def relu_backward(y: torch.Tensor, grad_y: torch.Tensor) -> torch.Tensor:
    out = torch.empty_like(grad_y)
    rc = lib().gnn_relu_backward(_dev(y, torch.float32, "y"), _dev(grad_y, torch.float32, "grad_y"), y.numel(),
                                 out.data_ptr(), _stream())
    _check(rc, "gnn_relu_backward")
    return out


def graph_pool_backward(graph_indicator: torch.Tensor, num_graphs: int, grad_out: torch.Tensor,
                        aggr: int = AGGR_MEAN) -> torch.Tensor:
    n, f = int(graph_indicator.shape[0]), int(grad_out.shape[1])
    gx = torch.empty((n, f), dtype=torch.float32, device=grad_out.device)
    rc = lib().gnn_graph_pool_backward(_dev(graph_indicator, torch.int32, "graph_indicator"), n, num_graphs,
                                       _dev(grad_out, torch.float32, "grad_out"), f, aggr, gx.data_ptr(), _stream())
    _check(rc, "gnn_graph_pool_backward")
    return gx


def dense_backward(x: torch.Tensor, w: torch.Tensor, grad_y: torch.Tensor):
    """-> (grad_x, grad_w, grad_b) of out = x w + b."""
    rows, k = x.shape
    n = int(w.shape[1])
    gx = torch.empty_like(x)
    gw = torch.empty_like(w)
    gb = torch.empty(n, dtype=torch.float32, device=x.device)
    ws = torch.empty(int(lib().gnn_dense_backward_workspace_bytes(rows, k, n)), dtype=torch.uint8, device=x.device)
    rc = lib().gnn_dense_backward(_dev(x, torch.float32, "x"), rows, k, _dev(w, torch.float32, "w"), n,
                                  _dev(grad_y, torch.float32, "grad_y"), gx.data_ptr(), gw.data_ptr(), gb.data_ptr(),
                                  ws.data_ptr(), ws.numel(), _stream())
    _check(rc, "gnn_dense_backward")
    return gx, gw, gb


def batchnorm_backward(x: torch.Tensor, gamma: Optional[torch.Tensor], mean: torch.Tensor, var: torch.Tensor,
                       grad_y: torch.Tensor, eps: float = 1e-5, y_relu: Optional[torch.Tensor] = None):
    """-> (grad_x, grad_gamma, grad_beta); y_relu = the output of a relu fused after the normalisation."""
    n, f = x.shape
    gx = torch.empty_like(x)
    gg = torch.empty(f, dtype=torch.float32, device=x.device)
    gb = torch.empty(f, dtype=torch.float32, device=x.device)
    ws = torch.empty(int(lib().gnn_batchnorm_backward_workspace_bytes(n, f)), dtype=torch.uint8, device=x.device)
    rc = lib().gnn_batchnorm_backward(_dev(x, torch.float32, "x"), n, f, _dev(gamma, torch.float32, "gamma"),
                                      _dev(mean, torch.float32, "mean"), _dev(var, torch.float32, "var"), float(eps),
                                      _dev(grad_y, torch.float32, "grad_y"), _dev(y_relu, torch.float32, "y_relu"),
                                      gx.data_ptr(), gg.data_ptr(), gb.data_ptr(), ws.data_ptr(), ws.numel(), _stream())
    _check(rc, "gnn_batchnorm_backward")
    return gx, gg, gb


def adam_step(p: torch.Tensor, m: torch.Tensor, v: torch.Tensor, g: torch.Tensor, lr: float, step: int,
              beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8) -> None:
    """Updates p, m, v in place."""
    rc = lib().gnn_adam_step(_dev(p, torch.float32, "p"), _dev(m, torch.float32, "m"), _dev(v, torch.float32, "v"),
                             _dev(g, torch.float32, "g"), p.numel(), float(lr), float(beta1), float(beta2), float(eps),
                             int(step), _stream())
    _check(rc, "gnn_adam_step")


def example_model_train_step(g: Graph, g_by_source: Graph, graph_indicator: torch.Tensor, num_graphs: int,
                             x: torch.Tensor, target: torch.Tensor, params: dict, adam_m: dict, adam_v: dict,
                             step: int, lr: float = 1e-4, bn_eps: float = 1e-5, beta1: float = 0.9,
                             beta2: float = 0.999, adam_eps: float = 1e-8, loss: Optional[torch.Tensor] = None,
                             workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """One training step of the example model (forward, MSE loss, gradients, Adam); params / adam_m / adam_v are
    dicts of device tensors keyed as PARAM_ORDER and are updated in place.  Returns the loss (1-element tensor)."""
    n, f0 = x.shape
    f1, f2, f3 = int(params["w1"].shape[1]), int(params["w2"].shape[1]), int(params["w3"].shape[1])
    if n != g.num_nodes or tuple(target.shape) != (num_graphs, f3) or int(graph_indicator.shape[0]) != n:
        raise ValueError("shape mismatch")
    need = int(lib().gnn_example_model_train_workspace_bytes(n, num_graphs, f0, f1, f2, f3))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    if loss is None:
        loss = torch.empty(1, dtype=torch.float32, device=x.device)
    arr = _vp * 8
    pp = arr(*[_dev(params[k], torch.float32, k) for k in PARAM_ORDER])
    pm = arr(*[_dev(adam_m[k], torch.float32, k) for k in PARAM_ORDER])
    pv = arr(*[_dev(adam_v[k], torch.float32, k) for k in PARAM_ORDER])
    rc = lib().gnn_example_model_train_step(g._h, g_by_source._h, _dev(graph_indicator, torch.int32, "graph_indicator"),
                                            num_graphs, _dev(x, torch.float32, "x"), f0, f1, f2, f3,
                                            _dev(target, torch.float32, "target"), pp, pm, pv, float(bn_eps), float(lr),
                                            float(beta1), float(beta2), float(adam_eps), int(step), loss.data_ptr(),
                                            workspace.data_ptr(), workspace.numel(), _stream())
    _check(rc, "gnn_example_model_train_step")
    return loss


def graph_pool(graph_indicator: torch.Tensor, num_graphs: int, x: torch.Tensor, aggr: int = AGGR_SUM,
               out: Optional[torch.Tensor] = None) -> torch.Tensor:
    n, f = x.shape
    if int(graph_indicator.shape[0]) != n:
        raise ValueError("graph_indicator must have one entry per node")
    if out is None:
        out = torch.empty((num_graphs, f), dtype=torch.float32, device=x.device)
    rc = lib().gnn_graph_pool(_dev(graph_indicator, torch.int32, "graph_indicator"), n, num_graphs,
                              _dev(x, torch.float32, "x"), f, aggr, _dev(out, torch.float32, "out"), _stream())
    _check(rc, "gnn_graph_pool")
    return out


def graph_pool_ws(graph_indicator: torch.Tensor, num_graphs: int, x: torch.Tensor, aggr: int = AGGR_SUM,
                  out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """gnn_graph_pool_ws: the readout with several blocks per graph for batches of few, large graphs."""
    n, f = x.shape
    if int(graph_indicator.shape[0]) != n:
        raise ValueError("graph_indicator must have one entry per node")
    if out is None:
        out = torch.empty((num_graphs, f), dtype=torch.float32, device=x.device)
    need = int(lib().gnn_graph_pool_workspace_bytes(n, num_graphs, f))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    rc = lib().gnn_graph_pool_ws(_dev(graph_indicator, torch.int32, "graph_indicator"), n, num_graphs,
                                 _dev(x, torch.float32, "x"), f, aggr, _dev(out, torch.float32, "out"),
                                 workspace.data_ptr(), workspace.numel(), _stream())
    _check(rc, "gnn_graph_pool_ws")
    return out


def gin_update(g: Graph, x: torch.Tensor, eps: float = 0.0, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    n, f = x.shape
    if n != g.num_nodes:
        raise ValueError("x must have one row per node")
    if out is None:
        out = torch.empty_like(x)
    rc = lib().gnn_gin_update(g._h, _dev(x, torch.float32, "x"), f, float(eps), _dev(out, torch.float32, "out"),
                              _stream())
    _check(rc, "gnn_gin_update")
    return out


def dense_xw(x: torch.Tensor, w: torch.Tensor, row_scale: Optional[torch.Tensor] = None,
             out: Optional[torch.Tensor] = None) -> torch.Tensor:
    rows, k = x.shape
    n = int(w.shape[1])
    if w.shape[0] != k:
        raise ValueError("shape mismatch")
    if out is None:
        out = torch.empty((rows, n), dtype=torch.float32, device=x.device)
    rc = lib().gnn_dense_xw(_dev(x, torch.float32, "x"), rows, k, _dev(w, torch.float32, "w"), n,
                            _dev(row_scale, torch.float32, "row_scale"), _dev(out, torch.float32, "out"), _stream())
    _check(rc, "gnn_dense_xw")
    return out
