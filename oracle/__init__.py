"""numpy front-end of the CPU oracle (``gnn_oracle.c``) -- TEST INFRASTRUCTURE ONLY.

The oracle is the plain definition of every operation on the message-passing
path (paper section 3, "Message Passing": apply_edges, aggregate_neighbors,
propagate; layers named in "Graph Convolutional Layers" / "Training Example").
Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package; the GPU library never does, and this package never imports it.

The wrapper does argument marshalling only: it checks dtypes/shapes, allocates
outputs and calls the C functions.  ``build()`` compiles the C file with gcc.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gnn_oracle.c")
_LIB = os.path.join(_HERE, "libgnn_oracle.so")

MSG_COPY_XJ, MSG_E_MUL_XJ, MSG_XJ_SUB_XI, MSG_XI_DOT_XJ = 0, 1, 2, 3
AGGR_SUM, AGGR_MEAN, AGGR_MAX, AGGR_MIN, AGGR_PROD = 0, 1, 2, 3, 4

_lib = None


class OracleError(RuntimeError):
    pass


def build(force: bool = True) -> str:
    """Compile the oracle (plain gcc, no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math",
                               "-Wall", "-Wextra", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _i32(a, name):
    a = np.ascontiguousarray(a)
    if a.dtype != np.int32:
        raise TypeError(f"{name} must be int32")
    return a


def _f32(a, name):
    a = np.ascontiguousarray(a)
    if a.dtype != np.float32:
        raise TypeError(f"{name} must be float32")
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc, what):
    if rc != 0:
        reason = {1: "index out of range", 2: "bad size or enum", 3: "out of memory"}.get(rc, "?")
        raise OracleError(f"{what}: {reason} (code {rc})")


def build_csr(src, dst, num_nodes: int):
    """-> (rowptr[N+1], colidx[E], perm[E], indeg[N]) int32; stable within a row."""
    src, dst = _i32(src, "src"), _i32(dst, "dst")
    e = src.shape[0]
    rowptr = np.empty(num_nodes + 1, np.int32)
    colidx = np.empty(e, np.int32)
    perm = np.empty(e, np.int32)
    indeg = np.empty(num_nodes, np.int32)
    rc = _load().oracle_build_csr(_p(src), _p(dst), ctypes.c_int64(e), ctypes.c_int32(num_nodes),
                                  _p(rowptr), _p(colidx), _p(perm), _p(indeg))
    _check(rc, "build_csr")
    return rowptr, colidx, perm, indeg


def _edge_data(e, num_edges, feat):
    if e is None:
        return None, 1
    e = _f32(e, "e")
    if e.ndim == 1:
        e = e.reshape(num_edges, 1)
    if e.shape[0] != num_edges:
        raise ValueError("e must have one row per edge")
    return e, int(e.shape[1])


def apply_edges(src, num_nodes: int, x, e=None, msg: int = MSG_COPY_XJ, dst=None, with_sabs: bool = False):
    """[E, F] message rows; for MSG_XI_DOT_XJ one scalar per edge, [E, 1] (with_sabs applies to it only)."""
    src, x = _i32(src, "src"), _f32(x, "x")
    dst = None if dst is None else _i32(dst, "dst")
    ne, f = src.shape[0], x.shape[1]
    e, e_dim = _edge_data(e, ne, f)
    m = np.empty((ne, 1 if msg == MSG_XI_DOT_XJ else f), np.float32)
    sabs = np.empty((ne, 1), np.float64) if (with_sabs and msg == MSG_XI_DOT_XJ) else None
    rc = _load().oracle_apply_edges(_p(src), _p(dst), ctypes.c_int64(ne), ctypes.c_int32(num_nodes), _p(x),
                                    ctypes.c_int32(f), _p(e), ctypes.c_int32(e_dim),
                                    ctypes.c_int32(msg), _p(m), _p(sabs))
    _check(rc, "apply_edges")
    return (m, sabs) if with_sabs else m


def aggregate_neighbors(dst, num_nodes: int, m, aggr: int = AGGR_SUM, with_sabs: bool = False):
    dst, m = _i32(dst, "dst"), _f32(m, "m")
    ne, f = m.shape
    out = np.empty((num_nodes, f), np.float32)
    sabs = np.empty((num_nodes, f), np.float64) if with_sabs else None
    rc = _load().oracle_aggregate_neighbors(_p(dst), ctypes.c_int64(ne), ctypes.c_int32(num_nodes),
                                            _p(m), ctypes.c_int32(f), ctypes.c_int32(aggr),
                                            _p(out), _p(sabs))
    _check(rc, "aggregate_neighbors")
    return (out, sabs) if with_sabs else out


def propagate(src, dst, num_nodes: int, x, e=None, msg: int = MSG_COPY_XJ, aggr: int = AGGR_SUM,
              with_sabs: bool = False):
    src, dst, x = _i32(src, "src"), _i32(dst, "dst"), _f32(x, "x")
    ne, f = src.shape[0], x.shape[1]
    e, e_dim = _edge_data(e, ne, f)
    if msg == MSG_E_MUL_XJ and e is None:
        raise ValueError("e_mul_xj needs edge data")
    out = np.empty((num_nodes, f), np.float32)
    sabs = np.empty((num_nodes, f), np.float64) if with_sabs else None
    rc = _load().oracle_propagate(_p(src), _p(dst), ctypes.c_int64(ne), ctypes.c_int32(num_nodes),
                                  _p(x), ctypes.c_int32(f), _p(e), ctypes.c_int32(e_dim),
                                  ctypes.c_int32(msg), ctypes.c_int32(aggr), _p(out), _p(sabs))
    _check(rc, "propagate")
    return (out, sabs) if with_sabs else out


def propagate_all_cores(src, dst, num_nodes: int, x, e=None, msg: int = MSG_COPY_XJ, aggr: int = AGGR_SUM):
    """propagate with the rows dealt to OpenMP threads (the all-cores CPU baseline) -> (out, threads used);
    bit-identical to propagate()."""
    src, dst, x = _i32(src, "src"), _i32(dst, "dst"), _f32(x, "x")
    ne, f = src.shape[0], x.shape[1]
    e, e_dim = _edge_data(e, ne, f)
    if msg == MSG_E_MUL_XJ and e is None:
        raise ValueError("e_mul_xj needs edge data")
    out = np.empty((num_nodes, f), np.float32)
    threads = ctypes.c_int32(0)
    rc = _load().oracle_propagate_all_cores(_p(src), _p(dst), ctypes.c_int64(ne), ctypes.c_int32(num_nodes),
                                            _p(x), ctypes.c_int32(f), _p(e), ctypes.c_int32(e_dim),
                                            ctypes.c_int32(msg), ctypes.c_int32(aggr), _p(out), ctypes.byref(threads))
    _check(rc, "propagate_all_cores")
    return out, int(threads.value)


def propagate_backward(src, dst, num_nodes: int, x, grad_out, e=None, msg: int = MSG_COPY_XJ,
                       aggr: int = AGGR_SUM, with_sabs: bool = False):
    """-> dict(grad_x, grad_e (None for copy_xj), argmax (max only), [sabs_x, sabs_e])."""
    src, dst, x, g = _i32(src, "src"), _i32(dst, "dst"), _f32(x, "x"), _f32(grad_out, "grad_out")
    ne, f = src.shape[0], x.shape[1]
    e, e_dim = _edge_data(e, ne, f)
    if msg == MSG_E_MUL_XJ and e is None:
        raise ValueError("e_mul_xj needs edge data")
    if g.shape != (num_nodes, f):
        raise ValueError("grad_out must be [N, F]")
    gx = np.empty((num_nodes, f), np.float32)
    ge = np.empty((ne, e_dim), np.float32) if msg == MSG_E_MUL_XJ else None
    am = np.empty((num_nodes, f), np.int32)
    sx = np.empty((num_nodes, f), np.float64) if with_sabs else None
    se = np.empty((ne, e_dim), np.float64) if (with_sabs and ge is not None) else None
    rc = _load().oracle_propagate_backward(_p(src), _p(dst), ctypes.c_int64(ne), ctypes.c_int32(num_nodes), _p(x),
                                           ctypes.c_int32(f), _p(e), ctypes.c_int32(e_dim), ctypes.c_int32(msg),
                                           ctypes.c_int32(aggr), _p(g), _p(gx), _p(ge), _p(am), _p(sx), _p(se))
    _check(rc, "propagate_backward")
    return {"grad_x": gx, "grad_e": ge, "argmax": am if aggr == AGGR_MAX else None, "sabs_x": sx, "sabs_e": se}


def gcnconv(src, dst, num_nodes: int, x, w, bias=None, add_self_loops: bool = True,
            with_sabs: bool = False):
    src, dst, x, w = _i32(src, "src"), _i32(dst, "dst"), _f32(x, "x"), _f32(w, "w")
    bias = None if bias is None else _f32(bias, "bias")
    ne, f_in, f_out = src.shape[0], x.shape[1], w.shape[1]
    if w.shape[0] != f_in:
        raise ValueError("w must be [f_in, f_out]")
    out = np.empty((num_nodes, f_out), np.float32)
    sabs = np.empty((num_nodes, f_out), np.float64) if with_sabs else None
    rc = _load().oracle_gcnconv(_p(src), _p(dst), ctypes.c_int64(ne), ctypes.c_int32(num_nodes),
                                _p(x), ctypes.c_int32(f_in), _p(w), _p(bias), ctypes.c_int32(f_out),
                                ctypes.c_int32(1 if add_self_loops else 0), _p(out), _p(sabs))
    _check(rc, "gcnconv")
    return (out, sabs) if with_sabs else out


def gcnconv_backward(src, dst, num_nodes: int, x, w, grad_out, add_self_loops: bool = True):
    """-> dict(grad_x, grad_w, grad_b, sabs_x, sabs_w, sabs_b)."""
    src, dst, x, w, g = _i32(src, "src"), _i32(dst, "dst"), _f32(x, "x"), _f32(w, "w"), _f32(grad_out, "grad_out")
    ne, f_in, f_out = src.shape[0], x.shape[1], w.shape[1]
    if w.shape[0] != f_in or g.shape != (num_nodes, f_out):
        raise ValueError("shape mismatch")
    gx, sx = np.empty((num_nodes, f_in), np.float32), np.empty((num_nodes, f_in), np.float64)
    gw, sw = np.empty((f_in, f_out), np.float32), np.empty((f_in, f_out), np.float64)
    gb, sb = np.empty(f_out, np.float32), np.empty(f_out, np.float64)
    rc = _load().oracle_gcnconv_backward(_p(src), _p(dst), ctypes.c_int64(ne), ctypes.c_int32(num_nodes), _p(x),
                                         ctypes.c_int32(f_in), _p(w), ctypes.c_int32(f_out),
                                         ctypes.c_int32(1 if add_self_loops else 0), _p(g), _p(gx), _p(gw), _p(gb),
                                         _p(sx), _p(sw), _p(sb))
    _check(rc, "gcnconv_backward")
    return {"grad_x": gx, "grad_w": gw, "grad_b": gb, "sabs_x": sx, "sabs_w": sw, "sabs_b": sb}


def segment_softmax(dst, num_nodes: int, scores) -> np.ndarray:
    dst, s = _i32(dst, "dst"), _f32(scores, "scores")
    ne = dst.shape[0]
    s2 = s.reshape(ne, -1)
    h = s2.shape[1] if ne else (s.shape[1] if s.ndim == 2 else 1)
    alpha = np.empty_like(s2)
    rc = _load().oracle_segment_softmax(_p(dst), ctypes.c_int64(ne), ctypes.c_int32(num_nodes),
                                        _p(s2), ctypes.c_int32(h), _p(alpha))
    _check(rc, "segment_softmax")
    return alpha.reshape(s.shape)


def gatconv(src, dst, num_nodes: int, x, w, a_src, a_dst, negative_slope: float = 0.2,
            with_sabs: bool = False):
    src, dst, x, w = _i32(src, "src"), _i32(dst, "dst"), _f32(x, "x"), _f32(w, "w")
    a_src, a_dst = _f32(a_src, "a_src"), _f32(a_dst, "a_dst")
    heads, ch = a_src.shape
    ne, f_in = src.shape[0], x.shape[1]
    if w.shape != (f_in, heads * ch) or a_dst.shape != (heads, ch):
        raise ValueError("shape mismatch")
    out = np.empty((num_nodes, heads * ch), np.float32)
    sabs = np.empty((num_nodes, heads * ch), np.float64) if with_sabs else None
    rc = _load().oracle_gatconv(_p(src), _p(dst), ctypes.c_int64(ne), ctypes.c_int32(num_nodes),
                                _p(x), ctypes.c_int32(f_in), _p(w), _p(a_src), _p(a_dst),
                                ctypes.c_int32(heads), ctypes.c_int32(ch),
                                ctypes.c_float(negative_slope), _p(out), _p(sabs))
    _check(rc, "gatconv")
    return (out, sabs) if with_sabs else out


def segment_softmax_backward(dst, num_nodes: int, alpha, grad_alpha, with_sabs: bool = False):
    """d scores from d alpha for the per-destination softmax (alpha = the forward result)."""
    dst, a, ga = _i32(dst, "dst"), _f32(alpha, "alpha"), _f32(grad_alpha, "grad_alpha")
    ne = dst.shape[0]
    if a.shape != ga.shape:
        raise ValueError("shape mismatch")
    a2, ga2 = a.reshape(ne, -1), ga.reshape(ne, -1)
    h = a2.shape[1] if ne else (a.shape[1] if a.ndim == 2 else 1)
    gs = np.empty_like(a2)
    sabs = np.empty(a2.shape, np.float64) if with_sabs else None
    rc = _load().oracle_segment_softmax_backward(_p(dst), ctypes.c_int64(ne), ctypes.c_int32(num_nodes), _p(a2),
                                                 _p(ga2), ctypes.c_int32(h), _p(gs), _p(sabs))
    _check(rc, "segment_softmax_backward")
    return (gs.reshape(a.shape), sabs.reshape(a.shape)) if with_sabs else gs.reshape(a.shape)


def gatconv_backward(src, dst, num_nodes: int, x, w, a_src, a_dst, grad_out, negative_slope: float = 0.2):
    """Gradients of the attention layer; returns a dict with grad_x, grad_w, grad_a_src, grad_a_dst and
    the matching sabs_* magnitudes."""
    src, dst, x, w = _i32(src, "src"), _i32(dst, "dst"), _f32(x, "x"), _f32(w, "w")
    a_src, a_dst, gout = _f32(a_src, "a_src"), _f32(a_dst, "a_dst"), _f32(grad_out, "grad_out")
    heads, ch = a_src.shape
    ne, f_in = src.shape[0], x.shape[1]
    if w.shape != (f_in, heads * ch) or a_dst.shape != (heads, ch) or gout.shape != (num_nodes, heads * ch):
        raise ValueError("shape mismatch")
    res = {"grad_x": np.empty((num_nodes, f_in), np.float32), "grad_w": np.empty((f_in, heads * ch), np.float32),
           "grad_a_src": np.empty((heads, ch), np.float32), "grad_a_dst": np.empty((heads, ch), np.float32),
           "sabs_x": np.empty((num_nodes, f_in), np.float64), "sabs_w": np.empty((f_in, heads * ch), np.float64),
           "sabs_a_src": np.empty((heads, ch), np.float64), "sabs_a_dst": np.empty((heads, ch), np.float64)}
    rc = _load().oracle_gatconv_backward(_p(src), _p(dst), ctypes.c_int64(ne), ctypes.c_int32(num_nodes),
                                         _p(x), ctypes.c_int32(f_in), _p(w), _p(a_src), _p(a_dst),
                                         ctypes.c_int32(heads), ctypes.c_int32(ch), ctypes.c_float(negative_slope),
                                         _p(gout), _p(res["grad_x"]), _p(res["grad_w"]), _p(res["grad_a_src"]),
                                         _p(res["grad_a_dst"]), _p(res["sabs_x"]), _p(res["sabs_w"]),
                                         _p(res["sabs_a_src"]), _p(res["sabs_a_dst"]))
    _check(rc, "gatconv_backward")
    return res


def dense(x, w, bias=None, relu: bool = False, with_sabs: bool = False):
    x, w = _f32(x, "x"), _f32(w, "w")
    bias = None if bias is None else _f32(bias, "bias")
    n_rows, k = x.shape
    if w.shape[0] != k or (bias is not None and bias.shape != (w.shape[1],)):
        raise ValueError("shape mismatch")
    out = np.empty((n_rows, w.shape[1]), np.float32)
    sabs = np.empty(out.shape, np.float64) if with_sabs else None
    rc = _load().oracle_dense(_p(x), ctypes.c_int32(n_rows), ctypes.c_int32(k), _p(w), ctypes.c_int32(w.shape[1]),
                              _p(bias), ctypes.c_int32(1 if relu else 0), _p(out), _p(sabs))
    _check(rc, "dense")
    return (out, sabs) if with_sabs else out


def batchnorm(x, gamma=None, beta=None, eps: float = 1e-5, relu: bool = False, mean=None, var=None):
    """-> (out, mean, var).  Batch statistics unless mean and var are given."""
    x = _f32(x, "x")
    n, f = x.shape
    gamma = None if gamma is None else _f32(gamma, "gamma")
    beta = None if beta is None else _f32(beta, "beta")
    given = mean is not None and var is not None
    mean_io = _f32(mean, "mean").copy() if given else np.empty(f, np.float32)
    var_io = _f32(var, "var").copy() if given else np.empty(f, np.float32)
    out = np.empty_like(x)
    rc = _load().oracle_batchnorm(_p(x), ctypes.c_int32(n), ctypes.c_int32(f), _p(gamma), _p(beta),
                                  ctypes.c_float(eps), ctypes.c_int32(1 if relu else 0),
                                  ctypes.c_int32(1 if given else 0), _p(mean_io), _p(var_io), _p(out))
    _check(rc, "batchnorm")
    return out, mean_io, var_io


def example_model_forward(src, dst, num_nodes: int, graph_indicator, num_graphs: int, x, params: dict,
                          eps: float = 1e-5):
    """The paper's example model (section 3, "Training Example"), step by step with the functions above:
    GCNConv(f0 => f1) -> BatchNorm(f1) over the nodes of the batch -> relu -> GCNConv(f1 => f2) + relu ->
    mean pooling per graph -> Dense(f2, f3).  Every intermediate is a stored float tensor.
    Returns the dict of all intermediates; "y" is the prediction [num_graphs, f3]."""
    h1 = gcnconv(src, dst, num_nodes, x, params["w1"], params["b1"], True)
    h2, mean, var = batchnorm(h1, params["gamma"], params["beta"], eps, relu=True)
    h3 = np.maximum(gcnconv(src, dst, num_nodes, h2, params["w2"], params["b2"], True), np.float32(0))
    pooled = graph_pool(graph_indicator, num_graphs, h3, AGGR_MEAN)
    y = dense(pooled, params["w3"], params["b3"])
    return {"h1": h1, "h2": h2, "mean": mean, "var": var, "h3": h3, "pooled": pooled, "y": y}


def round_bf16(x):
    """-> (codes uint16, widened float32): finite floats rounded to bfloat16, ties to even."""
    x = _f32(x, "x")
    flat = np.ascontiguousarray(x.reshape(-1))
    codes = np.empty(flat.shape, np.uint16)
    wide = np.empty(flat.shape, np.float32)
    rc = _load().oracle_round_bf16(_p(flat), ctypes.c_int64(flat.shape[0]), _p(codes), _p(wide))
    _check(rc, "round_bf16")
    return codes.reshape(x.shape), wide.reshape(x.shape)


def round_f16(x):
    """-> (codes uint16, widened float32): finite floats rounded to IEEE binary16, ties to even."""
    x = _f32(x, "x")
    flat = np.ascontiguousarray(x.reshape(-1))
    codes = np.empty(flat.shape, np.uint16)
    wide = np.empty(flat.shape, np.float32)
    rc = _load().oracle_round_f16(_p(flat), ctypes.c_int64(flat.shape[0]), _p(codes), _p(wide))
    _check(rc, "round_f16")
    return codes.reshape(x.shape), wide.reshape(x.shape)


def hetero_propagate(relations, num_dst_nodes: int, msg: int = MSG_COPY_XJ, aggr: int = AGGR_SUM,
                     with_sabs: bool = False):
    """Sum over the relations that end in one destination node type of each relation's propagate.
    relations: list of dicts with src, dst (indices into the relation's own source / the common
    destination node set), num_src_nodes, x [num_src_nodes, F] and optionally e [E] or [E, F]."""
    f = _f32(relations[0]["x"], "x").shape[1]
    out64 = np.zeros((num_dst_nodes, f), np.float64)
    sabs = np.zeros((num_dst_nodes, f), np.float64)
    for r in relations:
        src, dst, x = _i32(r["src"], "src"), _i32(r["dst"], "dst"), _f32(r["x"], "x")
        ne = src.shape[0]
        e, e_dim = _edge_data(r.get("e"), ne, f)
        rc = _load().oracle_propagate_relation_add(_p(src), _p(dst), ctypes.c_int64(ne),
                                                   ctypes.c_int32(int(r["num_src_nodes"])),
                                                   ctypes.c_int32(num_dst_nodes), _p(x), ctypes.c_int32(f), _p(e),
                                                   ctypes.c_int32(e_dim), ctypes.c_int32(msg), ctypes.c_int32(aggr),
                                                   _p(out64), _p(sabs))
        _check(rc, "hetero_propagate")
    out = out64.astype(np.float32)
    return (out, sabs) if with_sabs else out


def dense_backward(x, w, grad_out):
    x, w, gy = _f32(x, "x"), _f32(w, "w"), _f32(grad_out, "grad_out")
    n_rows, k = x.shape
    n = w.shape[1]
    gx, gw, gb = np.empty((n_rows, k), np.float32), np.empty((k, n), np.float32), np.empty(n, np.float32)
    rc = _load().oracle_dense_backward(_p(x), ctypes.c_int32(n_rows), ctypes.c_int32(k), _p(w), ctypes.c_int32(n),
                                       _p(gy), _p(gx), _p(gw), _p(gb))
    _check(rc, "dense_backward")
    return gx, gw, gb


def batchnorm_backward(x, gamma, grad_out, eps: float = 1e-5):
    x, gy = _f32(x, "x"), _f32(grad_out, "grad_out")
    gamma = None if gamma is None else _f32(gamma, "gamma")
    n, f = x.shape
    gx, gg, gb = np.empty_like(x), np.empty(f, np.float32), np.empty(f, np.float32)
    rc = _load().oracle_batchnorm_backward(_p(x), ctypes.c_int32(n), ctypes.c_int32(f), _p(gamma), ctypes.c_float(eps),
                                           _p(gy), _p(gx), _p(gg), _p(gb))
    _check(rc, "batchnorm_backward")
    return gx, gg, gb


def pool_backward(graph_indicator, num_graphs: int, grad_out, aggr: int = AGGR_MEAN):
    gi, go = _i32(graph_indicator, "graph_indicator"), _f32(grad_out, "grad_out")
    n, f = gi.shape[0], go.shape[1]
    gx = np.empty((n, f), np.float32)
    rc = _load().oracle_pool_backward(_p(gi), ctypes.c_int32(n), ctypes.c_int32(num_graphs), _p(go), ctypes.c_int32(f),
                                      ctypes.c_int32(aggr), _p(gx))
    _check(rc, "pool_backward")
    return gx


def adam_step(p, m, v, g, lr: float, t: int, b1: float = 0.9, b2: float = 0.999, eps: float = 1e-8):
    """-> (p, m, v) after one step; the inputs are not modified."""
    p2, m2, v2 = (np.ascontiguousarray(_f32(a, "a")).copy() for a in (p, m, v))
    g = np.ascontiguousarray(_f32(g, "g"))
    rc = _load().oracle_adam_step(_p(p2), _p(m2), _p(v2), _p(g), ctypes.c_int64(p2.size), ctypes.c_float(lr),
                                  ctypes.c_float(b1), ctypes.c_float(b2), ctypes.c_float(eps), ctypes.c_int32(t))
    _check(rc, "adam_step")
    return p2, m2, v2


def example_model_backward(src, dst, num_nodes: int, graph_indicator, num_graphs: int, x, params: dict, target,
                           eps: float = 1e-5):
    """Loss = mean squared error of the prediction against target [num_graphs, f3] (the example's loss) and its
    gradients with respect to every parameter, by the chain rule through the stages of example_model_forward
    in reverse.  Returns (loss, grads dict, forward intermediates)."""
    fw = example_model_forward(src, dst, num_nodes, graph_indicator, num_graphs, x, params, eps)
    diff = fw["y"].astype(np.float64) - _f32(target, "target").astype(np.float64)
    loss = float((diff ** 2).mean())
    gy = (2.0 * diff / diff.size).astype(np.float32)
    g_pooled, gw3, gb3 = dense_backward(fw["pooled"], params["w3"], gy)
    g_h3 = pool_backward(graph_indicator, num_graphs, g_pooled, AGGR_MEAN)
    g_z3 = np.where(fw["h3"] > 0, g_h3, np.float32(0)).astype(np.float32)          # relu of the second GCNConv
    r2 = gcnconv_backward(src, dst, num_nodes, fw["h2"], params["w2"], g_z3, True)
    g_bn = np.where(fw["h2"] > 0, r2["grad_x"], np.float32(0)).astype(np.float32)    # relu after the batch norm
    g_h1, ggamma, gbeta = batchnorm_backward(fw["h1"], params["gamma"], g_bn, eps)
    r1 = gcnconv_backward(src, dst, num_nodes, x, params["w1"], g_h1, True)
    grads = {"w1": r1["grad_w"], "b1": r1["grad_b"], "gamma": ggamma, "beta": gbeta, "w2": r2["grad_w"],
             "b2": r2["grad_b"], "w3": gw3, "b3": gb3}
    return loss, grads, fw


def gin_update(src, dst, num_nodes: int, x, eps: float = 0.0, with_sabs: bool = False):
    src, dst, x = _i32(src, "src"), _i32(dst, "dst"), _f32(x, "x")
    ne, f = src.shape[0], x.shape[1]
    out = np.empty((num_nodes, f), np.float32)
    sabs = np.empty((num_nodes, f), np.float64) if with_sabs else None
    rc = _load().oracle_gin_update(_p(src), _p(dst), ctypes.c_int64(ne), ctypes.c_int32(num_nodes),
                                   _p(x), ctypes.c_int32(f), ctypes.c_float(eps), _p(out), _p(sabs))
    _check(rc, "gin_update")
    return (out, sabs) if with_sabs else out


def graph_pool(graph_indicator, num_graphs: int, x, aggr: int = AGGR_SUM, with_sabs: bool = False):
    gi, x = _i32(graph_indicator, "graph_indicator"), _f32(x, "x")
    n, f = x.shape
    if gi.shape[0] != n:
        raise ValueError("graph_indicator must have one entry per node")
    out = np.empty((num_graphs, f), np.float32)
    sabs = np.empty((num_graphs, f), np.float64) if with_sabs else None
    rc = _load().oracle_graph_pool(_p(gi), ctypes.c_int32(n), ctypes.c_int32(num_graphs), _p(x),
                                   ctypes.c_int32(f), ctypes.c_int32(aggr), _p(out), _p(sabs))
    _check(rc, "graph_pool")
    return (out, sabs) if with_sabs else out
