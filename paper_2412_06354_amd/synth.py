"""Seeded synthetic workloads (graphs, features, weights, layer parameters).

This module only *draws inputs*.  It holds none of the message-passing
arithmetic: no CSR build, no gather/reduce, no normalisation, no softmax.
Both the HIP library's tests/bench and the CPU oracle's tests take their
inputs from here, so the two sides see byte-identical arrays.

Random numbers come from a counter-based generator written out below
(a splitmix64-style 64-bit mixer applied to ``key + counter * GOLDEN``), so
a value depends only on (seed, stream, counter) and never on numpy's own
bit-generators or on chunking.

The paper's own example builds its inputs the same way: ``rand_graph(n, m)``
topologies with ``randn(Float32, F, n)`` node features (section 3,
"Training Example").  The five workloads below follow the shapes of the
benchmark configurations; the public graph datasets whose sizes some of
them share are not used and not needed -- these generators stand in.

Index convention: nodes 0..N-1, edge k goes from ``src[k]`` to ``dst[k]``;
features are row-major ``[N, F]`` float32.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BASE_SEED = 241206354

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

# sub-stream tags (mixed into the seed)
STREAM_GRAPH = 1
STREAM_FEATURES = 2
STREAM_WEIGHTS = 3
STREAM_PARAMS = 4
STREAM_RELABEL = 5
STREAM_SIZES = 6

_CHUNK = 1 << 17  # counters hashed per numpy call (temporaries stay cache-sized)
_THREADS = 8      # chunks are independent (counter-based), so they are filled concurrently


def _for_chunks(count: int, body) -> None:
    """Run body(start, n) over [0, count) in _CHUNK pieces on a small thread pool
    (numpy releases the GIL inside its array loops).  Results do not depend on the split."""
    starts = range(0, count, _CHUNK)
    if count <= 4 * _CHUNK:
        for s in starts:
            body(s, min(_CHUNK, count - s))
        return
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=_THREADS) as pool:
        list(pool.map(lambda s: body(s, min(_CHUNK, count - s)), starts))


def _mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function on a uint64 array (wrap-around arithmetic)."""
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _key(seed: int, stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        k = _mix64(np.array([np.uint64(seed & 0xFFFFFFFFFFFFFFFF)], dtype=np.uint64))
        k = _mix64(k ^ (np.uint64(stream) * _GOLDEN))
    return k[0]


def hash_u64(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """64 random bits for counters start .. start+count-1."""
    key = _key(seed, stream)
    ctr = np.arange(start, start + count, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix64(key + (ctr + np.uint64(1)) * _GOLDEN)


def uniform01(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """float64 uniform on [0, 1) with 53 random bits."""
    return (hash_u64(seed, stream, start, count) >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)


def randint(seed: int, stream: int, start: int, count: int, lo: int, hi: int) -> np.ndarray:
    """Integers uniform on lo..hi inclusive (multiply-shift on the top 32 bits)."""
    span = np.uint64(hi - lo + 1)
    top = hash_u64(seed, stream, start, count) >> np.uint64(32)
    return (lo + ((top * span) >> np.uint64(32)).astype(np.int64)).astype(np.int64)


def normal_f32(seed: int, stream: int, count: int, out: Optional[np.ndarray] = None) -> np.ndarray:
    """``count`` standard normals as float32 (Box-Muller in float64, one value per pair)."""
    if out is None:
        out = np.empty(count, dtype=np.float32)
    flat = out.reshape(-1)

    def body(s, n):
        u = uniform01(seed, stream, 2 * s, 2 * n)
        u1 = 1.0 - u[0::2]                                               # (0, 1]
        u2 = u[1::2]
        flat[s:s + n] = (np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)).astype(np.float32)

    _for_chunks(count, body)
    return out


def uniform_f32(seed: int, stream: int, count: int, lo: float = 0.0, hi: float = 1.0) -> np.ndarray:
    out = np.empty(count, dtype=np.float32)

    def body(s, n):
        out[s:s + n] = (lo + (hi - lo) * uniform01(seed, stream, s, n)).astype(np.float32)

    _for_chunks(count, body)
    return out


def glorot_uniform(seed: int, stream: int, fan_in: int, fan_out: int, shape) -> np.ndarray:
    a = float(np.sqrt(6.0 / (fan_in + fan_out)))
    n = int(np.prod(shape))
    return uniform_f32(seed, stream, n, -a, a).reshape(shape)


def relabel_permutation(seed: int, n: int) -> np.ndarray:
    """A seeded bijection old id -> new id (rank of a per-node hash)."""
    keys = hash_u64(seed, STREAM_RELABEL, 0, n)
    order = np.argsort(keys, kind="stable")
    new_id = np.empty(n, dtype=np.int64)
    new_id[order] = np.arange(n, dtype=np.int64)
    return new_id


# --------------------------------------------------------------------------
# expected-degree (Chung-Lu) machinery
# --------------------------------------------------------------------------

def power_law_weights(n: int, total: float, inv_exponent: float, cap: float) -> np.ndarray:
    """w_i = min(c * (i+1)^(-inv_exponent), cap) with c chosen by bisection so sum(w) = total."""
    base = np.arange(1, n + 1, dtype=np.float64) ** (-inv_exponent)
    lo, hi = 0.0, float(total) / base[-1]
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if np.minimum(mid * base, cap).sum() < total:
            lo = mid
        else:
            hi = mid
    return np.minimum(hi * base, cap)


def _sample_endpoints(cdf: np.ndarray, seed: int, stream: int, start: int, count: int) -> np.ndarray:
    out = np.empty(count, dtype=np.int64)
    n = cdf.shape[0]

    def body(s, m):
        u = uniform01(seed, stream, start + s, m)
        out[s:s + m] = np.minimum(np.searchsorted(cdf, u, side="right"), n - 1)

    _for_chunks(count, body)
    return out


def chung_lu_directed(n: int, e: int, inv_exponent: float, cap: float, seed: int,
                      relabel: bool = True):
    """``e`` directed edges, endpoints independent with P(i) ~ w_i; self-loops redrawn,
    duplicate edges kept (a multigraph).  Returns (src, dst) int32 in draw order."""
    w = power_law_weights(n, float(e), inv_exponent, cap)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    src = _sample_endpoints(cdf, seed, STREAM_GRAPH, 0, e)
    dst = _sample_endpoints(cdf, seed, STREAM_GRAPH, e, e)
    ctr = 2 * e
    bad = np.flatnonzero(src == dst)
    while bad.size:
        m = bad.size
        src[bad] = _sample_endpoints(cdf, seed, STREAM_GRAPH, ctr, m)
        dst[bad] = _sample_endpoints(cdf, seed, STREAM_GRAPH, ctr + m, m)
        ctr += 2 * m
        bad = bad[src[bad] == dst[bad]]
    if relabel:
        new_id = relabel_permutation(seed, n)
        src, dst = new_id[src], new_id[dst]
    return src.astype(np.int32), dst.astype(np.int32)


def chung_lu_undirected_simple(n: int, pairs: int, inv_exponent: float, cap: float, seed: int,
                               relabel: bool = True):
    """Exactly ``pairs`` distinct unordered pairs (no self-pairs), endpoints ~ w;
    both directions emitted, interleaved: edge 2t = (u -> v), edge 2t+1 = (v -> u)."""
    w = power_law_weights(n, 2.0 * pairs, inv_exponent, cap)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    keys = np.empty(0, dtype=np.int64)
    ctr = 0
    while keys.size < pairs:
        m = int((pairs - keys.size) * 1.25) + 1024
        a = _sample_endpoints(cdf, seed, STREAM_GRAPH, ctr, m)
        b = _sample_endpoints(cdf, seed, STREAM_GRAPH, ctr + m, m)
        ctr += 2 * m
        keep = a != b
        lo = np.minimum(a[keep], b[keep])
        hi = np.maximum(a[keep], b[keep])
        cand = np.concatenate([keys, lo * n + hi])
        # keep first occurrences, in draw order
        _, first = np.unique(cand, return_index=True)
        first.sort()
        keys = cand[first]
    keys = keys[:pairs]
    u, v = keys // n, keys % n
    if relabel:
        new_id = relabel_permutation(seed, n)
        u, v = new_id[u], new_id[v]
    src = np.empty(2 * pairs, dtype=np.int32)
    dst = np.empty(2 * pairs, dtype=np.int32)
    src[0::2], dst[0::2] = u, v
    src[1::2], dst[1::2] = v, u
    return src, dst


def gnm_directed_simple(n: int, m: int, seed: int):
    """Exactly ``m`` distinct directed edges without self-loops, uniform, in draw order
    (the shape of ``rand_graph(n, m)`` in the paper's training example)."""
    keys = np.empty(0, dtype=np.int64)
    ctr = 0
    while keys.size < m:
        k = int((m - keys.size) * 1.25) + 64
        a = randint(seed, STREAM_GRAPH, ctr, k, 0, n - 1)
        b = randint(seed, STREAM_GRAPH, ctr + k, k, 0, n - 1)
        ctr += 2 * k
        keep = a != b
        cand = np.concatenate([keys, a[keep] * n + b[keep]])
        _, first = np.unique(cand, return_index=True)
        first.sort()
        keys = cand[first]
    keys = keys[:m]
    return (keys // n).astype(np.int32), (keys % n).astype(np.int32)


def multigraph_uniform(n: int, e: int, seed: int):
    """``e`` directed edges with uniform endpoints; self-loops and duplicates allowed."""
    return (randint(seed, STREAM_GRAPH, 0, e, 0, n - 1).astype(np.int32),
            randint(seed, STREAM_GRAPH, e, e, 0, n - 1).astype(np.int32))


def batched_er_graphs(num_graphs: int, n_lo: int, n_hi: int, p: float, seed: int):
    """Block-diagonal union of ``num_graphs`` Erdos-Renyi graphs (each unordered pair kept
    with probability p, both directions emitted, interleaved) with sizes uniform on
    n_lo..n_hi.  Returns (src, dst, graph_indicator, sizes)."""
    sizes = randint(seed, STREAM_SIZES, 0, num_graphs, n_lo, n_hi)
    offsets = np.concatenate([[0], np.cumsum(sizes)])
    src_parts, dst_parts = [], []
    ctr = 0
    tri = {n: np.triu_indices(n, 1) for n in range(n_lo, n_hi + 1)}
    for g in range(num_graphs):
        n = int(sizes[g])
        a, b = tri[n]
        u = uniform01(seed, STREAM_GRAPH, ctr, a.size)
        ctr += a.size
        keep = u < p
        ga = a[keep] + offsets[g]
        gb = b[keep] + offsets[g]
        s = np.empty(2 * ga.size, dtype=np.int32)
        d = np.empty(2 * ga.size, dtype=np.int32)
        s[0::2], d[0::2] = ga, gb
        s[1::2], d[1::2] = gb, ga
        src_parts.append(s)
        dst_parts.append(d)
    gi = np.repeat(np.arange(num_graphs, dtype=np.int32), sizes)
    return (np.concatenate(src_parts), np.concatenate(dst_parts), gi, sizes.astype(np.int32))


# --------------------------------------------------------------------------
# the five workloads
# --------------------------------------------------------------------------

@dataclass
class Workload:
    name: str
    num_nodes: int
    src: np.ndarray
    dst: np.ndarray
    x: np.ndarray
    edge_weight: Optional[np.ndarray] = None
    params: dict = field(default_factory=dict)
    graph_indicator: Optional[np.ndarray] = None
    num_graphs: int = 0

    @property
    def num_edges(self) -> int:
        return int(self.src.shape[0])

    def stats(self) -> dict:
        """Realised structure (reported next to every measurement)."""
        n, e = self.num_nodes, self.num_edges
        indeg = np.bincount(self.dst, minlength=n)
        key = self.src.astype(np.int64) * n + self.dst.astype(np.int64)
        return {"N": n, "E": e, "max_in_degree": int(indeg.max()) if n else 0,
                "isolated_in": int((indeg == 0).sum()),
                "duplicate_edges": int(e - np.unique(key).size),
                "self_loops": int((self.src == self.dst).sum())}


def seed_of(config_index: int) -> int:
    return BASE_SEED + config_index


def config0_tiny(num_nodes: int = 2708, num_edges: int = 10556, feat: int = 64) -> Workload:
    """Tiny propagate: distinct directed edges drawn uniformly, x ~ N(0,1)."""
    sd = seed_of(0)
    src, dst = gnm_directed_simple(num_nodes, num_edges, sd)
    x = normal_f32(sd, STREAM_FEATURES, num_nodes * feat).reshape(num_nodes, feat)
    return Workload("config0_tiny_propagate", num_nodes, src, dst, x)


def config1_gcn(num_nodes: int = 100_000, pairs: int = 500_000, f_in: int = 128,
                f_out: int = 128) -> Workload:
    """GCNConv forward: symmetrised power-law graph (degree exponent 2.1), Glorot W, zero bias."""
    sd = seed_of(1)
    cap = float(np.sqrt(2.0 * pairs))
    src, dst = chung_lu_undirected_simple(num_nodes, pairs, 1.0 / 1.1, cap, sd)
    x = normal_f32(sd, STREAM_FEATURES, num_nodes * f_in).reshape(num_nodes, f_in)
    w = glorot_uniform(sd, STREAM_PARAMS, f_in, f_out, (f_in, f_out))
    b = np.zeros(f_out, dtype=np.float32)
    return Workload("config1_gcnconv", num_nodes, src, dst, x, params={"w": w, "bias": b})


def config2_weighted(num_nodes: int = 1_000_000, num_edges: int = 20_000_000, feat: int = 64,
                     cap: float = 50_000.0) -> Workload:
    """Weighted propagate at scale: directed power-law multigraph (exponent 2.0), w ~ U(0,1)."""
    sd = seed_of(2)
    cap = min(cap, max(4.0, num_edges / 8.0))
    src, dst = chung_lu_directed(num_nodes, num_edges, 1.0, cap, sd)
    x = normal_f32(sd, STREAM_FEATURES, num_nodes * feat).reshape(num_nodes, feat)
    ew = uniform_f32(sd, STREAM_WEIGHTS, num_edges)
    return Workload("config2_weighted_propagate", num_nodes, src, dst, x, edge_weight=ew)


def config3_batched(num_graphs: int = 4096, n_lo: int = 20, n_hi: int = 30, p: float = 0.2,
                    feat: int = 32) -> Workload:
    """Batched small graphs for the GIN-style update and graph-level pooling."""
    sd = seed_of(3)
    src, dst, gi, _ = batched_er_graphs(num_graphs, n_lo, n_hi, p, sd)
    n = int(gi.shape[0])
    x = normal_f32(sd, STREAM_FEATURES, n * feat).reshape(n, feat)
    return Workload("config3_batched_gin_pool", n, src, dst, x, graph_indicator=gi,
                    num_graphs=num_graphs, params={"eps": 0.0})


def config4_gat(num_nodes: int = 2_449_029, num_edges: int = 123_718_280, f_in: int = 100,
                heads: int = 8, ch: int = 8, cap: float = 20_000.0) -> Workload:
    """GAT-style layer: directed power-law multigraph (exponent 2.1) plus one self-loop per node."""
    sd = seed_of(4)
    cap = min(cap, max(4.0, num_edges / 8.0))
    src, dst = chung_lu_directed(num_nodes, num_edges, 1.0 / 1.1, cap, sd)
    loops = np.arange(num_nodes, dtype=np.int32)
    src = np.concatenate([src, loops])
    dst = np.concatenate([dst, loops])
    x = normal_f32(sd, STREAM_FEATURES, num_nodes * f_in).reshape(num_nodes, f_in)
    f_out = heads * ch
    w = glorot_uniform(sd, STREAM_PARAMS, f_in, f_out, (f_in, f_out))
    a = float(np.sqrt(6.0 / (ch + 1)))
    a_src = uniform_f32(sd, STREAM_PARAMS + 16, f_out, -a, a).reshape(heads, ch)
    a_dst = uniform_f32(sd, STREAM_PARAMS + 32, f_out, -a, a).reshape(heads, ch)
    return Workload("config4_gat", num_nodes, src, dst, x,
                    params={"w": w, "a_src": a_src, "a_dst": a_dst, "heads": heads, "ch": ch,
                            "negative_slope": 0.2})


def config5_example_model(num_graphs: int = 32, n: int = 50, p: float = 0.08, f0: int = 16, f1: int = 64,
                          f2: int = 64, f3: int = 1) -> Workload:
    """A collated batch for the paper's example model (section 3, "Training Example"): ``num_graphs``
    random graphs of ``n`` nodes (the listing's n and m are not given: each unordered pair is kept with
    probability p, both directions emitted), standard-normal node features of width f0, and the model's
    parameters: Glorot-uniform weights, small uniform biases (so that the bias paths are exercised),
    batch-norm scale near 1 and shift near 0."""
    sd = seed_of(5)
    src, dst, gi, _ = batched_er_graphs(num_graphs, n, n, p, sd)
    nn = int(gi.shape[0])
    x = normal_f32(sd, STREAM_FEATURES, nn * f0).reshape(nn, f0)
    params = {
        "w1": glorot_uniform(sd, 20, f0, f1, (f0, f1)),
        "b1": uniform_f32(sd, 21, f1, -0.1, 0.1),
        "gamma": uniform_f32(sd, 22, f1, 0.9, 1.1),
        "beta": uniform_f32(sd, 23, f1, -0.1, 0.1),
        "w2": glorot_uniform(sd, 24, f1, f2, (f1, f2)),
        "b2": uniform_f32(sd, 25, f2, -0.1, 0.1),
        "w3": glorot_uniform(sd, 26, f2, f3, (f2, f3)),
        "b3": uniform_f32(sd, 27, f3, -0.1, 0.1),
    }
    return Workload("config5_example_model", nn, src, dst, x, graph_indicator=gi, num_graphs=num_graphs,
                    params=params)
