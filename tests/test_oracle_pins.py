"""Pins of the CPU oracle against things other than itself (CPU only).

The paper prints no numeric example, so each pin is a hand-worked tiny graph
(tests/golden), an invariant, a reduction to a library routine (dense matmul,
stable argsort, plain softmax) or brute force on graphs of at most 64 nodes.
"""
import numpy as np
import pytest

import oracle
from oracle import (AGGR_MAX, AGGR_MEAN, AGGR_MIN, AGGR_PROD, AGGR_SUM, MSG_COPY_XJ, MSG_E_MUL_XJ, MSG_XI_DOT_XJ,
                    MSG_XJ_SUB_XI)
from paper_2412_06354_amd import synth
from util import dense_adjacency, incoming, load_golden

AGGRS = {"sum": AGGR_SUM, "mean": AGGR_MEAN, "max": AGGR_MAX}


def rng_graph(seed, n, e, star=False):
    """Seeded random multigraph with self-loops, duplicates and isolated nodes."""
    src, dst = synth.multigraph_uniform(n, e, seed)
    if star:  # hub 0 receives an edge from every other node
        src = np.concatenate([src, np.arange(1, n, dtype=np.int32)])
        dst = np.concatenate([dst, np.zeros(n - 1, dtype=np.int32)])
    # make a few nodes isolated on the incoming side
    keep = dst % 7 != 3
    return src[keep], dst[keep]


# ----------------------------------------------------------------------------- hand-worked

def test_g5_csr(golden_dir):
    g = load_golden(golden_dir, "g5_propagate.json")
    src, dst = np.array(g["src"], np.int32), np.array(g["dst"], np.int32)
    rowptr, colidx, perm, indeg = oracle.build_csr(src, dst, g["num_nodes"])
    assert rowptr.tolist() == g["rowptr"]
    assert colidx.tolist() == g["colidx"]
    assert perm.tolist() == g["perm"]
    assert indeg.tolist() == g["indeg"]


@pytest.mark.parametrize("msg_name", ["copy_xj", "e_mul_xj"])
@pytest.mark.parametrize("aggr_name", ["sum", "mean", "max"])
def test_g5_propagate(golden_dir, msg_name, aggr_name):
    g = load_golden(golden_dir, "g5_propagate.json")
    src, dst = np.array(g["src"], np.int32), np.array(g["dst"], np.int32)
    x = np.array(g["x"], np.float32)
    w = np.array(g["w"], np.float32)
    msg = MSG_COPY_XJ if msg_name == "copy_xj" else MSG_E_MUL_XJ
    out = oracle.propagate(src, dst, g["num_nodes"], x, w if msg else None, msg, AGGRS[aggr_name])
    want = np.array(g[msg_name][aggr_name], np.float64).astype(np.float32)
    np.testing.assert_array_equal(out, want)


def test_g5_gin(golden_dir):
    g = load_golden(golden_dir, "g5_propagate.json")
    src, dst = np.array(g["src"], np.int32), np.array(g["dst"], np.int32)
    x = np.array(g["x"], np.float32)
    np.testing.assert_array_equal(oracle.gin_update(src, dst, 4, x, 0.0), np.array(g["gin_eps0"], np.float32))
    np.testing.assert_array_equal(oracle.gin_update(src, dst, 4, x, 0.5), np.array(g["gin_eps_half"], np.float32))


def test_g5_softmax(golden_dir):
    g = load_golden(golden_dir, "g5_softmax.json")
    dst = np.array(g["dst"], np.int32)
    s = np.array(g["scores"], np.float32).reshape(-1, 1)
    alpha = oracle.segment_softmax(dst, g["num_nodes"], s)
    np.testing.assert_allclose(alpha[:, 0], g["alpha"], rtol=3e-7)
    assert alpha[0, 0] == 1.0 and alpha[4, 0] == 1.0
    # shift invariance per destination, no overflow for huge scores
    s2 = s.copy()
    s2[1:4] += 1000.0
    alpha2 = oracle.segment_softmax(dst, g["num_nodes"], s2)
    np.testing.assert_allclose(alpha2[:, 0], g["alpha"], rtol=2e-4)  # fp32 input rounding of ln 2 + 1000
    assert np.isfinite(alpha2).all()


def test_path3_gcn(golden_dir):
    g = load_golden(golden_dir, "path3_gcn.json")
    src, dst = np.array(g["src"], np.int32), np.array(g["dst"], np.int32)
    x = np.array(g["x"], np.float32)
    out = oracle.gcnconv(src, dst, 3, x, np.array(g["w"], np.float32), None, True)
    np.testing.assert_allclose(out, np.array(g["out"]), rtol=1e-7)
    out2 = oracle.gcnconv(src, dst, 3, x, np.array(g["w2"], np.float32), np.array(g["bias2"], np.float32), True)
    np.testing.assert_allclose(out2, np.array(g["out2"]), rtol=1e-7)


# ----------------------------------------------------------------------------- library routines

@pytest.mark.parametrize("seed,n,e", [(1, 1, 5), (2, 7, 0), (3, 64, 700), (4, 1000, 20000)])
def test_csr_is_stable_sort(seed, n, e):
    src, dst = synth.multigraph_uniform(n, e, seed)
    rowptr, colidx, perm, indeg = oracle.build_csr(src, dst, n)
    order = np.argsort(dst, kind="stable")
    np.testing.assert_array_equal(perm, order.astype(np.int32))
    np.testing.assert_array_equal(colidx, src[order])
    np.testing.assert_array_equal(indeg, np.bincount(dst, minlength=n))
    np.testing.assert_array_equal(rowptr, np.searchsorted(dst[order], np.arange(n + 1)))


def test_csr_equals_dense_adjacency():
    src, dst = rng_graph(11, 40, 300, star=True)
    rowptr, colidx, _, _ = oracle.build_csr(src, dst, 40)
    a = np.zeros((40, 40))
    for i in range(40):
        for p in range(rowptr[i], rowptr[i + 1]):
            a[i, colidx[p]] += 1
    np.testing.assert_array_equal(a, dense_adjacency(src, dst, 40))


@pytest.mark.parametrize("seed,n,e,f", [(21, 64, 900, 5), (22, 33, 100, 8), (23, 64, 64, 3)])
def test_propagate_is_dense_matmul(seed, n, e, f):
    src, dst = rng_graph(seed, n, e, star=True)
    ne = src.shape[0]
    x = synth.normal_f32(seed, 2, n * f).reshape(n, f)
    w = synth.uniform_f32(seed, 3, ne, -1.0, 1.0)
    a = dense_adjacency(src, dst, n)
    deg = a.sum(1, keepdims=True)
    xs = x.astype(np.float64)
    # copy_xj + sum = (multiplicity adjacency) @ X ; mean = D^-1 A X
    np.testing.assert_allclose(oracle.propagate(src, dst, n, x), (a @ xs).astype(np.float32), rtol=0, atol=0)
    mean_ref = np.where(deg > 0, (a @ xs) / np.maximum(deg, 1), 0.0)
    np.testing.assert_allclose(oracle.propagate(src, dst, n, x, None, MSG_COPY_XJ, AGGR_MEAN),
                               mean_ref.astype(np.float32), rtol=1e-7, atol=1e-7)
    # e_mul_xj + sum = (weighted adjacency) @ X, up to the float rounding of each product
    aw = dense_adjacency(src, dst, n, w)
    got = oracle.propagate(src, dst, n, x, w, MSG_E_MUL_XJ, AGGR_SUM)
    np.testing.assert_allclose(got, aw @ xs, rtol=0, atol=1e-6 * (np.abs(aw) @ np.abs(xs)).max())
    # mean divides by the edge count, not by the weight sum
    got = oracle.propagate(src, dst, n, x, w, MSG_E_MUL_XJ, AGGR_MEAN)
    ref = np.where(deg > 0, (aw @ xs) / np.maximum(deg, 1), 0.0)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-6 * (np.abs(aw) @ np.abs(xs)).max())


@pytest.mark.parametrize("seed,n,e,f", [(31, 64, 500, 4), (32, 20, 30, 6)])
def test_propagate_max_brute_force(seed, n, e, f):
    src, dst = rng_graph(seed, n, e, star=True)
    ne = src.shape[0]
    x = synth.normal_f32(seed, 2, n * f).reshape(n, f)
    w = synth.uniform_f32(seed, 3, ne, -1.0, 1.0)
    inc = incoming(dst, n)
    for msg, e_arg in ((MSG_COPY_XJ, None), (MSG_E_MUL_XJ, w)):
        got = oracle.propagate(src, dst, n, x, e_arg, msg, AGGR_MAX)
        for i in range(n):
            if inc[i].size == 0:
                assert (got[i] == 0).all()
                continue
            rows = x[src[inc[i]]]
            if msg == MSG_E_MUL_XJ:
                rows = (w[inc[i]][:, None] * rows).astype(np.float32)   # float32 products
            np.testing.assert_array_equal(got[i], rows.max(0))


def test_max_of_signed_zeros_is_plus_zero():
    src = np.array([0, 1, 1, 0], np.int32)
    dst = np.array([2, 2, 3, 3], np.int32)
    x = np.array([[-0.0], [0.0], [5.0], [5.0]], np.float32)
    out = oracle.propagate(src, dst, 4, x, None, MSG_COPY_XJ, AGGR_MAX)
    assert not np.signbit(out[2, 0]) and not np.signbit(out[3, 0])
    x2 = np.array([[-0.0], [-0.0], [5.0], [5.0]], np.float32)
    out2 = oracle.propagate(src, dst, 4, x2, None, MSG_COPY_XJ, AGGR_MAX)
    assert np.signbit(out2[2, 0])   # all messages are -0 -> -0


def test_elementwise_edge_features():
    n, f = 30, 6
    src, dst = rng_graph(41, n, 200)
    ne = src.shape[0]
    x = synth.normal_f32(41, 2, n * f).reshape(n, f)
    ef = synth.normal_f32(41, 3, ne * f).reshape(ne, f)
    got = oracle.propagate(src, dst, n, x, ef, MSG_E_MUL_XJ, AGGR_SUM)
    ref = np.zeros((n, f))
    for k in range(ne):
        ref[dst[k]] += (ef[k] * x[src[k]]).astype(np.float64)
    np.testing.assert_allclose(got, ref, rtol=0, atol=2e-6 * np.abs(ref).max())


def test_two_step_equals_fused():
    n, f = 50, 7
    src, dst = rng_graph(51, n, 600, star=True)
    ne = src.shape[0]
    x = synth.normal_f32(51, 2, n * f).reshape(n, f)
    w = synth.uniform_f32(51, 3, ne)
    for msg, e_arg in ((MSG_COPY_XJ, None), (MSG_E_MUL_XJ, w)):
        m = oracle.apply_edges(src, n, x, e_arg, msg)
        assert m.shape == (ne, f)
        if msg == MSG_COPY_XJ:
            np.testing.assert_array_equal(m, x[src])          # gather
        else:
            np.testing.assert_array_equal(m, w[:, None] * x[src])
        for aggr in (AGGR_SUM, AGGR_MEAN, AGGR_MAX):
            two = oracle.aggregate_neighbors(dst, n, m, aggr)
            one = oracle.propagate(src, dst, n, x, e_arg, msg, aggr)
            np.testing.assert_array_equal(one, two)


# ----------------------------------------------------------------------------- invariants

def test_invariants_small_powerlaw():
    wl = synth.config2_weighted(num_nodes=3000, num_edges=40000, feat=8, cap=400.0)
    n, src, dst = wl.num_nodes, wl.src, wl.dst
    rowptr, _, _, indeg = oracle.build_csr(src, dst, n)
    ones = np.ones((n, 8), np.float32)
    s = oracle.propagate(src, dst, n, ones)
    np.testing.assert_array_equal(s[:, 0], indeg.astype(np.float32))         # sum of ones = in-degree
    np.testing.assert_array_equal(s[:, 0], np.diff(rowptr).astype(np.float32))
    c = np.full((n, 8), 2.5, np.float32)
    has = np.repeat((indeg > 0)[:, None], 8, axis=1)
    np.testing.assert_array_equal(oracle.propagate(src, dst, n, c, None, MSG_COPY_XJ, AGGR_MEAN), np.where(has, 2.5, 0).astype(np.float32))
    np.testing.assert_array_equal(oracle.propagate(src, dst, n, c, None, MSG_COPY_XJ, AGGR_MAX), np.where(has, 2.5, 0).astype(np.float32))
    # unit weights: e_mul_xj == copy_xj bit for bit
    w1 = np.ones(wl.num_edges, np.float32)
    for aggr in (AGGR_SUM, AGGR_MEAN, AGGR_MAX):
        np.testing.assert_array_equal(oracle.propagate(src, dst, n, wl.x, w1, MSG_E_MUL_XJ, aggr),
                                      oracle.propagate(src, dst, n, wl.x, None, MSG_COPY_XJ, aggr))
    # GIN of ones = 1 + in-degree
    np.testing.assert_array_equal(oracle.gin_update(src, dst, n, ones, 0.0)[:, 0], 1.0 + indeg)
    # sabs of a non-negative input equals the sum itself
    out, sabs = oracle.propagate(src, dst, n, np.abs(wl.x), None, MSG_COPY_XJ, AGGR_SUM, with_sabs=True)
    np.testing.assert_allclose(out, sabs, rtol=1e-6)


def test_gcn_sqrt_degree_is_fixed_point():
    wl = synth.config1_gcn(num_nodes=500, pairs=2000, f_in=4, f_out=4)
    n = wl.num_nodes
    d = np.bincount(wl.dst, minlength=n) + 1.0
    x = np.sqrt(d).astype(np.float32).reshape(n, 1)
    out = oracle.gcnconv(wl.src, wl.dst, n, x, np.ones((1, 1), np.float32), None, True)
    np.testing.assert_allclose(out, x, rtol=3e-7)


def test_gcn_regular_graph_rows_sum_to_one():
    n = 12  # ring: every node has in-degree 2 (+1 self-loop) -> each row of the operator sums to 1
    i = np.arange(n, dtype=np.int32)
    src = np.concatenate([i, (i + 1) % n]).astype(np.int32)
    dst = np.concatenate([(i + 1) % n, i]).astype(np.int32)
    x = np.full((n, 3), 7.0, np.float32)
    out = oracle.gcnconv(src, dst, n, x, np.eye(3, dtype=np.float32), None, True)
    np.testing.assert_allclose(out, x, rtol=3e-7)


@pytest.mark.parametrize("loops", [True, False])
def test_gcn_is_dense_operator(loops):
    n, f_in, f_out = 48, 5, 3
    src, dst = rng_graph(61, n, 400, star=True)
    x = synth.normal_f32(61, 2, n * f_in).reshape(n, f_in)
    w = synth.glorot_uniform(61, 4, f_in, f_out, (f_in, f_out))
    b = synth.uniform_f32(61, 5, f_out, -1, 1)
    a = dense_adjacency(src, dst, n) + (np.eye(n) if loops else 0.0)
    d = a.sum(1)
    dinv = np.where(d > 0, 1.0 / np.sqrt(np.maximum(d, 1e-300)), 0.0)
    ref = (dinv[:, None] * a * dinv[None, :]) @ (x.astype(np.float64) @ w.astype(np.float64)) + b
    got = oracle.gcnconv(src, dst, n, x, w, b, loops)
    np.testing.assert_allclose(got, ref, rtol=0, atol=2e-7 * np.abs(ref).max())


def test_gcn_equals_unfused_weighted_propagate():
    wl = synth.config1_gcn(num_nodes=800, pairs=3000, f_in=6, f_out=5)
    n = wl.num_nodes
    loops = np.arange(n, dtype=np.int32)
    s2, d2 = np.concatenate([wl.src, loops]), np.concatenate([wl.dst, loops])
    deg = np.bincount(d2, minlength=n).astype(np.float64)
    coef = (1.0 / np.sqrt(deg[s2] * deg[d2])).astype(np.float32)
    z = (wl.x.astype(np.float64) @ wl.params["w"].astype(np.float64)).astype(np.float32)
    unfused = oracle.propagate(s2, d2, n, z, coef, MSG_E_MUL_XJ, AGGR_SUM)
    fused, sabs = oracle.gcnconv(wl.src, wl.dst, n, wl.x, wl.params["w"], None, True, with_sabs=True)
    assert (np.abs(fused - unfused) <= 1e-6 * sabs + 1e-12).all()


def test_softmax_rows_and_plain_softmax():
    n, h = 40, 3
    src, dst = rng_graph(71, n, 500, star=True)
    ne = dst.shape[0]
    s = (4.0 * synth.normal_f32(71, 2, ne * h)).reshape(ne, h)
    alpha = oracle.segment_softmax(dst, n, s)
    inc = incoming(dst, n)
    for i in range(n):
        if inc[i].size == 0:
            continue
        seg = s[inc[i]].astype(np.float64)
        ex = np.exp(seg - seg.max(0))
        np.testing.assert_allclose(alpha[inc[i]], ex / ex.sum(0), rtol=2e-7)
        np.testing.assert_allclose(alpha[inc[i]].sum(0), 1.0, rtol=1e-6)
    # one-dimensional scores are accepted as one head
    a1 = oracle.segment_softmax(dst, n, s[:, 0].copy())
    np.testing.assert_array_equal(a1, alpha[:, 0])


def test_gat_brute_force():
    n, f_in, heads, ch = 30, 7, 3, 4
    src, dst = rng_graph(81, n, 300, star=True)
    loops = np.arange(n, dtype=np.int32)[::2]                      # some self-loops in the list
    src, dst = np.concatenate([src, loops]), np.concatenate([dst, loops])
    x = synth.normal_f32(81, 2, n * f_in).reshape(n, f_in)
    w = synth.glorot_uniform(81, 4, f_in, heads * ch, (f_in, heads * ch))
    a_s = synth.uniform_f32(81, 5, heads * ch, -1, 1).reshape(heads, ch)
    a_d = synth.uniform_f32(81, 6, heads * ch, -1, 1).reshape(heads, ch)
    got = oracle.gatconv(src, dst, n, x, w, a_s, a_d, 0.2)
    h = (x.astype(np.float64) @ w.astype(np.float64)).astype(np.float32).astype(np.float64).reshape(n, heads, ch)
    sl = (h * a_s[None]).sum(-1)
    sr = (h * a_d[None]).sum(-1)
    ref = np.zeros((n, heads, ch))
    inc = incoming(dst, n)
    for i in range(n):
        if inc[i].size == 0:
            continue
        j = src[inc[i]]
        sc = sl[j] + sr[i][None]
        sc = np.where(sc > 0, sc, 0.2 * sc)
        ex = np.exp(sc - sc.max(0))
        al = ex / ex.sum(0)
        ref[i] = (al[:, :, None] * h[j]).sum(0)
    np.testing.assert_allclose(got.reshape(n, heads, ch), ref, rtol=0, atol=3e-7 * np.abs(ref).max())


def test_gat_zero_attention_is_mean():
    wl = synth.config4_gat(num_nodes=400, num_edges=3000, f_in=10, heads=2, ch=4, cap=100.0)
    n = wl.num_nodes
    zero = np.zeros((2, 4), np.float32)
    got, sabs = oracle.gatconv(wl.src, wl.dst, n, wl.x, wl.params["w"], zero, zero, 0.2, with_sabs=True)
    hfeat = (wl.x.astype(np.float64) @ wl.params["w"].astype(np.float64)).astype(np.float32)
    ref = oracle.propagate(wl.src, wl.dst, n, hfeat, None, MSG_COPY_XJ, AGGR_MEAN)
    assert (np.abs(got - ref) <= 1e-6 * sabs + 1e-12).all()


def test_pool_and_batching():
    wl = synth.config3_batched(num_graphs=37, feat=4)
    n, g = wl.num_nodes, wl.num_graphs
    gi = wl.graph_indicator
    assert (np.diff(gi) >= 0).all()
    sizes = np.bincount(gi, minlength=g)
    ones = np.ones((n, 4), np.float32)
    np.testing.assert_array_equal(oracle.graph_pool(gi, g, ones)[:, 0], sizes)
    # sum-pool of propagate(ones) = edges per graph
    deg = oracle.propagate(wl.src, wl.dst, n, ones)
    np.testing.assert_array_equal(oracle.graph_pool(gi, g, deg)[:, 0], np.bincount(gi[wl.dst], minlength=g))
    c = np.full((n, 4), -3.0, np.float32)
    np.testing.assert_array_equal(oracle.graph_pool(gi, g, c, AGGR_MEAN), np.full((g, 4), -3.0, np.float32))
    # against per-graph numpy reductions
    off = np.concatenate([[0], np.cumsum(sizes)])
    for aggr, fn in ((AGGR_SUM, np.sum), (AGGR_MEAN, np.mean), (AGGR_MAX, np.max)):
        got = oracle.graph_pool(gi, g, wl.x, aggr)
        for q in range(g):
            np.testing.assert_allclose(got[q], fn(wl.x[off[q]:off[q + 1]].astype(np.float64), axis=0), rtol=1e-6, atol=1e-7)
    # a graph id without nodes gives a zero row
    got = oracle.graph_pool(gi, g + 2, wl.x, AGGR_MAX)
    assert (got[g:] == 0).all()
    # batched propagate = per-graph propagate, concatenated
    full = oracle.propagate(wl.src, wl.dst, n, wl.x)
    for q in (0, 5, g - 1):
        m = gi[wl.dst] == q
        part = oracle.propagate((wl.src[m] - off[q]).astype(np.int32), (wl.dst[m] - off[q]).astype(np.int32), int(sizes[q]), wl.x[off[q]:off[q + 1]])
        np.testing.assert_array_equal(part, full[off[q]:off[q + 1]])


# ----------------------------------------------------------------------------- backward

@pytest.mark.parametrize("aggr", [AGGR_SUM, AGGR_MEAN])
@pytest.mark.parametrize("e_kind", ["none", "scalar", "vector"])
def test_backward_is_the_adjoint(aggr, e_kind):
    """sum and mean are linear in x and in e, so <propagate(x), g> = <x, grad_x> = <e, grad_e>."""
    n, f = 50, 5
    src, dst = rng_graph(91, n, 600, star=True)
    ne = src.shape[0]
    x = synth.normal_f32(91, 2, n * f).reshape(n, f)
    g = synth.normal_f32(91, 7, n * f).reshape(n, f)
    e = {"none": None, "scalar": synth.uniform_f32(91, 3, ne, -1, 1),
         "vector": synth.normal_f32(91, 3, ne * f).reshape(ne, f)}[e_kind]
    msg = MSG_COPY_XJ if e is None else MSG_E_MUL_XJ
    out = oracle.propagate(src, dst, n, x, e, msg, aggr).astype(np.float64)
    bw = oracle.propagate_backward(src, dst, n, x, g, e, msg, aggr)
    lhs = (out * g).sum()
    np.testing.assert_allclose((x.astype(np.float64) * bw["grad_x"]).sum(), lhs, rtol=2e-5)
    if e is not None:
        np.testing.assert_allclose((e.reshape(ne, -1).astype(np.float64) * bw["grad_e"]).sum(), lhs, rtol=2e-5)
    else:
        assert bw["grad_e"] is None
    # dense form: grad_x = A^T (D^-1) g with A the (weighted) adjacency
    if e_kind != "vector":
        a = dense_adjacency(src, dst, n, e)
        gg = g.astype(np.float64)
        if aggr == AGGR_MEAN:
            deg = np.maximum(dense_adjacency(src, dst, n).sum(1, keepdims=True), 1)
            gg = gg / deg
        np.testing.assert_allclose(bw["grad_x"], a.T @ gg, rtol=0, atol=2e-6 * np.abs(a.T @ gg).max())


@pytest.mark.parametrize("e_kind", ["none", "scalar"])
def test_backward_max_finite_differences(e_kind):
    n, f = 25, 3
    src, dst = rng_graph(93, n, 160)
    ne = src.shape[0]
    x = synth.normal_f32(93, 2, n * f).reshape(n, f)
    g = synth.normal_f32(93, 7, n * f).reshape(n, f)
    e = None if e_kind == "none" else synth.uniform_f32(93, 3, ne, 0.5, 1.5)
    msg = MSG_COPY_XJ if e is None else MSG_E_MUL_XJ
    bw = oracle.propagate_backward(src, dst, n, x, g, e, msg, AGGR_MAX)

    def loss(xx, ee):
        return (oracle.propagate(src, dst, n, xx, ee, msg, AGGR_MAX).astype(np.float64) * g).sum()

    h = 1e-2   # messages are generic: no winner changes for this step
    for (j, c) in ((0, 0), (3, 1), (7, 2), (11, 0), (20, 1)):
        xp, xm = x.copy(), x.copy()
        xp[j, c] += h
        xm[j, c] -= h
        np.testing.assert_allclose(bw["grad_x"][j, c], (loss(xp, e) - loss(xm, e)) / (xp[j, c] - xm[j, c]), rtol=2e-3, atol=2e-3)
    if e is not None:
        for k in (0, 5, 17, 40):
            ep, em = e.copy(), e.copy()
            ep[k] += h
            em[k] -= h
            np.testing.assert_allclose(bw["grad_e"][k, 0], (loss(x, ep) - loss(x, em)) / (ep[k] - em[k]), rtol=2e-3, atol=2e-3)
    # the winner is an incoming edge whose message equals the forward output; ties go to the first edge
    out = oracle.propagate(src, dst, n, x, e, msg, AGGR_MAX)
    am = bw["argmax"]
    indeg = np.bincount(dst, minlength=n)
    assert ((am >= 0) == (indeg > 0)[:, None]).all()
    m = oracle.apply_edges(src, n, x, e, msg)
    for i in range(n):
        for c in range(f):
            if am[i, c] >= 0:
                k = am[i, c]
                assert dst[k] == i and m[k, c] == out[i, c]
                assert not (m[:k][dst[:k] == i][:, c] == out[i, c]).any()


def test_backward_max_ties_go_to_the_first_edge():
    src = np.array([0, 1, 2, 1], np.int32)
    dst = np.array([3, 3, 3, 3], np.int32)
    x = np.array([[1.0], [5.0], [5.0], [0.0]], np.float32)
    g = np.array([[0.0], [0.0], [0.0], [2.0]], np.float32)
    bw = oracle.propagate_backward(src, dst, 4, x, g, None, MSG_COPY_XJ, AGGR_MAX)
    assert bw["argmax"][3, 0] == 1
    np.testing.assert_array_equal(bw["grad_x"][:, 0], [0.0, 2.0, 0.0, 0.0])


@pytest.mark.parametrize("loops", [True, False])
def test_gcn_backward_dense_and_adjoint(loops):
    n, f_in, f_out = 40, 5, 3
    src, dst = rng_graph(95, n, 300, star=True)
    x = synth.normal_f32(95, 2, n * f_in).reshape(n, f_in)
    w = synth.glorot_uniform(95, 4, f_in, f_out, (f_in, f_out))
    b = synth.uniform_f32(95, 5, f_out, -1, 1)
    g = synth.normal_f32(95, 7, n * f_out).reshape(n, f_out)
    bw = oracle.gcnconv_backward(src, dst, n, x, w, g, loops)
    # dense operator
    a = dense_adjacency(src, dst, n) + (np.eye(n) if loops else 0.0)
    d = a.sum(1)
    dinv = np.where(d > 0, 1.0 / np.sqrt(np.maximum(d, 1e-300)), 0.0)
    ahat = dinv[:, None] * a * dinv[None, :]
    t = ahat.T @ g.astype(np.float64)
    np.testing.assert_allclose(bw["grad_x"], t @ w.astype(np.float64).T, rtol=0, atol=2e-7 * np.abs(t).max() * 3)
    np.testing.assert_allclose(bw["grad_w"], x.astype(np.float64).T @ t, rtol=0, atol=3e-7 * np.abs(x.T @ t).max())
    np.testing.assert_allclose(bw["grad_b"], g.astype(np.float64).sum(0), rtol=1e-6, atol=1e-6)
    # the loss <out, g> is linear in X, in W and in b: each gradient paired with its variable gives it back
    out = oracle.gcnconv(src, dst, n, x, w, b, loops).astype(np.float64)
    loss = (out * g).sum()
    bias_part = (b.astype(np.float64)[None, :] * g).sum()
    np.testing.assert_allclose((bw["grad_x"].astype(np.float64) * x).sum(), loss - bias_part, rtol=1e-5, atol=1e-5)
    np.testing.assert_allclose((bw["grad_w"].astype(np.float64) * w).sum(), loss - bias_part, rtol=1e-5, atol=1e-5)
    np.testing.assert_allclose((bw["grad_b"].astype(np.float64) * b).sum(), bias_part, rtol=1e-5, atol=1e-5)


def _gat_inputs(seed, n, e, f_in, heads, ch):
    src, dst = rng_graph(seed, n, e, star=True)
    loops = np.arange(n, dtype=np.int32)[::3]
    src, dst = np.concatenate([src, loops]), np.concatenate([dst, loops])
    x = synth.normal_f32(seed, 2, n * f_in).reshape(n, f_in)
    w = synth.glorot_uniform(seed, 4, f_in, heads * ch, (f_in, heads * ch))
    a_s = synth.uniform_f32(seed, 5, heads * ch, -1, 1).reshape(heads, ch)
    a_d = synth.uniform_f32(seed, 6, heads * ch, -1, 1).reshape(heads, ch)
    gout = synth.normal_f32(seed, 7, n * heads * ch).reshape(n, heads * ch)
    return src, dst, x, w, a_s, a_d, gout


def test_softmax_backward_is_the_autograd_gradient():
    """The segment-softmax Jacobian against reverse-mode differentiation of a float64 forward built from
    library scatter operations, plus what the Jacobian fixes: gradients of a segment sum to zero, a
    gradient that is constant over a segment gives zero, a one-edge segment gives zero."""
    import torch
    n, heads = 40, 3
    src, dst = rng_graph(95, n, 400, star=True)
    dst = np.concatenate([dst, np.array([n - 1], np.int32)])      # node n-1: make sure of a one-edge segment
    dst[:-1][dst[:-1] == n - 1] = 0
    e = dst.shape[0]
    s = (2.0 * synth.normal_f32(95, 2, e * heads)).reshape(e, heads)
    galpha = synth.normal_f32(95, 3, e * heads).reshape(e, heads)
    alpha = oracle.segment_softmax(dst, n, s)
    got = oracle.segment_softmax_backward(dst, n, alpha, galpha)
    st = torch.tensor(s, dtype=torch.float64, requires_grad=True)
    dt = torch.tensor(dst, dtype=torch.int64)
    ex = torch.exp(st - st.max())
    den = torch.zeros(n, heads, dtype=torch.float64).index_add_(0, dt, ex)
    (ex / den[dt] * torch.tensor(galpha, dtype=torch.float64)).sum().backward()
    ref = st.grad.numpy()
    np.testing.assert_allclose(got, ref, rtol=0, atol=2e-6 * np.abs(ref).max())
    sums = np.zeros((n, heads))
    np.add.at(sums, dst, got.astype(np.float64))
    assert np.abs(sums).max() <= 1e-6
    assert np.abs(got[-1]).max() <= 1e-7                            # the one-edge segment
    per_seg = synth.normal_f32(95, 4, n * heads).reshape(n, heads)[dst]
    const = oracle.segment_softmax_backward(dst, n, alpha, per_seg)
    assert np.abs(const).max() <= 1e-6


def test_gat_backward_is_the_autograd_gradient():
    """All four gradients of the attention layer against reverse-mode differentiation (float64, library
    gather / scatter-add operations) of an independent forward on a multigraph with a hub, duplicate
    edges, self-loops and nodes without incoming edges."""
    import torch
    n, f_in, heads, ch = 36, 6, 3, 4
    src, dst, x, w, a_s, a_d, gout = _gat_inputs(91, n, 350, f_in, heads, ch)
    res = oracle.gatconv_backward(src, dst, n, x, w, a_s, a_d, gout, 0.2)
    t = lambda a: torch.tensor(a, dtype=torch.float64, requires_grad=True)
    xt, wt, ast, adt = t(x), t(w), t(a_s), t(a_d)
    st, dt = torch.tensor(src, dtype=torch.int64), torch.tensor(dst, dtype=torch.int64)
    xw = xt @ wt
    h = (xw + (xw.detach().float().double() - xw.detach())).reshape(n, heads, ch)   # stored in float: value only
    sl, sr = (h * ast[None]).sum(-1), (h * adt[None]).sum(-1)
    v = sl[st] + sr[dt]
    sc = torch.where(v > 0, v, 0.2 * v)
    ex = torch.exp(sc - sc.max())
    den = torch.zeros(n, heads, dtype=torch.float64).index_add_(0, dt, ex)
    alpha = ex / den[dt]
    out = torch.zeros(n, heads, ch, dtype=torch.float64).index_add_(0, dt, alpha[:, :, None] * h[st])
    (out.reshape(n, heads * ch) * torch.tensor(gout, dtype=torch.float64)).sum().backward()
    for name, ref in (("grad_x", xt.grad), ("grad_w", wt.grad), ("grad_a_src", ast.grad), ("grad_a_dst", adt.grad)):
        ref = ref.numpy()
        np.testing.assert_allclose(res[name], ref, rtol=0, atol=2e-6 * np.abs(ref).max(), err_msg=name)
        # the magnitude outputs bound the values they belong to
        assert (np.abs(ref) <= res["sabs" + name[4:]] * (1 + 1e-6) + 1e-30).all(), name


def test_gat_backward_finite_differences():
    """Central differences of L = <G, out> through the oracle's own forward, in a few coordinates of
    every input (step 2e-3 on float inputs and a float result: agreement to ~1e-2 of the largest entry)."""
    n, f_in, heads, ch = 20, 5, 2, 3
    src, dst, x, w, a_s, a_d, gout = _gat_inputs(92, n, 120, f_in, heads, ch)
    res = oracle.gatconv_backward(src, dst, n, x, w, a_s, a_d, gout, 0.2)

    def loss(x_, w_, as_, ad_):
        return float((oracle.gatconv(src, dst, n, x_, w_, as_, ad_, 0.2).astype(np.float64) * gout).sum())

    args = [x, w, a_s, a_d]
    names = ["grad_x", "grad_w", "grad_a_src", "grad_a_dst"]
    step = 1.0 / 512
    for which in range(4):
        flat_n = args[which].size
        for q in range(0, flat_n, max(1, flat_n // 5)):
            hi = [a.copy() for a in args]
            lo = [a.copy() for a in args]
            hi[which].reshape(-1)[q] += step
            lo[which].reshape(-1)[q] -= step
            fd = (loss(*hi) - loss(*lo)) / (2 * step)
            an = float(res[names[which]].reshape(-1)[q])
            scale = max(1.0, float(np.abs(res[names[which]]).max()))
            assert abs(fd - an) <= 1e-2 * scale, (names[which], q, fd, an)


def test_gat_backward_zero_attention_is_mean_backward():
    """With zero attention vectors every weight is 1/in-degree, so grad_x reduces to the (already pinned)
    backward of mean aggregation followed by W^T."""
    wl = synth.config4_gat(num_nodes=300, num_edges=2500, f_in=9, heads=2, ch=4, cap=80.0)
    n = wl.num_nodes
    zero = np.zeros((2, 4), np.float32)
    gout = synth.normal_f32(93, 7, n * 8).reshape(n, 8)
    res = oracle.gatconv_backward(wl.src, wl.dst, n, wl.x, wl.params["w"], zero, zero, gout, 0.2)
    hfeat = (wl.x.astype(np.float64) @ wl.params["w"].astype(np.float64)).astype(np.float32)
    dh = oracle.propagate_backward(wl.src, wl.dst, n, hfeat, gout, None, MSG_COPY_XJ, AGGR_MEAN)["grad_x"]
    ref = dh.astype(np.float64) @ wl.params["w"].astype(np.float64).T
    np.testing.assert_allclose(res["grad_x"], ref, rtol=0, atol=3e-6 * np.abs(ref).max())
    ref_w = wl.x.astype(np.float64).T @ dh.astype(np.float64)
    np.testing.assert_allclose(res["grad_w"], ref_w, rtol=0, atol=3e-6 * np.abs(ref_w).max())


@pytest.mark.parametrize("seed,n,e,f", [(71, 40, 400, 5), (72, 12, 15, 3)])
def test_min_prod_and_target_messages_brute_force(seed, n, e, f):
    """min / prod reductions and the two messages that read the target node, against per-destination
    numpy loops written from the definitions; plus what they must reduce to: min(x) = -max(-x),
    sum of (x_j - x_i) = sum of x_j - indegree * x_i, and xi_dot_xj on a single feature = the product."""
    src, dst = rng_graph(seed, n, e, star=True)
    ne = src.shape[0]
    x = synth.uniform_f32(seed, 2, n * f, 0.5, 1.5).reshape(n, f)
    x[::3] *= -1.0
    w = synth.uniform_f32(seed, 3, ne, -1.0, 1.0)
    inc = incoming(dst, n)
    # messages
    sub = oracle.apply_edges(src, n, x, None, MSG_XJ_SUB_XI, dst=dst)
    np.testing.assert_array_equal(sub, x[src] - x[dst])
    dot, dot_abs = oracle.apply_edges(src, n, x, None, MSG_XI_DOT_XJ, dst=dst, with_sabs=True)
    ref_dot = (x[src].astype(np.float64) * x[dst].astype(np.float64)).sum(1, keepdims=True)
    assert dot.shape == (ne, 1)
    np.testing.assert_allclose(dot, ref_dot, rtol=0, atol=1e-7 * dot_abs.max())
    one = oracle.apply_edges(src, n, x[:, :1].copy(), None, MSG_XI_DOT_XJ, dst=dst)
    np.testing.assert_array_equal(one[:, 0], x[src, 0] * x[dst, 0])
    # reductions of a materialised message tensor and of the fused form
    for msg, edata, msgs in ((MSG_COPY_XJ, None, x[src]), (MSG_E_MUL_XJ, w, w[:, None] * x[src]),
                             (MSG_XJ_SUB_XI, None, x[src] - x[dst])):
        ref_min, ref_prod = np.zeros((n, f)), np.zeros((n, f))
        for i in range(n):
            if inc[i].size:
                ref_min[i] = msgs[inc[i]].min(0)
                ref_prod[i] = np.prod(msgs[inc[i]].astype(np.float64), axis=0)
        got_min = oracle.propagate(src, dst, n, x, edata, msg, AGGR_MIN)
        np.testing.assert_array_equal(got_min, ref_min.astype(np.float32))
        got_prod, sabs = oracle.propagate(src, dst, n, x, edata, msg, AGGR_PROD, with_sabs=True)
        np.testing.assert_allclose(got_prod, ref_prod, rtol=1e-6, atol=1e-300)
        assert (sabs >= np.abs(ref_prod) * (1 - 1e-12)).all()
        two_step = oracle.aggregate_neighbors(dst, n, msgs.astype(np.float32), AGGR_MIN)
        np.testing.assert_array_equal(two_step, got_min)
        neg_max = oracle.aggregate_neighbors(dst, n, (-msgs).astype(np.float32), AGGR_MAX)
        np.testing.assert_array_equal(got_min, -neg_max)
    s_sub = oracle.propagate(src, dst, n, x, None, MSG_XJ_SUB_XI, AGGR_SUM).astype(np.float64)
    s_cp = oracle.propagate(src, dst, n, x, None, MSG_COPY_XJ, AGGR_SUM).astype(np.float64)
    deg = np.bincount(dst, minlength=n)[:, None]
    np.testing.assert_allclose(s_sub, s_cp - deg * x, rtol=0, atol=2e-5)


def test_min_of_signed_zeros_is_minus_zero():
    src = np.array([1, 2, 2, 1], np.int32)
    dst = np.array([0, 0, 3, 3], np.int32)
    x = np.array([[0.0], [-0.0], [0.0], [0.0]], np.float32)
    out = oracle.propagate(src, dst, 4, x, None, MSG_COPY_XJ, AGGR_MIN)
    assert np.signbit(out[0, 0]) and np.signbit(out[3, 0])       # {-0, +0} in either order
    assert out[1, 0] == 0 and not np.signbit(out[1, 0])           # empty neighbourhood: +0
    prod = oracle.propagate(src, dst, 4, np.array([[3.0], [2.0], [-4.0], [1.0]], np.float32), None, MSG_COPY_XJ,
                            AGGR_PROD)
    np.testing.assert_array_equal(prod[:, 0], [-8.0, 0.0, 0.0, -8.0])


def test_batchnorm_and_dense_against_numpy():
    """Batch normalisation over the node dimension against numpy's float64 mean / variance, with what the
    definition fixes (zero mean and unit variance per feature when gamma = 1, beta = 0, eps = 0; a constant
    column maps to beta; stored statistics are used as given); the dense layer against a float64 matmul."""
    n, f = 300, 7
    x = (synth.normal_f32(97, 2, n * f).reshape(n, f) * np.arange(1, f + 1, dtype=np.float32) + 3.0).astype(np.float32)
    x[:, 3] = 2.5                                                   # a constant column
    gamma = synth.uniform_f32(97, 3, f, 0.5, 1.5)
    beta = synth.uniform_f32(97, 4, f, -1.0, 1.0)
    out, mean, var = oracle.batchnorm(x, gamma, beta, 1e-5)
    x64 = x.astype(np.float64)
    np.testing.assert_allclose(mean, x64.mean(0), rtol=1e-6)
    np.testing.assert_allclose(var, x64.var(0), rtol=1e-6, atol=1e-12)
    ref = gamma * (x64 - x64.mean(0)) / np.sqrt(x64.var(0) + np.float32(1e-5)) + beta
    np.testing.assert_allclose(out, ref, rtol=0, atol=2e-6)
    np.testing.assert_allclose(out[:, 3], beta[3], atol=1e-6)
    plain, _, _ = oracle.batchnorm(x[:, [0, 1, 2, 4]].copy(), None, None, 0.0)
    np.testing.assert_allclose(plain.astype(np.float64).mean(0), 0.0, atol=1e-6)
    np.testing.assert_allclose(plain.astype(np.float64).var(0), 1.0, rtol=1e-5)
    relu, _, _ = oracle.batchnorm(x, gamma, beta, 1e-5, relu=True)
    np.testing.assert_array_equal(relu, np.maximum(out, 0))
    m_given, v_given = np.zeros(f, np.float32), np.ones(f, np.float32)
    given, m2, v2 = oracle.batchnorm(x, gamma, beta, 0.0, mean=m_given, var=v_given)
    np.testing.assert_allclose(given, gamma * x64 + beta, rtol=1e-6, atol=1e-6)
    np.testing.assert_array_equal(m2, m_given)
    w = synth.glorot_uniform(97, 5, f, 4, (f, 4))
    b = synth.uniform_f32(97, 6, 4, -1, 1)
    y, sabs = oracle.dense(x, w, b, with_sabs=True)
    ref_y = x64 @ w.astype(np.float64) + b
    assert (np.abs(y - ref_y) <= 1e-7 * sabs).all()
    np.testing.assert_array_equal(oracle.dense(x, w, b, relu=True), np.maximum(y, 0))
    np.testing.assert_allclose(oracle.dense(x, w), x64 @ w.astype(np.float64), rtol=0, atol=1e-6 * sabs.max())


def test_example_model_against_dense_float64():
    """The example model end to end (GCNConv, batch norm over nodes, relu, GCNConv + relu, mean pooling,
    dense) against a float64 implementation with explicit dense adjacency and membership matrices on a
    small collated batch; intermediates are never rounded there, so agreement is to ~1e-5."""
    wl = synth.config5_example_model(num_graphs=5, n=12, p=0.3)
    n, g_cnt, p = wl.num_nodes, wl.num_graphs, wl.params
    res = oracle.example_model_forward(wl.src, wl.dst, n, wl.graph_indicator, g_cnt, wl.x, p)
    a = dense_adjacency(wl.src, wl.dst, n) + np.eye(n)
    deg = a.sum(1)
    ahat = a / np.sqrt(np.outer(deg, deg))
    f64 = lambda k: p[k].astype(np.float64)
    h1 = ahat @ (wl.x.astype(np.float64) @ f64("w1")) + f64("b1")
    h2 = np.maximum(f64("gamma") * (h1 - h1.mean(0)) / np.sqrt(h1.var(0) + np.float32(1e-5)) + f64("beta"), 0)
    h3 = np.maximum(ahat @ (h2 @ f64("w2")) + f64("b2"), 0)
    member = np.zeros((g_cnt, n))
    member[wl.graph_indicator, np.arange(n)] = 1.0
    pooled = (member @ h3) / member.sum(1, keepdims=True)
    y = pooled @ f64("w3") + f64("b3")
    np.testing.assert_allclose(res["h1"], h1, rtol=0, atol=1e-5 * np.abs(h1).max())
    np.testing.assert_allclose(res["h3"], h3, rtol=0, atol=2e-5 * np.abs(h3).max())
    np.testing.assert_allclose(res["y"], y, rtol=0, atol=2e-5 * np.abs(y).max())
    assert res["y"].shape == (g_cnt, 1)


def test_bf16_rounding(golden_dir):
    """Hand-worked bit patterns, and on random floats the defining property: the result is one of the two
    neighbouring codes, at most half a unit in the last place away, and a tie lands on the even code."""
    gd = load_golden(golden_dir, "bf16_rounding.json")
    bits = np.array([int(c["float_bits"], 16) for c in gd["cases"]], np.uint32)
    codes, wide = oracle.round_bf16(bits.view(np.float32))
    np.testing.assert_array_equal(codes, np.array([int(c["bf16"], 16) for c in gd["cases"]], np.uint16))
    np.testing.assert_array_equal(wide.view(np.uint32) >> 16, codes)
    x = (synth.normal_f32(99, 2, 20000) * np.float32(10.0) ** synth.randint(99, 3, 0, 20000, -20, 20)).astype(np.float32)
    codes, wide = oracle.round_bf16(x)
    ulp = np.abs(wide.astype(np.float64)) * 2.0 ** -7          # spacing is between 2^-8 and 2^-7 of the value
    assert (np.abs(wide.astype(np.float64) - x) <= 0.5 * ulp).all()
    trunc = (x.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)
    nxt = ((x.view(np.uint32) & np.uint32(0xFFFF0000)) + np.uint32(0x10000)).view(np.float32)
    assert ((wide == trunc) | (wide == nxt)).all()
    better = np.minimum(np.abs(trunc.astype(np.float64) - x), np.abs(nxt.astype(np.float64) - x))
    np.testing.assert_array_equal(np.abs(wide.astype(np.float64) - x), better)
    # representable values are fixed points
    np.testing.assert_array_equal(oracle.round_bf16(wide)[1], wide)


def test_f16_rounding(golden_dir):
    """Hand-worked bit patterns (ties, both ends of the subnormal range, overflow), numpy's own float16 conversion
    on random floats over the whole range (an independent IEEE implementation), and the defining property."""
    gd = load_golden(golden_dir, "f16_rounding.json")
    bits = np.array([int(c["float_bits"], 16) for c in gd["cases"]], np.uint32)
    codes, wide = oracle.round_f16(bits.view(np.float32))
    np.testing.assert_array_equal(codes, np.array([int(c["f16"], 16) for c in gd["cases"]], np.uint16))
    x = (synth.normal_f32(98, 2, 50000) * np.float32(10.0) ** synth.randint(98, 3, 0, 50000, -10, 6)).astype(np.float32)
    codes, wide = oracle.round_f16(x)
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16)
    np.testing.assert_array_equal(codes, ref.view(np.uint16))
    np.testing.assert_array_equal(wide.view(np.uint32), ref.astype(np.float32).view(np.uint32))
    # nearest: no representable value is closer (neighbouring codes of the same sign, where finite)
    fin = np.isfinite(wide) & (np.abs(x) < 60000)
    mag = (codes & 0x7FFF).astype(np.int32)
    for step in (-1, 1):
        nb = np.clip(mag + step, 0, 0x7BFF).astype(np.uint16) | (codes & 0x8000)
        nbv = nb.view(np.float16).astype(np.float64)
        assert (np.abs(wide[fin].astype(np.float64) - x[fin]) <= np.abs(nbv[fin] - x[fin])).all()
    # representable values are fixed points
    np.testing.assert_array_equal(oracle.round_f16(wide[fin])[1], wide[fin])


def _hetero_relations(seed, n_dst, sizes, edges, f):
    rels = []
    for r, (ns, ne) in enumerate(zip(sizes, edges)):
        src = synth.randint(seed, 10 + r, 0, ne, 0, ns - 1).astype(np.int32)
        dst = synth.randint(seed, 20 + r, 0, ne, 0, n_dst - 1).astype(np.int32)
        dst[dst % 5 == 2] = 0                                          # a hub and some empty destinations
        rels.append({"src": src, "dst": dst, "num_src_nodes": ns,
                     "x": synth.normal_f32(seed, 30 + r, ns * f).reshape(ns, f),
                     "e": synth.uniform_f32(seed, 40 + r, ne, -1.0, 1.0)})
    return rels


def test_hetero_propagate_is_a_sum_of_rectangular_products():
    """Relations into one node type: each is a rectangular (destinations x sources) adjacency product, the
    relations are summed; with the node types laid side by side it is one homogeneous propagate."""
    n_dst, sizes, edges, f = 23, [17, 40, 23], [150, 300, 90], 4
    rels = _hetero_relations(83, n_dst, sizes, edges, f)
    got = oracle.hetero_propagate(rels, n_dst, MSG_E_MUL_XJ, AGGR_SUM)
    ref = np.zeros((n_dst, f))
    ref_mean = np.zeros((n_dst, f))
    for r in rels:
        a = np.zeros((n_dst, r["num_src_nodes"]))
        np.add.at(a, (r["dst"], r["src"]), r["e"].astype(np.float64))
        ref += a @ r["x"].astype(np.float64)
        cnt = np.bincount(r["dst"], minlength=n_dst)[:, None]
        c = np.zeros((n_dst, r["num_src_nodes"]))
        np.add.at(c, (r["dst"], r["src"]), 1.0)
        ref_mean += np.where(cnt > 0, (c @ r["x"].astype(np.float64)) / np.maximum(cnt, 1), 0.0)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-6 * np.abs(ref).max())
    got_mean = oracle.hetero_propagate(rels, n_dst, MSG_COPY_XJ, AGGR_MEAN)
    np.testing.assert_allclose(got_mean, ref_mean, rtol=0, atol=1e-6 * np.abs(ref_mean).max())
    # one homogeneous graph: destination type first, then the source types one after the other
    offs = np.cumsum([n_dst] + sizes)
    src = np.concatenate([r["src"] + offs[k] for k, r in enumerate(rels)]).astype(np.int32)
    dst = np.concatenate([r["dst"] for r in rels]).astype(np.int32)
    x = np.concatenate([np.zeros((n_dst, f), np.float32)] + [r["x"] for r in rels])
    e = np.concatenate([r["e"] for r in rels])
    merged = oracle.propagate(src, dst, int(offs[-1]), x, e, MSG_E_MUL_XJ, AGGR_SUM)
    np.testing.assert_allclose(got, merged[:n_dst], rtol=0, atol=1e-6 * np.abs(ref).max())
    assert np.abs(merged[n_dst:]).max() == 0
    # a single relation on one node set is plain propagate
    one = oracle.hetero_propagate([rels[2]], n_dst, MSG_COPY_XJ, AGGR_MAX)
    np.testing.assert_array_equal(one, oracle.propagate(rels[2]["src"], rels[2]["dst"], n_dst, rels[2]["x"], None,
                                                        MSG_COPY_XJ, AGGR_MAX))


def test_example_model_backward_is_the_autograd_gradient():
    """Loss and all eight parameter gradients of the example model against reverse-mode differentiation of an
    independent float64 forward built from dense adjacency / membership matrices and library operations
    (including the library's own batch normalisation in training mode)."""
    import torch
    wl = synth.config5_example_model(num_graphs=6, n=14, p=0.25)
    n, ng, p = wl.num_nodes, wl.num_graphs, wl.params
    target = synth.normal_f32(77, 9, ng).reshape(ng, 1)
    loss, grads, _ = oracle.example_model_backward(wl.src, wl.dst, n, wl.graph_indicator, ng, wl.x, p, target)
    a = dense_adjacency(wl.src, wl.dst, n) + np.eye(n)
    deg = a.sum(1)
    ahat = torch.tensor(a / np.sqrt(np.outer(deg, deg)))
    member = np.zeros((ng, n))
    member[wl.graph_indicator, np.arange(n)] = 1.0
    member = torch.tensor(member / member.sum(1, keepdims=True))
    tp = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()}
    xt = torch.tensor(wl.x, dtype=torch.float64)
    h1 = ahat @ (xt @ tp["w1"]) + tp["b1"]
    h2 = torch.relu(torch.nn.functional.batch_norm(h1, None, None, tp["gamma"], tp["beta"], training=True, eps=1e-5))
    h3 = torch.relu(ahat @ (h2 @ tp["w2"]) + tp["b2"])
    y = (member @ h3) @ tp["w3"] + tp["b3"]
    ref_loss = ((y - torch.tensor(target, dtype=torch.float64)) ** 2).mean()
    ref_loss.backward()
    assert abs(loss - float(ref_loss.detach())) <= 1e-5 * abs(float(ref_loss.detach()))
    scale = max(float(tp[k].grad.abs().max()) for k in p)
    for k in p:
        ref = tp[k].grad.numpy()
        # (the gradient of b1 is exactly zero: the batch norm removes any constant shift)
        np.testing.assert_allclose(grads[k], ref, rtol=0, atol=2e-5 * np.abs(ref).max() + 1e-7 * scale, err_msg=k)
    assert np.abs(grads["b1"]).max() <= 1e-7 * scale


def test_dense_batchnorm_pool_backward_pieces():
    """The pieces on their own: dense backward against float64 products, pooling backward against its
    definition, batch-norm backward against what its Jacobian fixes (gradients orthogonal to constants and
    to xhat) and against reverse-mode differentiation."""
    import torch
    n, k, m = 50, 6, 3
    x = synth.normal_f32(79, 2, n * k).reshape(n, k)
    w = synth.glorot_uniform(79, 3, k, m, (k, m))
    gy = synth.normal_f32(79, 4, n * m).reshape(n, m)
    gx, gw, gb = oracle.dense_backward(x, w, gy)
    np.testing.assert_allclose(gx, gy.astype(np.float64) @ w.astype(np.float64).T, rtol=0, atol=1e-6)
    np.testing.assert_allclose(gw, x.astype(np.float64).T @ gy.astype(np.float64), rtol=0, atol=1e-5)
    np.testing.assert_allclose(gb, gy.astype(np.float64).sum(0), rtol=0, atol=1e-5)
    gi = np.repeat(np.arange(4, dtype=np.int32), [3, 1, 10, 36])
    go = synth.normal_f32(79, 5, 4 * k).reshape(4, k)
    np.testing.assert_array_equal(oracle.pool_backward(gi, 4, go, AGGR_SUM), go[gi])
    np.testing.assert_allclose(oracle.pool_backward(gi, 4, go, AGGR_MEAN), go[gi] / np.array([3, 1, 10, 36])[gi][:, None],
                               rtol=1e-7)
    gamma = synth.uniform_f32(79, 6, k, 0.5, 1.5)
    gyb = synth.normal_f32(79, 7, n * k).reshape(n, k)
    bx, bg, bb = oracle.batchnorm_backward(x, gamma, gyb, 1e-5)
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    gt = torch.tensor(gamma, dtype=torch.float64, requires_grad=True)
    bt = torch.zeros(k, dtype=torch.float64, requires_grad=True)
    out = torch.nn.functional.batch_norm(xt, None, None, gt, bt, training=True, eps=1e-5)
    (out * torch.tensor(gyb, dtype=torch.float64)).sum().backward()
    np.testing.assert_allclose(bx, xt.grad.numpy(), rtol=0, atol=1e-6)
    np.testing.assert_allclose(bg, gt.grad.numpy(), rtol=0, atol=1e-5)
    np.testing.assert_allclose(bb, bt.grad.numpy(), rtol=0, atol=1e-5)
    assert np.abs(bx.astype(np.float64).sum(0)).max() <= 1e-5            # shifting x does not change the output
    bx0, _, _ = oracle.batchnorm_backward(x, gamma, gyb, 0.0)
    xhat = (x - x.mean(0)) / np.sqrt(x.astype(np.float64).var(0))
    assert np.abs((bx0 * xhat).sum(0)).max() <= 1e-4                       # nor does scaling x - mean (eps = 0)


def test_adam_step_matches_the_library_optimizer():
    import torch
    n = 200
    p0 = synth.normal_f32(81, 2, n)
    pt = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([pt], lr=1e-2, betas=(0.9, 0.999), eps=1e-8)
    p, m, v = p0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    for t in range(1, 6):
        g = synth.normal_f32(81, 10 + t, n)
        pt.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        p, m, v = oracle.adam_step(p, m, v, g, 1e-2, t)
        np.testing.assert_allclose(p, pt.detach().numpy(), rtol=0, atol=2e-6)
    first, _, _ = oracle.adam_step(p0, np.zeros(n, np.float32), np.zeros(n, np.float32), np.ones(n, np.float32), 1e-2, 1)
    np.testing.assert_allclose(first, p0 - 1e-2, rtol=0, atol=1e-6)      # the first step moves by lr against the sign


def test_error_codes():
    src = np.array([0, 5], np.int32)
    dst = np.array([1, 0], np.int32)
    x = np.zeros((3, 2), np.float32)
    with pytest.raises(oracle.OracleError):
        oracle.build_csr(src, dst, 3)
    with pytest.raises(oracle.OracleError):
        oracle.propagate(src, dst, 3, x)
    with pytest.raises(oracle.OracleError):
        oracle.graph_pool(np.array([0, 1, 9], np.int32), 2, x)


# ----------------------------------------------------------------------------- gradients per edge and S_abs magnitudes

def test_g5_sabs_and_gradients_by_hand(golden_dir):
    """Hand-worked S_abs of the forward (a row whose signed terms cancel to zero keeps the sum of their absolute
    values) and hand-worked gradients with their S_abs, element by element."""
    g5 = load_golden(golden_dir, "g5_propagate.json")
    hw = load_golden(golden_dir, "sabs_handworked.json")["g5"]
    src, dst = np.array(g5["src"], np.int32), np.array(g5["dst"], np.int32)
    x, w = np.array(g5["x"], np.float32), np.array(g5["w"], np.float32)
    for msg_name, msg in (("copy_xj", MSG_COPY_XJ), ("e_mul_xj", MSG_E_MUL_XJ)):
        for aggr_name in ("sum", "mean"):
            _, sabs = oracle.propagate(src, dst, 4, x, w if msg else None, msg, AGGRS[aggr_name], with_sabs=True)
            np.testing.assert_allclose(sabs, np.array(hw[f"{msg_name}_{aggr_name}"]), rtol=1e-15, atol=0,
                                       err_msg=f"{msg_name} {aggr_name}")
    g = np.array(hw["grad_out"], np.float32)
    for aggr_name in ("sum", "mean"):
        bw = oracle.propagate_backward(src, dst, 4, x, g, w, MSG_E_MUL_XJ, AGGRS[aggr_name], with_sabs=True)
        np.testing.assert_allclose(bw["grad_e"][:, 0], np.array(hw[f"grad_e_{aggr_name}"]), rtol=1e-7)
        np.testing.assert_allclose(bw["sabs_e"][:, 0], np.array(hw[f"sabs_e_{aggr_name}"]), rtol=1e-15)
        np.testing.assert_allclose(bw["grad_x"], np.array(hw[f"grad_x_{aggr_name}"]), rtol=1e-7)
        np.testing.assert_allclose(bw["sabs_x"], np.array(hw[f"sabs_x_{aggr_name}"]), rtol=1e-15)


def test_path3_layer_sabs_by_hand(golden_dir):
    """GCN and attention layer on the 3-node path with inputs whose products cancel inside X W: the magnitude
    is built from |X||W|, not from |X W|; hand-worked values of the outputs, their S_abs and the GCN gradients."""
    hw = load_golden(golden_dir, "sabs_handworked.json")["path3"]
    src, dst = np.array(hw["src"], np.int32), np.array(hw["dst"], np.int32)
    x, w, b = np.array(hw["x"], np.float32), np.array(hw["w"], np.float32), np.array(hw["bias"], np.float32)
    out, sabs = oracle.gcnconv(src, dst, 3, x, w, b, True, with_sabs=True)
    np.testing.assert_allclose(out, np.array(hw["gcn_out"]), rtol=1e-7)
    np.testing.assert_allclose(sabs, np.array(hw["gcn_sabs"]), rtol=1e-15)
    g = np.array(hw["gcn_grad_out"], np.float32)
    t, tabs = np.array(hw["gcn_T"]), np.array(hw["gcn_Tabs"])
    bw = oracle.gcnconv_backward(src, dst, 3, x, w, g, True)
    np.testing.assert_allclose(bw["grad_x"], np.stack([t, t], 1), rtol=1e-6)               # W = [[1],[1]]
    np.testing.assert_allclose(bw["sabs_x"], np.stack([tabs, tabs], 1), rtol=1e-15)
    np.testing.assert_allclose(bw["grad_w"][:, 0], [1 * t[0] + 2 * t[1], -1 * t[0] + 3 * t[2]], rtol=1e-6)
    np.testing.assert_allclose(bw["sabs_w"][:, 0], [1 * tabs[0] + 2 * tabs[1], 1 * tabs[0] + 3 * tabs[2]], rtol=1e-15)
    np.testing.assert_allclose(bw["grad_b"], hw["gcn_grad_b"], rtol=0)
    np.testing.assert_allclose(bw["sabs_b"], hw["gcn_sabs_b"], rtol=0)
    a_s, a_d = np.array(hw["a_src"], np.float32), np.array(hw["a_dst"], np.float32)
    out, sabs = oracle.gatconv(src, dst, 3, x, w, a_s, a_d, 0.2, with_sabs=True)
    np.testing.assert_allclose(out, np.array(hw["gat_out"]), rtol=1e-7)
    np.testing.assert_allclose(sabs, np.array(hw["gat_sabs"]), rtol=1e-14)


@pytest.mark.parametrize("aggr", [AGGR_SUM, AGGR_MEAN])
@pytest.mark.parametrize("e_kind", ["scalar", "vector"])
def test_grad_e_and_backward_sabs_brute_force(aggr, e_kind):
    """Every element of grad_e, not only its pairing with e: grad_e[k] = <x[src k], g[dst k]> (one weight per edge)
    or the element-wise product (one weight per edge and feature), divided by the in-degree of dst k for the mean;
    and the S_abs outputs of the backward are the same sums over absolute values.  Python loops over the edges of a
    multigraph with a hub, duplicate edges, self-loops and isolated nodes."""
    n, f = 40, 4
    src, dst = rng_graph(97, n, 500, star=True)
    ne = src.shape[0]
    x = synth.normal_f32(97, 2, n * f).reshape(n, f)
    g = synth.normal_f32(97, 7, n * f).reshape(n, f)
    e = synth.uniform_f32(97, 3, ne, -1, 1) if e_kind == "scalar" else synth.normal_f32(97, 3, ne * f).reshape(ne, f)
    bw = oracle.propagate_backward(src, dst, n, x, g, e, MSG_E_MUL_XJ, aggr, with_sabs=True)
    indeg = np.bincount(dst, minlength=n)
    x64, g64, e64 = x.astype(np.float64), g.astype(np.float64), e.astype(np.float64).reshape(ne, -1)
    ge = np.zeros_like(e64)
    se = np.zeros_like(e64)
    gx, sx = np.zeros((n, f)), np.zeros((n, f))
    for k in range(ne):
        gi = g64[dst[k]] / (indeg[dst[k]] if aggr == AGGR_MEAN else 1.0)
        prod = x64[src[k]] * gi
        if e_kind == "scalar":
            ge[k, 0], se[k, 0] = prod.sum(), np.abs(prod).sum()
        else:
            ge[k], se[k] = prod, np.abs(prod)
        gx[src[k]] += e64[k] * gi
        sx[src[k]] += np.abs(e64[k] * gi)
    np.testing.assert_allclose(bw["grad_e"], ge, rtol=0, atol=2e-7 * np.abs(ge).max())
    np.testing.assert_allclose(bw["sabs_e"], se, rtol=1e-12)
    np.testing.assert_allclose(bw["grad_x"], gx, rtol=0, atol=2e-7 * np.abs(gx).max())
    np.testing.assert_allclose(bw["sabs_x"], sx, rtol=1e-12)


def test_forward_sabs_is_the_operator_on_absolute_values():
    """S_abs of propagate / GCNConv / the attention layer against dense float64 products of the absolute values
    (|A| |X|, Ahat |X||W| + |b|, alpha-weighted |X||W| with alpha from a per-row numpy softmax): a magnitude that is
    too large by any factor, or built from |X W| instead of |X||W|, fails."""
    n, f_in, f_out = 48, 5, 3
    src, dst = rng_graph(61, n, 400, star=True)
    ne = src.shape[0]
    x = synth.normal_f32(61, 2, n * f_in).reshape(n, f_in)
    e = synth.uniform_f32(61, 3, ne, -1, 1)
    indeg = np.bincount(dst, minlength=n)
    a_abs = dense_adjacency(src, dst, n, np.abs(e))
    for aggr in (AGGR_SUM, AGGR_MEAN):
        _, sabs = oracle.propagate(src, dst, n, x, e, MSG_E_MUL_XJ, aggr, with_sabs=True)
        # the product e * x is rounded to float before it is summed: its magnitude is that float's
        ref = np.zeros((n, f_in))
        for k in range(ne):
            ref[dst[k]] += np.abs((e[k] * x[src[k]]).astype(np.float32)).astype(np.float64)
        if aggr == AGGR_MEAN:
            ref = ref / np.maximum(indeg, 1)[:, None]
        np.testing.assert_allclose(sabs, ref, rtol=1e-12)
        np.testing.assert_allclose(sabs, (a_abs @ np.abs(x).astype(np.float64)) /
                                   (np.maximum(indeg, 1)[:, None] if aggr == AGGR_MEAN else 1.0), rtol=1e-6)
    w = synth.glorot_uniform(61, 4, f_in, f_out, (f_in, f_out))
    b = synth.uniform_f32(61, 5, f_out, -1, 1)
    zabs = np.abs(x).astype(np.float64) @ np.abs(w).astype(np.float64)
    for loops in (True, False):
        a = dense_adjacency(src, dst, n) + (np.eye(n) if loops else 0.0)
        d = a.sum(1)
        dinv = np.where(d > 0, 1.0 / np.sqrt(np.maximum(d, 1e-300)), 0.0)
        _, sabs = oracle.gcnconv(src, dst, n, x, w, b, loops, with_sabs=True)
        np.testing.assert_allclose(sabs, (dinv[:, None] * a * dinv[None, :]) @ zabs + np.abs(b), rtol=1e-12)
    heads, ch = 3, 1
    a_s = synth.uniform_f32(61, 6, heads * ch, -1, 1).reshape(heads, ch)
    a_d = synth.uniform_f32(61, 7, heads * ch, -1, 1).reshape(heads, ch)
    _, sabs = oracle.gatconv(src, dst, n, x, w, a_s, a_d, 0.2, with_sabs=True)
    h = (x.astype(np.float64) @ w.astype(np.float64)).astype(np.float32).astype(np.float64).reshape(n, heads, ch)
    sl, sr = (h * a_s[None]).sum(-1), (h * a_d[None]).sum(-1)
    ref = np.zeros((n, heads, ch))
    inc = incoming(dst, n)
    for i in range(n):
        if inc[i].size:
            j = src[inc[i]]
            sc = sl[j] + sr[i][None]
            sc = np.where(sc > 0, sc, 0.2 * sc)
            ex = np.exp(sc - sc.max(0))
            ref[i] = ((ex / ex.sum(0))[:, :, None] * zabs.reshape(n, heads, ch)[j]).sum(0)
    np.testing.assert_allclose(sabs.reshape(n, heads, ch), ref, rtol=1e-7)


def test_gcn_backward_sabs_is_the_operator_on_absolute_values():
    n, f_in, f_out = 40, 5, 3
    src, dst = rng_graph(95, n, 300, star=True)
    x = synth.normal_f32(95, 2, n * f_in).reshape(n, f_in)
    w = synth.glorot_uniform(95, 4, f_in, f_out, (f_in, f_out))
    g = synth.normal_f32(95, 7, n * f_out).reshape(n, f_out)
    for loops in (True, False):
        bw = oracle.gcnconv_backward(src, dst, n, x, w, g, loops)
        a = dense_adjacency(src, dst, n) + (np.eye(n) if loops else 0.0)
        d = a.sum(1)
        dinv = np.where(d > 0, 1.0 / np.sqrt(np.maximum(d, 1e-300)), 0.0)
        tabs = (dinv[:, None] * a * dinv[None, :]).T @ np.abs(g).astype(np.float64)
        np.testing.assert_allclose(bw["sabs_x"], tabs @ np.abs(w).astype(np.float64).T, rtol=1e-12)
        np.testing.assert_allclose(bw["sabs_w"], np.abs(x).astype(np.float64).T @ tabs, rtol=1e-12)
        np.testing.assert_allclose(bw["sabs_b"], np.abs(g).astype(np.float64).sum(0), rtol=1e-12)


@pytest.mark.parametrize("msg,aggr", [(MSG_COPY_XJ, AGGR_SUM), (MSG_E_MUL_XJ, AGGR_MEAN), (MSG_E_MUL_XJ, AGGR_MAX),
                                      (MSG_XJ_SUB_XI, AGGR_MIN), (MSG_COPY_XJ, AGGR_PROD)])
def test_all_cores_variant_is_the_same_function(msg, aggr):
    """The row-parallel variant timed as the all-cores CPU baseline: dense float64 A X for the sum, and the very
    bits of the single-threaded edge loop for every message and reduction."""
    wl = synth.config2_weighted(num_nodes=3000, num_edges=40000, feat=8, cap=400.0)
    n, src, dst = wl.num_nodes, wl.src, wl.dst
    e = wl.edge_weight if msg == MSG_E_MUL_XJ else None
    got, threads = oracle.propagate_all_cores(src, dst, n, wl.x, e, msg, aggr)
    assert threads >= 1
    np.testing.assert_array_equal(got.view(np.uint32), oracle.propagate(src, dst, n, wl.x, e, msg, aggr).view(np.uint32))
    if msg == MSG_COPY_XJ and aggr == AGGR_SUM:
        sub = slice(0, 64)   # dense check on the rows of the first 64 nodes
        a = np.zeros((64, n))
        m = dst < 64
        np.add.at(a, (dst[m], src[m]), 1.0)
        ref = a @ wl.x.astype(np.float64)
        np.testing.assert_allclose(got[sub], ref, rtol=0, atol=2e-7 * np.abs(ref).max())
