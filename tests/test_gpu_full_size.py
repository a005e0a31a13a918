"""GPU parity at the benchmark configurations' full sizes, in the launch configuration bench.py times.

The kernels run on the whole graph; the CPU oracle either runs on the whole graph too (where that takes
seconds) or on sampled destination rows: a destination's result depends only on its incoming edges and on
the features of their endpoints, so the test extracts those edges, relabels the touched nodes compactly and
runs the oracle on that subgraph (tests/util.subgraph_for_rows).  Hub rows, ordinary rows and rows without
incoming edges are all in the sample.
"""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from oracle import AGGR_MAX, AGGR_MEAN, AGGR_SUM, MSG_COPY_XJ, MSG_E_MUL_XJ
from paper_2412_06354_amd import synth
from util import assert_close_rel, assert_close_sabs, subgraph_for_rows

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def gnn():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2412_06354_amd import binding
    binding.lib()
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.cpu().numpy()


def sample_rows(dst, n, count, seed):
    """Random rows + the highest in-degree rows + some rows without incoming edges."""
    indeg = np.bincount(dst, minlength=n)
    rnd = synth.randint(seed, 9, 0, count, 0, n - 1)
    hubs = np.argsort(indeg)[-4:]
    empty = np.flatnonzero(indeg == 0)[:8]
    mid = np.flatnonzero((indeg > 400) & (indeg < 3000))[:16]
    return np.unique(np.concatenate([rnd, hubs, empty, mid])).astype(np.int64)


# ----------------------------------------------------------------------------- configuration 2

@pytest.fixture(scope="module")
def cfg2(gnn):
    say("config 2: generating 1M nodes / 20M edges")
    wl = synth.config2_weighted()
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), wl.num_nodes)
    say("config 2: graph built")
    yield wl, g
    g.close()


def test_config2_csr_bit_exact(cfg2):
    wl, g = cfg2
    rowptr, colidx, perm, indeg = oracle.build_csr(wl.src, wl.dst, wl.num_nodes)
    np.testing.assert_array_equal(host(g.indegree), indeg)
    np.testing.assert_array_equal(host(g.rowptr), rowptr)
    np.testing.assert_array_equal(host(g.perm), perm)
    np.testing.assert_array_equal(host(g.colidx), colidx)


@pytest.mark.parametrize("msg", [MSG_COPY_XJ, MSG_E_MUL_XJ])
def test_config2_propagate_sampled_rows(cfg2, gnn, msg):
    wl, g = cfg2
    n = wl.num_nodes
    rows = sample_rows(wl.dst, n, 3000, 21)
    s_src, s_dst, nodes, local_rows, eid = subgraph_for_rows(wl.src, wl.dst, rows)
    xs = wl.x[nodes]
    es = wl.edge_weight[eid] if msg == MSG_E_MUL_XJ else None
    x = dev(wl.x)
    e_csr = gnn.edge_data_to_csr(g, dev(wl.edge_weight)) if msg == MSG_E_MUL_XJ else None
    for aggr in (AGGR_SUM, AGGR_MEAN, AGGR_MAX):
        ref, sabs = oracle.propagate(s_src, s_dst, nodes.shape[0], xs, es, msg, aggr, with_sabs=True)
        got = host(gnn.propagate(g, x, e_csr, msg, aggr, e_order=gnn.EDGE_ORDER_CSR)[torch.from_numpy(rows).cuda()])
        if aggr == AGGR_MAX:
            np.testing.assert_array_equal(got.view(np.uint32), ref[local_rows].view(np.uint32))
        else:
            assert_close_sabs(got, ref[local_rows], sabs[local_rows], what=f"config2 msg={msg} aggr={aggr}")
        say(f"config 2: msg={msg} aggr={aggr} ok on {rows.shape[0]} sampled rows ({eid.shape[0]} edges)")


@pytest.mark.parametrize("msg,aggr", [(MSG_COPY_XJ, AGGR_SUM), (MSG_E_MUL_XJ, AGGR_SUM), (MSG_E_MUL_XJ, AGGR_MEAN),
                                      (MSG_E_MUL_XJ, AGGR_MAX)])
def test_config2_propagate_every_element(cfg2, gnn, msg, aggr):
    """All 1 M x 64 outputs of the headline launch (copy_xj + sum) and of the three weighted runs against the
    oracle's edge loop over the whole 20 M-edge list; edge weights in CSR order, as the benchmark times them."""
    wl, g = cfg2
    n = wl.num_nodes
    e = wl.edge_weight if msg == MSG_E_MUL_XJ else None
    say(f"config 2, every element: oracle msg={msg} aggr={aggr}")
    ref, sabs = oracle.propagate(wl.src, wl.dst, n, wl.x, e, msg, aggr, with_sabs=True)
    e_csr = gnn.edge_data_to_csr(g, dev(wl.edge_weight)) if msg == MSG_E_MUL_XJ else None
    got = host(gnn.propagate(g, dev(wl.x), e_csr, msg, aggr, e_order=gnn.EDGE_ORDER_CSR))
    if aggr == AGGR_MAX:
        np.testing.assert_array_equal(got.view(np.uint32), ref.view(np.uint32))
    else:
        assert_close_sabs(got, ref, sabs, what=f"config2 whole graph msg={msg} aggr={aggr}")
    say(f"config 2, every element: msg={msg} aggr={aggr} ok on {n} x {got.shape[1]} outputs")


def test_config2_invariants_at_full_size(cfg2, gnn):
    wl, g = cfg2
    n = wl.num_nodes
    indeg = np.bincount(wl.dst, minlength=n)
    ones = torch.ones((n, 64), dtype=torch.float32, device="cuda")
    out = gnn.propagate(g, ones)
    np.testing.assert_array_equal(host(out[:, 0]), indeg.astype(np.float32))      # exact: integers < 2^24
    np.testing.assert_array_equal(host(out[:, 63]), indeg.astype(np.float32))
    mx = gnn.propagate(g, ones * 2.5, None, MSG_COPY_XJ, AGGR_MAX)
    np.testing.assert_array_equal(host(mx[:, 7]), np.where(indeg > 0, 2.5, 0.0).astype(np.float32))
    # unit weights reproduce copy_xj bit for bit
    x = dev(wl.x)
    w1 = torch.ones(wl.num_edges, dtype=torch.float32, device="cuda")
    a = gnn.propagate(g, x)
    b = gnn.propagate(g, x, w1, MSG_E_MUL_XJ, AGGR_SUM)
    assert torch.equal(a, b)


def test_config2_segment_softmax_sampled_rows(cfg2, gnn):
    wl, g = cfg2
    n, e, heads = wl.num_nodes, wl.num_edges, 8
    s = (3.0 * synth.normal_f32(55, 2, e * heads)).reshape(e, heads)
    got_all = gnn.segment_softmax(g, dev(s))
    rows = sample_rows(wl.dst, n, 3000, 22)
    s_src, s_dst, nodes, local_rows, eid = subgraph_for_rows(wl.src, wl.dst, rows)
    ref = oracle.segment_softmax(s_dst, nodes.shape[0], s[eid])
    got = host(got_all[torch.from_numpy(eid).cuda()])
    assert_close_rel(got, ref, what="config2 segment softmax")


def test_config2_edge_route_every_element(cfg2, gnn):
    """The two-pass route for one float per edge at the full size: all 20 M weights land where e[perm] (perm from
    the oracle) says, the way back restores them, and propagate with COO-ordered weights through the route equals
    the CSR-ordered call bit for bit.  Runs last of the configuration-2 tests: it adds the route to the shared graph."""
    wl, g = cfg2
    _, _, perm, _ = oracle.build_csr(wl.src, wl.dst, wl.num_nodes)
    e = np.ascontiguousarray(wl.edge_weight, dtype=np.float32).reshape(-1)
    e_d, x = dev(e), dev(wl.x)
    before = gnn.propagate(g, x, e_d, MSG_E_MUL_XJ, AGGR_SUM)
    g.build_edge_route()
    e_csr = gnn.edge_data_to_csr(g, e_d)
    np.testing.assert_array_equal(host(e_csr), e[perm])
    np.testing.assert_array_equal(host(gnn.edge_data_to_coo(g, e_csr)), e)
    after = gnn.propagate(g, x, e_d, MSG_E_MUL_XJ, AGGR_SUM)
    assert torch.equal(after, before)
    from paper_2412_06354_amd.binding import EDGE_ORDER_CSR
    assert torch.equal(gnn.propagate(g, x, e_csr, MSG_E_MUL_XJ, AGGR_SUM, e_order=EDGE_ORDER_CSR), before)


# ----------------------------------------------------------------------------- configuration 1

def test_config1_gcnconv_full(gnn):
    say("config 1: generating 100k nodes / 1M edges")
    wl = synth.config1_gcn()
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), wl.num_nodes)
    rowptr, colidx, perm, _ = oracle.build_csr(wl.src, wl.dst, wl.num_nodes)
    np.testing.assert_array_equal(host(g.rowptr), rowptr)
    np.testing.assert_array_equal(host(g.perm), perm)
    w, b = wl.params["w"], wl.params["bias"]
    ref, sabs = oracle.gcnconv(wl.src, wl.dst, wl.num_nodes, wl.x, w, b, True, with_sabs=True)
    got = host(gnn.gcnconv(g, dev(wl.x), dev(w), dev(b), True))
    assert_close_sabs(got, ref, sabs, what="config1 gcnconv")
    g.close()


# ----------------------------------------------------------------------------- configuration 4

def test_config4_gatconv_sampled_rows(gnn):
    say("config 4: generating 2.45M nodes / 126M edges (about a minute)")
    wl = synth.config4_gat()
    p = wl.params
    n = wl.num_nodes
    say("config 4: building CSR on the GPU")
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), n)
    indeg = np.bincount(wl.dst, minlength=n)
    np.testing.assert_array_equal(host(g.indegree), indeg)
    rp = host(g.rowptr)
    assert rp[0] == 0 and rp[-1] == wl.num_edges
    np.testing.assert_array_equal(np.diff(rp), indeg)
    say("config 4: running the layer")
    out = gnn.gatconv(g, dev(wl.x), dev(p["w"]), dev(p["a_src"]), dev(p["a_dst"]), p["negative_slope"])
    torch.cuda.synchronize()
    rows = sample_rows(wl.dst, n, 400, 23)
    s_src, s_dst, nodes, local_rows, eid = subgraph_for_rows(wl.src, wl.dst, rows)
    say(f"config 4: oracle on {rows.shape[0]} sampled rows, {eid.shape[0]} edges, {nodes.shape[0]} nodes")
    # CSR order of the sampled rows: stable by original edge id
    perm = host(g.perm)
    colidx = host(g.colidx)
    for r in rows[:50]:
        seg = perm[rp[r]:rp[r + 1]]
        assert (np.diff(seg) > 0).all() and (wl.dst[seg] == r).all()
        np.testing.assert_array_equal(colidx[rp[r]:rp[r + 1]], wl.src[seg])
    ref, sabs = oracle.gatconv(s_src, s_dst, nodes.shape[0], wl.x[nodes], p["w"], p["a_src"], p["a_dst"],
                               p["negative_slope"], with_sabs=True)
    got = host(out[torch.from_numpy(rows).cuda()])
    assert_close_sabs(got, ref[local_rows], sabs[local_rows], what="config4 gatconv")

    # backward at the same size: grad_x of sampled source nodes.  Such a row needs the node's own
    # incoming edges and, for every edge it sends, the whole neighbourhood of that edge's destination.
    say("config 4: backward")
    hc = p["heads"] * p["ch"]
    gt = gnn.build_csr(dev(wl.dst), dev(wl.src), n)
    stats = torch.empty((n, p["heads"], 2), dtype=torch.float32, device="cuda")
    args = (dev(wl.x), dev(p["w"]), dev(p["a_src"]), dev(p["a_dst"]))
    out = gnn.gatconv(g, *args, p["negative_slope"], softmax_stats=stats)
    gout = synth.normal_f32(53, 7, n * hc).reshape(n, hc)
    gx, gw, gas, gad = gnn.gatconv_backward(g, gt, *args, out, stats, dev(gout), p["negative_slope"])
    torch.cuda.synchronize()
    assert all(bool(torch.isfinite(t).all()) for t in (gx, gw, gas, gad))
    # candidates: random nodes whose destinations' neighbourhoods total at most 30 000 edges (about a
    # third of all nodes; the oracle runs on everything those neighbourhoods touch), the first 12 of them
    pool = np.unique(synth.randint(29, 9, 0, 600, 0, n - 1)).astype(np.int64)
    lut = np.zeros(n, dtype=bool)
    lut[pool] = True
    pool_edges = np.flatnonzero(lut[wl.src])
    cost = np.zeros(n, dtype=np.int64)
    np.add.at(cost, wl.src[pool_edges], indeg[wl.dst[pool_edges]])
    cand = pool[(cost[pool] > 0) & (cost[pool] <= 30_000)][:12]
    lut[:] = False
    lut[cand] = True
    out_edges = np.flatnonzero(lut[wl.src])
    rows_b = np.unique(np.concatenate([cand, wl.dst[out_edges]]))
    b_src, b_dst, b_nodes, b_local, b_eid = subgraph_for_rows(wl.src, wl.dst, rows_b)
    say(f"config 4: backward oracle on {cand.shape[0]} sampled nodes: {b_eid.shape[0]} edges, {b_nodes.shape[0]} nodes")
    # leave out sampled nodes with an incident edge whose pre-activation is within rounding of the
    # leaky ReLU's kink (float and double may take different slopes there)
    h64 = (wl.x[b_nodes].astype(np.float64) @ p["w"].astype(np.float64)).reshape(-1, p["heads"], p["ch"])
    nl, nr = (h64 * p["a_src"][None]).sum(-1), (h64 * p["a_dst"][None]).sum(-1)
    near = np.abs(nl[b_src] + nr[b_dst]).min(axis=1) < 1e-5
    cand_local = np.searchsorted(b_nodes, cand)
    touched = np.zeros(b_nodes.shape[0], dtype=bool)
    touched[b_src[near]] = True
    touched[b_dst[near]] = True
    ok = ~touched[cand_local]
    assert ok.sum() >= 8
    ref_b = oracle.gatconv_backward(b_src, b_dst, b_nodes.shape[0], wl.x[b_nodes], p["w"], p["a_src"], p["a_dst"],
                                    gout[b_nodes], p["negative_slope"])
    got_b = host(gx[torch.from_numpy(cand[ok]).cuda()])
    assert_close_sabs(got_b, ref_b["grad_x"][cand_local[ok]], ref_b["sabs_x"][cand_local[ok]],
                      what="config4 gatconv backward grad_x")
    g.close()
    gt.close()


def test_gatconv_backward_mid_size_all_gradients(gnn):
    """All four gradients against the oracle on the whole graph, at a size where the row-chunked
    reductions use their maximum number of chunks and the default thresholds apply."""
    say("GAT backward, 100k nodes / 2M edges: generating")
    wl = synth.config4_gat(num_nodes=100_000, num_edges=2_000_000, cap=5000.0)
    p, n = wl.params, wl.num_nodes
    hc = p["heads"] * p["ch"]
    h64 = (wl.x.astype(np.float64) @ p["w"].astype(np.float64)).reshape(n, p["heads"], p["ch"])
    nl, nr = (h64 * p["a_src"][None]).sum(-1), (h64 * p["a_dst"][None]).sum(-1)
    keep = np.abs(nl[wl.src] + nr[wl.dst]).min(axis=1) > 1e-5     # see test_gatconv_backward in test_gpu_parity
    src, dst = wl.src[keep], wl.dst[keep]
    gout = synth.normal_f32(59, 7, n * hc).reshape(n, hc)
    g, gt = gnn.build_csr(dev(src), dev(dst), n), gnn.build_csr(dev(dst), dev(src), n)
    stats = torch.empty((n, p["heads"], 2), dtype=torch.float32, device="cuda")
    args = (dev(wl.x), dev(p["w"]), dev(p["a_src"]), dev(p["a_dst"]))
    out = gnn.gatconv(g, *args, p["negative_slope"], softmax_stats=stats)
    gx, gw, gas, gad = gnn.gatconv_backward(g, gt, *args, out, stats, dev(gout), p["negative_slope"])
    say("GAT backward: oracle")
    ref = oracle.gatconv_backward(src, dst, n, wl.x, p["w"], p["a_src"], p["a_dst"], gout, p["negative_slope"])
    assert_close_sabs(host(gx), ref["grad_x"], ref["sabs_x"], what="gat grad_x")
    assert_close_sabs(host(gw), ref["grad_w"], ref["sabs_w"], what="gat grad_w")
    assert_close_sabs(host(gas), ref["grad_a_src"], ref["sabs_a_src"], what="gat grad_a_src")
    assert_close_sabs(host(gad), ref["grad_a_dst"], ref["sabs_a_dst"], what="gat grad_a_dst")
    g.close()
    gt.close()


# ----------------------------------------------------------------------------- offsets beyond 2^31 elements

def test_element_offsets_beyond_2_to_31(gnn):
    """Feature and message arrays of more than 2^31 elements: N x F = 5 M x 512 (2.56 G floats) for the node side,
    E x F = 6 M x 512 (3.07 G floats) for the materialised messages.  A 32-bit element offset anywhere in the kernels
    would wrap in the upper half of these arrays; the sampled rows and edges are taken from both halves.  Features are
    a closed-form pattern (multiples of 1/64, exact in float) filled in on the device and recomputed on the host for
    the sampled rows only."""
    n, f, e = 5_000_000, 512, 6_000_000
    src = synth.randint(77, 1, 0, e, 0, n - 1).astype(np.int32)
    dst = synth.randint(77, 2, 0, e, 0, n - 1).astype(np.int32)

    def pattern(rows):   # x[i, c] = (((131 i + 7 c) mod 1001) - 500) / 64
        i = np.asarray(rows, np.int64).reshape(-1, 1)
        c = np.arange(f, dtype=np.int64).reshape(1, -1)
        return (((131 * i + 7 * c) % 1001 - 500) / 64.0).astype(np.float32)

    say("large offsets: filling 10 GB of features on the device")
    x = torch.empty((n, f), dtype=torch.float32, device="cuda")
    cols = torch.arange(f, dtype=torch.int64, device="cuda").reshape(1, -1)
    for r0 in range(0, n, 250_000):
        r1 = min(n, r0 + 250_000)
        i = torch.arange(r0, r1, dtype=torch.int64, device="cuda").reshape(-1, 1)
        x[r0:r1] = ((131 * i + 7 * cols) % 1001 - 500).to(torch.float32) / 64.0
    g = gnn.build_csr(dev(src), dev(dst), n)
    rows = np.unique(np.concatenate([synth.randint(77, 3, 0, 1500, 0, n - 1),
                                     synth.randint(77, 4, 0, 1500, n - n // 8, n - 1), [0, n - 1]])).astype(np.int64)
    s_src, s_dst, nodes, local_rows, eid = subgraph_for_rows(src, dst, rows)
    xs = pattern(nodes)
    rows_d = torch.from_numpy(rows).cuda()
    for aggr in (AGGR_SUM, AGGR_MAX):
        out = gnn.propagate(g, x, None, MSG_COPY_XJ, aggr)
        ref, sabs = oracle.propagate(s_src, s_dst, nodes.shape[0], xs, None, MSG_COPY_XJ, aggr, with_sabs=True)
        got = host(out[rows_d])
        if aggr == AGGR_MAX:
            np.testing.assert_array_equal(got.view(np.uint32), ref[local_rows].view(np.uint32))
        else:
            assert_close_sabs(got, ref[local_rows], sabs[local_rows], what="large offsets, sum")
        say(f"large offsets: propagate aggr={aggr} ok on {rows.shape[0]} rows")
    del out
    # materialised messages, 12 GB: message k is the source's row, bit for bit; reduced again they give the fused result
    m = gnn.apply_edges(g, x, None, MSG_COPY_XJ)
    ks = np.unique(np.concatenate([synth.randint(77, 5, 0, 2000, 0, e - 1),
                                   synth.randint(77, 6, 0, 2000, e - e // 8, e - 1), [0, e - 1]])).astype(np.int64)
    np.testing.assert_array_equal(host(m[torch.from_numpy(ks).cuda()]).view(np.uint32), pattern(src[ks]).view(np.uint32))
    again = gnn.aggregate_neighbors(g, m, AGGR_SUM)
    ref, sabs = oracle.propagate(s_src, s_dst, nodes.shape[0], xs, None, MSG_COPY_XJ, AGGR_SUM, with_sabs=True)
    assert_close_sabs(host(again[rows_d]), ref[local_rows], sabs[local_rows], what="large offsets, aggregate_neighbors")
    say("large offsets: apply_edges / aggregate_neighbors ok")
    g.close()
