"""GPU tests of the boundary itself: which calls allocate, the reservation of a graph's scratch memory, the
plain gnn_build_csr entry point, the batch build of temporal snapshots and the graph_indicator check.
All calls go through the C ABI; expected values come from the CPU oracle."""
import ctypes

import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from oracle import AGGR_MAX, AGGR_MEAN, AGGR_SUM, MSG_COPY_XJ, MSG_E_MUL_XJ
from paper_2412_06354_amd import synth
from util import assert_close_rel, assert_close_sabs

pytestmark = pytest.mark.gpu

ERR_INDEX_RANGE, ERR_NOT_SORTED, ERR_NOT_RESERVED = 3, 7, 8


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


def split_row_graph():
    """Power-law graph whose hub rows are cut into several wavefront pieces under the default thresholds."""
    return synth.config2_weighted(num_nodes=20_000, num_edges=300_000, feat=64, cap=6000.0)


def test_build_csr_entry_point_itself(gnn):
    """gnn_build_csr called directly through ctypes (not the variant with thresholds): CSR bit for bit."""
    wl = split_row_graph()
    src, dst = dev(wl.src), dev(wl.dst)
    lib = gnn.lib()
    out = ctypes.c_void_p()
    rc = lib.gnn_build_csr(src.data_ptr(), dst.data_ptr(), wl.num_edges, wl.num_nodes,
                           torch.cuda.current_stream().cuda_stream, ctypes.byref(out))
    assert rc == 0 and out.value
    g = gnn.Graph(out.value, src.device)
    rowptr, colidx, perm, indeg = oracle.build_csr(wl.src, wl.dst, wl.num_nodes)
    np.testing.assert_array_equal(host(g.rowptr), rowptr)
    np.testing.assert_array_equal(host(g.colidx), colidx)
    np.testing.assert_array_equal(host(g.perm), perm)
    np.testing.assert_array_equal(host(g.indegree), indeg)
    assert g.work_sizes()["split_rows"] > 0
    # the binding's default path is this very entry point
    g2 = gnn.build_csr(src, dst, wl.num_nodes)
    assert torch.equal(g2.perm, g.perm) and g2.work_sizes() == g.work_sizes()
    g.close()
    g2.close()


def test_first_propagate_can_be_captured(gnn):
    """Compute calls never allocate or synchronise: the FIRST propagate on a graph with split rows is recorded
    into a HIP graph (no warm-up call on this handle) and every replay reproduces the eager result."""
    wl = split_row_graph()
    n = wl.num_nodes
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), n)
    assert g.work_sizes()["split_rows"] > 0
    x, e = dev(wl.x), dev(wl.edge_weight)
    out = torch.empty((n, 64), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    gph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gph):
        gnn.propagate(g, x, e, MSG_E_MUL_XJ, AGGR_SUM, out=out)
    ref, sabs = oracle.propagate(wl.src, wl.dst, n, wl.x, wl.edge_weight, MSG_E_MUL_XJ, AGGR_SUM, with_sabs=True)
    first = None
    for it in range(4):
        out.fill_(float("nan"))
        gph.replay()
        torch.cuda.synchronize()
        got = host(out)
        assert_close_sabs(got, ref, sabs, what=f"captured propagate, replay {it}")
        if first is None:
            first = got.copy()
        assert np.array_equal(first.view(np.uint32), got.view(np.uint32))
        other = gnn.propagate(g, x, None, MSG_COPY_XJ, AGGR_MAX)     # eager work on the same handle between replays
        torch.cuda.synchronize()
        assert bool(torch.isfinite(other).all())
    eager = gnn.propagate(g, x, e, MSG_E_MUL_XJ, AGGR_SUM)
    assert np.array_equal(host(eager).view(np.uint32), first.view(np.uint32))
    del gph
    g.close()


def test_reservation_limits_and_reserve(gnn):
    """Beyond the sizes a fresh graph is reserved for, a compute call fails with GNN_ERR_NOT_RESERVED and
    launches nothing; after gnn_graph_reserve the same call matches the oracle."""
    lib, stream = gnn.lib(), torch.cuda.current_stream().cuda_stream
    # segment softmax: per-node statistics for 32 heads on 20 000 nodes exceed what the build set aside
    wl = split_row_graph()
    n, heads = wl.num_nodes, 32
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), n)
    assert 2 * n * heads > 3 * (2 * (wl.num_edges // 256) + 1) * 128, "the case must exceed the default reservation"
    s = (3.0 * synth.normal_f32(41, 2, wl.num_edges * heads)).reshape(wl.num_edges, heads)
    sd = dev(s)
    alpha = torch.full_like(sd, -7.0)
    rc = lib.gnn_segment_softmax(g._h, sd.data_ptr(), heads, 0, alpha.data_ptr(), stream)
    assert rc == ERR_NOT_RESERVED
    torch.cuda.synchronize()
    assert bool((alpha == -7.0).all())                          # nothing ran
    g.reserve(0, heads)
    rc = lib.gnn_segment_softmax(g._h, sd.data_ptr(), heads, 0, alpha.data_ptr(), stream)
    assert rc == 0
    ref = oracle.segment_softmax(wl.dst, n, s)
    assert_close_rel(host(alpha), ref, what="softmax after reserve")
    # a very wide propagate: the slots of this graph times 2 000 features exceed the default reservation
    wl2 = synth.config2_weighted(num_nodes=4000, num_edges=100_000, feat=8, cap=3000.0)
    n2 = wl2.num_nodes
    g2 = gnn.build_csr(dev(wl2.src), dev(wl2.dst), n2, 4, 64)      # many split rows
    f = 2000
    n_slots = int(g2.work_lists()["item_slot"].max()) + 1
    assert n_slots * f > 3 * (2 * (wl2.num_edges // 64) + 1) * 128, "the case must exceed the default reservation"
    xw = synth.normal_f32(41, 3, n2 * f).reshape(n2, f)
    xd = dev(xw)
    out = torch.full((n2, f), -7.0, dtype=torch.float32, device="cuda")
    rc = lib.gnn_propagate(g2._h, xd.data_ptr(), f, None, 1, 0, MSG_COPY_XJ, AGGR_SUM, out.data_ptr(), stream)
    assert rc == ERR_NOT_RESERVED
    torch.cuda.synchronize()
    assert bool((out == -7.0).all())
    g2.reserve(f, 0)
    got = host(gnn.propagate(g2, xd, None, MSG_COPY_XJ, AGGR_SUM, out=out))
    ref2, sabs2 = oracle.propagate(wl2.src, wl2.dst, n2, xw, None, MSG_COPY_XJ, AGGR_SUM, with_sabs=True)
    assert_close_sabs(got, ref2, sabs2, what="wide propagate after reserve")
    # reservations only grow: a smaller request afterwards changes nothing
    g.reserve(64, 1)
    rc = lib.gnn_segment_softmax(g._h, sd.data_ptr(), heads, 0, alpha.data_ptr(), stream)
    assert rc == 0
    assert_close_rel(host(alpha), ref, what="softmax after a smaller reserve")
    assert lib.gnn_graph_reserve(None, 1, 1) == 1 and lib.gnn_graph_reserve(g._h, -1, 0) == 2
    g.close()
    g2.close()


def test_batch_build_of_temporal_snapshots(gnn):
    """T snapshots over one node set: every handle equals the oracle's CSR of its snapshot bit for bit, has the
    work lists of a build on its own, and propagate per snapshot matches the oracle; handles are destroyed one
    by one in any order."""
    n, f = 6000, 32
    sizes = [90_000, 0, 25_000, 140_000, 1]
    snaps = []
    for t, e in enumerate(sizes):
        if e == 0:
            snaps.append((np.empty(0, np.int32), np.empty(0, np.int32)))
        else:
            snaps.append(synth.chung_lu_directed(n, e, 1.0, min(2500.0, max(4.0, e / 8.0)), 1000 + t))
    x = synth.normal_f32(77, 2, n * f).reshape(n, f)
    xd = dev(x)
    graphs = gnn.build_csr_batch([dev(s) for s, _ in snaps], [dev(d) for _, d in snaps], n)
    assert len(graphs) == len(sizes)
    assert any(g.work_sizes()["split_rows"] > 0 for g in graphs)
    for t, (g, (src, dst)) in enumerate(zip(graphs, snaps)):
        rowptr, colidx, perm, indeg = oracle.build_csr(src, dst, n)
        assert g.num_edges == sizes[t] and g.num_nodes == n
        np.testing.assert_array_equal(host(g.rowptr), rowptr, err_msg=f"snapshot {t}")
        np.testing.assert_array_equal(host(g.colidx), colidx, err_msg=f"snapshot {t}")
        np.testing.assert_array_equal(host(g.perm), perm, err_msg=f"snapshot {t}")
        np.testing.assert_array_equal(host(g.indegree), indeg, err_msg=f"snapshot {t}")
        alone = gnn.build_csr(dev(src), dev(dst), n)
        assert alone.work_sizes() == g.work_sizes()
        la, lb = alone.work_lists(), g.work_lists()
        assert all(torch.equal(la[k], lb[k]) for k in la)
        alone.close()
        e = synth.uniform_f32(78, t, max(sizes[t], 1))[:sizes[t]]
        for msg, aggr in ((MSG_COPY_XJ, AGGR_SUM), (MSG_E_MUL_XJ, AGGR_MEAN), (MSG_E_MUL_XJ, AGGR_MAX)):
            ref, sabs = oracle.propagate(src, dst, n, x, e if msg else None, msg, aggr, with_sabs=True)
            got = host(gnn.propagate(g, xd, dev(e) if msg else None, msg, aggr))
            if aggr == AGGR_MAX:
                np.testing.assert_array_equal(got.view(np.uint32), ref.view(np.uint32))
            else:
                assert_close_sabs(got, ref, sabs, what=f"snapshot {t} msg={msg} aggr={aggr}")
    # destroy out of order; the survivors stay valid until their own destroy
    graphs[3].close()
    graphs[0].close()
    ref = oracle.propagate(snaps[2][0], snaps[2][1], n, x, None, MSG_COPY_XJ, AGGR_MAX)
    np.testing.assert_array_equal(host(gnn.propagate(graphs[2], xd, None, MSG_COPY_XJ, AGGR_MAX)).view(np.uint32),
                                  ref.view(np.uint32))
    for g in graphs:
        g.close()
    # an out-of-range node id in any snapshot: no handle at all
    bad = snaps[2][1].copy()
    bad[17] = n
    with pytest.raises(gnn.GnnError) as err:
        gnn.build_csr_batch([dev(snaps[0][0]), dev(snaps[2][0])], [dev(snaps[0][1]), dev(bad)], n)
    assert err.value.code == ERR_INDEX_RANGE
    # host-side argument errors
    lib = gnn.lib()
    assert lib.gnn_build_csr_batch(0, None, None, None, n, None, None) == 1
    slots = (ctypes.c_void_p * 1)()
    assert lib.gnn_build_csr_batch(0, None, None, None, n, None, slots) == 2


def test_batch_build_of_many_small_snapshots(gnn):
    """Many small snapshots go through the same few launches (the snapshot is a grid dimension): CSR and work lists
    of every handle equal a build on its own.  A one-node graph takes the builds one after the other."""
    n = 700
    sizes = [int(v) for v in synth.randint(31, 6, 0, 37, 0, 3000)]
    sizes[5] = 0
    sizes[11] = 4096        # exactly one sort tile
    sizes[12] = 4097
    snaps = [synth.multigraph_uniform(n, e, seed=500 + t) if e else (np.empty(0, np.int32), np.empty(0, np.int32))
             for t, e in enumerate(sizes)]
    graphs = gnn.build_csr_batch([dev(s) for s, _ in snaps], [dev(d) for _, d in snaps], n)
    for t, (g, (src, dst)) in enumerate(zip(graphs, snaps)):
        rowptr, colidx, perm, indeg = oracle.build_csr(src, dst, n)
        np.testing.assert_array_equal(host(g.rowptr), rowptr, err_msg=f"snapshot {t}")
        np.testing.assert_array_equal(host(g.colidx), colidx, err_msg=f"snapshot {t}")
        np.testing.assert_array_equal(host(g.perm), perm, err_msg=f"snapshot {t}")
        np.testing.assert_array_equal(host(g.indegree), indeg, err_msg=f"snapshot {t}")
        alone = gnn.build_csr(dev(src), dev(dst), n)
        assert alone.work_sizes() == g.work_sizes()
        la, lb = alone.work_lists(), g.work_lists()
        assert all(torch.equal(la[k], lb[k]) for k in la)
        alone.close()
    for g in graphs:
        g.close()
    # one node: every edge is a self-loop
    loops = [np.zeros(e, np.int32) for e in (3, 0, 70)]
    graphs = gnn.build_csr_batch([dev(a) for a in loops], [dev(a) for a in loops], 1)
    for g, a in zip(graphs, loops):
        np.testing.assert_array_equal(host(g.rowptr), [0, a.shape[0]])
        np.testing.assert_array_equal(host(g.perm), np.arange(a.shape[0]))
        g.close()


def test_batch_and_single_builds_hand_their_arrays_on(gnn):
    """The arrays of a destroyed graph, or of a batch whose last handle is gone, serve the next build or batch of a
    similar size.  Whatever the block held before, every build equals the oracle's CSR and a fresh build's lists."""
    n = 3000
    snaps = [synth.chung_lu_directed(n, e, 1.0, 400.0, 900 + t) for t, e in enumerate((40_000, 35_000, 50_000))]
    whole = (np.concatenate([s for s, _ in snaps]), np.concatenate([d for _, d in snaps]))
    gnn.lib().gnn_release_cached_memory()
    fresh = [gnn.build_csr(dev(s), dev(d), n) for s, d in snaps]
    lists = [(g.work_sizes(), g.work_lists()) for g in fresh]
    for g in fresh:
        g.close()

    def check_batch(graphs):
        for t, (g, (src, dst)) in enumerate(zip(graphs, snaps)):
            rowptr, colidx, perm, _ = oracle.build_csr(src, dst, n)
            np.testing.assert_array_equal(host(g.rowptr), rowptr, err_msg=f"snapshot {t}")
            np.testing.assert_array_equal(host(g.colidx), colidx, err_msg=f"snapshot {t}")
            np.testing.assert_array_equal(host(g.perm), perm, err_msg=f"snapshot {t}")
            assert g.work_sizes() == lists[t][0]
            assert all(torch.equal(g.work_lists()[k], lists[t][1][k]) for k in lists[t][1])

    for _ in range(3):   # batch -> batch (the second and third take the block the previous one gave back)
        graphs = gnn.build_csr_batch([dev(s) for s, _ in snaps], [dev(d) for _, d in snaps], n)
        check_batch(graphs)
        for g in reversed(graphs):
            g.close()
    # batch -> single build of about the same total size -> batch
    g = gnn.build_csr(dev(whole[0]), dev(whole[1]), n)
    rowptr, colidx, perm, _ = oracle.build_csr(whole[0], whole[1], n)
    np.testing.assert_array_equal(host(g.rowptr), rowptr)
    np.testing.assert_array_equal(host(g.colidx), colidx)
    np.testing.assert_array_equal(host(g.perm), perm)
    g.close()
    graphs = gnn.build_csr_batch([dev(s) for s, _ in snaps], [dev(d) for _, d in snaps], n)
    check_batch(graphs)
    for g in graphs:
        g.close()
    assert gnn.lib().gnn_release_cached_memory() == 0


def test_batch_build_beyond_one_launch_group(gnn):
    """More snapshots than one launch takes in its second grid dimension (32 768): the batch is built in groups;
    handles on both sides of the group boundary, the first and the last equal the oracle's CSR."""
    n, t_snap, per = 5, 33_000, 3
    src_all, dst_all = synth.multigraph_uniform(n, t_snap * per, seed=77)
    src_d, dst_d = dev(src_all), dev(dst_all)
    srcs = [src_d[i * per:(i + 1) * per] for i in range(t_snap)]
    dsts = [dst_d[i * per:(i + 1) * per] for i in range(t_snap)]
    graphs = gnn.build_csr_batch(srcs, dsts, n)
    assert len(graphs) == t_snap
    for t in (0, 1, 32_766, 32_767, 32_768, 32_769, t_snap - 1):
        rowptr, colidx, perm, indeg = oracle.build_csr(src_all[t * per:(t + 1) * per], dst_all[t * per:(t + 1) * per], n)
        g = graphs[t]
        np.testing.assert_array_equal(host(g.rowptr), rowptr, err_msg=f"snapshot {t}")
        np.testing.assert_array_equal(host(g.colidx), colidx, err_msg=f"snapshot {t}")
        np.testing.assert_array_equal(host(g.perm), perm, err_msg=f"snapshot {t}")
        assert g.work_sizes()["small_rows"] == n
    for g in graphs:
        g.close()


def test_concurrent_builds_and_calls_from_two_threads(gnn):
    """Two host threads, each with its own stream, build graphs and run propagate at the same time: the buffer the
    builds share is handed to one build at a time (the other allocates its own temporaries), handles are
    independent, and every result equals the oracle's."""
    import threading
    n, f = 3000, 16
    work = []
    for t in range(2):
        src, dst = synth.chung_lu_directed(n, 60_000, 1.0, 900.0, 700 + t)
        x = synth.normal_f32(710 + t, 2, n * f).reshape(n, f)
        work.append((src, dst, x, oracle.build_csr(src, dst, n), oracle.propagate(src, dst, n, x, None, MSG_COPY_XJ, AGGR_MAX)))
    errors = []

    def body(t):
        try:
            src, dst, x, (rowptr, colidx, perm, _), ref = work[t]
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                sd, dd, xd = dev(src), dev(dst), dev(x)
                for _ in range(15):
                    g = gnn.build_csr(sd, dd, n)
                    out = gnn.propagate(g, xd, None, MSG_COPY_XJ, AGGR_MAX)
                    stream.synchronize()
                    assert np.array_equal(host(g.rowptr), rowptr) and np.array_equal(host(g.colidx), colidx)
                    assert np.array_equal(host(g.perm), perm)
                    assert np.array_equal(host(out).view(np.uint32), ref.view(np.uint32))
                    g.close()
        except Exception as exc:   # reported by the main thread
            errors.append((t, repr(exc)))

    threads = [threading.Thread(target=body, args=(t,)) for t in range(2)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors


def test_check_graph_indicator(gnn):
    wl = synth.config3_batched(num_graphs=200, feat=4)
    gi = wl.graph_indicator
    gnn.check_graph_indicator(dev(gi), wl.num_graphs)
    swapped = gi.copy()
    k = int(np.flatnonzero(np.diff(gi) > 0)[3])
    swapped[k], swapped[k + 1] = swapped[k + 1], swapped[k]
    with pytest.raises(gnn.GnnError) as err:
        gnn.check_graph_indicator(dev(swapped), wl.num_graphs)
    assert err.value.code == ERR_NOT_SORTED
    with pytest.raises(gnn.GnnError) as err:
        gnn.check_graph_indicator(dev(gi), wl.num_graphs - 1)
    assert err.value.code == ERR_INDEX_RANGE
    neg = gi.copy()
    neg[0] = -1
    with pytest.raises(gnn.GnnError) as err:
        gnn.check_graph_indicator(dev(neg), wl.num_graphs)
    assert err.value.code == ERR_INDEX_RANGE
