"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element,
on the same seeded inputs.  Integer / index work and max are compared bit for bit; sums, means,
softmax and the layers within 1e-5 (see util.assert_close_sabs)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from oracle import (AGGR_MAX, AGGR_MEAN, AGGR_MIN, AGGR_PROD, AGGR_SUM, MSG_COPY_XJ, MSG_E_MUL_XJ, MSG_XI_DOT_XJ,
                    MSG_XJ_SUB_XI)
from paper_2412_06354_amd import synth
from util import assert_close_rel, assert_close_sabs, load_golden

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gnn():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2412_06354_amd import binding
    binding.lib()   # fails loudly if the library has not been built
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.cpu().numpy()


def powerlaw(n, e, feat, cap):
    return synth.config2_weighted(num_nodes=n, num_edges=e, feat=feat, cap=cap)


GRAPHS = {
    # name: (builder, small_max, chunk)  -- thresholds chosen so every work-list kind appears
    "tiny": (lambda: synth.config0_tiny(), 0, 0),
    "powerlaw_default": (lambda: powerlaw(20_000, 300_000, 64, 6000.0), 0, 0),
    "powerlaw_split64": (lambda: powerlaw(5_000, 120_000, 64, 3000.0), 4, 64),
    "uniform_multi": (lambda: synth.Workload("u", 3000, *synth.multigraph_uniform(3000, 50_000, 77),
                                             synth.normal_f32(77, 2, 3000 * 64).reshape(3000, 64),
                                             edge_weight=synth.uniform_f32(77, 3, 50_000)), 16, 128),
}


@pytest.fixture(scope="module", params=list(GRAPHS))
def case(request, gnn):
    build, small_max, chunk = GRAPHS[request.param]
    wl = build()
    if wl.edge_weight is None:
        wl.edge_weight = synth.uniform_f32(5, 3, wl.num_edges)
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), wl.num_nodes, small_max, chunk)
    yield request.param, wl, g
    g.close()


# ----------------------------------------------------------------------------- CSR build

def test_csr_bit_exact(case, gnn):
    name, wl, g = case
    rowptr, colidx, perm, indeg = oracle.build_csr(wl.src, wl.dst, wl.num_nodes)
    np.testing.assert_array_equal(host(g.indegree), indeg)
    np.testing.assert_array_equal(host(g.rowptr), rowptr)
    np.testing.assert_array_equal(host(g.perm), perm)
    np.testing.assert_array_equal(host(g.colidx), colidx)
    sizes = g.work_sizes()
    if name == "powerlaw_split64":
        assert sizes["split_rows"] > 0 and sizes["items"] > sizes["split_rows"] and sizes["small_rows"] > 0


def test_csr_hand_worked_and_edge_cases(gnn, golden_dir):
    gd = load_golden(golden_dir, "g5_propagate.json")
    src, dst = np.array(gd["src"], np.int32), np.array(gd["dst"], np.int32)
    g = gnn.build_csr(dev(src), dev(dst), 4)
    assert host(g.rowptr).tolist() == gd["rowptr"]
    assert host(g.colidx).tolist() == gd["colidx"]
    assert host(g.perm).tolist() == gd["perm"]
    assert host(g.indegree).tolist() == gd["indeg"]
    x = dev(np.array(gd["x"], np.float32))
    w = dev(np.array(gd["w"], np.float32))
    for msg_name, msg in (("copy_xj", MSG_COPY_XJ), ("e_mul_xj", MSG_E_MUL_XJ)):
        for aggr_name, aggr in (("sum", AGGR_SUM), ("mean", AGGR_MEAN), ("max", AGGR_MAX)):
            out = gnn.propagate(g, x, w if msg else None, msg, aggr)
            want = np.array(gd[msg_name][aggr_name], np.float64).astype(np.float32)
            if aggr == AGGR_MAX:   # bit for bit
                np.testing.assert_array_equal(host(out).view(np.uint32), want.view(np.uint32), err_msg=f"{msg_name} max")
            else:
                np.testing.assert_allclose(host(out), want, rtol=1e-6, atol=0, err_msg=f"{msg_name} {aggr_name}")
    g.close()
    # no edges at all
    empty = torch.empty(0, dtype=torch.int32, device="cuda")
    g0 = gnn.build_csr(empty, empty, 5)
    assert host(g0.rowptr).tolist() == [0] * 6
    xx = dev(np.ones((5, 8), np.float32))
    for aggr in (AGGR_SUM, AGGR_MEAN, AGGR_MAX):
        assert (host(gnn.propagate(g0, xx, None, MSG_COPY_XJ, aggr)) == 0).all()
    g0.close()
    # one node, only self-loops
    s1 = dev(np.zeros(70, np.int32))
    g1 = gnn.build_csr(s1, s1, 1)
    assert host(g1.rowptr).tolist() == [0, 70]
    assert host(g1.perm).tolist() == list(range(70))
    assert host(gnn.propagate(g1, dev(np.full((1, 4), 2.0, np.float32))))[0].tolist() == [140.0] * 4
    g1.close()


def expected_work_lists(rowptr, small_max, chunk):
    """The degree-bucketed schedule as gnn.h states it, written out row by row."""
    small, item_row, item_start, item_slot, split_rows, split_slot0 = [], [], [], [], [], []
    slots = 0
    for r in range(len(rowptr) - 1):
        start, deg = int(rowptr[r]), int(rowptr[r + 1] - rowptr[r])
        if deg <= small_max:
            small.append(r)
            continue
        pieces = -(-deg // chunk)
        if pieces > 1:
            split_rows.append(r)
            split_slot0.append(slots)
        for c in range(pieces):
            item_row.append(r)
            item_start.append(start + c * chunk)
            item_slot.append(slots + c if pieces > 1 else -1)
        if pieces > 1:
            slots += pieces
    return {"small_rows": small, "item_row": item_row, "item_start": item_start, "item_slot": item_slot,
            "split_rows": split_rows, "split_slot0": split_slot0}


@pytest.mark.parametrize("n,e,small_max,chunk", [(20_000, 300_000, 16, 256), (5000, 120_000, 4, 64), (3000, 50_000, 0, 64),
                                                 (1, 700, 8, 128), (2500, 0, 16, 256), (4097, 30_000, 64, 65536)])
def test_work_lists(gnn, n, e, small_max, chunk):
    """Every entry of the work lists against the schedule computed on the host from the oracle's row pointers
    (several list-kernel blocks, a ragged last block, one-node, edge-free and all-short graphs)."""
    if e == 0:
        src = dst = np.zeros(0, np.int32)
    elif n == 1:
        src = dst = np.zeros(e, np.int32)
    else:
        wl = powerlaw(n, e, 4, max(50.0, e / 40.0))
        src, dst = wl.src, wl.dst
    g = gnn.build_csr(dev(src), dev(dst), n, small_max, chunk)
    rowptr, _, _, _ = oracle.build_csr(src, dst, n)
    want = expected_work_lists(rowptr, small_max, chunk)
    got = g.work_lists()
    sizes = g.work_sizes()
    assert sizes == {"small_rows": len(want["small_rows"]), "items": len(want["item_row"]),
                     "split_rows": len(want["split_rows"])}
    for name, ref in want.items():
        np.testing.assert_array_equal(host(got[name]), np.array(ref, np.int32), err_msg=name)
    g.close()


def test_build_after_destroy_reuses_arrays(gnn):
    """A destroyed graph's device arrays are handed to the next build of a similar size: builds of a larger, a
    slightly smaller, an empty and a much smaller graph in a row, each destroyed before the next, all bit-exact;
    then the cache is released and a build allocates again."""
    cases = [powerlaw(6000, 90_000, 4, 2000.0), powerlaw(5000, 70_000, 4, 2000.0),
             synth.Workload("empty", 5000, np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros((5000, 4), np.float32)),
             powerlaw(300, 2000, 4, 100.0), powerlaw(6000, 90_000, 4, 2000.0)]
    for step, wl in enumerate(cases):
        if step == 4:
            gnn.release_cached_memory()
        g = gnn.build_csr(dev(wl.src), dev(wl.dst), wl.num_nodes)
        rowptr, colidx, perm, indeg = oracle.build_csr(wl.src, wl.dst, wl.num_nodes)
        np.testing.assert_array_equal(host(g.rowptr), rowptr)
        np.testing.assert_array_equal(host(g.indegree), indeg)
        np.testing.assert_array_equal(host(g.perm), perm)
        np.testing.assert_array_equal(host(g.colidx), colidx)
        x = dev(wl.x)
        ref = oracle.propagate(wl.src, wl.dst, wl.num_nodes, wl.x, None, MSG_COPY_XJ, AGGR_MAX)
        np.testing.assert_array_equal(host(gnn.propagate(g, x, None, MSG_COPY_XJ, AGGR_MAX)).view(np.uint32),
                                      ref.view(np.uint32))
        g.close()
    gnn.release_cached_memory()


def test_csr_rejects_out_of_range(gnn):
    src = dev(np.array([0, 1, 7], np.int32))
    dst = dev(np.array([1, 2, 0], np.int32))
    with pytest.raises(gnn.GnnError) as ei:
        gnn.build_csr(src, dst, 3)
    assert ei.value.code == 3
    with pytest.raises(gnn.GnnError):
        gnn.build_csr(dst, dev(np.array([0, -1, 2], np.int32)), 3)


def test_edge_data_to_csr(case, gnn):
    _, wl, g = case
    _, _, perm, _ = oracle.build_csr(wl.src, wl.dst, wl.num_nodes)
    got = host(gnn.edge_data_to_csr(g, dev(wl.edge_weight)))
    np.testing.assert_array_equal(got, wl.edge_weight[perm])
    e3 = synth.normal_f32(9, 3, wl.num_edges * 3).reshape(wl.num_edges, 3)
    np.testing.assert_array_equal(host(gnn.edge_data_to_csr(g, dev(e3))), e3[perm])


# ----------------------------------------------------------------------------- propagate

@pytest.mark.parametrize("msg", [MSG_COPY_XJ, MSG_E_MUL_XJ])
@pytest.mark.parametrize("aggr", [AGGR_SUM, AGGR_MEAN, AGGR_MAX])
def test_propagate_f64(case, gnn, msg, aggr):
    name, wl, g = case
    e = wl.edge_weight if msg == MSG_E_MUL_XJ else None
    ref, sabs = oracle.propagate(wl.src, wl.dst, wl.num_nodes, wl.x, e, msg, aggr, with_sabs=True)
    x = dev(wl.x)
    got = host(gnn.propagate(g, x, dev(e) if e is not None else None, msg, aggr))
    if aggr == AGGR_MAX:
        np.testing.assert_array_equal(got.view(np.uint32), ref.view(np.uint32))
    else:
        assert_close_sabs(got, ref, sabs, what=f"{name} msg={msg} aggr={aggr}")
    if msg == MSG_E_MUL_XJ:   # edge data already in CSR order gives the same bits
        e_csr = gnn.edge_data_to_csr(g, dev(e))
        got2 = host(gnn.propagate(g, x, e_csr, msg, aggr, e_order=gnn.EDGE_ORDER_CSR))
        np.testing.assert_array_equal(got2.view(np.uint32), got.view(np.uint32))
    # run-to-run determinism (no atomics on the path)
    again = host(gnn.propagate(g, x, dev(e) if e is not None else None, msg, aggr))
    np.testing.assert_array_equal(again.view(np.uint32), got.view(np.uint32))


@pytest.mark.parametrize("feat", [4, 7, 12, 16, 32, 100, 128, 260, 515])
def test_propagate_feature_widths(gnn, feat):
    wl = powerlaw(4000, 60_000, feat, 2500.0)
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), wl.num_nodes, 8, 128)
    x = dev(wl.x)
    for msg, e in ((MSG_COPY_XJ, None), (MSG_E_MUL_XJ, wl.edge_weight)):
        for aggr in (AGGR_SUM, AGGR_MEAN, AGGR_MAX):
            ref, sabs = oracle.propagate(wl.src, wl.dst, wl.num_nodes, wl.x, e, msg, aggr, with_sabs=True)
            got = host(gnn.propagate(g, x, dev(e) if e is not None else None, msg, aggr))
            if aggr == AGGR_MAX:
                np.testing.assert_array_equal(got.view(np.uint32), ref.view(np.uint32))
            else:
                assert_close_sabs(got, ref, sabs, what=f"F={feat} msg={msg} aggr={aggr}")
    g.close()


@pytest.mark.parametrize("feat", [8, 64, 6])
def test_propagate_elementwise_edge_features(gnn, feat):
    wl = powerlaw(3000, 40_000, feat, 1500.0)
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), wl.num_nodes, 8, 64)
    ef = synth.normal_f32(13, 3, wl.num_edges * feat).reshape(wl.num_edges, feat)
    for aggr in (AGGR_SUM, AGGR_MEAN, AGGR_MAX):
        ref, sabs = oracle.propagate(wl.src, wl.dst, wl.num_nodes, wl.x, ef, MSG_E_MUL_XJ, aggr, with_sabs=True)
        got = host(gnn.propagate(g, dev(wl.x), dev(ef), MSG_E_MUL_XJ, aggr))
        if aggr == AGGR_MAX:
            np.testing.assert_array_equal(got.view(np.uint32), ref.view(np.uint32))
        else:
            assert_close_sabs(got, ref, sabs, what=f"elementwise F={feat} aggr={aggr}")
        got_csr = host(gnn.propagate(g, dev(wl.x), gnn.edge_data_to_csr(g, dev(ef)), MSG_E_MUL_XJ, aggr,
                                     e_order=gnn.EDGE_ORDER_CSR))
        np.testing.assert_array_equal(got_csr.view(np.uint32), got.view(np.uint32))
    g.close()


@pytest.mark.parametrize("msg", [MSG_COPY_XJ, MSG_E_MUL_XJ])
def test_apply_edges_then_aggregate(case, gnn, msg):
    name, wl, g = case
    n = wl.num_nodes
    e = wl.edge_weight if msg == MSG_E_MUL_XJ else None
    x = dev(wl.x)
    m_ref = oracle.apply_edges(wl.src, n, wl.x, e, msg)
    m = gnn.apply_edges(g, x, dev(e) if e is not None else None, msg)
    np.testing.assert_array_equal(host(m).view(np.uint32), m_ref.view(np.uint32))      # gather / one rounded product
    _, _, perm, _ = oracle.build_csr(wl.src, wl.dst, n)
    m_csr = gnn.apply_edges(g, x, dev(e) if e is not None else None, msg, m_order=gnn.EDGE_ORDER_CSR)
    np.testing.assert_array_equal(host(m_csr).view(np.uint32), m_ref[perm].view(np.uint32))
    for aggr in (AGGR_SUM, AGGR_MEAN, AGGR_MAX):
        ref, sabs = oracle.aggregate_neighbors(wl.dst, n, m_ref, aggr, with_sabs=True)
        got = host(gnn.aggregate_neighbors(g, m, aggr))
        got_csr = host(gnn.aggregate_neighbors(g, m_csr, aggr, m_order=gnn.EDGE_ORDER_CSR))
        np.testing.assert_array_equal(got.view(np.uint32), got_csr.view(np.uint32))
        if aggr == AGGR_MAX:
            np.testing.assert_array_equal(got.view(np.uint32), ref.view(np.uint32))
        else:
            assert_close_sabs(got, ref, sabs, what=f"{name} aggregate msg={msg} aggr={aggr}")
        if msg == MSG_COPY_XJ or aggr == AGGR_MAX:
            # the fused call walks the same rows in the same order: identical bits
            fused = host(gnn.propagate(g, x, dev(e) if e is not None else None, msg, aggr))
            np.testing.assert_array_equal(got.view(np.uint32), fused.view(np.uint32))


@pytest.mark.parametrize("msg", [MSG_COPY_XJ, MSG_E_MUL_XJ, MSG_XJ_SUB_XI])
def test_propagate_min_prod_and_target_message(case, gnn, msg):
    """min is compared bit for bit (like max); prod within one rounding per factor; x_j - x_i under
    every reduction; the two-step path (apply_edges, aggregate_neighbors) gives the fused result."""
    name, wl, g = case
    n = wl.num_nodes
    e = wl.edge_weight if msg == MSG_E_MUL_XJ else None
    de = dev(e) if e is not None else None
    x = dev(wl.x)
    ref_min = oracle.propagate(wl.src, wl.dst, n, wl.x, e, msg, AGGR_MIN)
    got_min = host(gnn.propagate(g, x, de, msg, AGGR_MIN))
    np.testing.assert_array_equal(got_min.view(np.uint32), ref_min.view(np.uint32))
    m = gnn.apply_edges(g, x, de, msg)
    m_ref = oracle.apply_edges(wl.src, n, wl.x, e, msg, dst=wl.dst)
    np.testing.assert_array_equal(host(m).view(np.uint32), m_ref.view(np.uint32))
    two_step = host(gnn.aggregate_neighbors(g, m, AGGR_MIN))
    np.testing.assert_array_equal(two_step.view(np.uint32), ref_min.view(np.uint32))
    # products: factors close to +-1 so that thousands of them stay in range
    xp = (1.0 + 1e-3 * wl.x).astype(np.float32)
    xp[::3] *= -1.0
    ep = None if e is None else (1.0 + 1e-3 * e).astype(np.float32)
    if msg == MSG_XJ_SUB_XI:
        xp = (wl.x * 1e-2 + np.arange(n, dtype=np.float32)[:, None] * 1e-6).astype(np.float32)
        xp[::2] += 1.0           # differences near +-1 (or tiny, where products underflow to 0 on both sides)
    ref_p, sabs_p = oracle.propagate(wl.src, wl.dst, n, xp, ep, msg, AGGR_PROD, with_sabs=True)
    got_p = host(gnn.propagate(g, dev(xp), dev(ep) if ep is not None else None, msg, AGGR_PROD)).astype(np.float64)
    assert np.isfinite(got_p).all()
    assert (np.abs(got_p - ref_p) <= 1.3e-7 * sabs_p + 1e-37).all(), f"{name} prod msg={msg}"
    if msg == MSG_XJ_SUB_XI:
        for aggr in (AGGR_SUM, AGGR_MEAN, AGGR_MAX):
            ref, sabs = oracle.propagate(wl.src, wl.dst, n, wl.x, None, msg, aggr, with_sabs=True)
            got = host(gnn.propagate(g, x, None, msg, aggr))
            if aggr == AGGR_MAX:
                np.testing.assert_array_equal(got.view(np.uint32), ref.view(np.uint32))
            else:
                assert_close_sabs(got, ref, sabs, what=f"{name} xj_sub_xi aggr={aggr}")


def test_apply_edges_dot_product(case, gnn):
    name, wl, g = case
    n = wl.num_nodes
    ref, sabs = oracle.apply_edges(wl.src, n, wl.x, None, MSG_XI_DOT_XJ, dst=wl.dst, with_sabs=True)
    got = gnn.apply_edges(g, dev(wl.x), None, MSG_XI_DOT_XJ)
    assert tuple(got.shape) == (wl.num_edges, 1)
    assert_close_sabs(host(got), ref, sabs, what=f"{name} xi_dot_xj")
    _, _, perm, _ = oracle.build_csr(wl.src, wl.dst, n)
    got_csr = gnn.apply_edges(g, dev(wl.x), None, MSG_XI_DOT_XJ, m_order=gnn.EDGE_ORDER_CSR)
    np.testing.assert_array_equal(host(got_csr), host(got)[perm])
    # the scalar messages can be reduced like any other: a width-1 aggregate
    ref_sum, sabs_sum = oracle.aggregate_neighbors(wl.dst, n, ref, AGGR_SUM, with_sabs=True)
    assert_close_sabs(host(gnn.aggregate_neighbors(g, dev(ref), AGGR_SUM)), ref_sum, sabs_sum,
                      what=f"{name} sum of dots")


def test_unsupported_backward_combinations(gnn):
    wl = powerlaw(500, 4000, 8, 200.0)
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), wl.num_nodes)
    gt = gnn.build_csr(dev(wl.dst), dev(wl.src), wl.num_nodes)
    x = dev(wl.x)
    for msg, aggr in ((MSG_XJ_SUB_XI, AGGR_SUM), (MSG_COPY_XJ, AGGR_MIN), (MSG_COPY_XJ, AGGR_PROD)):
        with pytest.raises(gnn.GnnError) as err:
            gnn.propagate_backward(g, gt, x, torch.ones_like(x), None, msg, aggr)
        assert err.value.code == 4
    g.close()
    gt.close()


def test_f32_to_bf16_bit_exact(gnn, golden_dir):
    gd = load_golden(golden_dir, "bf16_rounding.json")
    bits = np.array([int(c["float_bits"], 16) for c in gd["cases"]], np.uint32)
    x = np.concatenate([bits.view(np.float32),
                        (synth.normal_f32(98, 2, 100_003) * np.float32(10.0) ** synth.randint(98, 3, 0, 100_003, -30, 30)
                         ).astype(np.float32)])
    codes, _ = oracle.round_bf16(x)
    got = host(gnn.f32_to_bf16(dev(x))).view(np.uint16)
    np.testing.assert_array_equal(got, codes)


@pytest.mark.parametrize("msg", [MSG_COPY_XJ, MSG_E_MUL_XJ])
@pytest.mark.parametrize("aggr", [AGGR_SUM, AGGR_MEAN, AGGR_MAX])
def test_propagate_bf16_storage(case, gnn, msg, aggr):
    """Features stored as bfloat16, widened exactly, float arithmetic: the reference is the oracle's propagate
    on the oracle-rounded features, at the usual bar (max bit for bit)."""
    name, wl, g = case
    f = wl.x.shape[1]
    if f % 8 != 0:
        pytest.skip("bfloat16 rows are read eight values at a time")
    codes, wide = oracle.round_bf16(wl.x)
    e = wl.edge_weight if msg == MSG_E_MUL_XJ else None
    ref, sabs = oracle.propagate(wl.src, wl.dst, wl.num_nodes, wide, e, msg, aggr, with_sabs=True)
    xh = gnn.f32_to_bf16(dev(wl.x))
    np.testing.assert_array_equal(host(xh).view(np.uint16), codes)
    got = host(gnn.propagate_bf16(g, xh, dev(e) if e is not None else None, msg, aggr))
    if aggr == AGGR_MAX:
        np.testing.assert_array_equal(got.view(np.uint32), ref.view(np.uint32))
    else:
        assert_close_sabs(got, ref, sabs, what=f"{name} bf16 msg={msg} aggr={aggr}")
    if aggr == AGGR_MAX:     # the float path on the widened features gives the same maxima
        same = host(gnn.propagate(g, dev(wide), dev(e) if e is not None else None, msg, aggr))
        np.testing.assert_array_equal(got.view(np.uint32), same.view(np.uint32))


def test_propagate_bf16_wide_rows_and_rejections(gnn):
    wl = powerlaw(3000, 60_000, 256, 1500.0)
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), wl.num_nodes, 8, 128)
    codes, wide = oracle.round_bf16(wl.x)
    ref, sabs = oracle.propagate(wl.src, wl.dst, wl.num_nodes, wide, None, MSG_COPY_XJ, AGGR_SUM, with_sabs=True)
    xh = dev(codes.view(np.int16))
    assert_close_sabs(host(gnn.propagate_bf16(g, xh, None, MSG_COPY_XJ, AGGR_SUM)), ref, sabs, what="bf16 F=256")
    for msg, aggr in ((MSG_XJ_SUB_XI, AGGR_SUM), (MSG_COPY_XJ, AGGR_MIN)):
        with pytest.raises(gnn.GnnError) as err:
            gnn.propagate_bf16(g, xh, None, msg, aggr)
        assert err.value.code == 4
    with pytest.raises(gnn.GnnError) as err:      # feat_dim % 8 != 0
        gnn.propagate_bf16(g, xh[:, :12].contiguous(), None, MSG_COPY_XJ, AGGR_SUM)
    assert err.value.code == 4
    g.close()


def test_f32_to_f16_bit_exact(gnn, golden_dir):
    gd = load_golden(golden_dir, "f16_rounding.json")
    bits = np.array([int(c["float_bits"], 16) for c in gd["cases"]], np.uint32)
    x = np.concatenate([bits.view(np.float32),
                        (synth.normal_f32(97, 2, 100_003) * np.float32(10.0) ** synth.randint(97, 3, 0, 100_003, -12, 6)
                         ).astype(np.float32)])
    codes, _ = oracle.round_f16(x)
    got = host(gnn.f32_to_f16(dev(x))).view(np.uint16)
    np.testing.assert_array_equal(got, codes)


@pytest.mark.parametrize("msg", [MSG_COPY_XJ, MSG_E_MUL_XJ])
@pytest.mark.parametrize("aggr", [AGGR_SUM, AGGR_MEAN, AGGR_MAX])
def test_propagate_f16_storage(case, gnn, msg, aggr):
    """Features stored as IEEE binary16, widened exactly, float arithmetic: the reference is the oracle's propagate
    on the oracle-rounded features, at the usual bar (max bit for bit)."""
    name, wl, g = case
    f = wl.x.shape[1]
    if f % 8 != 0:
        pytest.skip("16-bit rows are read eight values at a time")
    codes, wide = oracle.round_f16(wl.x)
    e = wl.edge_weight if msg == MSG_E_MUL_XJ else None
    ref, sabs = oracle.propagate(wl.src, wl.dst, wl.num_nodes, wide, e, msg, aggr, with_sabs=True)
    xh = gnn.f32_to_f16(dev(wl.x))
    np.testing.assert_array_equal(host(xh).view(np.uint16), codes)
    got = host(gnn.propagate_f16(g, xh, dev(e) if e is not None else None, msg, aggr))
    if aggr == AGGR_MAX:
        np.testing.assert_array_equal(got.view(np.uint32), ref.view(np.uint32))
    else:
        assert_close_sabs(got, ref, sabs, what=f"{name} f16 msg={msg} aggr={aggr}")


def test_propagate_f16_subnormal_features_and_rejections(gnn):
    """Features deep in binary16's subnormal range are widened exactly (copy_xj + max returns them bit for bit)."""
    wl = powerlaw(3000, 60_000, 64, 1500.0)
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), wl.num_nodes, 8, 128)
    tiny = (wl.x * np.float32(2.0 ** -20)).astype(np.float32)          # |values| around 1e-6: subnormal halves
    codes, wide = oracle.round_f16(tiny)
    assert ((codes & 0x7C00) == 0).mean() > 0.9
    xh = dev(codes.view(np.int16))
    ref = oracle.propagate(wl.src, wl.dst, wl.num_nodes, wide, None, MSG_COPY_XJ, AGGR_MAX)
    np.testing.assert_array_equal(host(gnn.propagate_f16(g, xh, None, MSG_COPY_XJ, AGGR_MAX)).view(np.uint32),
                                  ref.view(np.uint32))
    ref, sabs = oracle.propagate(wl.src, wl.dst, wl.num_nodes, wide, None, MSG_COPY_XJ, AGGR_SUM, with_sabs=True)
    assert_close_sabs(host(gnn.propagate_f16(g, xh, None, MSG_COPY_XJ, AGGR_SUM)), ref, sabs, what="f16 subnormal sum")
    for msg, aggr in ((MSG_XJ_SUB_XI, AGGR_SUM), (MSG_COPY_XJ, AGGR_PROD)):
        with pytest.raises(gnn.GnnError) as err:
            gnn.propagate_f16(g, xh, None, msg, aggr)
        assert err.value.code == 4
    g.close()


def test_hetero_propagate(gnn):
    """Three relations into one destination node type (power-law destinations so that rows get split),
    against the oracle's sum over relations; a bipartite handle in plain propagate; and the rejections."""
    n_dst, f = 4000, 32
    sizes, edges = [2500, 7000, 4000], [60_000, 90_000, 30_000]
    w = synth.power_law_weights(n_dst, 1.0, 1.0, 0.05)
    cdf = np.cumsum(w / w.sum())
    rels = []
    for r, (ns, ne) in enumerate(zip(sizes, edges)):
        src = synth.randint(87, 10 + r, 0, ne, 0, ns - 1).astype(np.int32)
        dst = np.minimum(np.searchsorted(cdf, synth.uniform01(87, 20 + r, 0, ne)), n_dst - 1).astype(np.int32)
        rels.append({"src": src, "dst": dst, "num_src_nodes": ns,
                     "x": synth.normal_f32(87, 30 + r, ns * f).reshape(ns, f),
                     "e": synth.uniform_f32(87, 40 + r, ne, -1.0, 1.0)})
    graphs = [gnn.build_csr_bipartite(dev(r["src"]), dev(r["dst"]), r["num_src_nodes"], n_dst) for r in rels]
    assert any(g.work_sizes()["split_rows"] > 0 for g in graphs)
    xs, es = [dev(r["x"]) for r in rels], [dev(r["e"]) for r in rels]
    for msg, aggr in ((MSG_COPY_XJ, AGGR_SUM), (MSG_E_MUL_XJ, AGGR_SUM), (MSG_E_MUL_XJ, AGGR_MEAN),
                      (MSG_COPY_XJ, AGGR_MAX)):
        ref, sabs = oracle.hetero_propagate(rels, n_dst, msg, aggr, with_sabs=True)
        got = host(gnn.hetero_propagate(graphs, xs, es if msg == MSG_E_MUL_XJ else None, msg, aggr))
        assert_close_sabs(got, ref, sabs, what=f"hetero msg={msg} aggr={aggr}")
    # one relation through the plain entry points
    r0 = rels[0]
    one = oracle.hetero_propagate([r0], n_dst, MSG_COPY_XJ, AGGR_MAX)
    np.testing.assert_array_equal(host(gnn.propagate(graphs[0], xs[0], None, MSG_COPY_XJ, AGGR_MAX)), one)
    m = gnn.apply_edges(graphs[0], xs[0], es[0], MSG_E_MUL_XJ)
    np.testing.assert_array_equal(host(m), r0["e"][:, None] * r0["x"][r0["src"]])
    # what needs a node's own features is refused on a relation between two node sets
    # (relation 2 has as many sources as destinations: it is the handle that knows they are different sets)
    for fn in (lambda: gnn.gin_update(graphs[2], xs[2], 0.0),
               lambda: gnn.propagate(graphs[2], xs[2], None, MSG_XJ_SUB_XI, AGGR_SUM),
               lambda: gnn.apply_edges(graphs[2], xs[2], None, MSG_XI_DOT_XJ),
               lambda: gnn.gcnconv(graphs[2], xs[2], dev(np.ones((xs[2].shape[1], 4), np.float32)), None, False)):
        with pytest.raises(gnn.GnnError) as err:
            fn()
        assert err.value.code == 4
    with pytest.raises(gnn.GnnError):     # a source index beyond its node set
        gnn.build_csr_bipartite(dev(np.array([0, 2500], np.int32)), dev(np.array([1, 1], np.int32)), 2500, n_dst)
    for g in graphs:
        g.close()


def test_apply_edges_elementwise_and_odd_width(gnn):
    wl = powerlaw(2000, 30_000, 6, 900.0)
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), wl.num_nodes, 4, 64)
    ef = synth.normal_f32(19, 3, wl.num_edges * 6).reshape(wl.num_edges, 6)
    m_ref = oracle.apply_edges(wl.src, wl.num_nodes, wl.x, ef, MSG_E_MUL_XJ)
    m = gnn.apply_edges(g, dev(wl.x), dev(ef), MSG_E_MUL_XJ)
    np.testing.assert_array_equal(host(m).view(np.uint32), m_ref.view(np.uint32))
    ef_csr = gnn.edge_data_to_csr(g, dev(ef))
    m2 = gnn.apply_edges(g, dev(wl.x), ef_csr, MSG_E_MUL_XJ, e_order=gnn.EDGE_ORDER_CSR)
    np.testing.assert_array_equal(host(m2).view(np.uint32), m_ref.view(np.uint32))
    ref, sabs = oracle.aggregate_neighbors(wl.dst, wl.num_nodes, m_ref, AGGR_SUM, with_sabs=True)
    assert_close_sabs(host(gnn.aggregate_neighbors(g, m, AGGR_SUM)), ref, sabs, what="aggregate F=6")
    g.close()


@pytest.mark.parametrize("aggr", [AGGR_SUM, AGGR_MEAN])
@pytest.mark.parametrize("e_kind", ["none", "scalar", "vector"])
def test_propagate_backward(case, gnn, aggr, e_kind):
    name, wl, g = case
    n, ne, f = wl.num_nodes, wl.num_edges, wl.x.shape[1]
    gt = gnn.build_csr(dev(wl.dst), dev(wl.src), n, 4, 64)         # the same edges sorted by source
    gout = synth.normal_f32(17, 7, n * f).reshape(n, f)
    e = {"none": None, "scalar": wl.edge_weight,
         "vector": synth.normal_f32(23, 3, ne * f).reshape(ne, f)}[e_kind]
    msg = MSG_COPY_XJ if e is None else MSG_E_MUL_XJ
    ref = oracle.propagate_backward(wl.src, wl.dst, n, wl.x, gout, e, msg, aggr, with_sabs=True)
    gx, ge = gnn.propagate_backward(g, gt, dev(wl.x), dev(gout), dev(e) if e is not None else None, msg, aggr)
    assert_close_sabs(host(gx), ref["grad_x"], ref["sabs_x"], what=f"{name} grad_x {e_kind} aggr={aggr}")
    if e is None:
        assert ge is None
    else:
        assert_close_sabs(host(ge).reshape(ne, -1), ref["grad_e"], ref["sabs_e"], what=f"{name} grad_e {e_kind} aggr={aggr}")
    gt.close()


@pytest.mark.parametrize("e_kind", ["none", "scalar", "vector"])
def test_propagate_backward_max(case, gnn, e_kind):
    name, wl, g = case
    n, ne, f = wl.num_nodes, wl.num_edges, wl.x.shape[1]
    gt = gnn.build_csr(dev(wl.dst), dev(wl.src), n, 4, 64)
    gout = synth.normal_f32(27, 7, n * f).reshape(n, f)
    e = {"none": None, "scalar": wl.edge_weight,
         "vector": synth.normal_f32(29, 3, ne * f).reshape(ne, f)}[e_kind]
    msg = MSG_COPY_XJ if e is None else MSG_E_MUL_XJ
    x = wl.x.copy()
    x[:, :3] = np.round(x[:, :3])            # plenty of exact ties (and signed zeros) in three columns
    ref = oracle.propagate_backward(wl.src, wl.dst, n, x, gout, e, msg, AGGR_MAX, with_sabs=True)
    dx, de = dev(x), (dev(e) if e is not None else None)
    out = gnn.propagate(g, dx, de, msg, AGGR_MAX)
    am = gnn.propagate_argmax(g, dx, out, de, msg)
    np.testing.assert_array_equal(host(am), ref["argmax"])
    gx, ge = gnn.propagate_backward(g, gt, dx, dev(gout), de, msg, AGGR_MAX, argmax=am)
    assert_close_sabs(host(gx), ref["grad_x"], ref["sabs_x"], what=f"{name} max grad_x {e_kind}")
    if e is not None:
        assert_close_sabs(host(ge).reshape(ne, -1), ref["grad_e"], ref["sabs_e"], what=f"{name} max grad_e {e_kind}")
    if e_kind == "scalar":   # winners from CSR-ordered weights are the same edges
        am2 = gnn.propagate_argmax(g, dx, out, gnn.edge_data_to_csr(g, de), msg, e_order=gnn.EDGE_ORDER_CSR)
        assert torch.equal(am, am2)
    gt.close()


def test_propagate_backward_odd_width_and_errors(gnn):
    wl = powerlaw(2000, 30_000, 7, 900.0)
    n = wl.num_nodes
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), n)
    gt = gnn.build_csr(dev(wl.dst), dev(wl.src), n)
    gout = synth.normal_f32(18, 7, n * 7).reshape(n, 7)
    ref = oracle.propagate_backward(wl.src, wl.dst, n, wl.x, gout, wl.edge_weight, MSG_E_MUL_XJ, AGGR_MEAN, with_sabs=True)
    gx, ge = gnn.propagate_backward(g, gt, dev(wl.x), dev(gout), dev(wl.edge_weight), MSG_E_MUL_XJ, AGGR_MEAN)
    assert_close_sabs(host(gx), ref["grad_x"], ref["sabs_x"], what="grad_x F=7")
    assert_close_sabs(host(ge).reshape(-1, 1), ref["grad_e"], ref["sabs_e"], what="grad_e F=7")
    with pytest.raises(gnn.GnnError) as ei:
        gnn.propagate_backward(g, gt, dev(wl.x), dev(gout), None, MSG_COPY_XJ, AGGR_MAX)   # winners missing
    assert ei.value.code == 1
    small = gnn.build_csr(dev(wl.dst[:100]), dev(wl.src[:100]), n)
    with pytest.raises(gnn.GnnError):
        gnn.propagate_backward(g, small, dev(wl.x), dev(gout), None, MSG_COPY_XJ, AGGR_SUM)
    for h in (g, gt, small):
        h.close()


def test_propagate_invariants(case, gnn):
    _, wl, g = case
    n = wl.num_nodes
    indeg = np.bincount(wl.dst, minlength=n)
    ones = dev(np.ones((n, 64), np.float32))
    np.testing.assert_array_equal(host(gnn.propagate(g, ones))[:, 0], indeg.astype(np.float32))
    c = dev(np.full((n, 64), 2.5, np.float32))
    want = np.where(indeg > 0, 2.5, 0.0).astype(np.float32)
    np.testing.assert_array_equal(host(gnn.propagate(g, c, None, MSG_COPY_XJ, AGGR_MAX))[:, 5], want)
    np.testing.assert_allclose(host(gnn.propagate(g, c, None, MSG_COPY_XJ, AGGR_MEAN))[:, 5], want, rtol=1e-6)


def test_max_signed_zero(gnn):
    src = dev(np.array([0, 1, 1, 0, 0, 0], np.int32))
    dst = dev(np.array([2, 2, 3, 3, 1, 1], np.int32))
    g = gnn.build_csr(src, dst, 4)
    x = np.array([[-0.0] * 4, [0.0] * 4, [5.0] * 4, [5.0] * 4], np.float32)
    ref = oracle.propagate(host(src), host(dst), 4, x, None, MSG_COPY_XJ, AGGR_MAX)
    got = host(gnn.propagate(g, dev(x), None, MSG_COPY_XJ, AGGR_MAX))
    np.testing.assert_array_equal(got.view(np.uint32), ref.view(np.uint32))
    assert np.signbit(got[1]).all() and not np.signbit(got[2]).any()
    g.close()


def test_propagate_argument_errors(case, gnn):
    _, wl, g = case
    x = dev(wl.x)
    with pytest.raises(gnn.GnnError):
        gnn.propagate(g, x, None, MSG_E_MUL_XJ, AGGR_SUM)              # missing edge data
    with pytest.raises(gnn.GnnError):
        gnn.propagate(g, x, None, MSG_COPY_XJ, 7)                       # unknown aggregation
    with pytest.raises(gnn.GnnError):
        gnn.propagate(g, x, dev(np.zeros((wl.num_edges, 3), np.float32)), MSG_E_MUL_XJ, AGGR_SUM)  # e_dim


# ----------------------------------------------------------------------------- layers

def test_dense_xw_matches_the_oracle(gnn):
    """X W on the matrix cores against the oracle's double-precision triple loop (and its |X||W| magnitudes):
    every number of 32-wide k slices (1 .. 4, odd and even), partial last slices, 1 / 2 / 4 column tiles, ragged
    column counts, several column blocks, several tiles per wavefront, ragged last row tile; then the shapes that
    take the general kernel (k > 128 or not a multiple of 4)."""
    for rows, k, n in ((1000, 128, 128), (777, 100, 64), (130, 37, 50), (5, 8, 200), (4096, 16, 64),
                       (70_000, 128, 128), (500, 300, 128), (300, 520, 40), (900, 200, 64), (257, 64, 33),
                       (3000, 64, 100), (1500, 128, 36), (640, 100, 20), (333, 12, 4), (6000, 32, 300),
                       (150_000, 64, 128), (200_000, 96, 64), (140_001, 24, 32), (70_000, 72, 200), (33, 4, 4),
                       (90_000, 68, 36)):
        x = synth.normal_f32(rows + k, 2, rows * k).reshape(rows, k)
        w = synth.glorot_uniform(n, 4, k, n, (k, n))
        sc = synth.uniform_f32(3, 5, rows, 0.5, 2.0)
        ref, sabs = oracle.dense(x, w, with_sabs=True)
        assert_close_sabs(host(gnn.dense_xw(dev(x), dev(w))), ref, sabs, what=f"xw {rows}x{k}x{n}")
        assert_close_sabs(host(gnn.dense_xw(dev(x), dev(w), dev(sc))), ref.astype(np.float64) * sc[:, None],
                          sabs * sc[:, None], what=f"xw scaled {rows}x{k}x{n}")


@pytest.mark.parametrize("loops", [True, False])
def test_gcnconv(gnn, loops, golden_dir):
    gd = load_golden(golden_dir, "path3_gcn.json")
    g = gnn.build_csr(dev(np.array(gd["src"], np.int32)), dev(np.array(gd["dst"], np.int32)), 3)
    if loops:
        out = gnn.gcnconv(g, dev(np.array(gd["x"], np.float32)), dev(np.array(gd["w2"], np.float32)),
                          dev(np.array(gd["bias2"], np.float32)), True)
        np.testing.assert_allclose(host(out), np.array(gd["out2"]), rtol=1e-6)
    g.close()
    wl = synth.config1_gcn(num_nodes=20_000, pairs=100_000, f_in=128, f_out=128)
    bias = synth.uniform_f32(8, 5, 128, -1, 1)
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), wl.num_nodes, 8, 64)
    ref, sabs = oracle.gcnconv(wl.src, wl.dst, wl.num_nodes, wl.x, wl.params["w"], bias, loops, with_sabs=True)
    got = host(gnn.gcnconv(g, dev(wl.x), dev(wl.params["w"]), dev(bias), loops))
    assert_close_sabs(got, ref, sabs, what=f"gcnconv loops={loops}")
    # fixed point: X = sqrt(d) is reproduced by the normalised operator (W = 1)
    if loops:
        d = np.sqrt(np.bincount(wl.dst, minlength=wl.num_nodes) + 1.0).astype(np.float32).reshape(-1, 1)
        out = host(gnn.gcnconv(g, dev(d), dev(np.ones((1, 1), np.float32)), None, True))
        np.testing.assert_allclose(out, d, rtol=2e-6)
    g.close()


@pytest.mark.parametrize("loops,f_in,f_out,relu", [(True, 16, 64, True), (False, 16, 64, False), (True, 37, 50, False),
                                                   (True, 64, 16, True), (True, 3, 130, False)])
def test_gcnconv_widths(gnn, loops, f_in, f_out, relu):
    """Widening layers aggregate first and project afterwards, narrowing ones the other way round: both orders, odd
    widths and the activation against the same oracle."""
    wl = synth.config1_gcn(num_nodes=6000, pairs=30_000, f_in=f_in, f_out=f_out)
    bias = synth.uniform_f32(9, 5, f_out, -1, 1)
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), wl.num_nodes, 8, 64)
    ref, sabs = oracle.gcnconv(wl.src, wl.dst, wl.num_nodes, wl.x, wl.params["w"], bias, loops, with_sabs=True)
    if relu:
        ref = np.maximum(ref, 0.0)
    got = host(gnn.gcnconv(g, dev(wl.x), dev(wl.params["w"]), dev(bias), loops, relu=relu))
    assert_close_sabs(got, ref, sabs, what=f"gcnconv {f_in}->{f_out} loops={loops} relu={relu}")
    g.close()


@pytest.mark.parametrize("loops,f_in,f_out", [(True, 128, 128), (False, 128, 128), (True, 16, 64), (True, 37, 50),
                                              # grad_W through the LDS-staged kernel: every tile shape, ragged tiles, several
                                              # tiles per dimension
                                              (True, 100, 64), (True, 64, 128), (True, 48, 40), (True, 200, 192)])
def test_gcnconv_backward(gnn, loops, f_in, f_out):
    wl = synth.config1_gcn(num_nodes=20_000, pairs=100_000, f_in=f_in, f_out=f_out)
    n = wl.num_nodes
    w = wl.params["w"]
    gout = synth.normal_f32(33, 7, n * f_out).reshape(n, f_out)
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), n, 8, 64)
    gt = gnn.build_csr(dev(wl.dst), dev(wl.src), n, 8, 64)
    ref = oracle.gcnconv_backward(wl.src, wl.dst, n, wl.x, w, gout, loops)
    gx, gw, gb = gnn.gcnconv_backward(g, gt, dev(wl.x), dev(w), dev(gout), loops)
    assert_close_sabs(host(gx), ref["grad_x"], ref["sabs_x"], what="gcn grad_x")
    assert_close_sabs(host(gw), ref["grad_w"], ref["sabs_w"], what="gcn grad_w")
    assert_close_sabs(host(gb), ref["grad_b"], ref["sabs_b"], what="gcn grad_b")
    g.close()
    gt.close()


@pytest.mark.parametrize("n,f", [(5000, 64), (300, 7), (70_000, 200), (1, 5), (8192, 9), (8193, 9)])
def test_batchnorm(gnn, n, f):
    x = (synth.normal_f32(71, 2, n * f).reshape(n, f) * (1.0 + np.arange(f, dtype=np.float32) % 5) + 2.0).astype(np.float32)
    gamma = synth.uniform_f32(71, 3, f, 0.5, 1.5)
    beta = synth.uniform_f32(71, 4, f, -1.0, 1.0)
    for relu in (False, True):
        ref, mean, var = oracle.batchnorm(x, gamma, beta, 1e-5, relu=relu)
        got, gm, gv = gnn.batchnorm(dev(x), dev(gamma), dev(beta), 1e-5, relu=relu)
        np.testing.assert_allclose(host(gm), mean, rtol=1e-5, atol=1e-6)
        np.testing.assert_allclose(host(gv), var, rtol=1e-5, atol=1e-9)
        # the terms behind an element: gamma * (x - mean) / sqrt(var + eps) and beta
        inv = 1.0 / np.sqrt(var.astype(np.float64) + 1e-5)
        sabs = np.abs(gamma) * inv * (np.abs(x) + np.abs(mean)) + np.abs(beta)
        assert_close_sabs(host(got), ref, sabs, what=f"batchnorm {n}x{f} relu={relu}")
    # stored statistics; no scale / shift
    m0 = synth.uniform_f32(71, 5, f, -1.0, 1.0)
    v0 = synth.uniform_f32(71, 6, f, 0.5, 2.0)
    ref, _, _ = oracle.batchnorm(x, None, None, 1e-3, mean=m0, var=v0)
    got, _, _ = gnn.batchnorm(dev(x), None, None, 1e-3, mean=dev(m0), var=dev(v0))
    sabs = (np.abs(x) + np.abs(m0)) / np.sqrt(v0.astype(np.float64) + 1e-3)
    assert_close_sabs(host(got), ref, sabs, what="batchnorm stored statistics")


def test_dense_layer(gnn):
    for rows, k, n in ((32, 64, 1), (4096, 64, 1), (1000, 16, 64), (77, 30, 5)):
        x = synth.normal_f32(rows + n, 2, rows * k).reshape(rows, k)
        w = synth.glorot_uniform(n, 4, k, n, (k, n))
        b = synth.uniform_f32(n, 5, n, -1.0, 1.0)
        for relu in (False, True):
            ref, sabs = oracle.dense(x, w, b, relu=relu, with_sabs=True)
            assert_close_sabs(host(gnn.dense(dev(x), dev(w), dev(b), relu=relu)), ref, sabs, what=f"dense {rows}x{k}x{n}")
        ref, sabs = oracle.dense(x, w, with_sabs=True)
        assert_close_sabs(host(gnn.dense(dev(x), dev(w))), ref, sabs, what="dense without bias")


def test_example_model(gnn):
    """Every stage of the example model against the oracle's stage, each fed the oracle's previous
    intermediate (the strict per-operation bar); then the one-call chain, which runs the same kernels in
    the same order and must reproduce the stage-by-stage GPU result bit for bit, and agrees with the
    oracle's end-to-end prediction to 1e-4 (five stages of at most 1e-5 each, none of which amplifies:
    the normalisation bounds the activations)."""
    # widths: the default takes the fused normalisation in the second convolution's projection (as do 100 => 36:
    # four k quarters, the last one ragged); 32 => 64 widens (the gather reads the normalised rows: not fused),
    # 30 => 30 cannot be read in 128-bit pieces (general projection kernel: not fused)
    for kwargs in (dict(), dict(num_graphs=300, n=40, p=0.1), dict(num_graphs=300, n=40, p=0.1, f1=100, f2=36),
                   dict(num_graphs=40, n=30, p=0.1, f1=32, f2=64), dict(num_graphs=40, n=30, p=0.1, f1=30, f2=30)):
        wl = synth.config5_example_model(**kwargs)
        n, ng, p = wl.num_nodes, wl.num_graphs, wl.params
        ref = oracle.example_model_forward(wl.src, wl.dst, n, wl.graph_indicator, ng, wl.x, p)
        g = gnn.build_csr(dev(wl.src), dev(wl.dst), n)
        dp = {k: dev(v) for k, v in p.items()}
        gi = dev(wl.graph_indicator)
        # stage by stage on the oracle's intermediates
        r1, s1 = oracle.gcnconv(wl.src, wl.dst, n, wl.x, p["w1"], p["b1"], True, with_sabs=True)
        assert_close_sabs(host(gnn.gcnconv(g, dev(wl.x), dp["w1"], dp["b1"], True)), r1, s1, what="stage 1")
        got2, _, _ = gnn.batchnorm(dev(ref["h1"]), dp["gamma"], dp["beta"], 1e-5, relu=True)
        inv = 1.0 / np.sqrt(ref["var"].astype(np.float64) + 1e-5)
        s2 = np.abs(p["gamma"]) * inv * (np.abs(ref["h1"]) + np.abs(ref["mean"])) + np.abs(p["beta"])
        assert_close_sabs(host(got2), ref["h2"], s2, what="stage 2")
        r3, s3 = oracle.gcnconv(wl.src, wl.dst, n, ref["h2"], p["w2"], p["b2"], True, with_sabs=True)
        assert_close_sabs(host(gnn.gcnconv(g, dev(ref["h2"]), dp["w2"], dp["b2"], True, relu=True)), np.maximum(r3, 0),
                          s3, what="stage 3")
        r4, s4 = oracle.graph_pool(wl.graph_indicator, ng, ref["h3"], AGGR_MEAN, with_sabs=True)
        assert_close_sabs(host(gnn.graph_pool(gi, ng, dev(ref["h3"]), AGGR_MEAN)), r4, s4, what="stage 4")
        r5, s5 = oracle.dense(ref["pooled"], p["w3"], p["b3"], with_sabs=True)
        assert_close_sabs(host(gnn.dense(dev(ref["pooled"]), dp["w3"], dp["b3"])), r5, s5, what="stage 5")
        # the chain
        h1 = gnn.gcnconv(g, dev(wl.x), dp["w1"], dp["b1"], True)
        h2, _, _ = gnn.batchnorm(h1, dp["gamma"], dp["beta"], 1e-5, relu=True)
        h3 = gnn.gcnconv(g, h2, dp["w2"], dp["b2"], True, relu=True)
        y_steps = gnn.dense(gnn.graph_pool(gi, ng, h3, AGGR_MEAN), dp["w3"], dp["b3"])
        y = gnn.example_model_forward(g, gi, ng, dev(wl.x), dp)
        assert torch.equal(y, y_steps)
        err = np.abs(host(y).astype(np.float64) - ref["y"]).max()
        assert err <= 1e-4 * np.abs(ref["y"]).max(), err
        g.close()


def test_example_model_hip_graph_replay(gnn):
    """The chain only launches kernels once its scratch is reserved, so it can be captured into a HIP graph;
    every replay (with eager work and synchronisation in between) must reproduce the eager result."""
    wl = synth.config5_example_model()
    n, ng = wl.num_nodes, wl.num_graphs
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), n)
    dp = {k: dev(v) for k, v in wl.params.items()}
    gi, x = dev(wl.graph_indicator), dev(wl.x)
    f1, f2 = wl.params["w1"].shape[1], wl.params["w2"].shape[1]
    ws = torch.empty(int(gnn.lib().gnn_example_model_workspace_bytes(n, ng, f1, f2)), dtype=torch.uint8, device="cuda")
    y = torch.empty((ng, 1), dtype=torch.float32, device="cuda")
    eager = gnn.example_model_forward(g, gi, ng, x, dp).clone()
    gnn.example_model_forward(g, gi, ng, x, dp, out=y, workspace=ws)      # warm-up on the buffers to be captured
    torch.cuda.synchronize()
    gph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gph):
        gnn.example_model_forward(g, gi, ng, x, dp, out=y, workspace=ws)
    for it in range(4):
        y.fill_(float("nan"))
        ws.random_(0, 255)                                                  # stale scratch must not matter
        gph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, eager), it
        other = gnn.propagate(g, x, None, MSG_COPY_XJ, AGGR_SUM)            # eager work between replays
        torch.cuda.synchronize()
        assert bool(torch.isfinite(other).all())
    # new inputs in the captured buffers are picked up by the next replay
    x.mul_(0.5)
    expect = gnn.example_model_forward(g, gi, ng, x, dp).clone()
    gph.replay()
    torch.cuda.synchronize()
    assert torch.equal(y, expect)
    del gph
    g.close()


def test_training_pieces(gnn):
    """Loss, relu mask, pooling / dense / batch-norm backward and the Adam step, each against the oracle."""
    # mean squared error
    pred, target = synth.normal_f32(91, 2, 4096).reshape(4096, 1), synth.normal_f32(91, 3, 4096).reshape(4096, 1)
    loss, grad = gnn.mse_loss(dev(pred), dev(target))
    d = pred.astype(np.float64) - target
    assert abs(float(host(loss)[0]) - (d ** 2).mean()) <= 1e-5 * (d ** 2).mean()
    np.testing.assert_allclose(host(grad), 2 * d / d.size, rtol=1e-6, atol=1e-12)
    # relu mask
    yv, gv = synth.normal_f32(91, 4, 5000), synth.normal_f32(91, 5, 5000)
    np.testing.assert_array_equal(host(gnn.relu_backward(dev(yv), dev(gv))), np.where(yv > 0, gv, np.float32(0)))
    # pooling backward on batched graphs, one of them empty
    wl = synth.config3_batched(num_graphs=300)
    gi = wl.graph_indicator.copy()
    gi[gi >= 17] += 1
    ng, f = 301, 24
    go = synth.normal_f32(91, 6, ng * f).reshape(ng, f)
    np.testing.assert_array_equal(host(gnn.graph_pool_backward(dev(gi), ng, dev(go), AGGR_SUM)),
                                  oracle.pool_backward(gi, ng, go, AGGR_SUM))
    np.testing.assert_allclose(host(gnn.graph_pool_backward(dev(gi), ng, dev(go), AGGR_MEAN)),
                               oracle.pool_backward(gi, ng, go, AGGR_MEAN), rtol=2e-7)
    # dense backward
    for rows, k, n in ((32, 64, 1), (5000, 64, 1), (3000, 16, 64), (777, 30, 5)):
        x = synth.normal_f32(rows, 2, rows * k).reshape(rows, k)
        w = synth.glorot_uniform(n, 4, k, n, (k, n))
        gy = synth.normal_f32(rows, 7, rows * n).reshape(rows, n)
        rx, rw, rb = oracle.dense_backward(x, w, gy)
        gx, gw, gb = gnn.dense_backward(dev(x), dev(w), dev(gy))
        a = lambda t: np.abs(t).astype(np.float64)
        assert_close_sabs(host(gx), rx, a(gy) @ a(w).T, what=f"dense grad_x {rows}x{k}x{n}")
        assert_close_sabs(host(gw), rw, a(x).T @ a(gy), what=f"dense grad_w {rows}x{k}x{n}")
        assert_close_sabs(host(gb), rb, a(gy).sum(0), what=f"dense grad_b {rows}x{k}x{n}")
    # batch-norm backward, with and without the relu mask
    for n, f in ((5000, 64), (300, 7), (70_000, 40), (8192, 9), (8193, 9)):
        x = (synth.normal_f32(92, 2, n * f).reshape(n, f) * (1.0 + np.arange(f, dtype=np.float32) % 3) + 1.0).astype(np.float32)
        gamma, beta = synth.uniform_f32(92, 3, f, 0.5, 1.5), synth.uniform_f32(92, 4, f, -0.5, 0.5)
        gy = synth.normal_f32(92, 5, n * f).reshape(n, f)
        y, mean, var = oracle.batchnorm(x, gamma, beta, 1e-5, relu=True)
        for masked in (False, True):
            g_in = np.where(y > 0, gy, np.float32(0)).astype(np.float32) if masked else gy
            rx, rg, rb = oracle.batchnorm_backward(x, gamma, g_in, 1e-5)
            gx, gg, gb = gnn.batchnorm_backward(dev(x), dev(gamma), dev(mean), dev(var), dev(gy), 1e-5,
                                                y_relu=dev(y) if masked else None)
            inv = 1.0 / np.sqrt(var.astype(np.float64) + 1e-5)
            xh = (x.astype(np.float64) - mean) * inv
            s_b, s_g = np.abs(g_in).astype(np.float64).sum(0), (np.abs(g_in) * np.abs(xh)).sum(0)
            assert_close_sabs(host(gb), rb, s_b, what="bn grad_beta")
            assert_close_sabs(host(gg), rg, s_g, what="bn grad_gamma")
            s_x = np.abs(gamma) * inv * (np.abs(g_in) + s_b / n + np.abs(xh) * s_g / n)
            assert_close_sabs(host(gx), rx, s_x, what=f"bn grad_x {n}x{f} masked={masked}")
    # Adam
    cnt = 10_000
    p0, g0 = synth.normal_f32(93, 2, cnt), synth.normal_f32(93, 3, cnt)
    m0, v0 = 0.1 * synth.normal_f32(93, 4, cnt), np.abs(synth.normal_f32(93, 5, cnt)) * 0.01
    rp, rm, rv = oracle.adam_step(p0, m0, v0, g0, 1e-3, 7)
    p, m, v = dev(p0), dev(m0), dev(v0)
    gnn.adam_step(p, m, v, dev(g0), 1e-3, 7)
    np.testing.assert_allclose(host(m), rm, rtol=0, atol=3e-7 * (0.9 * np.abs(m0) + 0.1 * np.abs(g0)).max())   # two signed terms
    np.testing.assert_allclose(host(v), rv, rtol=1e-6, atol=1e-12)
    np.testing.assert_allclose(host(p), rp, rtol=0, atol=1e-3 * 1e-5 + 2.0 ** -23 * np.abs(rp).max())


def test_example_model_train_step(gnn):
    """Three training steps in one call each against the oracle's loop (forward, loss, backward, Adam):
    the loss of every step to 1e-4, the parameters after the last step to a small fraction of the total
    update.  (The gradient of b1 is exactly zero in exact arithmetic -- the batch norm removes it -- so
    Adam moves b1 by rounding noise of either sign; it is only checked to stay within the size of a step.)
    Then: two runs are bitwise identical, and a longer run drives the loss down."""
    wl = synth.config5_example_model(num_graphs=64)
    n, ng, p0 = wl.num_nodes, wl.num_graphs, wl.params
    target = synth.normal_f32(95, 9, ng).reshape(ng, 1)
    lr, steps = 1e-3, 3
    # oracle loop
    rp = {k: v.copy() for k, v in p0.items()}
    rm = {k: np.zeros_like(v) for k, v in p0.items()}
    rv = {k: np.zeros_like(v) for k, v in p0.items()}
    ref_losses = []
    for t in range(1, steps + 1):
        loss, grads, _ = oracle.example_model_backward(wl.src, wl.dst, n, wl.graph_indicator, ng, wl.x, rp, target)
        ref_losses.append(loss)
        for k in rp:
            a, b, c = oracle.adam_step(rp[k], rm[k], rv[k], grads[k], lr, t)
            rp[k], rm[k], rv[k] = a.reshape(rp[k].shape), b.reshape(rp[k].shape), c.reshape(rp[k].shape)
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), n)
    gt = gnn.build_csr(dev(wl.dst), dev(wl.src), n)
    gi, x, tg = dev(wl.graph_indicator), dev(wl.x), dev(target)

    def run(count, rate):
        dp = {k: dev(v.copy()) for k, v in p0.items()}
        dm = {k: torch.zeros_like(v) for k, v in dp.items()}
        dv = {k: torch.zeros_like(v) for k, v in dp.items()}
        losses = [float(host(gnn.example_model_train_step(g, gt, gi, ng, x, tg, dp, dm, dv, t, lr=rate))[0])
                  for t in range(1, count + 1)]
        return dp, losses

    dp, losses = run(steps, lr)
    np.testing.assert_allclose(losses, ref_losses, rtol=1e-4)
    for k in p0:
        moved = np.abs(host(dp[k]).astype(np.float64) - p0[k])
        assert moved.max() <= steps * lr * 1.2, k          # an Adam step is about lr at most in these first steps
        if k != "b1":
            np.testing.assert_allclose(host(dp[k]), rp[k], rtol=0, atol=2e-2 * lr, err_msg=k)
    dp2, losses2 = run(steps, lr)
    assert losses2 == losses and all(torch.equal(dp[k], dp2[k]) for k in p0)
    _, long_losses = run(150, 1e-2)
    assert long_losses[-1] < 0.6 * long_losses[0]
    g.close()
    gt.close()


@pytest.mark.parametrize("heads", [1, 8, 3])
def test_segment_softmax(case, gnn, heads):
    name, wl, g = case
    e = wl.num_edges
    s = (3.0 * synth.normal_f32(31 + heads, 2, e * heads)).reshape(e, heads)
    ref = oracle.segment_softmax(wl.dst, wl.num_nodes, s)
    got = host(gnn.segment_softmax(g, dev(s)))
    assert_close_rel(got, ref, what=f"softmax {name} H={heads}")
    # CSR-ordered input/output
    _, _, perm, _ = oracle.build_csr(wl.src, wl.dst, wl.num_nodes)
    got_csr = host(gnn.segment_softmax(g, dev(s[perm]), order=gnn.EDGE_ORDER_CSR))
    np.testing.assert_array_equal(got_csr, got[perm])
    # sums to one per non-empty destination; shift invariance
    sums = np.zeros((wl.num_nodes, heads))
    np.add.at(sums, wl.dst, got.astype(np.float64))
    has = np.bincount(wl.dst, minlength=wl.num_nodes) > 0
    np.testing.assert_allclose(sums[has], 1.0, rtol=2e-5)
    shift = (50.0 * synth.normal_f32(3, 9, wl.num_nodes)).astype(np.float32)
    got_shift = host(gnn.segment_softmax(g, dev((s + shift[wl.dst][:, None]).astype(np.float32))))
    np.testing.assert_allclose(got_shift, got, rtol=2e-4, atol=1e-9)


@pytest.mark.parametrize("heads,ch,f_in", [(8, 8, 100), (2, 4, 16), (3, 5, 12), (1, 64, 32), (5, 64, 20), (3, 30, 8)])
def test_gatconv(gnn, heads, ch, f_in):
    wl = synth.config4_gat(num_nodes=6000, num_edges=150_000, f_in=f_in, heads=heads, ch=ch, cap=3000.0)
    p = wl.params
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), wl.num_nodes, 8, 128)
    ref, sabs = oracle.gatconv(wl.src, wl.dst, wl.num_nodes, wl.x, p["w"], p["a_src"], p["a_dst"], 0.2, with_sabs=True)
    got = host(gnn.gatconv(g, dev(wl.x), dev(p["w"]), dev(p["a_src"]), dev(p["a_dst"]), 0.2))
    assert_close_sabs(got, ref, sabs, what=f"gatconv H={heads} ch={ch}")
    # zero attention vectors: uniform weights -> mean of the projected features
    zero = np.zeros((heads, ch), np.float32)
    got0 = host(gnn.gatconv(g, dev(wl.x), dev(p["w"]), dev(zero), dev(zero), 0.2))
    ref0, sabs0 = oracle.gatconv(wl.src, wl.dst, wl.num_nodes, wl.x, p["w"], zero, zero, 0.2, with_sabs=True)
    assert_close_sabs(got0, ref0, sabs0, what="gatconv zero attention")
    g.close()


@pytest.mark.parametrize("heads,ch,f_in", [(8, 8, 100), (2, 4, 16), (1, 64, 32), (4, 16, 24), (3, 2, 10), (2, 1, 6),
                                           (2, 128, 40), (3, 5, 12), (8, 5, 20), (2, 30, 9), (5, 12, 16), (4, 3, 7),
                                           (3, 30, 8), (12, 24, 10), (9, 10, 6)])
def test_gatconv_backward(gnn, heads, ch, f_in):
    wl = synth.config4_gat(num_nodes=5000, num_edges=120_000, f_in=f_in, heads=heads, ch=ch, cap=2500.0)
    p, n, hc = wl.params, wl.num_nodes, heads * ch
    gout = synth.normal_f32(41 + heads, 7, n * hc).reshape(n, hc)
    # the derivative of the leaky ReLU jumps at 0, and float and double may disagree about the sign of a
    # pre-activation within rounding of 0: the few edges that close are left out of the input (a
    # pre-activation depends on the endpoints' features only, so the others are unchanged)
    h64 = (wl.x.astype(np.float64) @ p["w"].astype(np.float64)).reshape(n, heads, ch)
    nl, nr = (h64 * p["a_src"][None]).sum(-1), (h64 * p["a_dst"][None]).sum(-1)
    keep = np.abs(nl[wl.src] + nr[wl.dst]).min(axis=1) > 1e-5
    assert keep.mean() > 0.999
    src, dst = wl.src[keep], wl.dst[keep]
    v = nl[src] + nr[dst]
    g = gnn.build_csr(dev(src), dev(dst), n, 8, 128)
    gt = gnn.build_csr(dev(dst), dev(src), n, 8, 128)
    assert g.work_sizes()["split_rows"] > 0 and gt.work_sizes()["split_rows"] > 0
    ref = oracle.gatconv_backward(src, dst, n, wl.x, p["w"], p["a_src"], p["a_dst"], gout, 0.2)
    stats = torch.empty((n, heads, 2), dtype=torch.float32, device="cuda")
    args = (dev(wl.x), dev(p["w"]), dev(p["a_src"]), dev(p["a_dst"]))
    out = gnn.gatconv(g, *args, 0.2, softmax_stats=stats)
    # the statistics: maximum of the scores and the denominator relative to it
    sc = np.where(v > 0, v, 0.2 * v)
    mx = np.full((n, heads), -np.inf)
    np.maximum.at(mx, dst, sc)
    den = np.zeros((n, heads))
    np.add.at(den, dst, np.exp(sc - mx[dst]))
    st = host(stats).astype(np.float64)
    has = np.isfinite(mx[:, 0])
    np.testing.assert_allclose(st[has, :, 0], mx[has], rtol=1e-5, atol=1e-5)
    np.testing.assert_allclose(st[has, :, 1] * np.exp(st[has, :, 0] - mx[has]), den[has], rtol=2e-4)
    assert (st[~has, :, 1] == 0).all()
    gx, gw, gas, gad = gnn.gatconv_backward(g, gt, *args, out, stats, dev(gout), 0.2)
    assert_close_sabs(host(gx), ref["grad_x"], ref["sabs_x"], what="gat grad_x")
    assert_close_sabs(host(gw), ref["grad_w"], ref["sabs_w"], what="gat grad_w")
    assert_close_sabs(host(gas), ref["grad_a_src"], ref["sabs_a_src"], what="gat grad_a_src")
    assert_close_sabs(host(gad), ref["grad_a_dst"], ref["sabs_a_dst"], what="gat grad_a_dst")
    # bitwise reproducible
    gx2, gw2, gas2, gad2 = gnn.gatconv_backward(g, gt, *args, out, stats, dev(gout), 0.2)
    for a, b in ((gx, gx2), (gw, gw2), (gas, gas2), (gad, gad2)):
        assert torch.equal(a, b)
    g.close()
    gt.close()


def test_gatconv_backward_rejects_unsupported_head_width(gnn):
    wl = synth.config4_gat(num_nodes=300, num_edges=2000, f_in=6, heads=2, ch=65, cap=100.0)   # a head wider than a wavefront
    p, n = wl.params, wl.num_nodes
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), n)
    gt = gnn.build_csr(dev(wl.dst), dev(wl.src), n)
    stats = torch.empty((n, 2, 2), dtype=torch.float32, device="cuda")
    args = (dev(wl.x), dev(p["w"]), dev(p["a_src"]), dev(p["a_dst"]))
    out = gnn.gatconv(g, *args, 0.2, softmax_stats=stats)
    with pytest.raises(RuntimeError):
        gnn.gatconv_backward(g, gt, *args, out, stats, torch.ones_like(out), 0.2)
    g.close()
    gt.close()


@pytest.mark.parametrize("heads", [1, 8, 3])
def test_segment_softmax_backward(case, gnn, heads):
    name, wl, g = case
    e = wl.num_edges
    s = (3.0 * synth.normal_f32(61 + heads, 2, e * heads)).reshape(e, heads)
    galpha = synth.normal_f32(61 + heads, 3, e * heads).reshape(e, heads)
    alpha = oracle.segment_softmax(wl.dst, wl.num_nodes, s)
    ref, sabs = oracle.segment_softmax_backward(wl.dst, wl.num_nodes, alpha, galpha, with_sabs=True)
    got = host(gnn.segment_softmax_backward(g, dev(alpha), dev(galpha)))
    assert_close_sabs(got, ref, sabs, what=f"softmax backward {name} H={heads}")
    _, _, perm, _ = oracle.build_csr(wl.src, wl.dst, wl.num_nodes)
    got_csr = host(gnn.segment_softmax_backward(g, dev(alpha[perm]), dev(galpha[perm]), order=gnn.EDGE_ORDER_CSR))
    np.testing.assert_array_equal(got_csr, got[perm])
    # a gradient that is constant over every segment is annihilated
    per_seg = synth.normal_f32(5, 4, wl.num_nodes * heads).reshape(wl.num_nodes, heads)[wl.dst]
    zero = host(gnn.segment_softmax_backward(g, dev(alpha), dev(np.ascontiguousarray(per_seg))))
    assert np.abs(zero).max() <= 2e-6


def test_segment_softmax_many_heads(gnn):
    wl = powerlaw(2000, 30_000, 4, 1500.0)
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), wl.num_nodes, 4, 64)
    # 70 and 300 take the one-head-per-lane kernels, 300 with more head groups per edge than a block has threads;
    # 1028 the same in the four-heads-per-lane kernels; 3 leaves threads of the element-wise blocks idle.
    for heads in (2, 3, 16, 70, 300, 1028):
        E = wl.num_edges if heads <= 70 else 3000
        gg = g if heads <= 70 else gnn.build_csr(dev(wl.src[:E]), dev(wl.dst[:E]), wl.num_nodes, 4, 64)
        dst = wl.dst[:E]
        s = (2.0 * synth.normal_f32(heads, 2, E * heads)).reshape(E, heads)
        ref = oracle.segment_softmax(dst, wl.num_nodes, s)
        assert_close_rel(host(gnn.segment_softmax(gg, dev(s))), ref, what=f"softmax H={heads}")
        galpha = synth.normal_f32(heads, 3, E * heads).reshape(E, heads)
        alpha = ref.astype(np.float32)
        refb, sabs = oracle.segment_softmax_backward(dst, wl.num_nodes, alpha, galpha, with_sabs=True)
        assert_close_sabs(host(gnn.segment_softmax_backward(gg, dev(alpha), dev(galpha))), refb, sabs,
                          what=f"softmax backward H={heads}")
        if gg is not g:
            gg.close()
    g.close()


def test_propagate_feature_width_one(gnn):
    wl = powerlaw(1500, 20_000, 1, 900.0)
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), wl.num_nodes, 4, 64)
    for msg, e in ((MSG_COPY_XJ, None), (MSG_E_MUL_XJ, wl.edge_weight)):
        for aggr in (AGGR_SUM, AGGR_MEAN, AGGR_MAX):
            ref, sabs = oracle.propagate(wl.src, wl.dst, wl.num_nodes, wl.x, e, msg, aggr, with_sabs=True)
            got = host(gnn.propagate(g, dev(wl.x), dev(e) if e is not None else None, msg, aggr))
            if aggr == AGGR_MAX:
                np.testing.assert_array_equal(got.view(np.uint32), ref.view(np.uint32))
            else:
                assert_close_sabs(got, ref, sabs, what=f"F=1 msg={msg} aggr={aggr}")
    g.close()


def test_gin_and_pool_batched(gnn):
    wl = synth.config3_batched()
    n, ng = wl.num_nodes, wl.num_graphs
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), n)
    for eps in (0.0, 0.25):
        ref, sabs = oracle.gin_update(wl.src, wl.dst, n, wl.x, eps, with_sabs=True)
        got = gnn.gin_update(g, dev(wl.x), eps)
        assert_close_sabs(host(got), ref, sabs, what=f"gin eps={eps}")
    gi = dev(wl.graph_indicator)
    upd = gnn.gin_update(g, dev(wl.x), 0.0)
    upd_h = host(upd)
    for aggr in (AGGR_SUM, AGGR_MEAN, AGGR_MAX):
        ref, sabs = oracle.graph_pool(wl.graph_indicator, ng, upd_h, aggr, with_sabs=True)
        got = host(gnn.graph_pool(gi, ng, upd, aggr))
        if aggr == AGGR_MAX:
            np.testing.assert_array_equal(got.view(np.uint32), ref.view(np.uint32))
        else:
            assert_close_sabs(got, ref, sabs, what=f"pool aggr={aggr}")
    ones = dev(np.ones((n, 32), np.float32))
    np.testing.assert_array_equal(host(gnn.graph_pool(gi, ng, ones))[:, 0], np.bincount(wl.graph_indicator, minlength=ng))
    np.testing.assert_array_equal(host(gnn.gin_update(g, ones, 0.0))[:, 0], 1.0 + np.bincount(wl.dst, minlength=n))
    # more graph ids than graphs present: trailing empty graphs give zero rows; odd feature width
    x7 = synth.normal_f32(4, 2, n * 7).reshape(n, 7)
    ref = oracle.graph_pool(wl.graph_indicator, ng + 3, x7, AGGR_MEAN)
    got = host(gnn.graph_pool(gi, ng + 3, dev(x7), AGGR_MEAN))
    np.testing.assert_allclose(got, ref, rtol=1e-5, atol=1e-6)
    assert (got[ng:] == 0).all()
    # wide and single-column features on the same small graphs (several feature passes per wavefront; 64 node slots)
    for f in (200, 1):
        xf = synth.normal_f32(5, f, n * f).reshape(n, f)
        for aggr in (AGGR_SUM, AGGR_MEAN, AGGR_MAX):
            ref, sabs = oracle.graph_pool(wl.graph_indicator, ng, xf, aggr, with_sabs=True)
            got = host(gnn.graph_pool(gi, ng, dev(xf), aggr))
            if aggr == AGGR_MAX:
                np.testing.assert_array_equal(got, ref)
            else:
                assert_close_sabs(got, ref, sabs, what=f"pool F={f} aggr={aggr}")
    g.close()


def test_pool_one_big_graph(gnn):
    n, f = 50_000, 48
    x = synth.normal_f32(6, 2, n * f).reshape(n, f)
    gi = np.zeros(n, np.int32)
    gi[n // 2:] = 2          # graph 1 is empty
    for aggr in (AGGR_SUM, AGGR_MEAN, AGGR_MAX):
        ref, sabs = oracle.graph_pool(gi, 3, x, aggr, with_sabs=True)
        got = host(gnn.graph_pool(dev(gi), 3, dev(x), aggr))
        if aggr == AGGR_MAX:
            np.testing.assert_array_equal(got, ref)
        else:
            assert_close_sabs(got, ref, sabs, what=f"big pool aggr={aggr}")


@pytest.mark.parametrize("n,f,bounds", [
    (300_000, 64, [0, 300_000]),                      # one graph that is the whole node set
    (400_000, 48, [0, 250_000, 250_000, 399_999, 400_000]),   # a large, an empty, a large and a one-node graph
    (70_000, 5, [0, 3, 70_000]),                      # a graph smaller than the number of its parts
    (40_000, 32, [0, 20_000, 40_000]),                # too small for parts: the plain path, no workspace needed
])
def test_pool_with_workspace_few_large_graphs(gnn, n, f, bounds):
    """gnn_graph_pool_ws: several blocks per graph, parts combined in a fixed order; against the oracle, and
    bit-identical from run to run.  Max equals gnn_graph_pool bit for bit."""
    ng = len(bounds) - 1
    x = synth.normal_f32(60 + f, 2, n * f).reshape(n, f)
    gi = np.zeros(n, np.int32)
    for g_ in range(ng):
        gi[bounds[g_]:bounds[g_ + 1]] = g_
    gid, xd = dev(gi), dev(x)
    need = int(gnn.lib().gnn_graph_pool_workspace_bytes(n, ng, f))
    assert (need > 0) == (n >= 8192 * ng)
    for aggr in (AGGR_SUM, AGGR_MEAN, AGGR_MAX):
        ref, sabs = oracle.graph_pool(gi, ng, x, aggr, with_sabs=True)
        got = gnn.graph_pool_ws(gid, ng, xd, aggr)
        again = gnn.graph_pool_ws(gid, ng, xd, aggr)
        assert torch.equal(got, again)
        if aggr == AGGR_MAX:
            np.testing.assert_array_equal(host(got), ref)
            assert torch.equal(got, gnn.graph_pool(gid, ng, xd, aggr))
        else:
            assert_close_sabs(host(got), ref, sabs, what=f"pool with workspace aggr={aggr}")
    if need:
        out = torch.empty((ng, f), dtype=torch.float32, device="cuda")
        small = torch.empty(need - 256, dtype=torch.uint8, device="cuda")
        rc = gnn.lib().gnn_graph_pool_ws(gid.data_ptr(), n, ng, xd.data_ptr(), f, AGGR_SUM, out.data_ptr(),
                                         small.data_ptr(), small.numel(), None)
        assert rc == 2      # workspace too small
        rc = gnn.lib().gnn_graph_pool_ws(gid.data_ptr(), n, ng, xd.data_ptr(), f, AGGR_SUM, out.data_ptr(), None, 0, None)
        assert rc == 1      # no workspace


def test_buffers_that_are_not_16_byte_aligned(gnn):
    """Every float buffer starts 4 bytes past a 16-byte boundary (feature widths that would otherwise take the
    128-bit paths): the calls fall back to their scalar paths and give the oracle's results."""
    wl = powerlaw(3000, 60_000, 32, 900.0)
    n, e, f = wl.num_nodes, wl.num_edges, 32
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), n, 8, 128)
    gt = gnn.build_csr(dev(wl.dst), dev(wl.src), n, 8, 128)

    def off(a):   # a device copy of `a` whose first element lies 4 bytes past a 16-byte boundary
        a = np.ascontiguousarray(a, dtype=np.float32)
        buf = torch.empty(a.size + 1, dtype=torch.float32, device="cuda")
        view = buf[1:].view(a.shape)
        view.copy_(torch.from_numpy(a))
        assert view.data_ptr() % 16 == 4
        return view

    def off_out(*shape):
        return torch.empty(int(np.prod(shape)) + 1, dtype=torch.float32, device="cuda")[1:].view(shape)

    w_e = synth.uniform_f32(901, 3, e, 0.0, 1.0)
    x_d, e_d = off(wl.x), off(w_e)
    for msg, aggr in ((MSG_COPY_XJ, AGGR_SUM), (MSG_E_MUL_XJ, AGGR_MEAN), (MSG_E_MUL_XJ, AGGR_MAX)):
        ref, sabs = oracle.propagate(wl.src, wl.dst, n, wl.x, w_e if msg else None, msg, aggr, with_sabs=True)
        got = host(gnn.propagate(g, x_d, e_d if msg else None, msg, aggr, out=off_out(n, f)))
        if aggr == AGGR_MAX:
            np.testing.assert_array_equal(got.view(np.uint32), ref.view(np.uint32))
        else:
            assert_close_sabs(got, ref, sabs, what=f"unaligned propagate {msg} {aggr}")
    gout = synth.normal_f32(902, 2, n * f).reshape(n, f)
    back = oracle.propagate_backward(wl.src, wl.dst, n, wl.x, gout, w_e, MSG_E_MUL_XJ, AGGR_SUM, with_sabs=True)
    gx, ge = gnn.propagate_backward(g, gt, x_d, off(gout), e_d, MSG_E_MUL_XJ, AGGR_SUM)
    assert_close_sabs(host(gx), back["grad_x"], back["sabs_x"], what="unaligned grad_x")
    assert_close_sabs(host(ge).reshape(-1, 1), back["grad_e"], back["sabs_e"], what="unaligned grad_e")
    # dense projection and the GCN layer
    wgt = synth.glorot_uniform(903, 3, f, 64, (f, 64))
    bias = synth.uniform_f32(904, 3, 64, -0.5, 0.5)
    ref = oracle.dense(wl.x, wgt, None, False)
    assert_close_sabs(host(gnn.dense_xw(x_d, off(wgt), out=off_out(n, 64))), ref,
                      np.abs(wl.x.astype(np.float64)) @ np.abs(wgt.astype(np.float64)), what="unaligned dense")
    ref, sabs = oracle.gcnconv(wl.src, wl.dst, n, wl.x, wgt, bias, True, with_sabs=True)
    assert_close_sabs(host(gnn.gcnconv(g, x_d, off(wgt), off(bias), True, out=off_out(n, 64))), ref, sabs, what="unaligned gcnconv")
    # segment softmax, attention layer, pooling
    heads, ch = 4, 8
    scores = (2.0 * synth.normal_f32(905, 2, e * heads)).reshape(e, heads)
    assert_close_rel(host(gnn.segment_softmax(g, off(scores), out=off_out(e, heads))), oracle.segment_softmax(wl.dst, n, scores),
                     what="unaligned softmax")
    wg = synth.glorot_uniform(906, 3, f, heads * ch, (f, heads * ch))
    a_s = synth.uniform_f32(907, 4, heads * ch, -0.8, 0.8).reshape(heads, ch)
    a_d = synth.uniform_f32(908, 4, heads * ch, -0.8, 0.8).reshape(heads, ch)
    ref, sabs = oracle.gatconv(wl.src, wl.dst, n, wl.x, wg, a_s, a_d, 0.2, with_sabs=True)
    got = gnn.gatconv(g, x_d, off(wg), off(a_s), off(a_d), 0.2, out=off_out(n, heads * ch))
    assert_close_sabs(host(got), ref, sabs, what="unaligned gatconv")
    # backward of the GCN layer and of the attention layer with unaligned inputs (outputs come from the binding)
    g64 = synth.normal_f32(910, 2, n * 64).reshape(n, 64)
    rb = oracle.gcnconv_backward(wl.src, wl.dst, n, wl.x, wgt, g64, True)
    bx, bw, bb = gnn.gcnconv_backward(g, gt, x_d, off(wgt), off(g64), True)
    assert_close_sabs(host(bx), rb["grad_x"], rb["sabs_x"], what="unaligned gcn grad_x")
    assert_close_sabs(host(bw), rb["grad_w"], rb["sabs_w"], what="unaligned gcn grad_w")
    assert_close_sabs(host(bb), rb["grad_b"], rb["sabs_b"], what="unaligned gcn grad_b")
    # (slope 1: the leaky ReLU has no kink, so no pre-activation can sit on the wrong side of it in float)
    stats = torch.empty(n * heads * 2 + 1, dtype=torch.float32, device="cuda")[1:].view(n, heads, 2)
    out_u = gnn.gatconv(g, x_d, off(wg), off(a_s), off(a_d), 1.0, out=off_out(n, heads * ch), softmax_stats=stats)
    gg = synth.normal_f32(911, 2, n * heads * ch).reshape(n, heads * ch)
    rg = oracle.gatconv_backward(wl.src, wl.dst, n, wl.x, wg, a_s, a_d, gg, 1.0)
    ax, aw, aas, aad = gnn.gatconv_backward(g, gt, x_d, off(wg), off(a_s), off(a_d), out_u, stats, off(gg), 1.0)
    assert_close_sabs(host(ax), rg["grad_x"], rg["sabs_x"], what="unaligned gat grad_x")
    assert_close_sabs(host(aw), rg["grad_w"], rg["sabs_w"], what="unaligned gat grad_w")
    assert_close_sabs(host(aas), rg["grad_a_src"], rg["sabs_a_src"], what="unaligned gat grad_a_src")
    # with slope 1 the destination half of a score cancels in the softmax: this gradient is exactly zero, the
    # computed one is rounding noise of its terms
    assert (np.abs(host(aad).astype(np.float64)) <= 1e-5 * rg["sabs_a_dst"]).all()
    gi = np.sort(synth.randint(909, 1, 0, n, 0, 39)).astype(np.int32)
    for aggr in (AGGR_SUM, AGGR_MAX):
        ref, sabs = oracle.graph_pool(gi, 40, wl.x, aggr, with_sabs=True)
        got = host(gnn.graph_pool(dev(gi), 40, x_d, aggr, out=off_out(40, f)))
        if aggr == AGGR_MAX:
            np.testing.assert_array_equal(got, ref)
        else:
            assert_close_sabs(got, ref, sabs, what="unaligned pool")
    g.close()
    gt.close()


@pytest.mark.parametrize("shape", ["in_star", "out_star", "one_pair"])
def test_star_graphs(gnn, shape):
    """One row with every edge (1 172 wavefront pieces at the smallest piece length) / one source gathered by every
    edge / one edge repeated 300 000 times: propagate, segment softmax, the attention layer and the backward passes against the oracle."""
    n, e, f, heads, ch = 4000, 300_000, 16, 2, 8
    other = synth.randint(321, 1, 0, e, 0, n - 1).astype(np.int32)
    hub = np.full(e, 7, np.int32)
    if shape == "one_pair":      # the same edge 300 000 times
        other = np.full(e, 3, np.int32)
    src, dst = (hub, other) if shape == "out_star" else (other, hub)
    x = synth.normal_f32(322, 2, n * f).reshape(n, f)
    w_e = synth.uniform_f32(323, 3, e, 0.0, 1.0)
    gout = synth.normal_f32(324, 2, n * f).reshape(n, f)
    g = gnn.build_csr(dev(src), dev(dst), n, 16, 256)
    gt = gnn.build_csr(dev(dst), dev(src), n, 16, 256)
    rowptr, colidx, perm, _ = oracle.build_csr(src, dst, n)
    np.testing.assert_array_equal(host(g.rowptr), rowptr)
    np.testing.assert_array_equal(host(g.perm), perm)
    xd, wd = dev(x), dev(w_e)
    for msg, aggr in ((MSG_COPY_XJ, AGGR_SUM), (MSG_E_MUL_XJ, AGGR_MEAN), (MSG_E_MUL_XJ, AGGR_MAX), (MSG_COPY_XJ, AGGR_MIN)):
        ref, sabs = oracle.propagate(src, dst, n, x, w_e if msg else None, msg, aggr, with_sabs=True)
        got = host(gnn.propagate(g, xd, wd if msg else None, msg, aggr))
        if aggr in (AGGR_MAX, AGGR_MIN):
            np.testing.assert_array_equal(got.view(np.uint32), ref.view(np.uint32))
        else:
            assert_close_sabs(got, ref, sabs, what=f"{shape} propagate {msg} {aggr}")
    back = oracle.propagate_backward(src, dst, n, x, gout, w_e, MSG_E_MUL_XJ, AGGR_SUM, with_sabs=True)
    gx, ge = gnn.propagate_backward(g, gt, xd, dev(gout), wd, MSG_E_MUL_XJ, AGGR_SUM)
    assert_close_sabs(host(gx), back["grad_x"], back["sabs_x"], what=f"{shape} grad_x")
    assert_close_sabs(host(ge).reshape(-1, 1), back["grad_e"], back["sabs_e"], what=f"{shape} grad_e")
    scores = (2.0 * synth.normal_f32(325, 2, e * heads)).reshape(e, heads)
    g.reserve(0, heads)
    assert_close_rel(host(gnn.segment_softmax(g, dev(scores))), oracle.segment_softmax(dst, n, scores), what=f"{shape} softmax")
    wgt = synth.glorot_uniform(326, 3, f, heads * ch, (f, heads * ch))
    a_s = synth.uniform_f32(327, 4, heads * ch, -0.8, 0.8).reshape(heads, ch)
    a_d = synth.uniform_f32(328, 4, heads * ch, -0.8, 0.8).reshape(heads, ch)
    ref, sabs = oracle.gatconv(src, dst, n, x, wgt, a_s, a_d, 0.2, with_sabs=True)
    stats = torch.empty((n, heads, 2), dtype=torch.float32, device="cuda")
    out = gnn.gatconv(g, xd, dev(wgt), dev(a_s), dev(a_d), 0.2, softmax_stats=stats)
    assert_close_sabs(host(out), ref, sabs, what=f"{shape} gatconv")
    g.close()
    gt.close()


def test_degenerate_graphs_through_every_entry_point(gnn):
    """No edges at all, a single node, a single self-loop: every entry point returns what the oracle
    returns (zeros for empty neighbourhoods, no fault, no stale memory)."""
    f = 8
    for n, src, dst in ((5, np.zeros(0, np.int32), np.zeros(0, np.int32)),
                        (1, np.zeros(0, np.int32), np.zeros(0, np.int32)),
                        (1, np.zeros(1, np.int32), np.zeros(1, np.int32)),
                        (3, np.array([2], np.int32), np.array([2], np.int32))):
        ne = src.shape[0]
        x = synth.normal_f32(7 + n, 2, n * f).reshape(n, f)
        w = synth.glorot_uniform(7, 3, f, f, (f, f))
        g = gnn.build_csr(dev(src), dev(dst), n)
        gt = gnn.build_csr(dev(dst), dev(src), n)
        e = synth.uniform_f32(7, 4, max(ne, 1))[:ne]
        de = dev(e) if ne else torch.zeros(0, dtype=torch.float32, device="cuda")
        for msg in (MSG_COPY_XJ, MSG_E_MUL_XJ, MSG_XJ_SUB_XI):
            for aggr in (AGGR_SUM, AGGR_MEAN, AGGR_MAX, AGGR_MIN, AGGR_PROD):
                ed = e if msg == MSG_E_MUL_XJ else None
                ref = oracle.propagate(src, dst, n, x, ed, msg, aggr)
                got = host(gnn.propagate(g, dev(x), de if msg == MSG_E_MUL_XJ else None, msg, aggr))
                np.testing.assert_allclose(got, ref, rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(host(gnn.gcnconv(g, dev(x), dev(w), None, True)),
                                   oracle.gcnconv(src, dst, n, x, w, None, True), rtol=1e-5, atol=1e-6)
        np.testing.assert_allclose(host(gnn.gcnconv(g, dev(x), dev(w), None, False)),
                                   oracle.gcnconv(src, dst, n, x, w, None, False), rtol=1e-5, atol=1e-6)
        np.testing.assert_allclose(host(gnn.gin_update(g, dev(x), 0.5)), oracle.gin_update(src, dst, n, x, 0.5),
                                   rtol=1e-6, atol=1e-7)
        gout = synth.normal_f32(7, 5, n * f).reshape(n, f)
        ref = oracle.propagate_backward(src, dst, n, x, gout, e if ne else np.zeros(0, np.float32), MSG_E_MUL_XJ, AGGR_SUM)
        gx, ge = gnn.propagate_backward(g, gt, dev(x), dev(gout), de, MSG_E_MUL_XJ, AGGR_SUM)
        np.testing.assert_allclose(host(gx), ref["grad_x"], rtol=1e-6, atol=1e-7)
        if ne:
            np.testing.assert_allclose(host(ge).reshape(-1), ref["grad_e"].reshape(-1), rtol=1e-5, atol=1e-6)
        rb = oracle.gcnconv_backward(src, dst, n, x, w, gout, True)
        bx, bw, bb = gnn.gcnconv_backward(g, gt, dev(x), dev(w), dev(gout), True)
        np.testing.assert_allclose(host(bx), rb["grad_x"], rtol=1e-5, atol=1e-6)
        np.testing.assert_allclose(host(bw), rb["grad_w"], rtol=1e-5, atol=1e-6)
        np.testing.assert_allclose(host(bb), rb["grad_b"], rtol=1e-5, atol=1e-6)
        heads, ch = 2, 4
        a_s = synth.uniform_f32(7, 6, heads * ch, -1, 1).reshape(heads, ch)
        a_d = synth.uniform_f32(7, 8, heads * ch, -1, 1).reshape(heads, ch)
        stats = torch.empty((n, heads, 2), dtype=torch.float32, device="cuda")
        out = gnn.gatconv(g, dev(x), dev(w), dev(a_s), dev(a_d), 0.2, softmax_stats=stats)
        np.testing.assert_allclose(host(out), oracle.gatconv(src, dst, n, x, w, a_s, a_d, 0.2), rtol=1e-5, atol=1e-6)
        rg = oracle.gatconv_backward(src, dst, n, x, w, a_s, a_d, gout, 0.2)
        got = gnn.gatconv_backward(g, gt, dev(x), dev(w), dev(a_s), dev(a_d), out, stats, dev(gout), 0.2)
        for t, k in zip(got, ("grad_x", "grad_w", "grad_a_src", "grad_a_dst")):
            np.testing.assert_allclose(host(t), rg[k], rtol=1e-4, atol=1e-5, err_msg=k)
        if ne:
            sc = synth.normal_f32(7, 9, ne * heads).reshape(ne, heads)
            al = gnn.segment_softmax(g, dev(sc))
            np.testing.assert_allclose(host(al), oracle.segment_softmax(dst, n, sc), rtol=1e-6)
            ga = synth.normal_f32(7, 10, ne * heads).reshape(ne, heads)
            np.testing.assert_allclose(host(gnn.segment_softmax_backward(g, al, dev(ga))),
                                       oracle.segment_softmax_backward(dst, n, host(al), ga), rtol=1e-5, atol=1e-6)
        g.close()
        gt.close()

