"""GPU tests of the two-pass route for one float per edge (gnn_graph_build_edge_route): the permutation into CSR
order and back is bit-exact against e[perm] with perm from the CPU oracle, and the compute calls that take the
route give what they give without it."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from oracle import AGGR_MEAN, AGGR_SUM, MSG_E_MUL_XJ
from paper_2412_06354_amd import synth
from util import assert_close_rel, assert_close_sabs

pytestmark = pytest.mark.gpu

TILE = 16384   # entries per tile / bucket of the route


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


def edge_values(count, seed):
    return synth.uniform_f32(seed, 2, count, -1.0, 1.0)


@pytest.mark.parametrize("num_nodes,num_edges", [
    (3, 1), (7, 5), (50, 1000), (300, TILE - 1), (300, TILE), (300, TILE + 1), (1000, 3 * TILE + 5),
    (20_000, 8 * TILE), (100_000, 1_000_003),
])
def test_route_is_the_permutation(gnn, num_nodes, num_edges):
    src, dst = synth.multigraph_uniform(num_nodes, num_edges, seed=900 + num_edges % 97)
    _, _, perm, _ = oracle.build_csr(src, dst, num_nodes)
    e = edge_values(num_edges, 11)
    g = gnn.build_csr(dev(src), dev(dst), num_nodes)
    e_d = dev(e)
    # the direct kernels
    direct = gnn.edge_data_to_csr(g, e_d)
    np.testing.assert_array_equal(host(direct), e[perm])
    np.testing.assert_array_equal(host(gnn.edge_data_to_coo(g, direct)), e)
    # the same two calls through the route, twice (the route's buffers are reused)
    g.build_edge_route()
    g.build_edge_route()
    for _ in range(2):
        routed = gnn.edge_data_to_csr(g, e_d)
        np.testing.assert_array_equal(host(routed), e[perm])
        np.testing.assert_array_equal(host(gnn.edge_data_to_coo(g, routed)), e)
    # wider records keep the direct path and stay correct on a graph that has a route
    e3 = edge_values(3 * num_edges, 12).reshape(num_edges, 3)
    wide = gnn.edge_data_to_csr(g, dev(e3))
    np.testing.assert_array_equal(host(wide), e3[perm])
    np.testing.assert_array_equal(host(gnn.edge_data_to_coo(g, wide)), e3)
    # buffers that are not 16-byte aligned keep the direct path
    if num_edges > 4:
        pad = torch.empty(num_edges + 1, dtype=torch.float32, device="cuda")
        pad[1:] = e_d
        np.testing.assert_array_equal(host(gnn.edge_data_to_csr(g, pad[1:])), e[perm])


def test_route_on_a_hub_graph_and_an_empty_one(gnn):
    wl = synth.config2_weighted(num_nodes=20_000, num_edges=300_000, feat=16, cap=6000.0)
    _, _, perm, _ = oracle.build_csr(wl.src, wl.dst, wl.num_nodes)
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), wl.num_nodes)
    g.build_edge_route()
    e = edge_values(wl.num_edges, 13)
    routed = gnn.edge_data_to_csr(g, dev(e))
    np.testing.assert_array_equal(host(routed), e[perm])
    np.testing.assert_array_equal(host(gnn.edge_data_to_coo(g, routed)), e)

    none = np.zeros(0, np.int32)
    g0 = gnn.build_csr(dev(none), dev(none), 5)
    g0.build_edge_route()
    assert gnn.edge_data_to_csr(g0, dev(np.zeros(0, np.float32))).numel() == 0


@pytest.mark.parametrize("aggr", [AGGR_SUM, AGGR_MEAN])
def test_compute_calls_take_the_route(gnn, aggr):
    """propagate(e_mul_xj) with COO-ordered weights and its backward, with and without a route: identical bits
    (the route only moves values), and both at the oracle's bar."""
    wl = synth.config2_weighted(num_nodes=20_000, num_edges=300_000, feat=32, cap=6000.0)
    n, f = wl.num_nodes, 32
    x = synth.normal_f32(77, 2, n * f).reshape(n, f)
    grad_out = synth.normal_f32(78, 2, n * f).reshape(n, f)
    e = np.ascontiguousarray(wl.edge_weight, dtype=np.float32).reshape(-1)
    src_d, dst_d, x_d, e_d, go_d = dev(wl.src), dev(wl.dst), dev(x), dev(e), dev(grad_out)

    plain = gnn.build_csr(src_d, dst_d, n)
    plain_t = gnn.build_csr(dst_d, src_d, n)
    out_plain = gnn.propagate(plain, x_d, e_d, MSG_E_MUL_XJ, aggr)
    gx_plain, ge_plain = gnn.propagate_backward(plain, plain_t, x_d, go_d, e_d, MSG_E_MUL_XJ, aggr)

    routed = gnn.build_csr(src_d, dst_d, n)
    routed_t = gnn.build_csr(dst_d, src_d, n)
    routed.build_edge_route()
    routed_t.build_edge_route()
    out_routed = gnn.propagate(routed, x_d, e_d, MSG_E_MUL_XJ, aggr)
    gx_routed, ge_routed = gnn.propagate_backward(routed, routed_t, x_d, go_d, e_d, MSG_E_MUL_XJ, aggr)
    # the caller's weights are untouched and a second call gives the same
    np.testing.assert_array_equal(host(e_d), e)
    np.testing.assert_array_equal(host(gnn.propagate(routed, x_d, e_d, MSG_E_MUL_XJ, aggr)), host(out_routed))

    if aggr == AGGR_SUM:   # the un-fused message tensor (rounded products: bit-exact against the oracle)
        m_ref = oracle.apply_edges(wl.src, n, x, e, MSG_E_MUL_XJ)
        np.testing.assert_array_equal(host(gnn.apply_edges(routed, x_d, e_d, MSG_E_MUL_XJ)), m_ref)
        np.testing.assert_array_equal(host(gnn.apply_edges(plain, x_d, e_d, MSG_E_MUL_XJ)), m_ref)
        # one dot product per edge: the same bits with and without a route, the oracle's value within its bar
        from oracle import MSG_XI_DOT_XJ
        d_ref, d_sabs = oracle.apply_edges(wl.src, n, x, None, MSG_XI_DOT_XJ, dst=wl.dst, with_sabs=True)
        d_routed = gnn.apply_edges(routed, x_d, None, MSG_XI_DOT_XJ)
        assert torch.equal(d_routed, gnn.apply_edges(plain, x_d, None, MSG_XI_DOT_XJ))
        assert_close_sabs(host(d_routed).reshape(-1, 1), d_ref, d_sabs, what="routed edge dot")
    np.testing.assert_array_equal(host(out_routed), host(out_plain))
    np.testing.assert_array_equal(host(gx_routed), host(gx_plain))
    np.testing.assert_array_equal(host(ge_routed), host(ge_plain))

    ref, sabs = oracle.propagate(wl.src, wl.dst, n, x, e, MSG_E_MUL_XJ, aggr, with_sabs=True)
    assert_close_sabs(host(out_routed), ref, sabs, what="routed propagate")
    back = oracle.propagate_backward(wl.src, wl.dst, n, x, grad_out, e, MSG_E_MUL_XJ, aggr, with_sabs=True)
    assert_close_sabs(host(gx_routed), back["grad_x"], back["sabs_x"], what="routed grad_x")
    assert_close_sabs(host(ge_routed).reshape(-1, 1), back["grad_e"], back["sabs_e"], what="routed grad_e")


def test_single_head_softmax_takes_the_route(gnn):
    """Segment softmax with one score per edge in COO order, forward and backward: the same bits with and without
    a route (the CSR-ordered kernels run on the moved scores), the oracle's values at its bar, inputs untouched."""
    wl = synth.config2_weighted(num_nodes=20_000, num_edges=300_000, feat=4, cap=6000.0)
    n, e = wl.num_nodes, wl.num_edges
    scores = (3.0 * synth.normal_f32(91, 2, e)).reshape(e, 1)
    dalpha = synth.normal_f32(92, 2, e).reshape(e, 1)
    src_d, dst_d = dev(wl.src), dev(wl.dst)
    plain, routed = gnn.build_csr(src_d, dst_d, n), gnn.build_csr(src_d, dst_d, n)
    routed.build_edge_route()
    s_d, da_d = dev(scores), dev(dalpha)
    a_plain, a_routed = gnn.segment_softmax(plain, s_d), gnn.segment_softmax(routed, s_d)
    assert torch.equal(a_plain, a_routed)
    np.testing.assert_array_equal(host(s_d), scores)
    assert_close_rel(host(a_routed), oracle.segment_softmax(wl.dst, n, scores), what="routed softmax")
    g_plain = gnn.segment_softmax_backward(plain, a_plain, da_d)
    g_routed = gnn.segment_softmax_backward(routed, a_routed, da_d)
    assert torch.equal(g_plain, g_routed)
    np.testing.assert_array_equal(host(da_d), dalpha)
    assert torch.equal(a_routed, a_plain)
    # several heads keep the direct path on a graph with a route
    s8 = (3.0 * synth.normal_f32(93, 2, e * 8)).reshape(e, 8)
    assert torch.equal(gnn.segment_softmax(routed, dev(s8)), gnn.segment_softmax(plain, dev(s8)))


def test_routed_calls_can_be_captured(gnn):
    """Calls that take the route only enqueue kernels: propagate with COO-ordered weights, its backward and the
    single-head softmax are recorded into one HIP graph; every replay (with eager work on the same handles in
    between) reproduces the eager results bit for bit."""
    wl = synth.config2_weighted(num_nodes=20_000, num_edges=300_000, feat=32, cap=6000.0)
    n, e, f = wl.num_nodes, wl.num_edges, 32
    x = dev(synth.normal_f32(81, 2, n * f).reshape(n, f))
    gout = dev(synth.normal_f32(82, 2, n * f).reshape(n, f))
    w = dev(np.ascontiguousarray(wl.edge_weight, dtype=np.float32).reshape(-1))
    scores = dev((2.0 * synth.normal_f32(83, 2, e)).reshape(e, 1))
    src_d, dst_d = dev(wl.src), dev(wl.dst)
    g, gt = gnn.build_csr(src_d, dst_d, n), gnn.build_csr(dst_d, src_d, n)
    g.build_edge_route()
    gt.build_edge_route()
    g.reserve(0, 1)
    ws = torch.empty(max(int(gnn.lib().gnn_propagate_backward_workspace_bytes(n, f, AGGR_SUM)), 16), dtype=torch.uint8,
                     device="cuda")
    out = torch.empty((n, f), dtype=torch.float32, device="cuda")
    gx, ge = torch.empty_like(out), torch.empty_like(w)
    alpha = torch.empty_like(scores)
    lib = gnn.lib()

    def calls():
        st = torch.cuda.current_stream().cuda_stream
        assert lib.gnn_propagate(g._h, x.data_ptr(), f, w.data_ptr(), 1, 0, MSG_E_MUL_XJ, AGGR_SUM, out.data_ptr(), st) == 0
        assert lib.gnn_propagate_backward(g._h, gt._h, x.data_ptr(), f, w.data_ptr(), 1, MSG_E_MUL_XJ, AGGR_SUM,
                                          gout.data_ptr(), None, gx.data_ptr(), ge.data_ptr(), ws.data_ptr(), ws.numel(),
                                          st) == 0
        assert lib.gnn_segment_softmax(g._h, scores.data_ptr(), 1, 0, alpha.data_ptr(), st) == 0

    calls()
    torch.cuda.synchronize()
    eager = [t.clone() for t in (out, gx, ge, alpha)]
    gph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gph):
        calls()
    for it in range(3):
        for t in (out, gx, ge, alpha):
            t.fill_(float("nan"))
        gph.replay()
        torch.cuda.synchronize()
        for got, want in zip((out, gx, ge, alpha), eager):
            assert torch.equal(got, want), f"replay {it}"
        gnn.edge_data_to_csr(g, w)      # eager use of the route's buffers between replays
        torch.cuda.synchronize()
    del gph
    g.close()
    gt.close()
