"""gnn_propagate_noalloc (the entry point for callers that cannot allocate) against gnn_propagate through the
C ABI: same kernels, so bit-identical results; two calls in a row share the library's fixed scratch array, the
second on a smaller graph."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2412_06354_amd import synth

pytestmark = pytest.mark.gpu

MSG_COPY_XJ, MSG_E_MUL_XJ = 0, 1
AGGR_SUM, AGGR_MEAN, AGGR_MAX = 0, 1, 2
ERR_SCRATCH_LIMIT = 9


@pytest.fixture(scope="module")
def gnn():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2412_06354_amd import binding
    binding.lib()
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def test_noalloc_matches_propagate_on_two_calls_in_a_row(gnn):
    big = synth.config2_weighted(num_nodes=30_000, num_edges=600_000, feat=64, cap=9000.0)
    small = synth.config2_weighted(num_nodes=5_000, num_edges=120_000, feat=64, cap=3000.0)
    cases = []
    for wl, small_max, chunk in ((big, 0, 0), (small, 4, 64)):
        g = gnn.build_csr(dev(wl.src), dev(wl.dst), wl.num_nodes, small_max, chunk)
        assert g.work_sizes()["split_rows"] > 0            # the scratch array is really used
        cases.append((wl, g, dev(wl.x), dev(wl.edge_weight)))
    for msg, aggr in ((MSG_COPY_XJ, AGGR_SUM), (MSG_E_MUL_XJ, AGGR_MEAN), (MSG_E_MUL_XJ, AGGR_MAX)):
        for wl, g, x, e in cases:                          # the larger graph first, then the smaller one
            want = gnn.propagate(g, x, e if msg else None, msg, aggr)
            out = torch.full_like(want, float("nan"))
            got = gnn.propagate_noalloc(g, x, e if msg else None, msg, aggr, gnn.EDGE_ORDER_COO, out)
            torch.cuda.synchronize()
            assert torch.equal(got.view(torch.int32), want.view(torch.int32)), (wl.num_nodes, msg, aggr)
    for _, g, _, _ in cases:
        g.close()


def test_noalloc_rejects_what_the_array_cannot_hold(gnn):
    wl = synth.config2_weighted(num_nodes=4000, num_edges=100_000, feat=8, cap=3000.0)
    g = gnn.build_csr(dev(wl.src), dev(wl.dst), wl.num_nodes, 4, 64)
    n_slots = int(g.work_lists()["item_slot"].max()) + 1
    f = 8192
    assert n_slots * f > 4 * 1024 * 1024
    x = torch.zeros((wl.num_nodes, f), dtype=torch.float32, device="cuda")
    out = torch.full((wl.num_nodes, f), -7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(gnn.GnnError) as err:
        gnn.propagate_noalloc(g, x, None, MSG_COPY_XJ, AGGR_SUM, gnn.EDGE_ORDER_COO, out)
    assert err.value.code == ERR_SCRATCH_LIMIT
    torch.cuda.synchronize()
    assert bool((out == -7.0).all())                       # nothing was launched
    g.close()
