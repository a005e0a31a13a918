"""Helpers shared by the tests: tolerance checks and tiny brute-force references.

Nothing here is used by the library or by the oracle.
"""
import json
import os

import numpy as np

RTOL = 1e-5   # fp32 bar for sum / mean / softmax-type results


def load_golden(golden_dir, name):
    with open(os.path.join(golden_dir, name)) as fh:
        return json.load(fh)


def assert_close_sabs(got, ref, sabs, rtol=RTOL, what=""):
    """Floating-point parity bar.

    (i)  component-wise, conditioned on the summation: |got - ref| <= rtol * S_abs, where S_abs
         is the sum of |terms| behind that element (exactly 0 where nothing was summed);
    (ii) norm-wise: max|got - ref| <= rtol * max|ref|.
    The double-accumulated oracle is exact to ~1e-16 * S_abs and any fp32 summation order is
    within depth * 2^-24 * S_abs, so a correct kernel passes for every order of summation.
    """
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    sabs = np.asarray(sabs, dtype=np.float64)
    assert got.shape == ref.shape == sabs.shape, (got.shape, ref.shape, sabs.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - ref)
    # one float rounding of the result itself is always allowed
    bound = rtol * sabs + 2.0 ** -24 * np.abs(ref)
    bad = err > bound
    if bad.any():
        q = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} elements beyond {rtol}*S_abs; worst at {q}: "
                             f"got {got[q]!r} ref {ref[q]!r} S_abs {sabs[q]!r}")
    scale = np.abs(ref).max() if ref.size else 0.0
    if scale > 0:
        assert err.max() <= rtol * scale, f"{what}: norm-wise error {err.max() / scale:.3e}"


def assert_close_rel(got, ref, rtol=RTOL, what=""):
    """Plain relative bar for results without cancellation (softmax weights are positive)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - ref)
    bound = rtol * np.abs(ref) + 1e-37
    assert (err <= bound).all(), f"{what}: worst rel err {np.max(err / (np.abs(ref) + 1e-300)):.3e}"


def incoming(dst, num_nodes):
    """List of edge-id arrays per destination, each in increasing edge id."""
    order = np.argsort(dst, kind="stable")
    bounds = np.searchsorted(dst[order], np.arange(num_nodes + 1))
    return [order[bounds[i]:bounds[i + 1]] for i in range(num_nodes)]


def dense_adjacency(src, dst, num_nodes, weight=None):
    """A[i, j] = number (or summed weight) of edges j -> i, float64."""
    a = np.zeros((num_nodes, num_nodes), dtype=np.float64)
    np.add.at(a, (dst, src), 1.0 if weight is None else weight.astype(np.float64))
    return a


def subgraph_for_rows(src, dst, rows):
    """Edges whose destination is in ``rows`` plus a compact relabelling of the nodes they
    touch.  A destination's result depends only on its incoming edges and their endpoints'
    features, so running a reference on this subgraph reproduces those rows of the full result.
    Returns (sub_src, sub_dst, nodes, local_rows, edge_ids)."""
    rows = np.asarray(rows)
    lut = np.zeros(int(max(dst.max(initial=0), rows.max(initial=0))) + 1, dtype=bool)
    lut[rows] = True
    mask = lut[dst]
    eid = np.flatnonzero(mask)
    nodes = np.unique(np.concatenate([rows, src[eid], dst[eid]]))
    s = np.searchsorted(nodes, src[eid]).astype(np.int32)
    d = np.searchsorted(nodes, dst[eid]).astype(np.int32)
    local_rows = np.searchsorted(nodes, rows)
    return s, d, nodes, local_rows, eid
