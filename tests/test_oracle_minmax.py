"""Pins for the max / min aggregator reference (paper Section 3.2: max() and min() keep the ids of the
contributing edges; a deleted contributor forces a from-scratch aggregation of that target).

The paper prints no numbers for these aggregators, so the reference is pinned to things the mathematics fixes: a
dense masked-adjacency formula written independently, the max/min duality, closed-form special cases, and the
invariant that the paper's incremental procedure, chained over snapshots, equals the from-scratch result."""
import numpy as np
import pytest

import oracle
from oracle import minmax
from paper_2501_15348_amd import synth


def _csr(n, src, dst):
    keys = oracle.canonicalise(np.asarray(src, np.int32), np.asarray(dst, np.int32), n)
    return oracle.csr_from_keys(keys, n)


def _dense(n, row_ptr, col, x, op, self_loop):
    a = np.zeros((n, n), dtype=bool)  # a[v, u]: u is a source of v
    for v in range(n):
        a[v, col[row_ptr[v]:row_ptr[v + 1]]] = True
    if self_loop:
        a |= np.eye(n, dtype=bool)
    fill = -np.inf if op == "max" else np.inf
    cube = np.where(a[:, :, None], x[None, :, :], fill)  # [v, u, j]
    m = cube.max(axis=1) if op == "max" else cube.min(axis=1)
    c = (cube.argmax(axis=1) if op == "max" else cube.argmin(axis=1)).astype(np.int32)  # first extremum = smallest id
    empty = ~a.any(axis=1)
    m[empty] = 0
    c[empty] = -1
    return m, c


@pytest.mark.parametrize("op", ["max", "min"])
@pytest.mark.parametrize("self_loop", [False, True])
@pytest.mark.parametrize("ties", [False, True])
def test_matches_dense_masked_adjacency(op, self_loop, ties):
    rng = np.random.default_rng(5)
    n, d, e = 60, 7, 400
    src, dst = rng.integers(0, n, e), rng.integers(0, n, e)
    dst[dst == 7] = 8  # node 7 gets no in-edge: the empty-target case without a self-loop
    row_ptr, col = _csr(n, src, dst)
    x = rng.integers(-2, 3, (n, d)).astype(np.float64) if ties else rng.standard_normal((n, d))
    m, c = minmax.aggregate_minmax(row_ptr, col, x, op, self_loop)
    md, cd = _dense(n, row_ptr, col, x, op, self_loop)
    assert np.array_equal(m, md) and np.array_equal(c, cd)
    if not self_loop:
        assert np.all(m[7] == 0) and np.all(c[7] == -1)


def test_min_is_max_of_the_negated_features():
    rng = np.random.default_rng(6)
    n, d = 80, 5
    row_ptr, col = _csr(n, rng.integers(0, n, 500), rng.integers(0, n, 500))
    x = rng.integers(-3, 4, (n, d)).astype(np.float64)
    mn, cn = minmax.aggregate_minmax(row_ptr, col, x, "min", True)
    mx, cx = minmax.aggregate_minmax(row_ptr, col, -x, "max", True)
    assert np.array_equal(mn, -mx) and np.array_equal(cn, cx)


def test_closed_forms():
    rng = np.random.default_rng(7)
    n, d = 12, 4
    x = rng.standard_normal((n, d))
    # complete graph with self-loops: every target sees every node
    src, dst = np.meshgrid(np.arange(n), np.arange(n))
    row_ptr, col = _csr(n, src.ravel(), dst.ravel())
    m, c = minmax.aggregate_minmax(row_ptr, col, x, "max", True)
    assert np.array_equal(m, np.broadcast_to(x.max(axis=0), (n, d))) and np.array_equal(c, np.broadcast_to(x.argmax(axis=0), (n, d)))
    # no edges: zeros / -1 without a self-loop, the node's own row with one
    row_ptr, col = _csr(n, [], [])
    m, c = minmax.aggregate_minmax(row_ptr, col, x, "min", False)
    assert not m.any() and np.all(c == -1)
    m, c = minmax.aggregate_minmax(row_ptr, col, x, "min", True)
    assert np.array_equal(m, x) and np.array_equal(c, np.broadcast_to(np.arange(n)[:, None], (n, d)))
    # a path 0 -> 1 -> 2: each target sees exactly its predecessor
    row_ptr, col = _csr(3, [0, 1], [1, 2])
    m, c = minmax.aggregate_minmax(row_ptr, col, x[:3], "max", False)
    assert np.array_equal(m[1], x[0]) and np.array_equal(m[2], x[1]) and not m[0].any()


def test_deleting_a_non_contributor_changes_nothing_and_a_contributor_forces_a_recompute():
    # target 3 has sources 0, 1, 2 with values 1, 5, 3: source 1 contributes the maximum
    x = np.array([[1.0], [5.0], [3.0], [0.0]])
    p0, c0 = _csr(4, [0, 1, 2], [3, 3, 3])
    m0, k0 = minmax.aggregate_minmax(p0, c0, x, "max", False)
    assert m0[3, 0] == 5.0 and k0[3, 0] == 1
    p1, c1 = _csr(4, [1, 2], [3, 3])  # drop the edge from source 0
    m1, k1, redo, touched = minmax.incremental_minmax_step(m0, k0, p0, c0, p1, c1, x, x, "max", False)
    assert m1[3, 0] == 5.0 and redo == set() and touched == {3}
    p2, c2 = _csr(4, [0, 2], [3, 3])  # drop the edge from source 1 instead
    m2, k2, redo, _ = minmax.incremental_minmax_step(m0, k0, p0, c0, p2, c2, x, x, "max", False)
    assert m2[3, 0] == 3.0 and k2[3, 0] == 2 and redo == {3}
    # the contributor's value drops without any edge change: also a lost contribution
    x2 = x.copy()
    x2[1, 0] = 2.0
    m3, k3, redo, _ = minmax.incremental_minmax_step(m0, k0, p0, c0, p0, c0, x, x2, "max", False)
    assert m3[3, 0] == 3.0 and k3[3, 0] == 2 and redo == {3}
    # a non-contributor rises above the old maximum: an insertion of its new value
    x3 = x.copy()
    x3[0, 0] = 9.0
    m4, k4, redo, _ = minmax.incremental_minmax_step(m0, k0, p0, c0, p0, c0, x, x3, "max", False)
    assert m4[3, 0] == 9.0 and k4[3, 0] == 0 and redo == set()


@pytest.mark.parametrize("arrivals_first", [False, True])
@pytest.mark.parametrize("op,self_loop,ties", [("max", True, False), ("min", False, True), ("max", False, True)])
def test_incremental_chain_equals_from_scratch(op, self_loop, ties, arrivals_first):
    wl = synth.WORKLOADS["tiny"].scaled(300, 6, edge_churn=0.05, feat_churn=0.05)
    seq = synth.make_sequence(wl)
    n = wl.num_nodes
    graphs = oracle.graphs_of(seq.edges, n)
    feats = [oracle.features_at(seq.x0, seq.feat_rows, seq.feat_vals, t).astype(np.float64) for t in range(wl.num_snapshots)]
    if ties:
        feats = [np.round(f * 1.5) for f in feats]
    m, c = minmax.aggregate_minmax(graphs[0].row_ptr, graphs[0].col, feats[0], op, self_loop)
    total_redo = total_touched = 0
    for t in range(1, wl.num_snapshots):
        before = m.copy()
        m, c, redo, touched = minmax.incremental_minmax_step(m, c, graphs[t - 1].row_ptr, graphs[t - 1].col, graphs[t].row_ptr,
                                                             graphs[t].col, feats[t - 1], feats[t], op, self_loop,
                                                             arrivals_first=arrivals_first)
        mf, cf = minmax.aggregate_minmax(graphs[t].row_ptr, graphs[t].col, feats[t], op, self_loop)
        assert np.array_equal(m, mf) and np.array_equal(c, cf), f"snapshot {t}"
        assert redo <= touched
        untouched = np.setdiff1d(np.arange(n), np.fromiter(touched, dtype=np.int64))
        assert np.array_equal(m[untouched], before[untouched])
        total_redo += len(redo)
        total_touched += len(touched)
    assert 0 < total_redo < total_touched  # both the fallback and the purely incremental path were exercised


def test_applying_arrivals_first_never_recomputes_more():
    wl = synth.WORKLOADS["tiny"].scaled(400, 5, edge_churn=0.10, feat_churn=0.05)
    seq = synth.make_sequence(wl)
    graphs = oracle.graphs_of(seq.edges, wl.num_nodes)
    feats = [np.round(oracle.features_at(seq.x0, seq.feat_rows, seq.feat_vals, t).astype(np.float64) * 2) for t in range(5)]
    m, c = minmax.aggregate_minmax(graphs[0].row_ptr, graphs[0].col, feats[0], "max", True)
    fewer = 0
    for t in range(1, 5):
        args = (m, c, graphs[t - 1].row_ptr, graphs[t - 1].col, graphs[t].row_ptr, graphs[t].col, feats[t - 1], feats[t], "max", True)
        m1, c1, redo1, _ = minmax.incremental_minmax_step(*args)
        m2, c2, redo2, _ = minmax.incremental_minmax_step(*args, arrivals_first=True)
        assert np.array_equal(m1, m2) and np.array_equal(c1, c2) and redo2 <= redo1
        fewer += len(redo1) - len(redo2)
        m, c = m1, c1
    assert fewer > 0
