"""Pins the from-scratch reference to the paper's incremental rule (Section 3.2, Eq. 2): a literal
set-based Eq. 2, chained from snapshot 0, must land on the from-scratch result at every step."""
import itertools
import os

import numpy as np
import pytest

import oracle
from oracle import incremental as inc
from paper_2501_15348_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _scaled_sources(x, rp, mode, self_loop):
    """Y = P X : the rows the targets gather (sym scales the source by deg^-1/2)."""
    if mode != "sym":
        return np.array(x, dtype=np.float64)
    deg = oracle.degrees(rp, self_loop)
    p = np.where(deg > 0, 1.0 / np.sqrt(np.maximum(deg, 1e-300)), 0.0)
    return x * p[:, None]


def _chain(edges, feats, n, mode, self_loop, form):
    """Runs `form` over consecutive snapshots and compares S_t with the from-scratch S_t."""
    g0 = oracle.Graph(oracle.canonicalise(*edges[0], n), n)
    s, _ = oracle.aggregate(g0.row_ptr, g0.col, feats[0], mode, self_loop)
    y_prev = _scaled_sources(feats[0], g0.row_ptr, mode, self_loop)
    e_prev = inc.edge_set(*edges[0])
    worst = 0.0
    for t in range(1, len(edges)):
        g = oracle.Graph(oracle.canonicalise(*edges[t], n), n)
        y_cur = _scaled_sources(feats[t], g.row_ptr, mode, self_loop)
        e_cur = inc.edge_set(*edges[t])
        s_new = form(s, y_prev, y_cur, e_prev, e_cur, self_loop)
        s_ref, _ = oracle.aggregate(g.row_ptr, g.col, feats[t], mode, self_loop)
        worst = max(worst, np.abs(s_new - s_ref).max())
        # rows outside the touched set keep their bits
        touched = inc.touched_rows(e_prev, e_cur, inc.changed_rows(y_prev, y_cur), n, self_loop)
        untouched = np.array(sorted(set(range(n)) - touched), dtype=int)
        assert np.array_equal(s_new[untouched], s[untouched])
        assert np.array_equal(s_ref[untouched], s_ref_prev[untouched]) if t > 1 else True
        s, y_prev, e_prev, s_ref_prev = s_new, y_cur, e_cur, s_ref
    return worst


FORMS = [inc.eq2_literal, inc.form_prev_features, inc.form_cur_features]


@pytest.mark.parametrize("form", FORMS)
@pytest.mark.parametrize("mode,self_loop", list(itertools.product(["sum", "mean", "sym"], [False, True])))
def test_incremental_equals_full_on_tiny_config(tiny_seq, form, mode, self_loop):
    n = tiny_seq.workload.num_nodes
    T = 5
    feats = [oracle.features_at(tiny_seq.x0, tiny_seq.feat_rows, tiny_seq.feat_vals, t) for t in range(T)]
    assert _chain(tiny_seq.edges[:T], feats, n, mode, self_loop, form) < 1e-10


def _case(n, steps, d=3, seed=0):
    """steps: list of (edge list [(u,v)], set of rows to re-draw)."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n, d))
    edges, feats = [], []
    for e, redraw in steps:
        x = x.copy()
        for r in redraw:
            x[r] = rng.standard_normal(d)
        src = np.array([u for u, _ in e], dtype=np.int64)
        dst = np.array([v for _, v in e], dtype=np.int64)
        edges.append((src, dst))
        feats.append(x)
    return edges, feats


ADVERSARIAL = {
    # an edge is deleted and its source's features change in the same step (counted once in G-)
    "delete_plus_changed_source": [([(0, 1), (0, 2), (3, 1)], []), ([(0, 2), (3, 1)], [0])],
    "delete_then_reinsert": [([(0, 1), (2, 1)], []), ([(2, 1)], []), ([(0, 1), (2, 1)], [])],
    "node_loses_all_in_edges": [([(0, 3), (1, 3), (2, 3)], []), ([(0, 1)], [])],
    "feature_only_step": [([(0, 1), (1, 2), (2, 0)], []), ([(0, 1), (1, 2), (2, 0)], [1, 2])],
    "edge_only_step": [([(0, 1), (1, 2)], []), ([(0, 1), (2, 1), (3, 0)], [])],
    "zero_churn": [([(0, 1), (1, 2)], []), ([(0, 1), (1, 2)], [])],
    "full_churn": [([(0, 1), (1, 2), (2, 3)], []), ([(3, 2), (2, 1), (1, 0)], [0, 1, 2, 3])],
    "insert_from_changed_source": [([(1, 2)], []), ([(1, 2), (0, 2)], [0])],
}


@pytest.mark.parametrize("name", sorted(ADVERSARIAL))
@pytest.mark.parametrize("form", FORMS)
def test_adversarial_cases(name, form):
    edges, feats = _case(5, ADVERSARIAL[name], seed=len(name))
    for mode, sl in itertools.product(["sum", "mean", "sym"], [False, True]):
        assert _chain(edges, feats, 5, mode, sl, form) < 1e-12


def test_zero_churn_is_bitwise_identity():
    edges, feats = _case(5, ADVERSARIAL["zero_churn"])
    g = oracle.Graph(oracle.canonicalise(*edges[0], 5), 5)
    s0, _ = oracle.aggregate(g.row_ptr, g.col, feats[0], "sum", True)
    s1 = inc.eq2_literal(s0, feats[0], feats[1], inc.edge_set(*edges[0]), inc.edge_set(*edges[1]), True)
    assert np.array_equal(s0, s1)


def test_worked_example_structure():
    """Section 3.2's example: B->E deleted, A->E inserted, A's features change."""
    spec = {}
    for line in open(os.path.join(GOLDEN, "worked_example_sec3_2.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        spec[k] = v
    ids = {name: i for i, name in enumerate(spec["nodes"])}
    parse = lambda toks: {(ids[a], ids[b]) for a, b in (tok.split("->") for tok in toks)}
    e_t, e_t1 = parse(spec["edges_t"]), parse(spec["edges_t1"])
    changed = {ids[a] for a in spec["feature_changed"]}
    g_minus, g_plus = inc.delta_graphs(e_t, e_t1, changed, len(ids), self_loop=False)
    assert g_minus == parse(spec["expect_gminus"])
    assert g_plus == parse(spec["expect_gplus"])
    # and the numbers follow: E's aggregate loses B's old row and gains A's new row
    rng = np.random.default_rng(0)
    f_t = rng.standard_normal((5, 2))
    f_t1 = f_t.copy()
    f_t1[ids["A"]] = rng.standard_normal(2)
    src, dst = zip(*e_t)
    g = oracle.Graph(oracle.canonicalise(src, dst, 5), 5)
    s_t, _ = oracle.aggregate(g.row_ptr, g.col, f_t, "sum", False)
    s_t1 = inc.eq2_literal(s_t, f_t, f_t1, e_t, e_t1, False)
    E, A, B, D = ids["E"], ids["A"], ids["B"], ids["D"]
    assert np.allclose(s_t1[E], f_t[D] + f_t1[A])
    assert np.allclose(s_t[E], f_t[D] + f_t[B])
    src, dst = zip(*e_t1)
    g1 = oracle.Graph(oracle.canonicalise(src, dst, 5), 5)
    assert np.allclose(s_t1, oracle.aggregate(g1.row_ptr, g1.col, f_t1, "sum", False)[0])


def test_a_planted_mistake_is_caught():
    """A dropped feature-change term must break the invariant (the pin has teeth)."""

    def broken(s_prev, y_prev, y_cur, e_prev, e_cur, self_loop):
        return inc.form_prev_features(s_prev, y_prev, y_prev, e_prev, e_cur, self_loop)

    edges, feats = _case(5, ADVERSARIAL["feature_only_step"])
    with pytest.raises(AssertionError):
        assert _chain(edges, feats, 5, "sum", True, broken) < 1e-12
