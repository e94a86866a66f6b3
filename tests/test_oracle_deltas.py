"""Pins for the reference edge deltas (paper Section 3.2: delta graphs of deletions and insertions)."""
import numpy as np

import oracle
from paper_2501_15348_amd import synth


def _pairs(rp, col):
    rows = np.repeat(np.arange(rp.size - 1), np.diff(rp))
    return list(zip(col.tolist(), rows.tolist()))  # (src, dst)


def test_matches_generator_ground_truth(tiny_seq):
    n = tiny_seq.workload.num_nodes
    keys = [oracle.canonicalise(s, d, n) for s, d in tiny_seq.edges]
    for t in range(1, len(keys)):
        (irp, icol), (drp, dcol) = oracle.edge_deltas(keys[t - 1], keys[t], n)
        ts, td = tiny_seq.truth_pairs(t, "ins")
        assert sorted(_pairs(irp, icol)) == sorted(zip(ts.tolist(), td.tolist()))
        ts, td = tiny_seq.truth_pairs(t, "del")
        assert sorted(_pairs(drp, dcol)) == sorted(zip(ts.tolist(), td.tolist()))
        assert irp.dtype == np.int64 and icol.dtype == np.int32
        for rp, col in ((irp, icol), (drp, dcol)):  # ascending columns inside every row
            for v in range(n):
                assert np.all(np.diff(col[rp[v] : rp[v + 1]]) > 0)


def test_closure_and_replay(tiny_seq):
    n = tiny_seq.workload.num_nodes
    keys = [oracle.canonicalise(s, d, n) for s, d in tiny_seq.edges]
    cur = set(keys[0].tolist())
    for t in range(1, len(keys)):
        (irp, icol), (drp, dcol) = oracle.edge_deltas(keys[t - 1], keys[t], n)
        ins = {(v << 32) | u for u, v in _pairs(irp, icol)}
        dele = {(v << 32) | u for u, v in _pairs(drp, dcol)}
        prev = set(keys[t - 1].tolist())
        assert dele <= prev and not (ins & prev)
        assert len(keys[t]) == len(keys[t - 1]) - len(dele) + len(ins)
        cur = (cur - dele) | ins
        assert cur == set(keys[t].tolist())


def test_brute_force_tiny():
    rng = np.random.default_rng(5)
    n = 9
    for trial in range(20):
        a = oracle.canonicalise(rng.integers(0, n, 30), rng.integers(0, n, 30), n)
        b = oracle.canonicalise(rng.integers(0, n, 30), rng.integers(0, n, 30), n)
        (irp, icol), (drp, dcol) = oracle.edge_deltas(a, b, n)
        ea = {(int(k) & 0xFFFFFFFF, int(k) >> 32) for k in a}
        eb = {(int(k) & 0xFFFFFFFF, int(k) >> 32) for k in b}
        ins = [(u, v) for v in range(n) for u in range(n) if (u, v) in eb and (u, v) not in ea]
        dele = [(u, v) for v in range(n) for u in range(n) if (u, v) in ea and (u, v) not in eb]
        assert _pairs(irp, icol) == ins and _pairs(drp, dcol) == dele


def test_degenerate():
    n = 4
    a = oracle.canonicalise([0, 1], [1, 2], n)
    e = np.empty(0, dtype=np.uint64)
    (irp, icol), (drp, dcol) = oracle.edge_deltas(a, a, n)
    assert icol.size == 0 and dcol.size == 0 and irp.tolist() == [0] * 5
    (irp, icol), (drp, dcol) = oracle.edge_deltas(a, e, n)  # everything deleted
    assert icol.size == 0 and _pairs(drp, dcol) == [(0, 1), (1, 2)]
    (irp, icol), (drp, dcol) = oracle.edge_deltas(e, a, n)
    assert dcol.size == 0 and _pairs(irp, icol) == [(0, 1), (1, 2)]


def test_change_counts_against_set_based_delta_graphs(tiny_seq):
    """The vectorised counts equal the sizes of the literal delta graphs of Section 3.2."""
    from oracle import incremental as inc

    n = tiny_seq.workload.num_nodes
    graphs = oracle.graphs_of(tiny_seq.edges, n)
    for mode, sl in (("sum", True), ("sym", True), ("mean", False)):
        for t in (1, 4):
            xp = oracle.features_at(tiny_seq.x0, tiny_seq.feat_rows, tiny_seq.feat_vals, t - 1)
            xc = oracle.features_at(tiny_seq.x0, tiny_seq.feat_rows, tiny_seq.feat_vals, t)
            c = oracle.change_counts(graphs[t - 1], graphs[t], xp, xc, mode, sl)
            assert c["n_ins"] == len(tiny_seq.truth_inserted[t]) and c["n_del"] == len(tiny_seq.truth_deleted[t])
            e_prev, e_cur = inc.edge_set(*tiny_seq.edges[t - 1]), inc.edge_set(*tiny_seq.edges[t])
            changed = set(np.nonzero(np.any(xp != xc, axis=1))[0].tolist())
            if mode == "sym":
                changed |= set(np.nonzero(np.diff(graphs[t - 1].row_ptr) != np.diff(graphs[t].row_ptr))[0].tolist())
            assert c["n_changed"] == len(changed)
            fchg = {e for e in inc.with_self_loops(e_cur, n, sl) if e[0] in changed}
            assert c["n_fchg_entries"] == len(fchg)
            assert c["n_entries"] == c["n_ins"] + c["n_del"] + len(fchg)
            assert c["n_rows"] == len(inc.touched_rows(e_prev, e_cur, changed, n, sl))
