"""GPU parity, integer side: the snapshot-diff builder (insert / delete CSRs, merged delta rows, change set)
against the CPU reference, bit for bit (paper Section 3.2: delta graphs)."""
import numpy as np
import pytest

import oracle
from helpers import expected_merged_delta, oracle_feats, oracle_graphs
from paper_2501_15348_amd import synth

pytestmark = pytest.mark.gpu


def _ctx(wl, arena=256 << 20, **kw):
    from paper_2501_15348_amd import reinc

    return reinc.Context.for_workload(wl, arena_bytes=arena, **kw)


def _check_all_steps(seq, delta_features=True, arena=256 << 20):
    wl = seq.workload
    ctx = _ctx(wl, arena=arena)
    ctx.load_sequence(seq, delta_features=delta_features)
    ctx.build_deltas(-1)
    graphs = oracle_graphs(seq)
    for t in range(seq.num_snapshots):
        rp, col = ctx.get_snapshot_csr(t)
        assert np.array_equal(rp, graphs[t].row_ptr) and np.array_equal(col, graphs[t].col), f"CSR t={t}"
    for t in range(1, seq.num_snapshots):
        print(f"[{wl.name}] step {t}", flush=True)
        exp_ins, exp_del, ent_ptr, ent, rows, changed = expected_merged_delta(
            graphs[t - 1], graphs[t], oracle_feats(seq, t - 1), oracle_feats(seq, t), wl.agg, wl.self_loop)
        for kind, (erp, ecol) in enumerate((exp_ins, exp_del)):
            rp, col = ctx.get_delta_csr(t, kind)
            assert rp.dtype == np.int64 and col.dtype == np.int32
            assert np.array_equal(rp, erp), f"t={t} kind={kind} row_ptr"
            assert np.array_equal(col, ecol), f"t={t} kind={kind} col"
        g_ptr, g_ent, g_rows, g_changed = ctx.get_merged_delta(t)
        assert np.array_equal(g_changed, changed), f"t={t} change set"
        assert np.array_equal(g_ptr, ent_ptr), f"t={t} entry_ptr"
        assert np.array_equal(g_ent, ent), f"t={t} entries"
        assert np.array_equal(g_rows, rows), f"t={t} row list"
        info = ctx.get_delta_info(t)
        assert info["n_ins"] == exp_ins[1].size and info["n_del"] == exp_del[1].size
        assert info["n_entries"] == ent.size and info["n_rows"] == rows.size and info["n_changed"] == changed.size
        assert info["num_edges_cur"] == graphs[t].col.size
    ctx.close()


def test_tiny_config_all_steps(tiny_seq):
    _check_all_steps(tiny_seq)


def test_generator_ground_truth(tiny_seq):
    ctx = _ctx(tiny_seq.workload)
    ctx.load_sequence(tiny_seq)
    ctx.build_deltas(-1)
    for t in range(1, tiny_seq.num_snapshots):
        for kind, which in ((0, "ins"), (1, "del")):
            rp, col = ctx.get_delta_csr(t, kind)
            rows = np.repeat(np.arange(ctx.n), np.diff(rp))
            ts, td = tiny_seq.truth_pairs(t, which)
            assert sorted(zip(col.tolist(), rows.tolist())) == sorted(zip(ts.tolist(), td.tolist()))
    ctx.close()


@pytest.mark.parametrize("mode", ["sum", "sym"])
def test_power_law_several_tiles_ragged(mode):
    wl = synth.WORKLOADS["c2"].scaled(4099, 4, agg=mode)
    _check_all_steps(synth.make_sequence(wl))


def test_full_feature_loads_find_the_same_change_set():
    wl = synth.WORKLOADS["c2"].scaled(1500, 3, agg="mean")
    _check_all_steps(synth.make_sequence(wl), delta_features=False)


def test_edge_lists_in_device_memory_give_the_same_snapshots(tiny_seq):
    """The raw edge list may already sit in device memory (on_device = 1): same canonical CSR and CSC."""
    import torch

    wl = tiny_seq.workload
    host, dev = _ctx(wl), _ctx(wl)
    for t in (0, 3):
        src, dst = tiny_seq.edges[t]
        host.load_edges(t, src, dst)
        dev.load_edges(t, torch.from_numpy(src).cuda(), torch.from_numpy(dst).cuda())
        for transpose in (False, True):
            a, b = host.get_snapshot_csr(t, transpose), dev.get_snapshot_csr(t, transpose)
            assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    host.close()
    dev.close()


def test_a_listed_row_with_unchanged_values_is_not_in_the_change_set():
    """Delta-mode loading ships (row, values) pairs; the change set is defined by the values: a row that is sent again
    with the values it already had belongs to it as little as it would after a full load."""
    import copy

    wl = synth.WORKLOADS["c2"].scaled(900, 3, agg="mean")
    seq = copy.deepcopy(synth.make_sequence(wl))
    t = 2
    x_prev = oracle_feats(seq, t - 1).astype(np.float32)
    extra = np.setdiff1d(np.arange(0, wl.num_nodes, 37, dtype=np.int32), seq.feat_rows[t])
    rows = np.concatenate([seq.feat_rows[t], extra])
    vals = np.concatenate([seq.feat_vals[t], x_prev[extra]])
    order = np.argsort(rows)
    seq.feat_rows[t], seq.feat_vals[t] = rows[order].astype(np.int32), vals[order]
    ctx = _ctx(wl)
    ctx.load_sequence(seq)
    ctx.build_deltas(-1)
    graphs = oracle_graphs(seq)
    counts = oracle.change_counts(graphs[t - 1], graphs[t], oracle_feats(seq, t - 1), oracle_feats(seq, t), wl.agg, wl.self_loop)
    info = ctx.get_delta_info(t)
    for k in ("n_changed", "n_fchg_entries", "n_entries", "n_rows"):
        assert info[k] == counts[k], (k, info[k], counts[k])
    _, _, _, changed = ctx.get_merged_delta(t)
    assert np.intersect1d(changed, extra).size == 0 and extra.size > 10
    ctx.close()
    _check_all_steps(seq)


def _manual_seq(n, steps, d=4, sl=True, agg="sum"):
    """steps: list of (src list, dst list, rows to re-draw)"""
    wl = synth.Workload("manual", n, 1.0, len(steps), "uniform", 0, 0, 0, "fp32", agg, sl, (d, d), "gru", d, len(steps))
    rng = np.random.default_rng(1)
    x0 = rng.standard_normal((n, d)).astype(np.float32)
    edges = [(np.array(s, dtype=np.int32), np.array(t, dtype=np.int32)) for s, t, _ in steps]
    rows = [np.array(sorted(r), dtype=np.int32) for _, _, r in steps]
    vals = [rng.standard_normal((len(r), d)).astype(np.float32) for r in rows]
    e = np.empty(0, dtype=np.uint64)
    return synth.SnapshotSequence(wl, edges, [e] * len(steps), [e] * len(steps), x0, rows, vals)


def test_degenerate_steps():
    n = 70
    ring = (list(range(n)), [(i + 1) % n for i in range(n)])
    hub_src = list(range(1, 65))
    steps = [
        (ring[0], ring[1], []),
        (ring[0], ring[1], []),  # zero churn
        ([], [], []),  # everything deleted: empty snapshot
        (hub_src, [0] * 64, [0, 3]),  # everything inserted, one 64-entry row, features change
        (hub_src + [0, 0, 5], [0] * 64 + [9, 9, 5], [3]),  # duplicates and a self-loop in the input
        (ring[1], ring[0], list(range(n))),  # 100 % churn, every row re-drawn
    ]
    seq = _manual_seq(n, steps)
    _check_all_steps(seq)
    ctx = _ctx(seq.workload)
    ctx.load_sequence(seq)
    ctx.build_deltas(1)
    info = ctx.get_delta_info(1)
    assert info["n_entries"] == 0 and info["n_rows"] == 0 and info["n_changed"] == 0
    ctx.close()


def test_long_rows_in_the_diff():
    n = 3000
    rng = np.random.default_rng(2)
    a = rng.choice(np.arange(1, n), 1500, replace=False)
    b = rng.choice(np.arange(1, n), 1400, replace=False)
    steps = [(a.tolist(), [0] * a.size, []), (b.tolist(), [0] * b.size, [7])]
    _check_all_steps(_manual_seq(n, steps))


def test_steps_built_in_several_groups_and_arena_exhaustion():
    """The builder takes as many steps per pass as the free arena allows: a generous arena (one group), one that
    forces several groups, and one that cannot hold the deltas at all (clean error, nothing half-built)."""
    from paper_2501_15348_amd import reinc

    wl = synth.WORKLOADS["c2"].scaled(6001, 9)
    seq = synth.make_sequence(wl)
    probe = _ctx(wl)
    probe.load_sequence(seq)
    loaded = probe.get_stats()["arena_used"]  # snapshots and features
    probe.build_deltas(-1)
    deltas = probe.get_stats()["arena_used"] - loaded
    probe.close()
    print(f"loaded {loaded >> 20} MiB, deltas {deltas >> 20} MiB", flush=True)
    _check_all_steps(seq, arena=256 << 20)
    _check_all_steps(seq, arena=loaded + deltas + (6 << 20))  # a step needs about 2.3 MiB of scratch: groups of one or two
    ctx = _ctx(wl, arena=loaded + deltas // 2)
    ctx.load_sequence(seq)
    with pytest.raises(reinc.ReincError) as e:
        ctx.build_deltas(-1)
    assert e.value.code == reinc.E_NOMEM
    built = 0
    for t in range(1, wl.num_snapshots):
        try:
            ctx.get_delta_info(t)
            built += 1
        except reinc.ReincError as err:
            assert err.code == reinc.E_STATE
    assert built < wl.num_snapshots - 1
    ctx.close()


def test_error_paths():
    from paper_2501_15348_amd import reinc

    wl = synth.WORKLOADS["tiny"].scaled(100, 3)
    ctx = _ctx(wl, arena=8 << 20)
    with pytest.raises(reinc.ReincError) as e:
        ctx.load_edges(0, np.array([0, 100], dtype=np.int32), np.array([1, 2], dtype=np.int32))
    assert e.value.code == reinc.E_ARG
    with pytest.raises(reinc.ReincError) as e:
        ctx.build_deltas(1)
    assert e.value.code == reinc.E_STATE
    with pytest.raises(reinc.ReincError) as e:
        ctx.get_delta_csr(1, 0)
    assert e.value.code == reinc.E_STATE
    with pytest.raises(reinc.ReincError) as e:
        ctx.load_edges(5, np.zeros(1, dtype=np.int32), np.ones(1, dtype=np.int32))
    assert e.value.code == reinc.E_ARG
    ctx.load_edges(0, np.array([0], dtype=np.int32), np.array([1], dtype=np.int32))
    with pytest.raises(reinc.ReincError) as e:
        ctx.load_edges(0, np.array([0], dtype=np.int32), np.array([1], dtype=np.int32))
    assert e.value.code == reinc.E_STATE
    with pytest.raises(reinc.ReincError) as e:
        ctx.load_features_delta(1, np.array([3, 2], dtype=np.int32), np.zeros((2, 16), dtype=np.float32))
    assert e.value.code in (reinc.E_ARG, reinc.E_STATE)
    ctx.close()
    small = _ctx(wl, arena=4096)
    with pytest.raises(reinc.ReincError) as e:
        small.load_features_full(0, np.zeros((100, 16), dtype=np.float32))
    assert e.value.code == reinc.E_NOMEM
    small.close()
