"""Pins of the node mini-batch reference (oracle.minibatch and the `loss_rows` argument of the window functions;
paper Section 4.2, "Rethinking Mini-batch Training") against facts it does not compute itself: hand-worked
graphs, breadth-first balls found by powers of a dense adjacency matrix, the full-graph model (the batch rows of
a model evaluated on the extracted computational graphs equal those of the model on the whole graph), additivity
of the loss and of its gradient over a partition of the nodes, and finite differences."""
import numpy as np
import pytest

import oracle
from oracle import minibatch
from paper_2501_15348_amd import synth


def _arr(pairs):
    a = np.array(pairs, dtype=np.int32).reshape(-1, 2)
    return a[:, 0].copy(), a[:, 1].copy()


def test_chain_by_hand():
    # 0 -> 1 -> 2 -> 3 -> 4 in the first snapshot, 5 -> 3 appears in the second
    edges = [_arr([(0, 1), (1, 2), (2, 3), (3, 4)]), _arr([(0, 1), (1, 2), (2, 3), (3, 4), (5, 3)])]
    levels = minibatch.closure(edges, [4], 2)
    assert levels == [{4}, {4, 3}, {4, 3, 2, 5}]
    node_list, sub, n_inner = minibatch.extract(edges, [4], 2)
    assert node_list.tolist() == [4, 3, 2, 5] and n_inner == 2  # the batch, then one hop (3), then two hops (2, 5)
    # kept: edges into 3 or 4.  new ids: 4 -> 0, 3 -> 1, 2 -> 2, 5 -> 3
    assert list(zip(*[a.tolist() for a in sub[0]])) == [(2, 1), (1, 0)]
    assert list(zip(*[a.tolist() for a in sub[1]])) == [(2, 1), (1, 0), (3, 1)]


def test_star_and_batch_order():
    # leaves 1..4 point at the hub 0; the batch keeps its given order, the others ascend within their hop count
    edges = [_arr([(1, 0), (2, 0), (3, 0), (4, 0)])]
    node_list, sub, n_inner = minibatch.extract(edges, [3, 0], 1)
    assert node_list.tolist() == [3, 0, 1, 2, 4] and n_inner == 2
    assert sorted(zip(*[a.tolist() for a in sub[0]])) == [(0, 1), (2, 1), (3, 1), (4, 1)]
    with pytest.raises(ValueError):
        minibatch.extract(edges, [1, 1], 1)


def test_every_hop_set_is_a_prefix_of_the_numbering():
    rng = np.random.default_rng(5)
    edges = [(rng.integers(0, 60, 90).astype(np.int32), rng.integers(0, 60, 90).astype(np.int32)) for _ in range(3)]
    batch = [17, 3, 41]
    levels = minibatch.closure(edges, batch, 3)
    node_list, _, n_inner = minibatch.extract(edges, batch, 3)
    assert node_list[:3].tolist() == batch and n_inner == len(levels[2])
    for k in range(4):
        first = node_list[:len(levels[k])].tolist()
        assert set(first) == levels[k]
        if k:  # ascending ids among the nodes first reached in k hops
            new = first[len(levels[k - 1]):]
            assert new == sorted(new)
    assert len(levels[1]) < len(levels[2]) < len(levels[3]) < 60  # (the case does separate the sets)


def test_zero_hops_is_the_batch_alone():
    edges = [_arr([(1, 0), (2, 1)])]
    node_list, sub, n_inner = minibatch.extract(edges, [1], 0)
    assert node_list.tolist() == [1] and n_inner == 0 and sub[0][0].size == 0


@pytest.mark.parametrize("seed,hops", [(0, 1), (1, 2), (2, 3)])
def test_closure_is_the_ball_of_the_union_graph(seed, hops):
    rng = np.random.default_rng(seed)
    n, T = 40, 3
    edges = []
    union = np.zeros((n, n), dtype=np.int64)  # union[v, u] = 1 iff u -> v in some snapshot
    for _ in range(T):
        src, dst = rng.integers(0, n, 60).astype(np.int32), rng.integers(0, n, 60).astype(np.int32)
        edges.append((src, dst))
        union[dst, src] = 1
    batch = rng.choice(n, 3, replace=False)
    reach = np.zeros(n, dtype=np.int64)
    reach[batch] = 1
    step = union.T + np.eye(n, dtype=np.int64)  # one hop backwards along the edges, or stay
    for k in range(hops):
        reach = (step @ reach > 0).astype(np.int64)
    levels = minibatch.closure(edges, batch, hops)
    assert levels[hops] == set(np.nonzero(reach)[0].tolist())
    for a, b in zip(levels, levels[1:]):
        assert a <= b


def _model(mode, rnn, layers, n=60, T=4, seed=3):
    dims = (4,) + (5,) * layers
    wl = synth.Workload("mb", n, 3.0, T, "uniform", 0.0, 0.2, 0.2, "fp32", mode, True, dims, rnn, 3, T, seed)
    seq = synth.make_sequence(wl)
    feats = [oracle.features_at(seq.x0, seq.feat_rows, seq.feat_vals, t) for t in range(T)]
    flat = synth.make_params(wl, bias_scale=0.3).astype(np.float64)
    target = synth.make_target(wl).astype(np.float64)
    return wl, seq, feats, flat, target


def _run(wl, graphs, feats, flat, target, rows):
    p = synth.split_params(wl, flat)
    L = len(wl.dims) - 1
    loss, h, saved = oracle.forward_window(graphs, feats, p, L, wl.agg, wl.self_loop, wl.rnn, target, keep=True, loss_rows=rows)
    g = oracle.backward_window(graphs, saved, h, p, L, wl.agg, wl.self_loop, wl.rnn, target, loss_rows=rows)
    return loss, h, np.concatenate([g[name].ravel() for name, _ in synth.param_shapes(wl)])


@pytest.mark.parametrize("mode,rnn,layers", [("sum", "gru", 1), ("mean", "lstm", 2), ("sym", "gru", 2)])
def test_extracted_graphs_reproduce_the_full_graph_on_the_batch(mode, rnn, layers):
    wl, seq, feats, flat, target = _model(mode, rnn, layers)
    n = wl.num_nodes
    graphs = oracle.graphs_of(seq.edges, n)
    batch = np.random.default_rng(5).choice(n, 7, replace=False)
    full_loss, full_h, full_g = _run(wl, graphs, feats, flat, target, batch)
    hops = layers + (1 if mode == "sym" else 0)
    node_list, sub, _ = minibatch.extract(seq.edges, batch, hops)
    assert len(node_list) < n  # the test means something only if the sub-sequence is smaller
    sub_graphs = oracle.graphs_of(sub, len(node_list))
    sub_feats = [x[node_list] for x in feats]
    loss, h, g = _run(wl, sub_graphs, sub_feats, flat, target[node_list], np.arange(len(batch)))
    assert loss == pytest.approx(full_loss, rel=1e-12)
    np.testing.assert_allclose(h[:len(batch)], full_h[batch], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g, full_g, rtol=1e-10, atol=1e-14)
    # one hop fewer is not enough (so the hop count is not slack)
    short_list, short_sub, _ = minibatch.extract(seq.edges, batch, hops - 1)
    _, h_short, _ = _run(wl, oracle.graphs_of(short_sub, len(short_list)), [x[short_list] for x in feats], flat,
                         target[short_list], np.arange(len(batch)))
    assert not np.allclose(h_short[:len(batch)], full_h[batch], rtol=1e-9, atol=1e-12)


def test_batch_losses_and_gradients_add_up_over_a_partition():
    wl, seq, feats, flat, target = _model("mean", "gru", 2)
    n = wl.num_nodes
    graphs = oracle.graphs_of(seq.edges, n)
    full_loss, _, full_g = _run(wl, graphs, feats, flat, target, None)
    perm = np.random.default_rng(1).permutation(n)
    parts = [perm[:11], perm[11:30], perm[30:]]
    loss = sum(len(b) / n * _run(wl, graphs, feats, flat, target, b)[0] for b in parts)
    grad = sum(len(b) / n * _run(wl, graphs, feats, flat, target, b)[2] for b in parts)
    assert loss == pytest.approx(full_loss, rel=1e-12)
    np.testing.assert_allclose(grad, full_g, rtol=1e-10, atol=1e-15)
    # all rows, listed, is the plain loss
    assert _run(wl, graphs, feats, flat, target, np.arange(n))[0] == pytest.approx(full_loss, rel=1e-13)


def test_batch_gradient_by_finite_differences():
    wl, seq, feats, flat, target = _model("sum", "lstm", 1, n=25, T=3)
    graphs = oracle.graphs_of(seq.edges, wl.num_nodes)
    batch = np.array([3, 17, 8])
    _, _, grad = _run(wl, graphs, feats, flat, target, batch)
    eps = 1e-6
    for i in np.random.default_rng(0).choice(flat.size, 25, replace=False):
        fp, fm = flat.copy(), flat.copy()
        fp[i] += eps
        fm[i] -= eps
        num = (_run(wl, graphs, feats, fp, target, batch)[0] - _run(wl, graphs, feats, fm, target, batch)[0]) / (2 * eps)
        assert abs(num - grad[i]) <= 1e-6 * max(1.0, abs(num)) + 1e-9, (i, num, grad[i])


def test_the_batch_loss_ignores_features_outside_its_computational_graph():
    wl, seq, feats, flat, target = _model("mean", "gru", 2)
    graphs = oracle.graphs_of(seq.edges, wl.num_nodes)
    batch = np.array([0, 9])
    inside = minibatch.closure(seq.edges, batch, 2)[2]
    outside = np.array(sorted(set(range(wl.num_nodes)) - inside))
    assert outside.size > 0
    base = _run(wl, graphs, feats, flat, target, batch)[0]
    moved = [x.copy() for x in feats]
    for x in moved:
        x[outside] += 10.0
    assert _run(wl, graphs, moved, flat, target, batch)[0] == base
    for x in moved:
        x[list(inside)[-1]] += 10.0
    assert _run(wl, graphs, moved, flat, target, batch)[0] != base


# ---- the integrated model (graph operations inside the gates): its receptive field grows by one hop per timestep,
# so a window of L timesteps needs the batch's neighbourhood of L hops (one more under the symmetric normalisation)

def _model_integrated(mode, rnn, n=300, T=3, degree=2.0, seed=4):
    import dataclasses

    wl = synth.Workload("mbi", n, degree, T, "uniform", 0.0, 0.2, 0.2, "fp32", mode, True, (4, 5), rnn, 3, T, seed)
    wli = dataclasses.replace(wl, dims=(4,))  # parameter shapes: the cell only
    seq = synth.make_sequence(wl)
    feats = [oracle.features_at(seq.x0, seq.feat_rows, seq.feat_vals, t) for t in range(T)]
    flat = synth.make_params(wli, bias_scale=0.3).astype(np.float64)
    target = synth.make_target(wl).astype(np.float64)
    return wl, wli, seq, feats, flat, target


def _run_integrated(wl, wli, graphs, feats, flat, target, rows):
    p = synth.split_params(wli, flat)
    loss, h, saved = oracle.forward_window_integrated(graphs, feats, p, wl.agg, wl.self_loop, wl.rnn, target, keep=True,
                                                      loss_rows=rows)
    g = oracle.backward_window_integrated(graphs, saved, h, p, wl.agg, wl.self_loop, wl.rnn, target, loss_rows=rows)
    return loss, h, np.concatenate([g[name].ravel() for name, _ in synth.param_shapes(wli)])


@pytest.mark.parametrize("mode,rnn", [("sum", "gru"), ("mean", "lstm"), ("sym", "gru")])
def test_integrated_model_on_extracted_graphs_needs_one_hop_per_timestep(mode, rnn):
    wl, wli, seq, feats, flat, target = _model_integrated(mode, rnn)
    n, T = wl.num_nodes, wl.num_snapshots
    graphs = oracle.graphs_of(seq.edges, n)
    batch = np.random.default_rng(2).choice(n, 4, replace=False)
    full_loss, full_h, full_g = _run_integrated(wl, wli, graphs, feats, flat, target, batch)
    hops = T + (1 if mode == "sym" else 0)
    node_list, sub, _ = minibatch.extract(seq.edges, batch, hops)
    reach = [len(f) for f in minibatch.closure(seq.edges, batch, hops)]
    assert all(a < b for a, b in zip(reach, reach[1:])) and reach[-1] < n, reach  # every hop adds nodes, and not all
    rows = np.arange(len(batch))
    loss, h, g = _run_integrated(wl, wli, oracle.graphs_of(sub, len(node_list)), [x[node_list] for x in feats], flat,
                                 target[node_list], rows)
    assert loss == pytest.approx(full_loss, rel=1e-12)
    np.testing.assert_allclose(h[:len(batch)], full_h[batch], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g, full_g, rtol=1e-10, atol=1e-14)
    short_list, short_sub, _ = minibatch.extract(seq.edges, batch, hops - 1)
    _, h_short, _ = _run_integrated(wl, wli, oracle.graphs_of(short_sub, len(short_list)), [x[short_list] for x in feats], flat,
                                    target[short_list], rows)
    assert not np.allclose(h_short[:len(batch)], full_h[batch], rtol=1e-9, atol=1e-12)


def test_integrated_batch_losses_add_up_and_match_finite_differences():
    wl, wli, seq, feats, flat, target = _model_integrated("mean", "gru", n=30, degree=2.0)
    n = wl.num_nodes
    graphs = oracle.graphs_of(seq.edges, n)
    full_loss, _, full_g = _run_integrated(wl, wli, graphs, feats, flat, target, None)
    perm = np.random.default_rng(1).permutation(n)
    parts = [perm[:7], perm[7:19], perm[19:]]
    runs = [_run_integrated(wl, wli, graphs, feats, flat, target, b) for b in parts]
    assert sum(len(b) / n * r[0] for b, r in zip(parts, runs)) == pytest.approx(full_loss, rel=1e-12)
    np.testing.assert_allclose(sum(len(b) / n * r[2] for b, r in zip(parts, runs)), full_g, rtol=1e-10, atol=1e-15)
    batch, grad, eps = parts[0], runs[0][2], 1e-6
    for i in np.random.default_rng(0).choice(flat.size, 20, replace=False):
        fp, fm = flat.copy(), flat.copy()
        fp[i] += eps
        fm[i] -= eps
        num = (_run_integrated(wl, wli, graphs, feats, fp, target, batch)[0] -
               _run_integrated(wl, wli, graphs, feats, fm, target, batch)[0]) / (2 * eps)
        assert abs(num - grad[i]) <= 1e-6 * max(1.0, abs(num)) + 1e-9, (i, num, grad[i])
