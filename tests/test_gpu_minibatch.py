"""GPU parity for node mini-batches (paper Section 4.2, "Rethinking Mini-batch Training"): the computational graphs
of a node set extracted on the device (bit-exact against the set-based reference), and windows run on the
extracted sub-sequence against the from-scratch reference of the WHOLE graph with the loss taken over the batch
rows -- the extraction must lose nothing the batch depends on.  (The library takes as many hops as there are GCN
layers and carries the degree scales over from the whole graph; the set-based reference, which recomputes degrees
from the kept edges, needs one hop more under the symmetric normalisation: the extraction test passes that count.)"""
import numpy as np
import pytest

import oracle
from oracle import minibatch
from helpers import GRAD_RTOL_FP32, RTOL_FP32, assert_close, assert_gradients_close, oracle_feats, oracle_graphs
from paper_2501_15348_amd import synth

pytestmark = pytest.mark.gpu


def _dev(a):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _workload(mode, rnn, layers, n=3000, T=6, degree=2.5, seed=11, dist="uniform", dims=None):
    dims = dims or (16,) + (32,) * layers
    return synth.Workload("mb", n, degree, T, dist, 2.1 if dist == "chunglu" else 0.0, 0.05, 0.02, "fp32", mode, True, dims, rnn,
                          32, 4, seed)


def _parent(wl, arena=1 << 28):
    from paper_2501_15348_amd import reinc

    seq = synth.make_sequence(wl)
    ctx = reinc.Context.for_workload(wl, arena_bytes=arena)
    ctx.load_sequence(seq)
    return seq, ctx


@pytest.mark.parametrize("mode,hops,dist", [("sum", 1, "uniform"), ("mean", 2, "uniform"), ("sym", 3, "uniform"), ("mean", 2, "chunglu")])
def test_extraction_is_exact(mode, hops, dist):
    wl = _workload(mode, "gru", 2, dist=dist)
    seq, ctx = _parent(wl)
    batch = np.random.default_rng(3).choice(wl.num_nodes, 40, replace=False).astype(np.int32)  # not sorted
    ref_list, ref_sub, ref_inner = minibatch.extract(seq.edges, batch, hops)
    total, inner = ctx.batch_plan(batch, hops)
    assert (total, inner) == (len(ref_list), ref_inner)
    assert np.array_equal(ctx.batch_node_list(total), ref_list)
    child = ctx.batch_context(batch, 1 << 27, hops)
    assert child.n == total
    ref_graphs = oracle.graphs_of(ref_sub, total)
    for t in range(wl.num_snapshots):
        ptr, idx = child.get_snapshot_csr(t)
        assert np.array_equal(ptr, ref_graphs[t].row_ptr) and np.array_equal(idx, ref_graphs[t].col), t
        # the transpose (by source, targets ascending): counting sort of the reference rows
        src, dst = ref_graphs[t].col, np.repeat(np.arange(total), np.diff(ref_graphs[t].row_ptr))
        order = np.lexsort((dst, src))
        tptr, tidx = child.get_snapshot_csr(t, transpose=True)
        assert np.array_equal(tptr, np.concatenate(([0], np.cumsum(np.bincount(src, minlength=total))))), t
        assert np.array_equal(tidx, dst[order]), t
        # aggregation over the extracted structure (row order lists, long-row lists, both directions) against the
        # dense definition on the same graph
        x = np.random.default_rng(t).standard_normal((total, 16)).astype(np.float32)
        dense = np.zeros((total, total))
        dense[dst, src] = 1.0
        # (source-side scales under the symmetric normalisation: the degrees of the WHOLE graph, carried over)
        scale = np.ones(total)
        if mode == "sym":
            scale = (1.0 + np.bincount(seq.edges[t][1], minlength=wl.num_nodes))[ref_list] ** -0.5
        a = dense + np.eye(total)
        for transpose in (False, True):
            got = child.aggregate_full(t, _dev(x), transpose=transpose).cpu().numpy()
            want = scale[:, None] * (a.T @ x) if transpose else a @ (scale[:, None] * x)
            assert_close(got, want, RTOL_FP32, f"aggregate over the extracted snapshot {t}, transpose {transpose}")
    assert total < wl.num_nodes
    child.close()
    # a second plan on the same context replaces the first
    other = np.arange(5, dtype=np.int32)
    total2, _ = ctx.batch_plan(other, hops)
    assert np.array_equal(ctx.batch_node_list(total2), minibatch.extract(seq.edges, other, hops)[0])
    ctx.close()


@pytest.mark.parametrize("mode,rnn,layers", [("sum", "gru", 1), ("mean", "lstm", 2), ("sym", "gru", 2)])
def test_batch_windows_match_the_whole_graph_reference(mode, rnn, layers):
    _check_batch_windows(mode, rnn, layers)


@pytest.mark.parametrize("mode,rnn,dims", [("sum", "gru", (16, 32, 32, 32)), ("mean", "lstm", (16, 32, 16)),
                                           ("sym", "gru", (16, 32, 16, 16)), ("mean", "gru", (16, 32, 32, 16))])
def test_layers_below_the_last_run_on_their_hop_sets(mode, rnn, dims):
    """Layer l of L is computed on the nodes within L - l hops of the batch only (a prefix of the numbering); three
    layers, and layers that narrow their input (linear map before the aggregation) in every position."""
    _check_batch_windows(mode, rnn, len(dims) - 1, degree=1.5, dims=dims, prefixes=True)


@pytest.mark.parametrize("mode,rnn,dims", [("mean", "lstm", (16, 32, 32)), ("sym", "gru", (16, 32, 16, 16))])
def test_batch_windows_with_every_row_of_the_layers_below(mode, rnn, dims, monkeypatch):
    """The same with the restriction of the layers below the last switched off: only the last layer and the cell work
    on the batch rows."""
    monkeypatch.setenv("REINC_LAYER_ROWS", "1e12")
    _check_batch_windows(mode, rnn, len(dims) - 1, dims=dims)


def test_batch_windows_with_three_timesteps_per_launch(monkeypatch):
    """A window of four timesteps in launches of three and one: the compact slices of the last layer and of the cell
    are adjacent within a launch's timesteps only."""
    monkeypatch.setenv("REINC_BATCH", "3")
    _check_batch_windows("mean", "lstm", 2)
    _check_batch_windows("sum", "gru", 2)


def test_batch_windows_with_hub_rows_and_columns():
    """A power-law graph: the batch graph has rows and columns beyond the length at which the aggregation kernels
    switch to a block per row, in the forward pass (rows) and in the backward pass (columns)."""
    _check_batch_windows("sym", "gru", 2, dist="chunglu", degree=12.0, hubs=True)


def _check_batch_windows(mode, rnn, layers, dist="uniform", degree=2.5, hubs=False, dims=None, prefixes=False):
    import torch

    wl = _workload(mode, rnn, layers, dist=dist, degree=degree, dims=dims)
    seq, ctx = _parent(wl)
    n, T, L, H = wl.num_nodes, wl.num_snapshots, 4, wl.hidden
    batch = np.random.default_rng(8).choice(n, 64, replace=False).astype(np.int32)
    if hubs:  # the node with the most in-edges joins the batch
        batch[0] = np.argmax(np.bincount(seq.edges[0][1], minlength=n))
        batch = np.unique(batch).astype(np.int32)
    if prefixes:
        # a batch context whose memory starts out as NaN: a row that no layer computes must not be read by any other
        from paper_2501_15348_amd import reinc

        total, _ = ctx.batch_plan(batch)
        child = reinc.Context(total, ctx.T, ctx.dims, ctx.rnn, ctx.hidden, mode, True, "fp32", arena_bytes=1 << 28)
        child.arena[:child.arena.numel() // 4 * 4].view(torch.float32).fill_(float("nan"))
        ctx._ck(ctx.lib.reinc_batch_load(ctx.handle, child.handle))
    else:
        child = ctx.batch_context(batch, 1 << 28)  # default hop count
    node_list = ctx.batch_node_list(child.n)
    assert child.n < n or hubs
    if prefixes:  # the case does separate the hop sets: every layer has its own row count
        reach = [len(f) for f in minibatch.closure(seq.edges, batch, layers)]
        assert all(a < b for a, b in zip(reach, reach[1:])) and reach[-1] == child.n, reach
    if hubs:
        ptr, idx = child.get_snapshot_csr(0)
        assert np.diff(ptr).max() > 64 and np.bincount(idx).max() > 64
    child.build_deltas(-1)
    flat = synth.make_params(wl, bias_scale=0.2)
    target = synth.make_target(wl)
    params, tgt = _dev(flat), _dev(target[node_list])
    loss = torch.zeros(1, device="cuda")
    h_last = torch.empty((child.n, H), device="cuda")
    grads = torch.empty_like(params)
    graphs = oracle_graphs(seq)
    p = synth.split_params(wl, flat.astype(np.float64))
    names = [name for name, _ in synth.param_shapes(wl)]
    for t0 in (0, 1, T - L):  # seq-first: the windows of one batch slide over the sequence
        print(f"[{wl.name} {mode} {rnn}] window t0={t0}", flush=True)
        child.forward_window(t0, L, params, tgt, loss, h_last)
        child.backward_window(t0, L, params, tgt, grads)
        torch.cuda.synchronize()
        g = graphs[t0:t0 + L]
        feats = [oracle_feats(seq, t) for t in range(t0, t0 + L)]
        ref_loss, ref_h, saved = oracle.forward_window(g, feats, p, layers, wl.agg, wl.self_loop, wl.rnn, target, keep=True,
                                                       loss_rows=batch)
        assert_close(h_last.cpu().numpy()[:len(batch)], ref_h[batch], RTOL_FP32, "h_last on the batch rows")
        assert abs(loss.item() - ref_loss) <= RTOL_FP32 * abs(ref_loss), (loss.item(), ref_loss)
        assert_gradients_close(
            synth.split_params(wl, grads.cpu().numpy()), saved,
            lambda sv: oracle.backward_window(g, sv, ref_h, p, layers, wl.agg, wl.self_loop, wl.rnn, target, loss_rows=batch),
            names, GRAD_RTOL_FP32)
    st = child.get_stats()
    assert st["global_hits"] == 3 + 3 and st["global_misses"] == 4 + 1 + 1  # the batch's cache serves its later windows
    child.close()
    ctx.close()


def test_bf16_features_and_a_cache_budget_in_the_batch_context():
    """bfloat16 feature rows are gathered as bit patterns; the batch context takes a cache budget like any other."""
    import dataclasses

    import torch

    from helpers import RTOL_BF16

    wl = dataclasses.replace(_workload("mean", "gru", 2), feat_dtype="bf16")
    seq, ctx = _parent(wl)
    n, T, L, H = wl.num_nodes, wl.num_snapshots, 4, wl.hidden
    batch = np.random.default_rng(2).choice(n, 48, replace=False).astype(np.int32)
    child = ctx.batch_context(batch, 1 << 28)
    node_list = ctx.batch_node_list(child.n)
    child.build_deltas(-1)
    child.cache_configure("score", 2 * child.aggregate_bytes(), window=L, stride=1)
    flat, target = synth.make_params(wl, bias_scale=0.2), synth.make_target(wl)
    params, tgt = _dev(flat), _dev(target[node_list])
    loss = torch.zeros(1, device="cuda")
    h_last = torch.empty((child.n, H), device="cuda")
    graphs = oracle_graphs(seq)
    p = synth.split_params(wl, flat.astype(np.float64))
    for t0 in range(T - L + 1):
        child.forward_window(t0, L, params, tgt, loss, h_last)
        torch.cuda.synchronize()
        feats = [oracle_feats(seq, t) for t in range(t0, t0 + L)]
        ref_loss, ref_h, _ = oracle.forward_window(graphs[t0:t0 + L], feats, p, 2, wl.agg, wl.self_loop, wl.rnn, target, loss_rows=batch)
        assert_close(h_last.cpu().numpy()[:len(batch)], ref_h[batch], RTOL_BF16, f"h_last on the batch rows, window {t0}")
        assert abs(loss.item() - ref_loss) <= RTOL_BF16 * abs(ref_loss)
    st = child.get_stats()
    assert 0 < st["global_hits"] <= 2 * (T - L) and st["global_peak_bytes"] <= 2 * child.aggregate_bytes()
    child.close()
    ctx.close()


def test_loss_rows_on_an_ordinary_context():
    import torch

    wl = _workload("mean", "gru", 1, n=500, T=4)
    seq, ctx = _parent(wl)
    ctx.build_deltas(-1)
    flat, target = synth.make_params(wl, bias_scale=0.2), synth.make_target(wl)
    params, tgt = _dev(flat), _dev(target)
    loss = torch.zeros(1, device="cuda")
    grads = torch.empty_like(params)
    graphs = oracle_graphs(seq)
    feats = [oracle_feats(seq, t) for t in range(4)]
    p = synth.split_params(wl, flat.astype(np.float64))
    from paper_2501_15348_amd import reinc

    # growing and shrinking row counts: the compact slices of the recurrent state move, the zero state must stay zero
    for rows in (123, 0, 300, 50):
        ctx.set_loss_rows(rows)
        with pytest.raises(reinc.ReincError, match="forward pass"):
            ctx.backward_window(0, 4, params, tgt, grads)  # the rows changed: the last forward pass does not count
        ctx.forward_window(0, 4, params, tgt, loss)
        ctx.backward_window(0, 4, params, tgt, grads)
        torch.cuda.synchronize()
        sel = np.arange(rows) if rows else None
        ref_loss, ref_h, saved = oracle.forward_window(graphs, feats, p, 1, wl.agg, wl.self_loop, wl.rnn, target, keep=True, loss_rows=sel)
        assert abs(loss.item() - ref_loss) <= RTOL_FP32 * abs(ref_loss)
        assert_gradients_close(
            synth.split_params(wl, grads.cpu().numpy()), saved,
            lambda sv: oracle.backward_window(graphs, sv, ref_h, p, 1, wl.agg, wl.self_loop, wl.rnn, target, loss_rows=sel),
            [name for name, _ in synth.param_shapes(wl)], GRAD_RTOL_FP32)
    ctx.close()


def test_error_paths():
    from paper_2501_15348_amd import reinc

    wl = _workload("mean", "gru", 1, n=400, T=3)
    seq, ctx = _parent(wl, arena=1 << 26)
    with pytest.raises(reinc.ReincError, match="twice"):
        ctx.batch_plan(np.array([5, 9, 5], dtype=np.int32))
    with pytest.raises(reinc.ReincError, match="out of range"):
        ctx.batch_plan(np.array([5, 400], dtype=np.int32))
    with pytest.raises(reinc.ReincError, match="between 1 and"):
        ctx.batch_plan(np.array([], dtype=np.int32))
    with pytest.raises(reinc.ReincError, match="no node batch"):
        ctx.batch_node_list(1)  # the failed plans left nothing behind
    with pytest.raises(reinc.ReincError, match="loss rows"):
        ctx.set_loss_rows(401)
    total, _ = ctx.batch_plan(np.array([7, 3], dtype=np.int32))
    wrong = reinc.Context(total + 1, wl.num_snapshots, wl.dims, wl.rnn, wl.hidden, wl.agg, wl.self_loop, arena_bytes=1 << 24)
    rc = ctx.lib.reinc_batch_load(ctx.handle, wrong.handle)
    assert rc == reinc.E_ARG and b"needs" in ctx.lib.reinc_last_error(ctx.handle)
    wrong.close()
    # the whole graph as a batch: every node is a batch node, the loss covers every row
    everyone = np.random.default_rng(0).permutation(400).astype(np.int32)
    child = ctx.batch_context(everyone, 1 << 26)
    assert child.n == 400 and np.array_equal(ctx.batch_node_list(400), everyone)
    child.close()
    # a context without its snapshots cannot plan
    empty = reinc.Context.for_workload(wl, arena_bytes=1 << 24)
    with pytest.raises(reinc.ReincError, match="must be loaded"):
        empty.batch_plan(np.array([1], dtype=np.int32))
    empty.close()
    ctx.close()


def test_integrated_model_on_a_batch_context_reads_every_row():
    """After a stacked window the cached layer-1 sums of a batch context hold the rows that layer 1 needs; the integrated
    model's first timestep needs more of them (here every row: three timesteps on a two-hop sub-sequence), so its window
    drops the short sums and computes longer ones: h against the reference model run on the extracted graphs (sum
    aggregation: no scales carried over from the whole graph), on the batch rows, and on every row once the loss rows
    are taken back."""
    import dataclasses
    import torch

    wl = _workload("sum", "gru", 2)
    seq, ctx = _parent(wl)
    batch = np.random.default_rng(5).choice(wl.num_nodes, 50, replace=False).astype(np.int32)
    node_list, sub, _ = minibatch.extract(seq.edges, batch, 2)
    child = ctx.batch_context(batch, 1 << 28)
    assert child.n == len(node_list)
    child.build_deltas(-1)
    L, H = 3, wl.hidden
    flat = _dev(synth.make_params(wl, bias_scale=0.2))
    nb = len(batch)
    h_stacked = torch.empty((child.n, H), device="cuda")
    child.forward_window(0, L, flat, h_last=h_stacked)  # fills the cache with short buffers
    torch.cuda.synchronize()
    first = h_stacked[:nb].clone()
    wli = dataclasses.replace(wl, dims=(wl.dims[0],))
    flat_i = synth.make_params(wli, bias_scale=0.2)
    h_last = torch.empty((child.n, H), device="cuda")
    child.forward_window_integrated(0, L, _dev(flat_i), h_last=h_last)
    torch.cuda.synchronize()
    graphs = oracle.graphs_of(sub, child.n)
    feats = [oracle_feats(seq, t)[node_list] for t in range(L)]
    p = synth.split_params(wli, flat_i.astype(np.float64))
    _, ref_h, _ = oracle.forward_window_integrated(graphs[:L], feats, p, wl.agg, wl.self_loop, wl.rnn, None)
    # (the last timestep exists on the batch rows only; with the loss rows taken back every row is computed)
    assert_close(h_last.cpu().numpy()[:nb], ref_h[:nb], RTOL_FP32, "integrated h_last on a batch context")
    # and the stacked model afterwards finds whole cached sums, of which it reads its rows: the same batch rows as before
    child.forward_window(0, L, flat, h_last=h_stacked)
    torch.cuda.synchronize()
    assert_close(h_stacked[:nb].cpu().numpy(), first.cpu().numpy(), 1e-6, "stacked h_last after the integrated window")
    child.set_loss_rows(0)
    child.forward_window_integrated(0, L, _dev(flat_i), h_last=h_last)
    torch.cuda.synchronize()
    assert_close(h_last.cpu().numpy(), ref_h, RTOL_FP32, "integrated h_last on every row of the sub-sequence")
    child.close()
    ctx.close()


@pytest.mark.parametrize("mode,rnn", [("sum", "gru"), ("mean", "lstm"), ("sym", "gru")])
def test_integrated_model_on_a_batch_of_one_hop_per_timestep(mode, rnn):
    """The integrated model aggregates the hidden state inside the gates (Section 2.1), so what a batch row depends on
    grows by one hop per timestep: a sub-sequence extracted with as many hops as the window is long gives the batch rows,
    the batch loss and the gradients of the whole graph (Section 4.2: the loss of a batch is taken over its nodes)."""
    import dataclasses
    import torch

    wl = _workload(mode, rnn, 1, n=6000, T=5, degree=2.0)
    wli = dataclasses.replace(wl, dims=(wl.dims[0],))
    seq, ctx = _parent(wl)
    n, T, L, H = wl.num_nodes, wl.num_snapshots, 3, wl.hidden
    batch = np.random.default_rng(3).choice(n, 24, replace=False).astype(np.int32)
    # (the library computes timestep i of the window on the nodes within L - 1 - i hops of the batch only: the batch
    # context's memory starts out as NaN, so that a read of a row that no timestep computes shows)
    from paper_2501_15348_amd import reinc

    total, _ = ctx.batch_plan(batch, hops=L)
    child = reinc.Context(total, ctx.T, ctx.dims, ctx.rnn, ctx.hidden, mode, True, "fp32", arena_bytes=1 << 28)
    child.arena[:child.arena.numel() // 4 * 4].view(torch.float32).fill_(float("nan"))
    ctx._ck(ctx.lib.reinc_batch_load(ctx.handle, child.handle))
    node_list = ctx.batch_node_list(child.n)
    reach = [len(f) for f in minibatch.closure(seq.edges, batch, L)]
    assert all(a < b for a, b in zip(reach, reach[1:])) and reach[-1] == child.n < n, reach
    child.build_deltas(-1)
    flat = synth.make_params(wli, bias_scale=0.2)
    target = synth.make_target(wl)
    params, tgt = _dev(flat), _dev(target[node_list])
    loss = torch.zeros(1, device="cuda")
    h_last = torch.empty((child.n, H), device="cuda")
    grads = torch.empty_like(params)
    graphs = oracle_graphs(seq)
    p = synth.split_params(wli, flat.astype(np.float64))
    for t0 in (0, T - L):
        print(f"[{wl.name} {mode} {rnn}] integrated batch window t0={t0}", flush=True)
        child.forward_window_integrated(t0, L, params, tgt, loss, h_last)
        child.backward_window_integrated(t0, L, params, tgt, grads)
        torch.cuda.synchronize()
        g = graphs[t0:t0 + L]
        feats = [oracle_feats(seq, t) for t in range(t0, t0 + L)]
        ref_loss, ref_h, saved = oracle.forward_window_integrated(g, feats, p, wl.agg, wl.self_loop, wl.rnn, target, keep=True,
                                                                  loss_rows=batch)
        assert_close(h_last.cpu().numpy()[:len(batch)], ref_h[batch], RTOL_FP32, "integrated h_last on the batch rows")
        assert abs(loss.item() - ref_loss) <= RTOL_FP32 * abs(ref_loss), (loss.item(), ref_loss)
        ref_g = oracle.backward_window_integrated(g, saved, ref_h, p, wl.agg, wl.self_loop, wl.rnn, target, loss_rows=batch)
        got = synth.split_params(wli, grads.cpu().numpy())
        for name, _ in synth.param_shapes(wli):
            assert_close(got[name], ref_g[name], GRAD_RTOL_FP32, f"grad {name} (t0={t0})")
    child.close()
    ctx.close()
