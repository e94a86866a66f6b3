"""GPU parity at the full sizes of the benchmark workloads, in the launch configuration bench.py times:
integer outputs in full, float outputs in full where the host can recompute them in seconds and on
sampled rows otherwise (paper Section 3.2 for the aggregation, Sections 2.2 / 3.3 for the window)."""
import numpy as np
import pytest

import oracle
from helpers import GRAD_RTOL_FP32, RTOL_BF16, RTOL_FP32, assert_close, assert_gradients_close, oracle_feats
from paper_2501_15348_amd import synth

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


def _setup(name, T, arena_gb, **kw):
    from paper_2501_15348_amd import reinc

    base = synth.WORKLOADS[name]
    wl = base.scaled(base.num_nodes, T, **kw)
    print(f"[{wl.name}] generating {wl.num_nodes} nodes, {wl.num_edges} edges, {T} snapshots", flush=True)
    seq = synth.make_sequence(wl, shuffle_edges=False)
    ctx = reinc.Context.for_workload(wl, arena_bytes=int(arena_gb * (1 << 30)))
    print(f"[{wl.name}] loading", flush=True)
    ctx.load_sequence(seq)
    ctx.build_deltas(-1)
    return wl, seq, ctx


def _check_deltas(ctx, seq, graphs, t):
    n = seq.workload.num_nodes
    (irp, icol), (drp, dcol) = oracle.edge_deltas(graphs[t - 1].keys, graphs[t].keys, n)
    for kind, (erp, ecol) in enumerate(((irp, icol), (drp, dcol))):
        rp, col = ctx.get_delta_csr(t, kind)
        assert np.array_equal(rp, erp) and np.array_equal(col, ecol), f"delta CSR kind {kind} step {t}"
    # the generator's own lists are the ground truth of the diff
    ts, td = seq.truth_pairs(t, "ins")
    assert irp[-1] == ts.size
    counts = oracle.change_counts(graphs[t - 1], graphs[t], oracle_feats(seq, t - 1), oracle_feats(seq, t),
                                  seq.workload.agg, seq.workload.self_loop)
    info = ctx.get_delta_info(t)
    for k in ("n_ins", "n_del", "n_changed", "n_fchg_entries", "n_entries", "n_rows"):
        assert info[k] == counts[k], (k, info[k], counts[k])


def _check_window_full(ctx, wl, seq, graphs, t0, L, rtol, grad_rtol, say):
    """One window at full size through the driver the benchmark times -- layer-1 sums chained by Eq. 2 from the cached
    predecessor, time-batched dense steps, back-propagation through time -- against the from-scratch reference:
    h_last, the loss and every gradient, all rows."""
    import torch

    flat = synth.make_params(wl, bias_scale=0.1)
    target = synth.make_target(wl)
    params, tgt = torch.from_numpy(flat).cuda(), torch.from_numpy(target).cuda()
    loss = torch.zeros(1, device="cuda")
    h = torch.empty((wl.num_nodes, wl.hidden), device="cuda")
    grads = torch.empty_like(params)
    st0 = ctx.get_stats()
    if t0 > 0:
        ctx.forward_window(t0 - 1, 1, params, tgt, loss)  # caches the predecessor's sums: the window's steps chain from it
    ctx.forward_window(t0, L, params, tgt, loss, h)
    ctx.backward_window(t0, L, params, tgt, grads)
    torch.cuda.synchronize()
    st1 = ctx.get_stats()
    assert st1["steps_incremental"] - st0["steps_incremental"] == (L if t0 > 0 else L - 1), (st0, st1)
    say(f"[{wl.name}] window [{t0}, {t0 + L}) done on the GPU; reference forward")
    layers = len(wl.dims) - 1
    feats = [oracle_feats(seq, t) for t in range(t0, t0 + L)]
    p = synth.split_params(wl, flat.astype(np.float64))
    ref_loss, ref_h, saved = oracle.forward_window(graphs[t0:t0 + L], feats, p, layers, wl.agg, wl.self_loop, wl.rnn, target, keep=True)
    del feats
    assert_close(h.cpu().numpy(), ref_h, rtol, f"{wl.name} full-size h_last")
    assert abs(loss.item() - ref_loss) <= rtol * abs(ref_loss), (loss.item(), ref_loss)
    say(f"[{wl.name}] h_last and loss match; reference backward")
    got = synth.split_params(wl, grads.cpu().numpy())
    assert_gradients_close(
        got, saved,
        lambda sv: oracle.backward_window(graphs[t0:t0 + L], sv, ref_h, p, layers, wl.agg, wl.self_loop, wl.rnn, target),
        [name for name, _ in synth.param_shapes(wl)], grad_rtol)
    say(f"[{wl.name}] gradients match")


@pytest.fixture
def say(capsys):
    """Progress lines that reach the terminal while the test runs (the largest cases take minutes on the host side)."""
    def emit(msg):
        with capsys.disabled():
            print(msg, flush=True)
    return emit


def test_bench_workload_c2_full():
    """100k nodes, 1M edges, sym normalisation: deltas, both aggregation paths, and a 3-snapshot window."""
    import torch

    wl, seq, ctx = _setup("c2", 4, 2)
    graphs = oracle.graphs_of(seq.edges, wl.num_nodes)
    for t in (1, 3):
        _check_deltas(ctx, seq, graphs, t)
    s = ctx.aggregate_full(0)
    for t in range(1, 4):
        s = ctx.aggregate_incremental(t, s)
        s_ref, agg_ref = oracle.aggregate(graphs[t].row_ptr, graphs[t].col, oracle_feats(seq, t), wl.agg, wl.self_loop)
        assert_close(s.cpu().numpy(), s_ref, RTOL_FP32, f"incremental S t={t}")
        assert_close(ctx.aggregate_full(t, apply_q=True).cpu().numpy(), agg_ref, RTOL_FP32, f"full Agg t={t}")
    flat = synth.make_params(wl, bias_scale=0.1)
    target = synth.make_target(wl)
    params, tgt = torch.from_numpy(flat).cuda(), torch.from_numpy(target).cuda()
    loss = torch.zeros(1, device="cuda")
    h = torch.empty((wl.num_nodes, wl.hidden), device="cuda")
    grads = torch.empty_like(params)
    ctx.forward_window(1, 3, params, tgt, loss, h)
    ctx.backward_window(1, 3, params, tgt, grads)
    feats = [oracle_feats(seq, t) for t in range(1, 4)]
    p = synth.split_params(wl, flat.astype(np.float64))
    ref_loss, ref_h, saved = oracle.forward_window(graphs[1:4], feats, p, 2, wl.agg, wl.self_loop, wl.rnn, target, keep=True)
    assert_close(h.cpu().numpy(), ref_h, RTOL_FP32, "h_last")
    assert abs(loss.item() - ref_loss) <= RTOL_FP32 * abs(ref_loss)
    ref_g = oracle.backward_window(graphs[1:4], saved, ref_h, p, 2, wl.agg, wl.self_loop, wl.rnn, target)
    got = synth.split_params(wl, grads.cpu().numpy())
    for name, _ in synth.param_shapes(wl):
        assert_close(got[name], ref_g[name], GRAD_RTOL_FP32, f"grad {name}")
    # a node mini-batch extracted at this size (Section 4.2): the same window on the batch's computational graphs
    # against the whole-graph reference with the loss over the batch rows
    batch = np.random.default_rng(4).choice(wl.num_nodes, 2000, replace=False).astype(np.int32)
    print(f"[{wl.name}] node mini-batch of {batch.size}", flush=True)
    child = ctx.batch_context(batch, 2 << 30)
    node_list = ctx.batch_node_list(child.n)
    rest = node_list[batch.size:]
    # the batch as given, then the nodes first reached in one hop by ascending id, then those reached in two
    assert np.array_equal(node_list[:batch.size], batch) and np.sum(np.diff(rest) <= 0) <= 1
    assert np.intersect1d(rest, batch).size == 0 and np.unique(node_list).size == child.n <= wl.num_nodes
    child.build_deltas(-1)
    tgt_b = torch.from_numpy(target[node_list]).cuda()
    hb = torch.empty((child.n, wl.hidden), device="cuda")
    child.forward_window(1, 3, params, tgt_b, loss, hb)
    child.backward_window(1, 3, params, tgt_b, grads)
    assert_close(hb.cpu().numpy()[:batch.size], ref_h[batch], RTOL_FP32, "mini-batch h_last")
    ref_loss_b = float(np.mean((ref_h[batch] - target[batch].astype(np.float64)) ** 2))
    assert abs(loss.item() - ref_loss_b) <= RTOL_FP32 * abs(ref_loss_b)
    ref_gb = oracle.backward_window(graphs[1:4], saved, ref_h, p, 2, wl.agg, wl.self_loop, wl.rnn, target, loss_rows=batch)
    got = synth.split_params(wl, grads.cpu().numpy())
    for name, _ in synth.param_shapes(wl):
        assert_close(got[name], ref_gb[name], GRAD_RTOL_FP32, f"mini-batch grad {name}")
    child.close()
    # the integrated model on a batch planned with one hop per timestep of its window (Section 2.1, Section 4.2)
    import dataclasses

    wli = dataclasses.replace(wl, dims=(wl.dims[0],))
    flat_i = synth.make_params(wli, bias_scale=0.1)
    pi = synth.split_params(wli, flat_i.astype(np.float64))
    small = batch[:200]
    print(f"[{wl.name}] integrated model on a node mini-batch of {small.size}, two hops", flush=True)
    child = ctx.batch_context(small, 2 << 30, hops=2)
    node_list = ctx.batch_node_list(child.n)
    child.build_deltas(-1)
    params_i, grads_i = torch.from_numpy(flat_i).cuda(), torch.empty(flat_i.size, device="cuda")
    tgt_b = torch.from_numpy(target[node_list]).cuda()
    hb = torch.empty((child.n, wl.hidden), device="cuda")
    child.forward_window_integrated(1, 2, params_i, tgt_b, loss, hb)
    child.backward_window_integrated(1, 2, params_i, tgt_b, grads_i)
    ref_loss_i, ref_hi, saved_i = oracle.forward_window_integrated(graphs[1:3], feats[:2], pi, wl.agg, wl.self_loop, wl.rnn, target,
                                                                   keep=True, loss_rows=small)
    assert_close(hb.cpu().numpy()[:small.size], ref_hi[small], RTOL_FP32, "integrated mini-batch h_last")
    assert abs(loss.item() - ref_loss_i) <= RTOL_FP32 * abs(ref_loss_i)
    ref_gi = oracle.backward_window_integrated(graphs[1:3], saved_i, ref_hi, pi, wl.agg, wl.self_loop, wl.rnn, target, loss_rows=small)
    got = synth.split_params(wli, grads_i.cpu().numpy())
    for name, _ in synth.param_shapes(wli):
        assert_close(got[name], ref_gi[name], GRAD_RTOL_FP32, f"integrated mini-batch grad {name}")
    child.close()
    ctx.close()


def test_churn_sweep_workload_c5_full():
    """500k nodes, 6M edges, sum aggregation, 10 % churn: incremental chain against the from-scratch reference."""
    wl, seq, ctx = _setup("c5_10", 3, 4)
    graphs = oracle.graphs_of(seq.edges, wl.num_nodes)
    _check_deltas(ctx, seq, graphs, 2)
    s = ctx.aggregate_full(0)
    for t in (1, 2):
        ctx.aggregate_incremental(t, s, s)
        s_ref, _ = oracle.aggregate(graphs[t].row_ptr, graphs[t].col, oracle_feats(seq, t), wl.agg, wl.self_loop)
        assert_close(s.cpu().numpy(), s_ref, RTOL_FP32, f"S t={t}")
    ctx.close()


def test_window_workload_c3_full(say):
    """1M nodes, 16M edges, d = 128, mean aggregation, LSTM 128: deltas in full, aggregates on sampled rows (hubs
    included), and a 3-snapshot window forward + backward against the reference on every row."""
    wl, seq, ctx = _setup("c3", 4, 56)
    n = wl.num_nodes
    say(f"[{wl.name}] loaded; canonical graphs on the host")
    graphs = oracle.graphs_of(seq.edges, n)
    _check_deltas(ctx, seq, graphs, 1)
    rng = np.random.default_rng(0)
    s0 = ctx.aggregate_full(0)
    s1 = ctx.aggregate_incremental(1, s0)
    full1 = ctx.aggregate_full(1, apply_q=True)
    _, _, rows_changed, _ = ctx.get_merged_delta(1)
    deg = np.diff(graphs[1].row_ptr)
    sample = np.unique(np.concatenate([rng.integers(0, n, 300), rng.choice(rows_changed, 300), np.argsort(deg)[-20:], [0, n - 1]]))
    x1 = oracle_feats(seq, 1)
    s_ref, agg_ref = oracle.aggregate_rows(graphs[1].row_ptr, graphs[1].col, x1, sample, wl.agg, wl.self_loop)
    assert_close(s1.cpu().numpy()[sample], s_ref, RTOL_FP32, "incremental S (sampled rows)")
    assert_close(full1.cpu().numpy()[sample], agg_ref, RTOL_FP32, "full Agg (sampled rows)")
    untouched = np.setdiff1d(sample, rows_changed)
    assert np.array_equal(s1.cpu().numpy()[untouched], s0.cpu().numpy()[untouched])
    del s0, s1, full1
    _check_window_full(ctx, wl, seq, graphs, 1, 3, RTOL_FP32, GRAD_RTOL_FP32, say)
    ctx.close()


def test_incremental_chain_of_31_steps_c3(say):
    """Drift of a long chain of Eq. 2 steps (Section 3.2; nothing corrects it): the layer-1 sums of the last of
    workload c3's 32 snapshots, reached by 31 chained incremental steps from the first, against the from-scratch
    fp64 reference on sampled rows (hubs and often-changed rows included) and against the GPU's own from-scratch
    aggregation on every row.  The measured worst errors are recorded with the test's other figures."""
    wl, seq, ctx = _setup("c3", 32, 72)
    n, T = wl.num_nodes, wl.num_snapshots
    s = ctx.aggregate_full(0)
    touched = np.zeros(n, dtype=np.int32)
    for t in range(1, T):
        ctx.aggregate_incremental(t, s, s)
        _, _, rows_changed, _ = ctx.get_merged_delta(t)
        touched[rows_changed] += 1
    say(f"[{wl.name}] 31 chained steps done; rows changed at most {touched.max()} times")
    last = T - 1
    g = oracle.Graph(oracle.canonicalise(*seq.edges[last], n), n)
    x = oracle_feats(seq, last)
    rng = np.random.default_rng(5)
    deg = np.diff(g.row_ptr)
    sample = np.unique(np.concatenate([rng.integers(0, n, 400), np.argsort(deg)[-20:], np.argsort(touched)[-200:], [0, n - 1]]))
    s_ref, _ = oracle.aggregate_rows(g.row_ptr, g.col, x, sample, wl.agg, wl.self_loop)
    s_host = s.cpu().numpy()
    assert_close(s_host[sample], s_ref, RTOL_FP32, "S after 31 chained Eq. 2 steps (sampled rows, vs fp64)")
    scratch = ctx.aggregate_full(last).cpu().numpy()
    assert_close(s_host, scratch, RTOL_FP32, "S after 31 chained Eq. 2 steps (all rows, vs from scratch in fp32)")
    never = touched == 0
    assert never.any() and np.array_equal(s_host[never], ctx.aggregate_full(0).cpu().numpy()[never])
    ctx.close()


def test_bf16_workload_c4_full(say):
    """2.5M nodes, 50M edges, bf16 features of width 256, 10 % churn, 256 -> 256 -> 128, GRU 128: deltas in full,
    aggregates on sampled rows, and a 2-snapshot window forward + backward against the reference on every row."""
    wl, seq, ctx = _setup("c4", 3, 96)
    n = wl.num_nodes
    say(f"[{wl.name}] loaded; canonical graphs on the host")
    graphs = oracle.graphs_of(seq.edges, n)
    _check_deltas(ctx, seq, graphs, 1)
    rng = np.random.default_rng(1)
    s0 = ctx.aggregate_full(0)
    s1 = ctx.aggregate_incremental(1, s0, s0)
    _, _, rows_changed, _ = ctx.get_merged_delta(1)
    deg = np.diff(graphs[1].row_ptr)
    sample = np.unique(np.concatenate([rng.integers(0, n, 200), rng.choice(rows_changed, 200), np.argsort(deg)[-10:]]))
    x1 = seq.x0.copy()
    x1[seq.feat_rows[1]] = seq.feat_vals[1]
    s_ref, _ = oracle.aggregate_rows(graphs[1].row_ptr, graphs[1].col, x1, sample, wl.agg, wl.self_loop)
    assert_close(s1[torch_index(sample)].cpu().numpy(), s_ref, RTOL_BF16, "incremental S (sampled rows)")
    full = ctx.aggregate_full(1)
    assert_close(full[torch_index(sample)].cpu().numpy(), s_ref, RTOL_BF16, "full S (sampled rows)")
    del s0, s1, full, x1
    _check_window_full(ctx, wl, seq, graphs, 1, 2, RTOL_BF16, RTOL_BF16, say)
    ctx.close()


def torch_index(rows):
    import torch

    return torch.from_numpy(np.asarray(rows, dtype=np.int64)).cuda()


def _sampled_rows(n, rng, count=600):
    """Random rows plus the first and last rows of the matrix, of a 32-row tile and of a persistent block's range."""
    edges = [0, 1, 31, 32, n // 2, n - 33, n - 32, n - 2, n - 1]
    return np.unique(np.concatenate([rng.integers(0, n, count), np.asarray(edges)]))


@pytest.mark.parametrize("n,k,m,relu,scale,bias", [
    (800_000, 64, 64, True, True, True),      # a batch of 8 timesteps of workload c2: layer update
    (800_000, 192, 64, False, False, False),  # c2: gate gradients back through W_i
    (1_000_000, 128, 128, True, True, True),  # c3: layer update
    (1_000_000, 512, 128, False, False, False),  # c3: LSTM gate gradients, two passes over K
    (1_000_003, 256, 256, True, True, True),  # c4's first layer width, ragged last tile
])
def test_row_gemm_at_full_size(n, k, m, relu, scale, bias):
    """The dense layer update at the row counts of the benchmark (persistent grid, one block per compute unit):
    sampled output rows against the fp64 reference."""
    import torch
    from paper_2501_15348_amd import reinc

    rng = np.random.default_rng(k + m)
    ctx = reinc.Context(64, 1, (16, 16), "gru", 16, "sum", True, arena_bytes=1 << 20)
    a = torch.randn(n, k, device="cuda")
    w = (rng.standard_normal((k, m)) / np.sqrt(k)).astype(np.float32)
    b = rng.standard_normal(m).astype(np.float32) if bias else None
    rs = torch.rand(n, device="cuda") * 0.9 + 0.1 if scale else None
    print(f"row gemm {n} x {k} -> {m}", flush=True)
    out = ctx.gcn_transform(a, torch.from_numpy(w).cuda(), torch.from_numpy(b).cuda() if bias else None, rs, relu=relu)
    rows = _sampled_rows(n, rng)
    idx = torch_index(rows)
    a_s = a[idx].cpu().numpy().astype(np.float64)
    if scale:
        a_s = a_s * rs[idx].cpu().numpy().astype(np.float64)[:, None]
    ref = oracle.dense_layer(a_s, w, b, relu)
    assert_close(out[idx].cpu().numpy(), ref, RTOL_FP32, f"rows of {n}x{k}x{m}")
    ctx.close()


@pytest.mark.parametrize("kind,n,d,h", [
    ("gru", 100_000, 64, 64),       # c2
    ("lstm", 1_000_000, 128, 128),  # c3: 16 hidden units per wave, two gates per tile
    ("gru", 1_000_003, 128, 128),   # c4's cell, ragged last tile
])
def test_recurrent_step_at_full_size(kind, n, d, h):
    """The fused recurrent step at the row counts of the benchmark: sampled rows against the fp64 cell."""
    import torch
    from paper_2501_15348_amd import reinc

    rng = np.random.default_rng(n % 1000 + d + h)
    ctx = reinc.Context(64, 1, (16, 16), "gru", 16, "sum", True, arena_bytes=1 << 20)
    kg = 3 if kind == "gru" else 4
    x, hp, cp = (torch.randn(n, w, device="cuda") for w in (d, h, h))
    wi = (rng.standard_normal((d, kg * h)) / np.sqrt(d)).astype(np.float32)
    wh = (rng.standard_normal((h, kg * h)) / np.sqrt(h)).astype(np.float32)
    bi = (rng.standard_normal(kg * h) * 0.3).astype(np.float32)
    bh = (rng.standard_normal(kg * h) * 0.3).astype(np.float32)
    saved = torch.empty((n, 4 * h), device="cuda")
    print(f"{kind} step {n} x {d} / {h}", flush=True)
    dev = lambda v: torch.from_numpy(v).cuda()
    h_out, c_out = ctx.rnn_step(kind, x, hp, cp if kind == "lstm" else None, dev(wi), dev(wh), dev(bi), dev(bh), saved)
    rows = _sampled_rows(n, rng)
    idx = torch_index(rows)
    f = lambda t: t[idx].cpu().numpy().astype(np.float64)
    g = lambda v: v.astype(np.float64)
    if kind == "gru":
        ref_h, gates = oracle.gru_cell(f(x), f(hp), g(wi), g(wh), g(bi), g(bh))
    else:
        ref_h, ref_c, gates = oracle.lstm_cell(f(x), f(hp), f(cp), g(wi), g(wh), g(bi), g(bh))
        assert_close(c_out[idx].cpu().numpy(), ref_c, RTOL_FP32, "c")
    assert_close(h_out[idx].cpu().numpy(), ref_h, RTOL_FP32, "h")
    assert_close(saved[idx].cpu().numpy(), np.concatenate(gates, axis=1), RTOL_FP32, "saved gates")
    ctx.close()
