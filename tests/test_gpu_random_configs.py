"""GPU parity on seeded random configurations of the window driver: node counts around tile boundaries, one to three
GCN layers of widths 16..256, GRU / LSTM of 16..128 hidden units, every aggregator, with and without self-loops,
every fallback setting, with and without a cache budget, features loaded whole or as deltas; the stacked model over
every window of the sequence and the integrated model on the first (paper Sections 2.2, 3.2, 3.3)."""
import dataclasses
import random

import numpy as np
import pytest

import oracle
from helpers import GRAD_RTOL_FP32, RTOL_FP32, assert_close, assert_gradients_close, oracle_feats, oracle_graphs
from paper_2501_15348_amd import synth

pytestmark = pytest.mark.gpu


def _config(case):
    rng = random.Random(1000 + case)
    n = rng.choice([31, 33, 64, 95, 257, 1000, 2049, 3333, 5000])
    T = rng.randint(3, 6)
    L = rng.randint(1, min(T, 4))
    agg = rng.choice(["sum", "mean", "sym"])
    layers = rng.choice([1, 2, 2, 3])
    kw = dict(dims=tuple(rng.choice([16, 32, 64, 128, 256]) for _ in range(layers + 1)), hidden=rng.choice([16, 32, 64, 128]),
              agg=agg, rnn=rng.choice(["gru", "lstm"]), self_loop=rng.choice([True, True, False]))
    wl = synth.WORKLOADS[rng.choice(["c2", "c3", "c5_10"])].scaled(n, T, **kw)
    budget = (rng.choice(["score", "lru", "lfu"]), rng.randint(0, L)) if rng.random() < 0.4 else None
    return wl, L, rng.choice([0.5, -1.0, 0.0]), budget, rng.random() < 0.7


@pytest.mark.parametrize("case", range(16))
def test_random_configuration(case):
    import torch
    from paper_2501_15348_amd import reinc

    wl, L, fallback, budget, delta_features = _config(case)
    T = wl.num_snapshots
    print(f"{wl.name}: T={T} L={L} dims={wl.dims} {wl.rnn}{wl.hidden} {wl.agg} self_loop={wl.self_loop} fallback={fallback} "
          f"budget={budget} delta_features={delta_features}", flush=True)
    seq = synth.make_sequence(wl)
    ctx = reinc.Context.for_workload(wl, arena_bytes=1 << 30, fallback_ratio=fallback)
    ctx.load_sequence(seq, delta_features=delta_features)
    ctx.build_deltas(-1)
    if budget:
        ctx.cache_configure(budget[0], budget[1] * ctx.aggregate_bytes(), window=L, stride=1)
    flat = synth.make_params(wl, bias_scale=0.2)
    if wl.agg == "sum":
        # an un-normalised sum multiplies the activations by about the degree at every layer: the layer weights are drawn
        # that much smaller, as trained weights of such a model would be, so that every layer's output stays of order one
        views = synth.split_params(wl, flat)
        for l in range(1, len(wl.dims)):
            views[f"W{l}"] *= np.float32(1.0 / (1.0 + wl.mean_degree))
    target = synth.make_target(wl)
    params, tgt = torch.from_numpy(flat).cuda(), torch.from_numpy(target).cuda()
    loss = torch.zeros(1, device="cuda")
    h_last = torch.empty((wl.num_nodes, wl.hidden), device="cuda")
    grads = torch.empty_like(params)
    graphs_all = oracle_graphs(seq)
    p = synth.split_params(wl, flat.astype(np.float64))
    layers = len(wl.dims) - 1
    for t0 in range(T - L + 1):
        ctx.forward_window(t0, L, params, tgt, loss, h_last)
        ctx.backward_window(t0, L, params, tgt, grads)
        torch.cuda.synchronize()
        graphs = graphs_all[t0:t0 + L]
        feats = [oracle_feats(seq, t) for t in range(t0, t0 + L)]
        ref_loss, ref_h, saved = oracle.forward_window(graphs, feats, p, layers, wl.agg, wl.self_loop, wl.rnn, target, keep=True)
        assert_close(h_last.cpu().numpy(), ref_h, RTOL_FP32, f"h_last (t0={t0})")
        assert abs(loss.item() - ref_loss) <= RTOL_FP32 * abs(ref_loss), (loss.item(), ref_loss)
        assert_gradients_close(
            synth.split_params(wl, grads.cpu().numpy()), saved,
            lambda sv: oracle.backward_window(graphs, sv, ref_h, p, layers, wl.agg, wl.self_loop, wl.rnn, target),
            [name for name, _ in synth.param_shapes(wl)], GRAD_RTOL_FP32)
    # the integrated model (graph operations inside the gates) on the first window of the same sequence
    wli = dataclasses.replace(wl, dims=(wl.dims[0],))
    flat_i = synth.make_params(wli, bias_scale=0.2)
    pi = synth.split_params(wli, flat_i.astype(np.float64))
    params_i = torch.from_numpy(flat_i).cuda()
    grads_i = torch.empty_like(params_i)
    ctx.forward_window_integrated(0, L, params_i, tgt, loss, h_last)
    ctx.backward_window_integrated(0, L, params_i, tgt, grads_i)
    torch.cuda.synchronize()
    feats = [oracle_feats(seq, t) for t in range(L)]
    ref_loss, ref_h, saved = oracle.forward_window_integrated(graphs_all[:L], feats, pi, wl.agg, wl.self_loop, wl.rnn, target, keep=True)
    assert_close(h_last.cpu().numpy(), ref_h, RTOL_FP32, "integrated h_last")
    ref_g = oracle.backward_window_integrated(graphs_all[:L], saved, ref_h, pi, wl.agg, wl.self_loop, wl.rnn, target)
    got = synth.split_params(wli, grads_i.cpu().numpy())
    for name, _ in synth.param_shapes(wli):
        assert_close(got[name], ref_g[name], GRAD_RTOL_FP32, f"integrated grad {name}")
    ctx.close()
