"""Pins for the reference window forward/backward (Section 2.2: the forward pass runs over the whole
sequence and gradients flow back across timesteps): central finite differences in fp64 and
torch.autograd on the same model written with a dense normalised adjacency."""
import itertools

import numpy as np
import pytest
import torch

import oracle
from paper_2501_15348_amd import synth


def _setup(mode, rnn, layers, n=30, T=3, d=4, hid=3, seed=0):
    dims = (d,) + (5,) * layers
    wl = synth.Workload("fd", n, 3.0, T, "uniform", 0.0, 0.2, 0.2, "fp32", mode, True, dims, rnn, hid, T, seed)
    seq = synth.make_sequence(wl)
    graphs = oracle.graphs_of(seq.edges, n)
    feats = [oracle.features_at(seq.x0, seq.feat_rows, seq.feat_vals, t) for t in range(T)]
    flat = synth.make_params(wl, bias_scale=0.3).astype(np.float64)
    target = synth.make_target(wl).astype(np.float64)
    return wl, graphs, feats, flat, target


def _loss(wl, graphs, feats, flat, target):
    p = synth.split_params(wl, flat)
    return oracle.forward_window(graphs, feats, p, len(wl.dims) - 1, wl.agg, wl.self_loop, wl.rnn, target)[0]


def _grads(wl, graphs, feats, flat, target):
    p = synth.split_params(wl, flat)
    L = len(wl.dims) - 1
    loss, h, saved = oracle.forward_window(graphs, feats, p, L, wl.agg, wl.self_loop, wl.rnn, target, keep=True)
    g = oracle.backward_window(graphs, saved, h, p, L, wl.agg, wl.self_loop, wl.rnn, target)
    return loss, np.concatenate([g[name].ravel() for name, _ in synth.param_shapes(wl)])


@pytest.mark.parametrize("mode,rnn,layers", [("sum", "gru", 1), ("sym", "gru", 2), ("mean", "lstm", 2)])
def test_finite_differences(mode, rnn, layers):
    wl, graphs, feats, flat, target = _setup(mode, rnn, layers)
    _, grad = _grads(wl, graphs, feats, flat, target)
    rng = np.random.default_rng(0)
    idx = rng.choice(flat.size, 40, replace=False)
    eps = 1e-6
    for i in idx:
        fp, fm = flat.copy(), flat.copy()
        fp[i] += eps
        fm[i] -= eps
        num = (_loss(wl, graphs, feats, fp, target) - _loss(wl, graphs, feats, fm, target)) / (2 * eps)
        assert abs(num - grad[i]) <= 1e-6 * max(1.0, abs(num)) + 1e-9, (i, num, grad[i])


def _dense_ahat(g, mode, self_loop):
    n = g.n
    a = np.zeros((n, n))
    rows = np.repeat(np.arange(n), np.diff(g.row_ptr))
    a[rows, g.col] = 1.0
    if self_loop:
        a += np.eye(n)
    deg = a.sum(1)
    if mode == "mean":
        a = a / np.where(deg > 0, deg, 1)[:, None]
    elif mode == "sym":
        s = np.where(deg > 0, deg, 1) ** -0.5
        a = s[:, None] * a * s[None, :]
    return torch.from_numpy(a)


@pytest.mark.parametrize("mode,rnn,layers", [("sum", "gru", 1), ("sym", "gru", 2), ("mean", "lstm", 2), ("sum", "lstm", 1)])
def test_against_torch_autograd(mode, rnn, layers):
    wl, graphs, feats, flat, target = _setup(mode, rnn, layers, seed=1)
    loss, grad = _grads(wl, graphs, feats, flat, target)
    tflat = torch.tensor(flat, requires_grad=True)
    p = {}
    off = 0
    for name, shp in synth.param_shapes(wl):
        sz = int(np.prod(shp))
        p[name] = tflat[off : off + sz].reshape(shp)
        off += sz
    hid = wl.hidden
    h = torch.zeros(wl.num_nodes, hid, dtype=torch.float64)
    c = torch.zeros_like(h)
    for g, x in zip(graphs, feats):
        a = _dense_ahat(g, mode, wl.self_loop)
        hl = torch.from_numpy(x)
        for l in range(1, layers + 1):
            hl = torch.relu(a @ hl @ p[f"W{l}"] + p[f"b{l}"])
        if rnn == "gru":
            h = torch._VF.gru_cell(hl, h, p["W_i"].T, p["W_h"].T, p["b_i"], p["b_h"])
        else:
            h, c = torch._VF.lstm_cell(hl, (h, c), p["W_i"].T, p["W_h"].T, p["b_i"], p["b_h"])
    tl = torch.mean((h - torch.from_numpy(target)) ** 2)
    tl.backward()
    assert abs(tl.item() - loss) < 1e-12
    assert np.allclose(grad, tflat.grad.numpy(), rtol=1e-9, atol=1e-12)


def test_layer1_aggregate_is_weight_independent():
    """Reuse across sequences applies to the first layer because its aggregate does not depend on the
    weights (Section 3.1)."""
    wl, graphs, feats, flat, target = _setup("mean", "gru", 2)
    L = 2
    _, _, s1 = oracle.forward_window(graphs, feats, synth.split_params(wl, flat), L, "mean", True, "gru", target, keep=True)
    _, _, s2 = oracle.forward_window(graphs, feats, synth.split_params(wl, flat * 1.7 + 0.1), L, "mean", True, "gru", target, keep=True)
    for a, b in zip(s1, s2):
        assert np.array_equal(a["aggs"][0], b["aggs"][0])
        assert not np.array_equal(a["aggs"][1], b["aggs"][1])
