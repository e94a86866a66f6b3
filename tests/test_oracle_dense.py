"""Pins for the dense side of the reference: GCN update (Listing 1 of Section 3.5) and the
recurrent cells (three gates for GRU, four for LSTM: Section 3.3)."""
import numpy as np
import pytest
import torch

import oracle


def test_dense_layer_identity_and_loops():
    rng = np.random.default_rng(0)
    agg = rng.standard_normal((7, 4))
    assert np.array_equal(oracle.dense_layer(agg, np.eye(4), np.zeros(4)), np.maximum(agg, 0))
    w, b = rng.standard_normal((4, 3)), rng.standard_normal(3)
    ref = np.zeros((7, 3))
    for i in range(7):
        for j in range(3):
            acc = b[j]
            for k in range(4):
                acc += agg[i, k] * w[k, j]
            ref[i, j] = acc
    assert np.allclose(oracle.dense_layer(agg, w, b, relu=False), ref, atol=1e-13)
    assert np.allclose(oracle.dense_layer(agg, w, b), np.maximum(ref, 0), atol=1e-13)


def _rand(rng, *shape):
    return rng.standard_normal(shape)


def test_gru_matches_torch_cell():
    rng = np.random.default_rng(1)
    n, d, h = 6, 5, 4
    x, hp = _rand(rng, n, d), _rand(rng, n, h)
    wi, wh, bi, bh = _rand(rng, d, 3 * h), _rand(rng, h, 3 * h), _rand(rng, 3 * h), _rand(rng, 3 * h)
    cell = torch.nn.GRUCell(d, h).double()
    with torch.no_grad():
        cell.weight_ih.copy_(torch.from_numpy(wi.T))
        cell.weight_hh.copy_(torch.from_numpy(wh.T))
        cell.bias_ih.copy_(torch.from_numpy(bi))
        cell.bias_hh.copy_(torch.from_numpy(bh))
        ref = cell(torch.from_numpy(x), torch.from_numpy(hp)).numpy()
    out, _ = oracle.gru_cell(x, hp, wi, wh, bi, bh)
    assert np.allclose(out, ref, atol=1e-13)


def test_lstm_matches_torch_cell():
    rng = np.random.default_rng(2)
    n, d, h = 6, 5, 4
    x, hp, cp = _rand(rng, n, d), _rand(rng, n, h), _rand(rng, n, h)
    wi, wh, bi, bh = _rand(rng, d, 4 * h), _rand(rng, h, 4 * h), _rand(rng, 4 * h), _rand(rng, 4 * h)
    cell = torch.nn.LSTMCell(d, h).double()
    with torch.no_grad():
        cell.weight_ih.copy_(torch.from_numpy(wi.T))
        cell.weight_hh.copy_(torch.from_numpy(wh.T))
        cell.bias_ih.copy_(torch.from_numpy(bi))
        cell.bias_hh.copy_(torch.from_numpy(bh))
        rh, rc = cell(torch.from_numpy(x), (torch.from_numpy(hp), torch.from_numpy(cp)))
    out_h, out_c, _ = oracle.lstm_cell(x, hp, cp, wi, wh, bi, bh)
    assert np.allclose(out_h, rh.numpy(), atol=1e-13) and np.allclose(out_c, rc.numpy(), atol=1e-13)


def test_zero_weight_closed_forms():
    rng = np.random.default_rng(3)
    n, d, h = 5, 3, 4
    x, hp, cp = _rand(rng, n, d), _rand(rng, n, h), _rand(rng, n, h)
    z3 = (np.zeros((d, 3 * h)), np.zeros((h, 3 * h)), np.zeros(3 * h), np.zeros(3 * h))
    out, _ = oracle.gru_cell(x, hp, *z3)
    assert np.allclose(out, 0.5 * hp)  # z = 1/2, n = 0
    z4 = (np.zeros((d, 4 * h)), np.zeros((h, 4 * h)), np.zeros(4 * h), np.zeros(4 * h))
    oh, oc, _ = oracle.lstm_cell(x, hp, cp, *z4)
    assert np.allclose(oc, 0.5 * cp) and np.allclose(oh, 0.5 * np.tanh(0.5 * cp))
