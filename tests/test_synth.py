"""Generator invariants: sizes, distinctness, ground-truth lists, determinism."""
import numpy as np

from paper_2501_15348_amd import synth


def _keys(src, dst):
    return (dst.astype(np.int64) << 32) | src.astype(np.int64)


def test_tiny_shapes(tiny_seq):
    wl = tiny_seq.workload
    assert tiny_seq.num_snapshots == 8
    for t, (s, d) in enumerate(tiny_seq.edges):
        assert s.dtype == np.int32 and d.dtype == np.int32
        assert len(s) == 5000 and np.all(s != d)
        assert np.unique(_keys(s, d)).size == 5000
        assert s.min() >= 0 and s.max() < wl.num_nodes
    assert tiny_seq.x0.shape == (1000, 16) and tiny_seq.x0.dtype == np.float32
    for t in range(1, 8):
        assert len(tiny_seq.truth_inserted[t]) == 50 == len(tiny_seq.truth_deleted[t])
        r = tiny_seq.feat_rows[t]
        assert len(r) == 10 and np.all(np.diff(r) > 0)
        assert tiny_seq.feat_vals[t].shape == (10, 16)


def test_truth_lists_replay(tiny_seq):
    cur = set(_keys(*tiny_seq.edges[0]).tolist())
    for t in range(1, tiny_seq.num_snapshots):
        ins = set(_keys(*tiny_seq.truth_pairs(t, "ins")).tolist())
        dele = set(_keys(*tiny_seq.truth_pairs(t, "del")).tolist())
        assert dele <= cur and not (ins & cur)
        cur = (cur - dele) | ins
        assert cur == set(_keys(*tiny_seq.edges[t]).tolist())


def test_deterministic():
    wl = synth.WORKLOADS["c2"].scaled(2000, 3)
    a, b = synth.make_sequence(wl), synth.make_sequence(wl)
    for (s1, d1), (s2, d2) in zip(a.edges, b.edges):
        assert np.array_equal(s1, s2) and np.array_equal(d1, d2)
    assert np.array_equal(a.x0, b.x0)
    c = synth.make_sequence(synth.dataclasses.replace(wl, seed=1))
    assert not np.array_equal(a.x0, c.x0)


def test_power_law_has_hubs():
    wl = synth.WORKLOADS["c2"].scaled(20000, 2)
    s = synth.make_sequence(wl)
    indeg = np.bincount(s.edges[0][1], minlength=wl.num_nodes)
    assert len(s.edges[0][0]) == 200000
    assert indeg.max() > 20 * indeg.mean()  # heavy tail
    assert indeg.max() <= 3 * int(np.sqrt(200000))  # capped near sqrt(E)
    assert np.median(indeg) < indeg.mean()


def test_bf16_rounding():
    x = np.array([1.0, 1.00390625, 1.01171875, -3.14159, 1e-8, 65504.0], dtype=np.float32)
    r = synth.round_to_bf16(x)
    import torch

    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(r, ref)
    assert np.array_equal(synth.bf16_bits(r), torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))


def test_params_layout():
    wl = synth.WORKLOADS["c3"]
    flat = synth.make_params(wl, bias_scale=0.1)
    p = synth.split_params(wl, flat)
    assert p["W1"].shape == (128, 128) and p["W_i"].shape == (128, 512) and p["b_h"].shape == (512,)
    assert abs(p["W1"]).max() <= 1 / np.sqrt(128)
    assert synth.make_target(wl.scaled(100)).shape == (100, 128)


def test_impossible_edge_count_is_refused():
    """More edges than distinct pairs exist: the generator says so instead of drawing for ever."""
    import pytest

    with pytest.raises(ValueError):
        synth.make_sequence(synth.WORKLOADS["c5_10"].scaled(3, 2))
