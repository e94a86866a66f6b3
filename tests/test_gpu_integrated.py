"""GPU parity for the integrated model (paper Sections 2.1 and 3.1: the recurrent gates work on Agg(x_t) and
Agg(h_{t-1}), each aggregated once per timestep and shared by all gates): forward, loss and back-propagation through
time against the CPU reference, with the layer-1 aggregate coming from the global cache / the incremental rule."""
import dataclasses

import numpy as np
import pytest

import oracle
from helpers import GRAD_RTOL_FP32, RTOL_FP32, assert_close, oracle_feats, oracle_graphs
from paper_2501_15348_amd import synth

pytestmark = pytest.mark.gpu


def _dev(a):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


CASES = [
    ("tiny", None, None, {}),                                              # 16 -> 16, GRU, sum + self-loop
    ("c2", 3001, 6, {}),                                                   # sym, GRU, 64 / 64
    ("c3", 2003, 5, dict(dims=(128, 128, 128))),                           # mean, LSTM, 128 / 128
    ("c5_10", 2500, 5, dict(rnn="lstm", self_loop=False)),                 # sum without self-loops
    ("c4", 1200, 4, {}),                                                   # bf16 features 256, GRU 128
]


@pytest.mark.parametrize("name,n,T,kw", CASES)
def test_forward_and_backward_match_reference(name, n, T, kw):
    import torch
    from paper_2501_15348_amd import reinc

    wl = synth.WORKLOADS[name]
    if n:
        wl = wl.scaled(n, T, **kw)
    wli = dataclasses.replace(wl, dims=(wl.dims[0],))  # parameter shapes of the integrated model: the cell only
    seq = synth.make_sequence(wl)
    ctx = reinc.Context.for_workload(wl, arena_bytes=1 << 30)
    ctx.load_sequence(seq)
    ctx.build_deltas(-1)
    flat = synth.make_params(wli, bias_scale=0.2)
    target = synth.make_target(wl)
    graphs = oracle_graphs(seq)
    T = wl.num_snapshots
    L = min(T, 4)
    params, tgt = _dev(flat), _dev(target)
    loss = torch.zeros(1, device="cuda")
    h_last = torch.empty((wl.num_nodes, wl.hidden), device="cuda")
    grads = torch.empty_like(params)
    p = synth.split_params(wli, flat.astype(np.float64))
    for t0 in (0, T - L):
        print(f"[{wl.name}] integrated window t0={t0} L={L}", flush=True)
        ctx.forward_window_integrated(t0, L, params, tgt, loss, h_last)
        ctx.backward_window_integrated(t0, L, params, tgt, grads)
        torch.cuda.synchronize()
        feats = [oracle_feats(seq, t) for t in range(t0, t0 + L)]
        ref_loss, ref_h, saved = oracle.forward_window_integrated(graphs[t0:t0 + L], feats, p, wl.agg, wl.self_loop, wl.rnn, target,
                                                                  keep=True)
        assert_close(h_last.cpu().numpy(), ref_h, RTOL_FP32, "h_last")
        assert abs(loss.item() - ref_loss) <= RTOL_FP32 * abs(ref_loss), (loss.item(), ref_loss)
        ref_g = oracle.backward_window_integrated(graphs[t0:t0 + L], saved, ref_h, p, wl.agg, wl.self_loop, wl.rnn, target)
        got = synth.split_params(wli, grads.cpu().numpy())
        for name_, _ in synth.param_shapes(wli):
            assert_close(got[name_], ref_g[name_], GRAD_RTOL_FP32, f"grad {name_} (t0={t0})")
    st = ctx.get_stats()
    assert st["global_hits"] + st["global_misses"] == 2 * L  # the input aggregates went through the global cache
    ctx.close()


def test_stacked_and_integrated_windows_can_alternate():
    """Both models share the layer-1 cache and take turns with the local cache; a backward call must follow the
    forward call of its own model."""
    import torch
    from paper_2501_15348_amd import reinc

    wl = synth.WORKLOADS["tiny"]
    wli = dataclasses.replace(wl, dims=(wl.dims[0],))
    seq = synth.make_sequence(wl)
    ctx = reinc.Context.for_workload(wl, arena_bytes=1 << 28)
    ctx.load_sequence(seq)
    ctx.build_deltas(-1)
    ps, pi = _dev(synth.make_params(wl)), _dev(synth.make_params(wli))
    tgt = _dev(synth.make_target(wl))
    loss = torch.zeros(1, device="cuda")
    gs, gi = torch.empty_like(ps), torch.empty_like(pi)
    ctx.forward_window(0, 4, ps, tgt, loss)
    l_stacked = loss.item()
    ctx.forward_window_integrated(0, 4, pi, tgt, loss)
    with pytest.raises(reinc.ReincError) as e:  # the local cache now belongs to the integrated model
        ctx.backward_window(0, 4, ps, tgt, gs)
    assert e.value.code == reinc.E_STATE
    ctx.backward_window_integrated(0, 4, pi, tgt, gi)
    ctx.forward_window(0, 4, ps, tgt, loss)
    ctx.backward_window(0, 4, ps, tgt, gs)
    torch.cuda.synchronize()
    assert loss.item() == l_stacked and bool(torch.isfinite(gs).all()) and bool(torch.isfinite(gi).all())
    ctx.close()
