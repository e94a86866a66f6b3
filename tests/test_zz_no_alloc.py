"""The incremental max / min step through the entry point that allocates nothing (its work area is a static device
array inside the library): results must equal those of reinc_aggregate_incremental_minmax, which takes the work
buffer from the caller -- values, contributor ids and the count of re-aggregated rows bit for bit -- on two calls
in a row, the second on a smaller graph (the shared work area keeps the first call's contents)."""
import numpy as np
import pytest

from paper_2501_15348_amd import synth

pytestmark = pytest.mark.gpu


def _ctx(wl, arena=1 << 30):
    from paper_2501_15348_amd import reinc

    seq = synth.make_sequence(wl)
    ctx = reinc.Context.for_workload(wl, arena_bytes=arena)
    ctx.load_sequence(seq)
    ctx.build_deltas(-1)
    return ctx


def _compare_chain(ctx, op, label):
    """Chains both entry points over every step, in place and into new buffers; returns the re-aggregated row counts."""
    import torch

    m0, c0 = ctx.aggregate_full_minmax(0, op)
    m_ref, c_ref = m0.clone(), c0.clone()      # in place, caller's work buffer
    m_new, c_new = m0.clone(), c0.clone()      # in place, static work area
    out_m, out_c = torch.empty_like(m0), torch.empty_like(c0)
    redone = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    counts = []
    for t in range(1, ctx.T):
        print(f"[{label}] {op} step {t}", flush=True)
        # into new buffers from the same previous state
        exp_m, exp_c, work = ctx.aggregate_incremental_minmax(t, op, m_ref, c_ref)
        ctx.aggregate_incremental_minmax_static(t, op, m_new, c_new, out_m, out_c, redone)
        torch.cuda.synchronize()
        assert torch.equal(out_m, exp_m) and torch.equal(out_c, exp_c), f"{label} step {t}: new buffers"
        assert int(redone.item()) == int(work[0].item()), f"{label} step {t}: count"
        # in place along the chain
        _, _, work = ctx.aggregate_incremental_minmax(t, op, m_ref, c_ref, m_ref, c_ref)
        ctx.aggregate_incremental_minmax_static(t, op, m_new, c_new, m_new, c_new, redone)
        torch.cuda.synchronize()
        assert torch.equal(m_new, m_ref) and torch.equal(c_new, c_ref), f"{label} step {t}: in place"
        assert int(redone.item()) == int(work[0].item()), f"{label} step {t}: count in place"
        counts.append(int(redone.item()))
    return counts


def test_static_work_area_matches_caller_buffer_twice_second_smaller():
    big = _ctx(synth.WORKLOADS["c2"].scaled(6001, 4, agg="sum"))        # power-law: hub rows take the block path
    small = _ctx(synth.WORKLOADS["tiny"].scaled(700, 4, edge_churn=0.08, feat_churn=0.05))
    a = _compare_chain(big, "max", "6001 nodes")
    b = _compare_chain(small, "max", "700 nodes")      # second call, smaller input, same static array
    c = _compare_chain(small, "min", "700 nodes")
    assert any(x > 0 for x in a) and any(x > 0 for x in b + c)
    big.close()
    small.close()


def test_count_pointer_is_optional_and_sizes_beyond_the_maximum_are_refused():
    import torch
    from paper_2501_15348_amd import reinc

    ctx = _ctx(synth.WORKLOADS["tiny"])
    m, c = ctx.aggregate_full_minmax(0, "max")
    exp_m, exp_c, _ = ctx.aggregate_incremental_minmax(1, "max", m, c)
    out_m, out_c = torch.empty_like(m), torch.empty_like(c)
    ctx.aggregate_incremental_minmax_static(1, "max", m, c, out_m, out_c, None)
    torch.cuda.synchronize()
    assert torch.equal(out_m, exp_m) and torch.equal(out_c, exp_c)
    with pytest.raises(reinc.ReincError) as e:  # values in place, contributors not: same checks as the other entry
        ctx.aggregate_incremental_minmax_static(1, "max", m, c, m, out_c)
    assert e.value.code == reinc.E_ARG
    ctx.close()
    too_big = reinc.Context((1 << 20) + 1, 2, (16, 16), "gru", 16, "sum", True, arena_bytes=1 << 20)
    dummy_f = torch.empty(16, device="cuda")
    dummy_i = torch.empty(16, dtype=torch.int32, device="cuda")
    with pytest.raises(reinc.ReincError) as e:
        too_big.aggregate_incremental_minmax_static(1, "max", dummy_f, dummy_i, dummy_f, dummy_i)
    assert e.value.code == reinc.E_ARG and "at most" in str(e.value)
    too_big.close()
