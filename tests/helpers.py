"""Shared by the GPU parity tests: tolerance rule and oracle-side expectations."""
import json
import os

import numpy as np

import oracle

RTOL_FP32 = 1e-4  # fp32 path
RTOL_BF16 = 2e-2  # bf16 inputs, fp32 accumulation
GRAD_RTOL_FP32 = 1e-4  # gradients of the fp32 path: the same bound as the outputs

_ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
_ERROR_LOG = os.path.join(_ROOT, "gpurun_out", "parity_errors.jsonl")


def record(what, worst, rtol):
    """Notes the measured worst error of one comparison (in the units of the tolerance rule: the rtol that would just
    pass) next to the tolerance it was held to, one JSON line per comparison, where a results folder exists."""
    if not os.path.isdir(os.path.dirname(_ERROR_LOG)):
        return
    try:
        with open(_ERROR_LOG, "a") as f:
            f.write(json.dumps({"test": os.environ.get("PYTEST_CURRENT_TEST", "").split(" ")[0], "what": what,
                                "worst": float(worst), "rtol": float(rtol)}) + "\n")
    except OSError:
        pass


def assert_close(got, ref, rtol, what=""):
    """|got - ref| <= rtol * |ref| + rtol * rms(ref), element-wise.  A purely relative bound is ill-defined
    where sums of zero-mean values cancel, so the absolute floor is tied to the tensor's own scale."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    if ref.size == 0:
        return
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    rms = float(np.sqrt(np.mean(ref * ref)))
    err = np.abs(got - ref)
    bound = rtol * np.abs(ref) + rtol * rms
    denom = np.abs(ref) + rms
    if what:
        record(what, float(np.max(np.where(denom > 0, err / np.where(denom > 0, denom, 1.0), np.where(err > 0, np.inf, 0.0)))), rtol)
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {ref.size} outside tolerance; worst at {i}: got {got[i]!r} ref {ref[i]!r} "
                             f"(rms {rms:.3g}, rtol {rtol})")


def oracle_graphs(seq):
    return oracle.graphs_of(seq.edges, seq.workload.num_nodes)


def oracle_feats(seq, t):
    return oracle.features_at(seq.x0, seq.feat_rows, seq.feat_vals, t)


def expected_merged_delta(g_prev, g_cur, x_prev, x_cur, mode, self_loop):
    """The library's merged delta rows, derived from the oracle's CSRs: per row the inserted sources, the
    deleted sources, then positions (in the ascending change set) of changed sources among the row's
    current in-edges, the row's own entry last."""
    n = g_cur.n
    (irp, icol), (drp, dcol) = oracle.edge_deltas(g_prev.keys, g_cur.keys, n)
    flags = np.any(np.asarray(x_prev, dtype=np.float32).view(np.uint32) != np.asarray(x_cur, dtype=np.float32).view(np.uint32), axis=1)
    if mode == "sym":
        flags |= np.diff(g_prev.row_ptr) != np.diff(g_cur.row_ptr)
    changed = np.nonzero(flags)[0].astype(np.int32)
    index_of = np.full(n, -1, dtype=np.int64)
    index_of[changed] = np.arange(changed.size)
    ent_ptr = np.zeros(n + 1, dtype=np.int64)
    ent = []
    for v in range(n):
        row = [int(u) for u in icol[irp[v]:irp[v + 1]]]
        row += [(1 << 30) | int(u) for u in dcol[drp[v]:drp[v + 1]]]
        cur = g_cur.col[g_cur.row_ptr[v]:g_cur.row_ptr[v + 1]]
        row += [(2 << 30) | int(index_of[u]) for u in cur if index_of[u] >= 0]
        if self_loop and index_of[v] >= 0:
            row.append((2 << 30) | int(index_of[v]))
        ent += row
        ent_ptr[v + 1] = len(ent)
    rows = np.nonzero(np.diff(ent_ptr) > 0)[0].astype(np.int32)
    return (irp, icol), (drp, dcol), ent_ptr, np.array(ent, dtype=np.uint32), rows, changed


def undecided_relu(saved, threshold=3e-7, limit=3):
    """Pre-activations so close to zero (relative to their layer's rms) that fp32 rounding, not the model, decides
    on which side of the ReLU they fall: [(timestep, layer index, row, column)], at most `limit` (None if more)."""
    found = []
    for i, s in enumerate(saved):
        for l, z in enumerate(s["zs"]):
            rms = np.sqrt(np.mean(z * z))
            for r, c in np.argwhere(np.abs(z) < threshold * rms):
                found.append((i, l, int(r), int(c)))
    return found if len(found) <= limit else None


def assert_gradients_close(got, saved, backward, names, rtol):
    """got[name] against backward(saved)[name].  Where the ReLU decision of a unit is not unique in fp32 (see
    undecided_relu) either decision is right: the gradients then have to match the reference under one of the
    combinations of decisions for those units (a flip is made by changing the sign of the tiny pre-activation)."""
    import itertools

    def check(ref):
        for name in names:
            assert_close(got[name], ref[name], rtol, f"grad {name}")

    try:
        check(backward(saved))
        return
    except AssertionError as first:
        units = undecided_relu(saved)
        if not units:
            raise
        for k in range(1, len(units) + 1):
            for flips in itertools.combinations(units, k):
                for i, l, r, c in flips:
                    saved[i]["zs"][l][r, c] *= -1.0
                try:
                    check(backward(saved))
                    print(f"gradients match with the ReLU decision of {flips} taken the other way", flush=True)
                    return
                except AssertionError:
                    pass
                finally:
                    for i, l, r, c in flips:
                        saved[i]["zs"][l][r, c] *= -1.0
        raise first
