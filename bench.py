#!/usr/bin/env python3
"""Benchmark of the incremental dynamic-GNN hot path on one MI355X.

One "step" is one cold pass of the whole path over one synthetic snapshot sequence that is already
resident in HBM: build the per-step deltas, then slide a window of L snapshots over the sequence and
run forward + backward + SGD for every window (the first epoch: the layer-1 sums are computed once,
by the incremental rule of Section 3.2, Eq. 2 or, above the change-ratio threshold, from scratch, and
reused by every later window).

`value` is the throughput of the incremental aggregation inside that timed region: effective delta
edges consumed by Eq. 2 steps / summed duration of the incremental kernel's launches (each stamped
by events attached to the launch).  `ms_per_step` is the whole step (the snapshot-window epoch time);
`delta_edges_per_s_of_epoch` relates the same delta edges to it.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4] [--extras core|full|none]
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E
LONG_ROW = 64  # rows with more entries than this are aggregated by the block-per-row kernel
MAX_BATCH = 8  # timesteps of a window that the driver hands to one launch
DEFAULT_WORKLOAD = "c4"  # the largest configuration that fits one GPU


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--nodes", type=int, default=0, help="scale the workload down to this many nodes (debug)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--extras", choices=("auto", "core", "full", "none"), default="auto",
                    help="measurements after the timed region: core = per-kernel figures; full = also the widened "
                         "parts (max aggregation, integrated model, cache budgets, node mini-batches); auto = core "
                         "for workloads of a million nodes or more, full below")
    ap.add_argument("--no-extras", action="store_true", help="same as --extras none")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device copy (a kernel of known traffic, for scaling rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def agg_bytes(num_edges: float, n: int, d: int, elem: int) -> float:
    """Algorithmic bytes of one from-scratch aggregation launch: a column index and one source row per edge,
    one row pointer pair and one fp32 output row per node."""
    return num_edges * (4 + d * elem) + n * (d * 4 + 16)


def inc_bytes(info: dict, n: int, d: int, elem: int, new_buffer: bool) -> float:
    """Algorithmic bytes of one incremental step: per inserted / deleted entry its tag and one source row of the
    stored features, per feature-change entry its tag and one fp32 row of dY; per changed row of S its offsets,
    the old sums and the new sums; into a new buffer additionally the copy of every unchanged row."""
    structural = info["n_ins"] + info["n_del"]
    b = structural * (4 + d * elem) + info["n_fchg_entries"] * (4 + d * 4) + info["n_rows"] * (2 * d * 4 + 16)
    if new_buffer:
        b += 2 * (n - info["n_rows"]) * d * 4
    return float(b)


def diff_bytes(info: dict, n: int) -> float:
    """Algorithmic bytes of the snapshot-diff builder for one step: both column lists and row pointers read, the
    insert / delete lists, the merged entries and three row-pointer arrays written."""
    return float(4 * (info["num_edges_prev"] + info["num_edges_cur"]) + 16 * n
                 + 4 * (info["n_ins"] + info["n_del"]) + 4 * info["n_entries"] + 24 * (n + 1))


def measured_traffic(workload: str, kernel_prefix: str):
    """HBM bytes per launch of a kernel from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary of this command
    (profiles/bench_<workload>_hbm_traffic_pmc.txt: last column, MB per launch, counters scaled by a copy kernel of
    known size).  None when the workload has no such summary or the kernel is not in it."""
    path = os.path.join(ROOT, "profiles", f"bench_{workload}_hbm_traffic_pmc.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith(kernel_prefix):
            m = re.findall(r"[-+]?\d+\.?\d*", line[44:])
            if len(m) >= 6:
                return float(m[-1]) * 1e6
    return None


def _progress(stage, t, total):
    """Progress lines on stderr: generating and loading the largest workloads takes a while."""
    print(f"[bench] {stage} {t + 1}/{total}", file=sys.stderr, flush=True)


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_2501_15348_amd import reinc, synth

    wl = synth.WORKLOADS[args.workload]
    if args.nodes:
        wl = wl.scaled(args.nodes)
    n, T, L = wl.num_nodes, wl.num_snapshots, min(wl.window, wl.num_snapshots)
    d0 = wl.dims[0]
    elem = 2 if wl.feat_dtype == "bf16" else 4
    extras_level = "none" if args.no_extras else args.extras
    if extras_level == "auto":
        extras_level = "core" if n >= 1_000_000 else "full"
    t_gen = time.perf_counter()
    seq = synth.make_sequence(wl, progress=_progress)
    t_gen = time.perf_counter() - t_gen

    # arena: snapshots + features + deltas + caches, with head-room
    feat_bytes = T * n * d0 * elem
    edge_bytes = T * (wl.num_edges * 8 + n * 24)
    cache_bytes = T * n * d0 * 4
    local_bytes = (L + 4) * n * (sum(wl.dims[1:]) * 2 + 6 * wl.hidden + 4 * max(wl.dims)) * 4
    delta_bytes = T * (wl.num_edges * 8 + n * 40 + n * d0 * 4)
    arena = int(1.25 * (feat_bytes + edge_bytes + cache_bytes + local_bytes + delta_bytes)) + (256 << 20)
    # the estimate is generous; at the largest workload it exceeds the card, where everything still fits: take what
    # is free (less room for the few matrices the per-kernel measurements allocate) and let the library size its
    # scratch (it lowers the time-batch depth) or report that it ran out
    free_bytes, _ = torch.cuda.mem_get_info()
    arena = min(arena, free_bytes - (8 << 30) - 4 * n * d0 * 4)
    ctx = reinc.Context.for_workload(wl, arena_bytes=arena, fallback_ratio=0.5)
    t_load = time.perf_counter()
    ctx.load_sequence(seq, progress=_progress)
    torch.cuda.synchronize()
    t_load = time.perf_counter() - t_load

    params0 = torch.from_numpy(synth.make_params(wl)).cuda()
    params = params0.clone()
    target = torch.from_numpy(synth.make_target(wl)).cuda()
    grads = torch.empty_like(params)
    loss = torch.zeros(1, device="cuda")
    windows = T - L + 1

    def step():
        ctx.reset_derived()
        ctx.build_deltas(-1)
        for t0 in range(windows):
            ctx.forward_window(t0, L, params, target, loss)
            ctx.backward_window(t0, L, params, target, grads)
            ctx.sgd_step(params, grads, 1e-2)

    if args.calibrate_copy:
        src = torch.empty(64 << 20, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)  # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    print(f"[bench] generated in {t_gen:.1f} s, loaded in {t_load:.1f} s; warm-up", file=sys.stderr, flush=True)
    for i in range(args.warmup):
        step()
        torch.cuda.synchronize()
        _progress("warm-up step", i, args.warmup)
    torch.cuda.synchronize()
    st0 = ctx.get_stats()
    # the two aggregation kernels are stamped by events attached to their launches (the kernel's own begin / end)
    ctx.profile_begin(("agg_full", "agg_inc"))
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = ctx.profile_end()
    print(f"[bench] {args.steps} timed steps in {elapsed:.2f} s", file=sys.stderr, flush=True)
    st1 = ctx.get_stats()
    ms_per_step = elapsed * 1e3 / args.steps
    loss_value = float(loss.item())

    infos = [ctx.get_delta_info(t) for t in range(1, T)]
    delta_edges = sum(i["n_entries"] for i in infos)
    per_step = lambda k: (st1[k] - st0[k]) / args.steps
    inc_steps, full_steps, fallback_steps = per_step("steps_incremental"), per_step("steps_full"), per_step("steps_fallback")
    consumed = per_step("delta_entries_processed")  # effective delta edges that went through Eq. 2, per step

    # ---- the incremental kernel inside the timed region (one launch per Eq. 2 step; the driver writes each
    # snapshot's sums into a buffer of their own, so a launch also copies the unchanged rows)
    inc_launches, inc_ms = prof["agg_inc"]
    # which steps ran incrementally: every step under the threshold whose predecessor was cached (all but step 0)
    ratio_ok = [i["n_entries"] <= 0.5 * max(i["num_edges_cur"], 1) for i in infos]
    inc_alg = [inc_bytes(i, n, d0, elem, True) for i, ok in zip(infos, ratio_ok) if ok]
    inc_bytes_per_launch = float(np.mean(inc_alg)) if inc_alg else 0.0
    if inc_launches:
        inc_avg_ms = inc_ms / inc_launches
        value = consumed * args.steps / (inc_ms * 1e-3)
        achieved = inc_bytes_per_launch / (inc_avg_ms * 1e-3) / 1e9
        traffic = measured_traffic(wl.name, "incremental_segmented")
        roofline = {
            "bound": "hbm", "kernel": "incremental_segmented (Eq. 2, into a new buffer: unchanged rows copied through)",
            "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": traffic,
            "traffic_frac": round(traffic / (inc_avg_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if traffic else None,
            "traffic_source": f"profiles/bench_{wl.name}_hbm_traffic_pmc.txt" if traffic else None,
            "launches": int(inc_launches), "avg_us": round(inc_avg_ms * 1e3, 2),
            "algorithmic_bytes_per_launch": int(inc_bytes_per_launch),
            "share_of_step_time": round(inc_ms / (elapsed * 1e3), 4),
        }
    else:
        # every step exceeded the change-ratio threshold (Section 3.2's fallback): Eq. 2 never ran in the timed
        # region and there is no throughput of it to report
        value = 0.0
        roofline = {"bound": "hbm", "kernel": "incremental_segmented", "achieved": 0.0, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": 0.0, "traffic": None, "launches": 0,
                    "note": "no incremental step in the timed region: every step is above the fallback threshold"}

    # ---- second block: aggregate_rows_grouped, the from-scratch gather (layer-1 steps that are not incremental,
    # and every layer above the first, forward and adjoint).  It takes every row of at most LONG_ROW entries (longer
    # rows go to a block-per-row kernel that is not part of this figure): algorithmic bytes of exactly the rows it
    # handles / its measured launch time
    launches, total_ms = prof["agg_full"]
    layers = len(wl.dims) - 1
    fwd_short, adj_short = [], []  # per snapshot: (edges, rows) handled by the grouped kernel, CSR and CSC side
    for t in range(T):
        for transpose, acc in ((False, fwd_short), (True, adj_short)):
            ptr, _ = ctx.get_snapshot_csr(t, transpose)
            deg = np.diff(ptr)
            short = deg <= LONG_ROW
            acc.append((float(deg[short].sum()), float(short.sum())))

    def short_bytes(t, side, d, el):
        e_s, n_s = (fwd_short if side == "fwd" else adj_short)[t]
        return e_s * (4 + d * el) + n * 16 + n_s * d * 4

    total_bytes, count = 0.0, 0.0
    mean_l1 = float(np.mean([short_bytes(t, "fwd", d0, elem) for t in range(T)]))
    total_bytes += full_steps * mean_l1
    count += full_steps
    batches = -(-L // MAX_BATCH)  # above layer 1 one launch aggregates up to MAX_BATCH snapshots of a window
    for t0_ in range(windows):
        for l in range(2, layers + 1):  # forward aggregate and backward adjoint of layer l
            count += 2 * batches
            # a layer that narrows its input applies its linear map first and gathers rows of its own width
            width = wl.dims[l] if wl.dims[l] < wl.dims[l - 1] else wl.dims[l - 1]
            for t in range(t0_, t0_ + L):
                total_bytes += short_bytes(t, "fwd", width, 4) + short_bytes(t, "adj", width, 4)
    # (a launch covers one snapshot at layer 1 and up to MAX_BATCH snapshots above it -- fewer where the arena leaves
    # less scratch -- so the bytes of all launches are set against their total duration)
    bytes_per_launch = total_bytes * args.steps / max(launches, 1)
    avg_ms = total_ms / max(launches, 1)
    full_achieved = bytes_per_launch / (avg_ms * 1e-3) / 1e9 if launches else 0.0
    full_traffic = measured_traffic(wl.name, "aggregate_rows_grouped")
    roofline_full = {
        "bound": "hbm", "kernel": "aggregate_rows_grouped (Eq. 1 and its adjoint, rows of at most 64 entries)",
        "achieved": round(full_achieved, 1), "peak": HBM_PEAK_GBS,
        "unit": "GB/s", "frac": round(full_achieved / HBM_PEAK_GBS, 4), "traffic": full_traffic,
        "traffic_frac": round(full_traffic / (avg_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if full_traffic and launches else None,
        "launches": int(launches), "avg_us": round(avg_ms * 1e3, 2),
        "algorithmic_bytes_per_launch": int(bytes_per_launch),
        "share_of_step_time": round(total_ms / (elapsed * 1e3), 3),
    }
    if full_achieved > HBM_PEAK_GBS:
        roofline_full["note"] = ("cache-served: the gathered matrix fits the caches, so the algorithmic rate exceeds the "
                                 "HBM peak; the counter traffic is the HBM-side figure")

    out = {
        "metric": "delta-edges/sec", "value": round(value, 1), "unit": "delta-edges/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32" if elem == 4 else "bf16-in/f32-acc", "data": "synthetic",
        "config": {"workload": wl.name, "num_nodes": n, "num_edges": wl.num_edges, "snapshots": T, "window": L,
                   "windows_per_step": windows, "edge_churn": wl.edge_churn, "feat_churn": wl.feat_churn, "agg": wl.agg,
                   "dims": list(wl.dims), "rnn": wl.rnn, "hidden": wl.hidden, "fallback_ratio": 0.5,
                   "step": "build deltas + cold epoch of forward/backward/SGD over all windows",
                   "dense_products": ("fp32 matrix instructions" if os.environ.get("REINC_DENSE") == "fp32" else
                                      "f32 operands as three bfloat16 terms each, six products on the bf16 matrix cores, "
                                      "f32 accumulation (error as the fp32 instructions)")},
        "value_definition": "effective delta edges consumed by Eq. 2 steps in the timed region / summed duration of the "
                            "incremental kernel's launches in the timed region",
        "delta_edges_per_step": int(delta_edges), "delta_edges_through_eq2_per_step": int(consumed),
        "snapshot_window_epoch_ms": round(ms_per_step, 3),
        "delta_edges_per_s_of_epoch": round(delta_edges / (ms_per_step * 1e-3), 1),
        "layer1_steps": {"incremental": int(inc_steps), "full": int(full_steps), "fallback": int(fallback_steps)},
        "loss": loss_value, "host_load_s": round(t_load, 3), "generate_s": round(t_gen, 3),
        "roofline": roofline, "roofline_aggregate_full": roofline_full,
    }

    if extras_level != "none":
        out["kernels"] = extras(ctx, wl, seq, infos, params0, target, step, elapsed / args.steps, extras_level == "full")
    ctx.close()
    del ctx
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, seq, delta_edges)
    print(json.dumps(out), flush=True)


def extras(ctx, wl, seq, infos, params, target, step, step_s, full):
    """Per-kernel figures measured after the timed region (not part of `value`); `full` adds the widened parts."""
    import numpy as np
    import torch

    n, T, d = wl.num_nodes, wl.num_snapshots, wl.dims[0]
    elem = 2 if wl.feat_dtype == "bf16" else 4
    res = {}
    # time share per kernel class over one more cold step
    ctx.profile_begin(reinc_kinds())
    step()
    prof = ctx.profile_end()
    res["breakdown_ms"] = {k: {"launches": int(c), "total_ms": round(ms, 3)} for k, (c, ms) in prof.items() if c}

    def timed(fn, reps=10):
        fn()
        torch.cuda.synchronize()
        evs = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            evs.append((a, b))
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) for a, b in evs)
        return ts[len(ts) // 2]

    # incremental (forced) versus from-scratch layer-1 aggregation, per step: in place (rows of R_t only) and into
    # a new buffer (what the window driver does: unchanged rows are copied through)
    s = ctx.aggregate_full(0)
    work = s.clone()
    out = torch.empty_like(s)
    ip_ms, nb_ms, full_ms, ip_b, nb_b = [], [], [], [], []
    for t in range(1, T):
        i = infos[t - 1]
        ip_ms.append(timed(lambda: ctx.aggregate_incremental(t, work, work)))
        nb_ms.append(timed(lambda: ctx.aggregate_incremental(t, s, out)))
        full_ms.append(timed(lambda: ctx.aggregate_full(t, out=out)))
        ip_b.append(inc_bytes(i, n, d, elem, False))
        nb_b.append(inc_bytes(i, n, d, elem, True))
    e_mean = float(np.mean([len(a) for a, _ in seq.edges]))
    ent = sum(i["n_entries"] for i in infos)

    def inc_row(ms, nbytes):
        rate = sum(nbytes) / (sum(ms) * 1e-3) / 1e9
        return {"delta_edges_per_s": round(ent / (sum(ms) * 1e-3), 1), "mean_us": round(1e3 * sum(ms) / len(ms), 2),
                "algorithmic_GBps": round(rate, 1), "hbm_frac": round(rate / HBM_PEAK_GBS, 4),
                "speedup_over_full": round(sum(full_ms) / sum(ms), 3)}

    res["aggregate_incremental"] = {
        "in_place": inc_row(ip_ms, ip_b), "new_buffer": inc_row(nb_ms, nb_b),
        "mean_changed_row_fraction": round(float(np.mean([i["n_rows"] for i in infos])) / n, 4),
        "mean_delta_to_edge_ratio": round(ent / (len(infos) * e_mean), 4),
    }
    fb = agg_bytes(e_mean, n, d, elem)
    full_rate = fb * len(full_ms) / (sum(full_ms) * 1e-3) / 1e9
    res["aggregate_full"] = {"mean_us": round(1e3 * sum(full_ms) / len(full_ms), 2), "algorithmic_GBps": round(full_rate, 1),
                             "hbm_frac": round(full_rate / HBM_PEAK_GBS, 4),
                             "note": "both kernels of a from-scratch aggregation (rows of up to 64 entries, hub rows)"}
    if full_rate > HBM_PEAK_GBS:
        res["aggregate_full"]["note"] += "; cache-served: above the HBM peak because gathered rows are re-used out of the caches"
    res["incremental_speedup_over_full"] = round(sum(full_ms) / sum(ip_ms), 3)
    del s, work, out
    if full:
        res["aggregate_max"] = max_rows(ctx, wl, seq, infos, timed)
    # snapshot-diff builder
    ctx.reset_derived()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ctx.build_deltas(-1)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    db = sum(diff_bytes(i, n) for i in infos)
    res["build_deltas"] = {"ms_per_step": round(dt * 1e3 / (T - 1), 3),
                           "edges_per_s": round(sum(i["num_edges_prev"] + i["num_edges_cur"] for i in infos) / dt, 1),
                           "algorithmic_GBps": round(db / dt / 1e9, 1), "hbm_frac": round(db / dt / 1e9 / HBM_PEAK_GBS, 4),
                           "note": "wall time of reinc_build_deltas for all steps (every kernel and both host waits)"}
    res["gcn_transform"], res["rnn_step"] = dense_rows(ctx, wl, timed)
    # warm epoch: every layer-1 sum comes from the global cache
    L = min(wl.window, T)
    loss = torch.zeros(1, device="cuda")
    grads = torch.empty_like(params)
    p = params.clone()

    def epoch():
        for t0_ in range(T - L + 1):
            ctx.forward_window(t0_, L, p, target, loss)
            ctx.backward_window(t0_, L, p, target, grads)
            ctx.sgd_step(p, grads, 1e-2)

    epoch()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    epoch()
    torch.cuda.synchronize()
    res["warm_epoch_ms"] = round((time.perf_counter() - t0) * 1e3, 3)
    res["cold_epoch_ms"] = round(step_s * 1e3, 3)
    if not full:
        return res
    # the integrated model (graph operations inside the recurrent gates): warm epoch, same windows
    import dataclasses

    from paper_2501_15348_amd import synth

    wli = dataclasses.replace(wl, dims=(wl.dims[0],))
    pi = torch.from_numpy(synth.make_params(wli)).cuda()
    gi = torch.empty_like(pi)

    def epoch_integrated():
        for t0_ in range(T - L + 1):
            ctx.forward_window_integrated(t0_, L, pi, target, loss)
            ctx.backward_window_integrated(t0_, L, pi, target, gi)
            ctx.sgd_step(pi, gi, 1e-2)

    epoch_integrated()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    epoch_integrated()
    torch.cuda.synchronize()
    res["integrated_model_warm_epoch_ms"] = round((time.perf_counter() - t0) * 1e3, 3)
    # budgeted layer-1 cache: one cold epoch (deltas built, no aggregate cached) per policy and budget
    size = ctx.aggregate_bytes()
    rows = []
    for policy, slots in (("keep_all", T), ("score", L - 1), ("lru", L - 1), ("score", L // 2), ("lru", L // 2), ("score", 0)):
        ctx.cache_configure(policy, slots * size, window=L, stride=1)
        torch.cuda.synchronize()
        st0 = ctx.get_stats()
        t0 = time.perf_counter()
        epoch()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3
        st1 = ctx.get_stats()
        hits, misses = st1["global_hits"] - st0["global_hits"], st1["global_misses"] - st0["global_misses"]
        rows.append({"policy": policy, "budget_aggregates": slots, "cold_epoch_ms": round(ms, 3), "hits": hits, "misses": misses,
                     "full": st1["steps_full"] - st0["steps_full"],
                     "retained_peak_MB": round((T * size if policy == "keep_all" else st1["global_peak_bytes"]) / 1e6, 1)})
    ctx.cache_configure("keep_all")
    res["cache_budget"] = rows
    # (both parts need a second context of up to the size of the first: skipped where the card has no room for it)
    free_bytes, _ = torch.cuda.mem_get_info()
    if free_bytes < 2.2 * int(ctx.cfg.arena_bytes) + (2 << 30):
        res["node_minibatch"] = "skipped: no room for a second context of this workload's size"
        return res
    res["node_minibatch"] = minibatch_rows(ctx, wl, seq, params, target, L, "bench workload")
    # the same model on a road-network-like graph (uniform, mean degree 3, mean aggregation: the paper's forecasting
    # data sets are sensor networks of that sparsity), where the computational graphs of a batch stay small
    from paper_2501_15348_amd import reinc

    wl2 = dataclasses.replace(wl, name="sparse", mean_degree=3.0, structure="uniform", gamma=0.0, agg="mean")
    seq2 = synth.make_sequence(wl2)
    ctx2 = reinc.Context.for_workload(wl2, arena_bytes=int(ctx.cfg.arena_bytes))
    ctx2.load_sequence(seq2)
    res["node_minibatch"] += minibatch_rows(ctx2, wl2, seq2, params, target, L, "uniform degree 3, mean")
    ctx2.close()
    return res


MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 matrix-core peak of MI355X
MFMA_F32_PEAK_TFLOPS = 157.3


def dense_rows(ctx, wl, timed):
    """K5 per GCN layer and K6 at the workload's row count, one timestep per call (inside a window the driver hands
    them up to MAX_BATCH timesteps as one taller matrix): algorithmic bytes against the HBM peak, and the matrix-core
    rate -- fp32-equivalent flops, and the six bf16 products per fp32 product that the three-term split really
    issues, against the bf16 peak.  With REINC_DENSE=fp32 the products run on the fp32 matrix instructions instead."""
    import torch

    n = wl.num_nodes
    split = os.environ.get("REINC_DENSE") != "fp32"
    g = torch.Generator(device="cuda").manual_seed(3)

    def row(ms, nbytes, flops):
        r = {"us": round(ms * 1e3, 1), "algorithmic_GBps": round(nbytes / ms / 1e6, 1),
             "hbm_frac": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4), "f32_equivalent_TFLOPs": round(flops / ms / 1e9, 1)}
        if split:
            r["bf16_products_TFLOPs"] = round(6 * flops / ms / 1e9, 1)
            r["mfma_frac"] = round(6 * flops / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4)
        else:
            r["mfma_frac"] = round(flops / ms / 1e9 / MFMA_F32_PEAK_TFLOPS, 4)
        return r

    layers = []
    for l in range(1, len(wl.dims)):
        k, m = wl.dims[l - 1], wl.dims[l]
        a = torch.randn(n, k, device="cuda", generator=g)
        w = torch.randn(k, m, device="cuda", generator=g) / k ** 0.5
        b = torch.zeros(m, device="cuda")
        out = torch.empty(n, m, device="cuda")
        ms = timed(lambda: ctx.gcn_transform(a, w, b, None, True, out))
        layers.append({"rows": n, "d_in": k, "d_out": m, **row(ms, n * (k + m) * 4 + k * m * 4, 2.0 * n * k * m)})
        del a, out
    d, h = wl.dims[-1], wl.hidden
    kg = 4 if wl.rnn == "lstm" else 3
    x = torch.randn(n, d, device="cuda", generator=g)
    hp = 0.5 * torch.randn(n, h, device="cuda", generator=g)
    cp = 0.5 * torch.randn(n, h, device="cuda", generator=g) if wl.rnn == "lstm" else None
    wi = torch.randn(d, kg * h, device="cuda", generator=g) / d ** 0.5
    wh = torch.randn(h, kg * h, device="cuda", generator=g) / h ** 0.5
    bi, bh = torch.zeros(kg * h, device="cuda"), torch.zeros(kg * h, device="cuda")
    saved = torch.empty(n, 4 * h, device="cuda")
    ms = timed(lambda: ctx.rnn_step(wl.rnn, x, hp, cp, wi, wh, bi, bh, saved))
    # x, h (and c) read; h (and c) and the four saved gate rows written
    nbytes = n * 4 * (d + h * (2 if cp is not None else 1) * 2 + 4 * h)
    cell = {"rows": n, "d_in": d, "hidden": h, "kind": wl.rnn, **row(ms, nbytes, 2.0 * n * (d + h) * kg * h)}
    return layers, cell


def max_rows(ctx, wl, seq, infos, timed):
    """Max aggregation with contributing source ids (Section 3.2): from scratch versus the incremental procedure."""
    import numpy as np
    import torch

    n, T, d = wl.num_nodes, wl.num_snapshots, wl.dims[0]
    elem = 2 if wl.feat_dtype == "bf16" else 4
    e_mean = float(np.mean([len(a) for a, _ in seq.edges]))
    # max aggregation with contributing source ids (Section 3.2): from scratch versus the incremental procedure
    # (in place; rows whose contributor was lost are aggregated from scratch inside the same call)
    mm, cc = ctx.aggregate_full_minmax(0, "max")
    mo, co = torch.empty_like(mm), torch.empty_like(cc)
    tm, tc = torch.empty_like(mm), torch.empty_like(cc)
    wk = torch.empty(2 * n + 4, dtype=torch.int32, device="cuda")
    mm_inc, mm_full, redone = [], [], []

    def timed_step_in_place(t, reps=5):
        ts = []
        for _ in range(reps + 1):
            tm.copy_(mm)  # the state of step t-1, restored outside the timed region
            tc.copy_(cc)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            ctx.aggregate_incremental_minmax(t, "max", tm, tc, tm, tc, wk)
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b))
        ts = sorted(ts[1:])
        return ts[len(ts) // 2]

    for t in range(1, T):
        mm_full.append(timed(lambda: ctx.aggregate_full_minmax(t, "max", out=mo, contrib=co)))
        mm_inc.append(timed_step_in_place(t))
        ctx.aggregate_incremental_minmax(t, "max", mm, cc, mm, cc, wk)  # advance the chain
        redone.append(int(wk[0].item()))
    mm_bytes = e_mean * (4 + d * elem) + n * (16 + 2 * d * 4)
    return {
        "full_mean_us": round(1e3 * sum(mm_full) / len(mm_full), 2),
        "full_algorithmic_GBps": round(mm_bytes * len(mm_full) / (sum(mm_full) * 1e-3) / 1e9, 1),
        "incremental_mean_us_in_place": round(1e3 * sum(mm_inc) / len(mm_inc), 2),
        "rows_reaggregated_fraction_of_changed_rows": round(sum(redone) / max(sum(i["n_rows"] for i in infos), 1), 4),
        "rows_reaggregated_fraction_of_all_rows": round(sum(redone) / (n * len(redone)), 4),
        "incremental_speedup_over_full": round(sum(mm_full) / sum(mm_inc), 3),
    }


def minibatch_rows(ctx, wl, seq, params, target, L, label):
    """Seq-first node mini-batches: for a few batch sizes, the first batches of a seeded partition of the nodes are
    extracted into their own context and every window of the sequence is trained on each (forward, backward, SGD)
    before the next batch is taken; node-first order is imitated by dropping the batch's aggregate cache before every
    window.  Times are per batch."""
    import numpy as np
    import torch

    from paper_2501_15348_amd import synth

    n, T = wl.num_nodes, wl.num_snapshots
    perm = np.random.default_rng(wl.seed + 77).permutation(n).astype(np.int32)
    full_edges = float(sum(len(s_) for s_, _ in seq.edges))
    rows = []
    for parts, take in ((8, 2), (64, 3)):
        size = n // parts
        acc = {"extract_ms": [], "deltas_ms": [], "seq_first_epoch_ms": [], "node_first_epoch_ms": [], "nodes": [], "inner": [], "edges": [],
               "cache_MB": [], "hits": [], "misses": [], "hits_node_first": []}
        for b in range(take):
            batch = perm[b * size:(b + 1) * size]
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            total, inner = ctx.batch_plan(batch)
            frac = total / n
            child_arena = int(frac * ctx.cfg.arena_bytes) + (512 << 20)
            child = ctx.batch_context(batch, child_arena, planned_total=total)
            torch.cuda.synchronize()
            acc["extract_ms"].append((time.perf_counter() - t0) * 1e3)
            t0 = time.perf_counter()
            child.build_deltas(-1)
            torch.cuda.synchronize()
            acc["deltas_ms"].append((time.perf_counter() - t0) * 1e3)
            node_list = torch.from_numpy(ctx.batch_node_list(total).astype(np.int64)).cuda()
            tgt = target[node_list].contiguous()
            p = params.clone()
            grads = torch.empty_like(p)
            loss = torch.zeros(1, device="cuda")

            def epoch(node_first):
                for t0_ in range(T - L + 1):
                    if node_first:
                        child.cache_clear()
                    child.forward_window(t0_, L, p, tgt, loss)
                    child.backward_window(t0_, L, p, tgt, grads)
                    child.sgd_step(p, grads, 1e-2)

            for node_first in (False, True):
                child.cache_clear()
                st0 = child.get_stats()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                epoch(node_first)
                torch.cuda.synchronize()
                ms = (time.perf_counter() - t0) * 1e3
                st1 = child.get_stats()
                if node_first:
                    acc["node_first_epoch_ms"].append(ms)
                    acc["hits_node_first"].append(st1["global_hits"] - st0["global_hits"])
                else:
                    acc["seq_first_epoch_ms"].append(ms)
                    acc["hits"].append(st1["global_hits"] - st0["global_hits"])
                    acc["misses"].append(st1["global_misses"] - st0["global_misses"])
            acc["nodes"].append(total)
            acc["inner"].append(inner)
            acc["edges"].append(sum(child.get_snapshot_csr(t)[1].size for t in range(T)) / full_edges)
            cached_rows = inner if len(wl.dims) > 2 else batch.size  # the rows that layer 1 is needed on
            acc["cache_MB"].append(T * cached_rows * wl.dims[0] * 4 / 1e6)
            child.close()
            del child
        mean = lambda k: float(np.mean(acc[k]))
        rows.append({"graph": label, "batch_nodes": size, "batches_timed": take, "batches_per_pass": parts,
                     "sub_sequence_nodes": round(mean("nodes")), "nodes_within_one_hop": round(mean("inner")),
                     "edges_kept_frac": round(mean("edges"), 4),
                     "extract_ms": round(mean("extract_ms"), 3), "build_deltas_ms": round(mean("deltas_ms"), 3),
                     "seq_first_epoch_ms": round(mean("seq_first_epoch_ms"), 3), "node_first_epoch_ms": round(mean("node_first_epoch_ms"), 3),
                     "layer1_cache_MB": round(mean("cache_MB"), 1), "hits": round(mean("hits")), "misses": round(mean("misses")),
                     "hits_node_first": round(mean("hits_node_first"))})
    return rows


def reinc_kinds():
    from paper_2501_15348_amd import reinc

    return reinc.KERNEL_KINDS


def cpu_baseline(wl, seq, delta_edges_epoch):
    """The CPU reference as it stands, timed on this host on a bounded sample: the from-scratch layer-1 aggregation
    (Section 3.2, Eq. 1, fp64) of ONE snapshot of the same workload, with all host threads and with one thread, scaled
    to the T-1 snapshots the sequence's delta edges lead to (the reference recomputes every snapshot)."""
    import ctypes

    import numpy as np

    import oracle

    n, T = wl.num_nodes, wl.num_snapshots
    t_s = 1 if T > 1 else 0
    g = oracle.graphs_of(seq.edges[t_s:t_s + 1], n)[0]
    x = oracle.features_at(seq.x0, seq.feat_rows, seq.feat_vals, t_s)
    cores = oracle.num_threads()
    omp = ctypes.CDLL("libgomp.so.1")

    def timed():
        t0 = time.perf_counter()
        oracle.aggregate(g.row_ptr, g.col, x, wl.agg, wl.self_loop)
        return time.perf_counter() - t0

    timed()  # page in
    all_s = timed()
    one_s = None
    if all_s * cores < 60.0:  # keep the whole leg bounded: one thread is about `cores` times slower
        omp.omp_set_num_threads(1)
        one_s = timed()
        omp.omp_set_num_threads(cores)
    steps = max(T - 1, 1)
    out = {"value": round(delta_edges_epoch / (all_s * steps), 1), "unit": "delta-edges/s", "cores": cores, "kind": "oracle",
           "sample": f"from-scratch fp64 layer-1 aggregation of snapshot {t_s} of the same workload ({g.col.size} edges x "
                     f"{wl.dims[0]} features): {all_s:.2f} s on {cores} threads, scaled to the {steps} snapshots that the "
                     f"sequence's delta edges update",
           "sample_seconds_all_cores": round(all_s, 3)}
    if one_s is not None:
        out["value_1_thread"] = round(delta_edges_epoch / (one_s * steps), 1)
        out["sample_seconds_1_thread"] = round(one_s, 3)
    return out


if __name__ == "__main__":
    main()
