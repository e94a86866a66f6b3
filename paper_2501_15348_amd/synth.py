"""Seeded synthetic snapshot sequences (inputs only).

This module draws the inputs that both the HIP path and the CPU checker consume:
edge lists per snapshot, feature matrices and their per-step row replacements,
model parameters and regression targets.  It holds none of the method's
arithmetic: no aggregation, no delta extraction, no neural-network maths.  The
generator does know which edges it deleted and inserted at every step; those
lists are kept as ground truth for tests of the snapshot-diff builder.

Workload shapes follow the paper's evaluation set-up (Section 5.1): graphs with
millions of nodes, average degree around 8-25, feature width around 100-128,
and dynamic versions made from a static graph by random edge deletion and
insertion plus re-assignment of node features.  The public datasets used there
are replaced by Chung-Lu power-law graphs of the same shape.

All randomness comes from numpy's counter-based Philox generator keyed by
(seed, stream id), so every array is reproducible independently of the others.
"""
from __future__ import annotations

import dataclasses
import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np

# stream ids for the Philox key
_S_GRAPH, _S_PERM, _S_STEP, _S_FEAT0, _S_FEATSTEP, _S_PARAM, _S_TARGET, _S_SHUFFLE = range(8)


def _rng(seed: int, stream: int, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed << 16) ^ sub, stream]))


# The largest workloads hold tens of millions of edges per snapshot; the array passes below are split into pieces
# that a few threads work on (numpy releases the interpreter lock inside them).  The pieces and their results do
# not depend on the number of threads.
_PIECE = 1 << 20
_THREADS = max(1, min(16, os.cpu_count() or 1))


def _pieces(n: int, piece: int = _PIECE):
    return [(a, min(a + piece, n)) for a in range(0, n, piece)]


def _pmap(fn, n: int, piece: int = _PIECE):
    """fn(a, b) for every piece [a, b) of range(n); results in order."""
    parts = _pieces(n, piece)
    if len(parts) <= 1 or _THREADS == 1:
        return [fn(a, b) for a, b in parts]
    with ThreadPoolExecutor(_THREADS) as pool:
        return list(pool.map(lambda ab: fn(*ab), parts))


def _in_sorted(ref_sorted: np.ndarray, x: np.ndarray) -> np.ndarray:
    """Mask of the entries of x that occur in ref_sorted."""
    out = np.zeros(x.size, dtype=bool)
    if ref_sorted.size == 0:
        return out

    def run(a, b):
        pos = np.minimum(np.searchsorted(ref_sorted, x[a:b]), ref_sorted.size - 1)
        out[a:b] = ref_sorted[pos] == x[a:b]

    _pmap(run, x.size)
    return out


def _first_occurrences(k: np.ndarray) -> np.ndarray:
    """The entries of k without repeats of an earlier value, in their order.  (Repeats are rare: the values that
    occur more than once are found from one plain sort, and only their occurrences are ranked by position.)"""
    ks = np.sort(k)
    rep = ks[1:][ks[1:] == ks[:-1]]
    if rep.size == 0:
        return k, ks
    rep = rep[np.concatenate([[True], rep[1:] != rep[:-1]])]
    idx = np.nonzero(_in_sorted(rep, k))[0]
    _, first = np.unique(k[idx], return_index=True)
    keep = np.ones(k.size, dtype=bool)
    keep[idx] = False
    keep[idx[first]] = True
    uk = ks[np.concatenate([[True], ks[1:] != ks[:-1]])]
    return k[keep], uk


def _replace_sorted(keys: np.ndarray, drop: np.ndarray, ins: np.ndarray) -> np.ndarray:
    """keys (sorted, distinct) without the entries at the sorted positions `drop`, united with `ins` (sorted,
    disjoint from keys); sorted.  Piece by piece: a piece of the old array and the new values that fall into
    its range are merged on their own."""
    if keys.size == 0:
        return ins.copy()
    parts = _pieces(keys.size)
    lo = [0] + [int(x) for x in np.searchsorted(ins, keys[[a for a, _ in parts[1:]]])] if len(parts) > 1 else [0]
    hi = lo[1:] + [ins.size]
    dlo = np.searchsorted(drop, [a for a, _ in parts])
    dhi = np.append(dlo[1:], drop.size)

    def run(i):
        a, b = parts[i]
        keep = np.ones(b - a, dtype=bool)
        keep[drop[dlo[i]:dhi[i]] - a] = False
        return np.sort(np.concatenate([keys[a:b][keep], ins[lo[i]:hi[i]]]))

    if len(parts) == 1 or _THREADS == 1:
        out = [run(i) for i in range(len(parts))]
    else:
        with ThreadPoolExecutor(_THREADS) as pool:
            out = list(pool.map(run, range(len(parts))))
    return np.concatenate(out)


@dataclass(frozen=True)
class Workload:
    """Shape of one synthetic dynamic-graph workload."""

    name: str
    num_nodes: int
    mean_degree: float
    num_snapshots: int
    structure: str  # "uniform" or "chunglu"
    gamma: float  # power-law exponent (chunglu only)
    edge_churn: float  # fraction of |E_{t-1}| deleted AND inserted per step
    feat_churn: float  # fraction of rows re-drawn per step
    feat_dtype: str  # "fp32" or "bf16"
    agg: str  # "sum" | "mean" | "sym"
    self_loop: bool
    dims: Tuple[int, ...]  # (d0, d1, ..., d_last) : len-1 GCN layers
    rnn: str  # "gru" | "lstm"
    hidden: int
    window: int
    seed: int = 0

    @property
    def num_edges(self) -> int:
        return int(round(self.num_nodes * self.mean_degree))

    @property
    def feat_dim(self) -> int:
        return self.dims[0]

    def scaled(self, num_nodes: int, num_snapshots: Optional[int] = None, **kw) -> "Workload":
        """Same recipe on fewer nodes (and optionally fewer snapshots)."""
        return dataclasses.replace(
            self,
            name=f"{self.name}@{num_nodes}",
            num_nodes=num_nodes,
            num_snapshots=num_snapshots or self.num_snapshots,
            **kw,
        )


WORKLOADS = {
    # 1,000 nodes, 5,000 uniform edges, 1 % + 1 % churn, 1 % feature rows, GCN 16->16 sum+self-loop, GRU 16
    "tiny": Workload("tiny", 1000, 5.0, 8, "uniform", 0.0, 0.01, 0.01, "fp32", "sum", True, (16, 16), "gru", 16, 8),
    # 100k nodes, Chung-Lu 2.1, mean degree 10, 5 % + 5 %, 2 % rows, 2-layer sym-normalised GCN 64, GRU 64
    "c2": Workload("c2", 100_000, 10.0, 20, "chunglu", 2.1, 0.05, 0.02, "fp32", "sym", True, (64, 64, 64), "gru", 64, 8),
    # 1M nodes, exponent 2.2, mean degree 16, 1 % + 1 %, 1 % rows, mean aggregation, LSTM 128, window 8
    "c3": Workload("c3", 1_000_000, 16.0, 32, "chunglu", 2.2, 0.01, 0.01, "fp32", "mean", True, (128, 128, 128), "lstm", 128, 8),
    # 2.5M nodes, exponent 2.0, mean degree 20, 10 % churn, bf16 features 256, GCN 256->256->128, GRU 128
    "c4": Workload("c4", 2_500_000, 20.0, 16, "chunglu", 2.0, 0.10, 0.0, "bf16", "mean", True, (256, 256, 128), "gru", 128, 8),
    # churn sweep: 500k nodes, exponent 2.1, mean degree 12, 12 snapshots, fp32 64, sum + self-loop
    "c5_01": Workload("c5_01", 500_000, 12.0, 12, "chunglu", 2.1, 0.01, 0.0, "fp32", "sum", True, (64, 64, 64), "gru", 64, 8),
    "c5_10": Workload("c5_10", 500_000, 12.0, 12, "chunglu", 2.1, 0.10, 0.0, "fp32", "sum", True, (64, 64, 64), "gru", 64, 8),
    "c5_25": Workload("c5_25", 500_000, 12.0, 12, "chunglu", 2.1, 0.25, 0.0, "fp32", "sum", True, (64, 64, 64), "gru", 64, 8),
    "c5_50": Workload("c5_50", 500_000, 12.0, 12, "chunglu", 2.1, 0.50, 0.0, "fp32", "sum", True, (64, 64, 64), "gru", 64, 8),
}


# --------------------------------------------------------------------------- edges


def _pack(src: np.ndarray, dst: np.ndarray) -> np.ndarray:
    """Generator-internal identity of a directed edge, used only to reject duplicates."""
    out = np.empty(src.size, dtype=np.uint64)

    def run(a, b):
        out[a:b] = (dst[a:b].astype(np.uint64) << np.uint64(32)) | src[a:b].astype(np.uint64)

    _pmap(run, src.size)
    return out


def _unpack(keys: np.ndarray, order: Optional[Tuple[int, int]] = None) -> Tuple[np.ndarray, np.ndarray]:
    """(src, dst) of packed edges; with order = (a, b) entry i is taken from keys[(a * i + b) % len(keys)]."""
    n = keys.size
    src = np.empty(n, dtype=np.int32)
    dst = np.empty(n, dtype=np.int32)

    def run(lo, hi):
        k = keys[lo:hi] if order is None else keys[(np.arange(lo, hi, dtype=np.int64) * order[0] + order[1]) % n]
        src[lo:hi] = (k & np.uint64(0xFFFFFFFF)).astype(np.int32)
        dst[lo:hi] = (k >> np.uint64(32)).astype(np.int32)

    _pmap(run, n)
    return src, dst


class _EndpointSampler:
    """Draws (src, dst) pairs: uniform, or proportional to Chung-Lu weights."""

    def __init__(self, wl: Workload):
        n, e = wl.num_nodes, wl.num_edges
        self.n = n
        if wl.structure == "uniform":
            self.cdf = None
            self.perm = None
            return
        if wl.structure != "chunglu":
            raise ValueError(f"unknown structure {wl.structure!r}")
        expo = -1.0 / (wl.gamma - 1.0)
        idx = np.arange(n, dtype=np.float64)
        cap = max(float(math.isqrt(e)), 1.5 * e / n)

        def max_deg(i0: float) -> float:
            w = (idx + i0) ** expo
            return e * w[0] / w.sum()

        lo, hi = 1e-9, float(n) * 1e3
        for _ in range(200):  # max_deg is decreasing in i0
            mid = math.sqrt(lo * hi)
            if max_deg(mid) > cap:
                lo = mid
            else:
                hi = mid
        w = (idx + hi) ** expo
        self.cdf = np.cumsum(w)
        self.cdf /= self.cdf[-1]
        self.perm = _rng(wl.seed, _S_PERM).permutation(n).astype(np.int32)

    def draw(self, rng: np.random.Generator, m: int) -> Tuple[np.ndarray, np.ndarray]:
        if self.cdf is None:
            return (rng.integers(0, self.n, m, dtype=np.int32), rng.integers(0, self.n, m, dtype=np.int32))
        out = []
        for _ in range(2):
            u = rng.random(m)
            ids = np.empty(m, dtype=np.int32)

            def run(a, b):
                ids[a:b] = self.perm[np.minimum(np.searchsorted(self.cdf, u[a:b]), self.n - 1)]

            _pmap(run, m)
            out.append(ids)
        return out[0], out[1]


def _draw_round(rng, sampler: _EndpointSampler, m: int):
    """m endpoint pairs as packed edges without self-loops and repeats: (in draw order, the same values sorted)."""
    s, d = sampler.draw(rng, m)
    ok = s != d
    return _first_occurrences(_pack(s[ok], d[ok]))


def _round_size(missing: int) -> int:
    return int(missing * 1.25) + 64


def _draw_new_edges(rng, sampler: _EndpointSampler, need: int, existing_sorted: np.ndarray, first_round=None) -> np.ndarray:
    """`need` distinct edges, none a self-loop, none in `existing_sorted`; returned sorted.  first_round: the result
    of _draw_round(rng, sampler, _round_size(need)) if the caller has drawn it already."""
    room = sampler.n * (sampler.n - 1) - existing_sorted.size
    if need > room:
        raise ValueError(f"{need} new edges requested, but only {room} distinct edges without self-loops are left on {sampler.n} nodes")
    got = np.empty(0, dtype=np.uint64)
    while got.size < need:
        if first_round is not None:
            k, uk = first_round
            first_round = None
        else:
            k, uk = _draw_round(rng, sampler, _round_size(need - got.size))
        taken = uk[_in_sorted(existing_sorted, uk) | _in_sorted(got, uk)]
        if taken.size:
            k = k[~_in_sorted(taken, k)]
        k = k[: need - got.size]
        got = np.sort(np.concatenate([got, k]))
    return got


@dataclass
class SnapshotSequence:
    """Everything one workload feeds to the loader, plus the generator's own change lists."""

    workload: Workload
    # raw loader input per snapshot: unsorted (src, dst) int32 arrays
    edges: List[Tuple[np.ndarray, np.ndarray]]
    # ground truth of what the generator did at step t (index 0 unused): sorted packed ids
    truth_inserted: List[np.ndarray]
    truth_deleted: List[np.ndarray]
    # features: X0 dense; per step (rows sorted unique int32, values [len(rows), d]); fp32 storage.
    # For feat_dtype == "bf16" every value is exactly representable in bfloat16.
    x0: np.ndarray
    feat_rows: List[np.ndarray]
    feat_vals: List[np.ndarray]

    @property
    def num_snapshots(self) -> int:
        return len(self.edges)

    def truth_pairs(self, t: int, which: str) -> Tuple[np.ndarray, np.ndarray]:
        """(src, dst) of the edges inserted ("ins") or deleted ("del") going from t-1 to t."""
        keys = self.truth_inserted[t] if which == "ins" else self.truth_deleted[t]
        return _unpack(keys)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bfloat16 (ties to even); result stays in fp32 storage."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of fp32 values that are already bfloat16-representable."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


_ROW_BLOCK = 1 << 16


def _normal_rows(seed: int, stream: int, n: int, d: int, to_bf16: bool) -> np.ndarray:
    """[n, d] fp32 N(0,1), drawn in blocks of 65,536 rows, block j from sub-stream j of the Philox key (the blocks
    are independent of each other, so several threads can draw them)."""
    x = np.empty((n, d), dtype=np.float32)

    def run(a, b):
        blk = _rng(seed, stream, a // _ROW_BLOCK).standard_normal((b - a, d), dtype=np.float32)
        x[a:b] = round_to_bf16(blk) if to_bf16 else blk

    _pmap(run, n, _ROW_BLOCK)
    return x


def make_sequence(wl: Workload, shuffle_edges: bool = True, progress=None) -> SnapshotSequence:
    """Generate the seeded snapshot sequence of a workload.

    `progress`, if given, is called as progress(stage, t, T) after each snapshot's edges ("edges") and
    feature rows ("features") are drawn; it does not influence the generated values.
    """
    n, e0, T, d = wl.num_nodes, wl.num_edges, wl.num_snapshots, wl.feat_dim
    tell = progress if progress is not None else (lambda stage, t, total: None)
    sampler = _EndpointSampler(wl)
    keys = _draw_new_edges(_rng(wl.seed, _S_GRAPH), sampler, e0, np.empty(0, dtype=np.uint64))

    def emit(k: np.ndarray, t: int):
        # The loader's input is an edge list in no particular order: the sorted keys are handed over through a seeded
        # index map i -> (a i + b) mod E with a coprime to E (a bijection; neighbours in the list are far apart in key
        # order).  Nothing downstream depends on this order.
        if not shuffle_edges or k.size < 2:
            return _unpack(k)
        r = _rng(wl.seed, _S_SHUFFLE, t)
        a = int(r.integers(k.size // 3, k.size)) | 1
        while math.gcd(a, k.size) != 1:
            a += 2
        return _unpack(k, (a % k.size, int(r.integers(0, k.size))))

    edges = [emit(keys, 0)]
    tell("edges", 0, T)
    t_ins: List[np.ndarray] = [np.empty(0, dtype=np.uint64)]
    t_del: List[np.ndarray] = [np.empty(0, dtype=np.uint64)]
    m = int(math.floor(wl.edge_churn * keys.size))  # (the edge count stays the same from step to step)

    def prepare(t: int):
        # what step t needs that does not depend on the edges of step t-1: which positions leave, and the first round
        # of candidate edges.  Each step has its own generator, so the steps can be prepared ahead by other threads.
        rng = _rng(wl.seed, _S_STEP, t)
        drop = np.sort(rng.choice(keys.size, m, replace=False)) if m else np.empty(0, dtype=np.int64)
        return rng, drop, (_draw_round(rng, sampler, _round_size(m)) if m else None)

    with ThreadPoolExecutor(max(1, min(4, _THREADS // 2))) as ahead:
        prepared = [ahead.submit(prepare, t) for t in range(1, T)]
        for t in range(1, T):
            rng, drop, first_round = prepared[t - 1].result()
            prepared[t - 1] = None
            ins = _draw_new_edges(rng, sampler, m, keys, first_round)  # rejects anything in E_{t-1}, deleted ones included
            t_del.append(keys[drop])
            t_ins.append(ins)
            keys = _replace_sorted(keys, drop, ins)
            edges.append(emit(keys, t))
            tell("edges", t, T)

    x0 = _normal_rows(wl.seed, _S_FEAT0, n, d, wl.feat_dtype == "bf16")
    rows_l = [np.empty(0, dtype=np.int32)]
    vals_l = [np.empty((0, d), dtype=np.float32)]
    for t in range(1, T):
        rng = _rng(wl.seed, _S_FEATSTEP, t)
        m = int(math.floor(wl.feat_churn * n))
        rows = np.sort(rng.choice(n, m, replace=False)).astype(np.int32) if m else np.empty(0, dtype=np.int32)
        vals = rng.standard_normal((m, d), dtype=np.float32)
        if wl.feat_dtype == "bf16":
            vals = round_to_bf16(vals)
        rows_l.append(rows)
        vals_l.append(vals)
        tell("features", t, T)
    return SnapshotSequence(wl, edges, t_ins, t_del, x0, rows_l, vals_l)


# --------------------------------------------------------------------------- model inputs


def num_gates(rnn: str) -> int:
    return {"gru": 3, "lstm": 4}[rnn]


def param_shapes(wl: Workload) -> List[Tuple[str, Tuple[int, ...]]]:
    """Flat parameter order shared by every consumer: per GCN layer W[d_in,d_out], b[d_out];
    then the recurrent cell W_i[d_last,K*H], W_h[H,K*H], b_i[K*H], b_h[K*H]."""
    out: List[Tuple[str, Tuple[int, ...]]] = []
    for l in range(len(wl.dims) - 1):
        out.append((f"W{l + 1}", (wl.dims[l], wl.dims[l + 1])))
        out.append((f"b{l + 1}", (wl.dims[l + 1],)))
    kh = num_gates(wl.rnn) * wl.hidden
    out += [("W_i", (wl.dims[-1], kh)), ("W_h", (wl.hidden, kh)), ("b_i", (kh,)), ("b_h", (kh,))]
    return out


def make_params(wl: Workload, bias_scale: float = 0.0, seed_offset: int = 0) -> np.ndarray:
    """Flat fp32 parameter vector: weights U(-1/sqrt(fan_in), 1/sqrt(fan_in)); biases
    bias_scale * U(-1, 1) (zero by default)."""
    rng = _rng(wl.seed + seed_offset, _S_PARAM)
    parts = []
    for name, shp in param_shapes(wl):
        if len(shp) == 2:
            a = 1.0 / math.sqrt(shp[0])
            parts.append(rng.uniform(-a, a, shp).astype(np.float32).ravel())
        else:
            parts.append((bias_scale * rng.uniform(-1.0, 1.0, shp)).astype(np.float32))
    return np.concatenate(parts)


def split_params(wl: Workload, flat: np.ndarray) -> dict:
    out, off = {}, 0
    for name, shp in param_shapes(wl):
        sz = int(np.prod(shp))
        out[name] = flat[off : off + sz].reshape(shp)
        off += sz
    if off != flat.size:
        raise ValueError(f"parameter vector has {flat.size} entries, layout needs {off}")
    return out


def make_target(wl: Workload) -> np.ndarray:
    return _rng(wl.seed, _S_TARGET).standard_normal((wl.num_nodes, wl.hidden), dtype=np.float32)
