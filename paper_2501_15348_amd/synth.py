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
from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np

# stream ids for the Philox key
_S_GRAPH, _S_PERM, _S_STEP, _S_FEAT0, _S_FEATSTEP, _S_PARAM, _S_TARGET, _S_SHUFFLE = range(8)


def _rng(seed: int, stream: int, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed << 16) ^ sub, stream]))


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
    return (dst.astype(np.uint64) << np.uint64(32)) | src.astype(np.uint64)


def _unpack(keys: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    src = (keys & np.uint64(0xFFFFFFFF)).astype(np.int32)
    dst = (keys >> np.uint64(32)).astype(np.int32)
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
        s = np.minimum(np.searchsorted(self.cdf, rng.random(m)), self.n - 1)
        d = np.minimum(np.searchsorted(self.cdf, rng.random(m)), self.n - 1)
        return self.perm[s], self.perm[d]


def _draw_new_edges(rng, sampler: _EndpointSampler, need: int, existing_sorted: np.ndarray) -> np.ndarray:
    """`need` distinct edges, none a self-loop, none in `existing_sorted`; returned sorted."""
    room = sampler.n * (sampler.n - 1) - existing_sorted.size
    if need > room:
        raise ValueError(f"{need} new edges requested, but only {room} distinct edges without self-loops are left on {sampler.n} nodes")
    got = np.empty(0, dtype=np.uint64)
    while got.size < need:
        m = int((need - got.size) * 1.25) + 64
        s, d = sampler.draw(rng, m)
        ok = s != d
        k = _pack(s[ok], d[ok])
        _, first = np.unique(k, return_index=True)
        k = k[np.sort(first)]  # distinct, in draw order
        for ref in (existing_sorted, got):
            if ref.size:
                pos = np.minimum(np.searchsorted(ref, k), ref.size - 1)
                k = k[ref[pos] != k]
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
        if shuffle_edges:
            k = k[_rng(wl.seed, _S_SHUFFLE, t).permutation(k.size)]
        return _unpack(k)

    edges = [emit(keys, 0)]
    tell("edges", 0, T)
    t_ins: List[np.ndarray] = [np.empty(0, dtype=np.uint64)]
    t_del: List[np.ndarray] = [np.empty(0, dtype=np.uint64)]
    for t in range(1, T):
        rng = _rng(wl.seed, _S_STEP, t)
        m = int(math.floor(wl.edge_churn * keys.size))
        drop = np.sort(rng.choice(keys.size, m, replace=False)) if m else np.empty(0, dtype=np.int64)
        ins = _draw_new_edges(rng, sampler, m, keys)  # rejects anything in E_{t-1}, deleted ones included
        keep = np.ones(keys.size, dtype=bool)
        keep[drop] = False
        t_del.append(keys[drop])
        t_ins.append(ins)
        keys = np.sort(np.concatenate([keys[keep], ins]))
        edges.append(emit(keys, t))
        tell("edges", t, T)

    x0 = _rng(wl.seed, _S_FEAT0).standard_normal((n, d), dtype=np.float32)
    if wl.feat_dtype == "bf16":
        x0 = round_to_bf16(x0)
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
