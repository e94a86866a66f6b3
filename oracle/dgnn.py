"""From-scratch fp64 reference of the stacked dynamic GNN (GCN layers, then a GRU/LSTM over time).

TEST INFRASTRUCTURE: see the package docstring for who may import this.

Orientation (paper Section 3.2): an edge goes from a source to a target and the target
aggregates the source's features, so the adjacency is stored as a CSR by destination whose row v
lists the sources u of the edges (u -> v).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

__all__ = [
    "build_native",
    "num_threads",
    "canonicalise",
    "csr_from_keys",
    "edge_deltas",
    "features_at",
    "change_counts",
    "degrees",
    "aggregate",
    "aggregate_adjoint",
    "aggregate_rows",
    "dense_layer",
    "gru_cell",
    "lstm_cell",
    "Graph",
    "graphs_of",
    "forward_window",
    "backward_window",
    "forward_window_integrated",
    "backward_window_integrated",
    "AGG_MODES",
]

AGG_MODES = {"sum": 0, "mean": 1, "sym": 2}

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle_agg.so")
_lib = None


def build_native(force: bool = False) -> str:
    """Compile agg.c with gcc (plain C, OpenMP row partition)."""
    src = os.path.join(_HERE, "agg.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC", src, "-o", _SO, "-lm"])
    return _SO


def _native():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_native())
        i64, i32, p = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
        lib.oracle_aggregate.argtypes = [i64, i32, p, p, p, ctypes.c_int, ctypes.c_int, p, p]
        lib.oracle_aggregate.restype = ctypes.c_int
        lib.oracle_aggregate_adjoint.argtypes = [i64, i32, p, p, p, ctypes.c_int, ctypes.c_int, p]
        lib.oracle_aggregate_adjoint.restype = ctypes.c_int
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_native().oracle_num_threads())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


# ----------------------------------------------------------------------------- graph side


def canonicalise(src: np.ndarray, dst: np.ndarray, n: int) -> np.ndarray:
    """A snapshot is a set of directed edges without self-loops: drop u == v, order by
    (target, source), remove duplicates.  Returns 64-bit ids target * 2^32 + source."""
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    if src.shape != dst.shape:
        raise ValueError("src and dst differ in length")
    if src.size and (src.min() < 0 or dst.min() < 0 or src.max() >= n or dst.max() >= n):
        raise ValueError("node id out of range")
    keep = src != dst
    ids = dst[keep] * (1 << 32) + src[keep]
    return np.unique(ids).astype(np.uint64)


def csr_from_keys(keys: np.ndarray, n: int) -> Tuple[np.ndarray, np.ndarray]:
    """CSR by destination from sorted unique ids (counting sort on the target)."""
    k = keys.astype(np.int64)
    tgt = k >> 32
    counts = np.bincount(tgt, minlength=n).astype(np.int64)
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    col = (k & 0xFFFFFFFF).astype(np.int32)
    return row_ptr, col


def edge_deltas(keys_prev: np.ndarray, keys_cur: np.ndarray, n: int):
    """Edge insertions E_t \\ E_{t-1} and deletions E_{t-1} \\ E_t (Section 3.2), each as a CSR
    by destination with ascending columns.  Returns ((ins_row_ptr, ins_col), (del_row_ptr, del_col))."""
    ins = np.setdiff1d(keys_cur, keys_prev, assume_unique=True)
    dele = np.setdiff1d(keys_prev, keys_cur, assume_unique=True)
    return csr_from_keys(ins, n), csr_from_keys(dele, n)


def features_at(x0: np.ndarray, feat_rows: Sequence[np.ndarray], feat_vals: Sequence[np.ndarray], t: int) -> np.ndarray:
    """X_t: X_0 with the rows listed for steps 1..t replaced in order (fp64 copy)."""
    x = np.array(x0, dtype=np.float64)
    for s in range(1, t + 1):
        if len(feat_rows[s]):
            x[feat_rows[s]] = feat_vals[s]
    return x


def change_counts(g_prev: "Graph", g_cur: "Graph", x_prev, x_cur, mode: str, self_loop: bool) -> Dict[str, int]:
    """Size of one step's change (Section 3.2): inserted and deleted edges, the nodes whose scaled feature row
    differs (for "sym" a degree change alters the scaling), the current out-edges of those nodes (self-loop
    included) -- together the effective delta edges -- and the number of target rows they touch."""
    n = g_cur.n
    ins = np.setdiff1d(g_cur.keys, g_prev.keys, assume_unique=True)
    dele = np.setdiff1d(g_prev.keys, g_cur.keys, assume_unique=True)
    changed = np.any(np.asarray(x_prev) != np.asarray(x_cur), axis=1)
    if mode == "sym":
        changed |= np.diff(g_prev.row_ptr) != np.diff(g_cur.row_ptr)
    hit = changed[g_cur.col]
    rows_cur = np.repeat(np.arange(n), np.diff(g_cur.row_ptr))
    touched = np.zeros(n, dtype=bool)
    touched[(ins >> np.uint64(32)).astype(np.int64)] = True
    touched[(dele >> np.uint64(32)).astype(np.int64)] = True
    touched[rows_cur[hit]] = True
    n_f = int(hit.sum())
    if self_loop:
        touched |= changed
        n_f += int(changed.sum())
    return dict(n_ins=int(ins.size), n_del=int(dele.size), n_changed=int(changed.sum()), n_fchg_entries=n_f,
                n_entries=int(ins.size + dele.size + n_f), n_rows=int(touched.sum()))


def degrees(row_ptr: np.ndarray, self_loop: bool) -> np.ndarray:
    return np.diff(row_ptr).astype(np.float64) + (1.0 if self_loop else 0.0)


def aggregate(row_ptr, col, x, mode: str, self_loop: bool) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 1 from scratch.  Returns (S, Agg): the un-normalised sums over scaled sources and the
    aggregate after target-side scaling (identical for "sum")."""
    n = row_ptr.size - 1
    x = np.ascontiguousarray(x, dtype=np.float64)
    if x.shape[0] != n:
        raise ValueError("feature rows != nodes")
    d = x.shape[1]
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
    col = np.ascontiguousarray(col, dtype=np.int32)
    s = np.empty((n, d), dtype=np.float64)
    agg = np.empty((n, d), dtype=np.float64)
    rc = _native().oracle_aggregate(n, d, _ptr(row_ptr), _ptr(col), _ptr(x), AGG_MODES[mode], int(self_loop), _ptr(s), _ptr(agg))
    if rc:
        raise ValueError("column index out of range")
    return s, agg


def aggregate_adjoint(row_ptr, col, g, mode: str, self_loop: bool) -> np.ndarray:
    """dLoss/dX given g = dLoss/dAgg for Agg = aggregate(X)."""
    n = row_ptr.size - 1
    g = np.ascontiguousarray(g, dtype=np.float64)
    d = g.shape[1]
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
    col = np.ascontiguousarray(col, dtype=np.int32)
    dx = np.empty((n, d), dtype=np.float64)
    rc = _native().oracle_aggregate_adjoint(n, d, _ptr(row_ptr), _ptr(col), _ptr(g), AGG_MODES[mode], int(self_loop), _ptr(dx))
    if rc:
        raise ValueError("column index out of range")
    return dx


def aggregate_rows(row_ptr, col, x, rows, mode: str, self_loop: bool) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 1 for a sample of target rows only, one row at a time from the definition (for graphs too large
    to aggregate in full on the host).  x may be fp32; sums are fp64.  Returns (S[rows], Agg[rows])."""
    deg = np.diff(row_ptr).astype(np.float64) + (1.0 if self_loop else 0.0)
    with np.errstate(divide="ignore"):
        if mode == "sym":
            p = np.where(deg > 0, 1.0 / np.sqrt(deg), 0.0)
            q = p
        elif mode == "mean":
            p = np.ones_like(deg)
            q = np.where(deg > 0, 1.0 / deg, 0.0)
        else:
            p = q = np.ones_like(deg)
    d = x.shape[1]
    s = np.zeros((len(rows), d), dtype=np.float64)
    for k, v in enumerate(rows):
        u = col[row_ptr[v]:row_ptr[v + 1]]
        acc = (p[u, None] * x[u].astype(np.float64)).sum(axis=0) if u.size else np.zeros(d)
        if self_loop:
            acc = acc + p[v] * x[v].astype(np.float64)
        s[k] = acc
    return s, s * q[np.asarray(rows)][:, None]


# ----------------------------------------------------------------------------- dense side


def dense_layer(agg: np.ndarray, w: np.ndarray, b: Optional[np.ndarray], relu: bool = True) -> np.ndarray:
    """GCN update step (Listing 1 of Section 3.5): aggregate first, then a linear map, then ReLU."""
    z = np.asarray(agg, dtype=np.float64) @ np.asarray(w, dtype=np.float64)
    if b is not None:
        z = z + np.asarray(b, dtype=np.float64)
    return np.maximum(z, 0.0) if relu else z


def _sigmoid(a: np.ndarray) -> np.ndarray:
    return 1.0 / (1.0 + np.exp(-a))


def gru_cell(x, h, w_i, w_h, b_i, b_h):
    """GRU with gate order (r, z, n); weights are [in, 3H] and [H, 3H]:
    r = sig(x W_ir + b_ir + h W_hr + b_hr), z likewise, n = tanh(x W_in + b_in + r * (h W_hn + b_hn)),
    h' = (1 - z) * n + z * h.   (Three gates: Section 3.3.)"""
    hd = h.shape[1]
    gi = x @ w_i + b_i
    gh = h @ w_h + b_h
    r = _sigmoid(gi[:, :hd] + gh[:, :hd])
    z = _sigmoid(gi[:, hd : 2 * hd] + gh[:, hd : 2 * hd])
    nn = np.tanh(gi[:, 2 * hd :] + r * gh[:, 2 * hd :])
    h_new = (1.0 - z) * nn + z * h
    return h_new, (r, z, nn, gh[:, 2 * hd :])


def lstm_cell(x, h, c, w_i, w_h, b_i, b_h):
    """LSTM with gate order (i, f, g, o); weights are [in, 4H] and [H, 4H]:
    c' = f * c + i * g,  h' = o * tanh(c').   (Four gates: Section 3.3.)"""
    hd = h.shape[1]
    a = x @ w_i + b_i + h @ w_h + b_h
    i = _sigmoid(a[:, :hd])
    f = _sigmoid(a[:, hd : 2 * hd])
    g = np.tanh(a[:, 2 * hd : 3 * hd])
    o = _sigmoid(a[:, 3 * hd :])
    c_new = f * c + i * g
    h_new = o * np.tanh(c_new)
    return h_new, c_new, (i, f, g, o)


# ----------------------------------------------------------------------------- the stacked model


class Graph:
    """One canonical snapshot."""

    def __init__(self, keys: np.ndarray, n: int):
        self.n = n
        self.keys = keys
        self.row_ptr, self.col = csr_from_keys(keys, n)


def graphs_of(edges: Sequence[Tuple[np.ndarray, np.ndarray]], n: int) -> List[Graph]:
    return [Graph(canonicalise(s, d, n), n) for s, d in edges]


def _f64(p: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    return {k: np.asarray(v, dtype=np.float64) for k, v in p.items()}


def forward_window(
    graphs: Sequence[Graph],
    feats: Sequence[np.ndarray],
    params: Dict[str, np.ndarray],
    num_layers: int,
    mode: str,
    self_loop: bool,
    rnn: str,
    target: Optional[np.ndarray] = None,
    keep: bool = False,
    loss_rows: Optional[np.ndarray] = None,
):
    """Forward over one window (Section 2.2: a sequence of consecutive snapshots is one sample and the
    recurrent state runs across it).  graphs[i], feats[i] are snapshot t0+i.  Every timestep recomputes
    H^l = ReLU(Agg(H^{l-1}; G_t) W_l + b_l) for l = 1..num_layers from H^0 = X_t, then steps the
    recurrent cell from zero state.  loss = mean((h_last - target)^2), over all nodes or, for a node mini-batch
    (Section 4.2: the sample is the sequence of computational graphs of the selected nodes), over the rows
    `loss_rows` of h_last and target only.
    Returns (loss or None, h_last, saved) where saved feeds backward_window when keep is set."""
    p = _f64(params)
    n = graphs[0].n
    hd = p["W_h"].shape[0]
    h = np.zeros((n, hd))
    c = np.zeros((n, hd))
    saved = []
    for g, x in zip(graphs, feats):
        hl = np.asarray(x, dtype=np.float64)
        aggs, zs = [], []
        for l in range(1, num_layers + 1):
            _, agg = aggregate(g.row_ptr, g.col, hl, mode, self_loop)
            z = agg @ p[f"W{l}"] + p[f"b{l}"]
            hl = np.maximum(z, 0.0)
            aggs.append(agg)
            zs.append(z)
        if rnn == "gru":
            h_new, gates = gru_cell(hl, h, p["W_i"], p["W_h"], p["b_i"], p["b_h"])
            c_new = c
        else:
            h_new, c_new, gates = lstm_cell(hl, h, c, p["W_i"], p["W_h"], p["b_i"], p["b_h"])
        if keep:
            saved.append(dict(aggs=aggs, zs=zs, x=hl, h_prev=h, c_prev=c, c_new=c_new, gates=gates))
        h, c = h_new, c_new
    loss = None
    if target is not None:
        diff = h - np.asarray(target, dtype=np.float64)
        loss = float(np.mean((diff if loss_rows is None else diff[np.asarray(loss_rows)]) ** 2))
    return loss, h, saved


def backward_window(
    graphs: Sequence[Graph],
    saved,
    h_last: np.ndarray,
    params: Dict[str, np.ndarray],
    num_layers: int,
    mode: str,
    self_loop: bool,
    rnn: str,
    target: np.ndarray,
    loss_rows: Optional[np.ndarray] = None,
) -> Dict[str, np.ndarray]:
    """Back-propagation through time over the window (Section 2.2) for the loss of forward_window (the same
    `loss_rows`).  Gradients for every parameter; nothing is propagated to the input features."""
    p = _f64(params)
    hd = p["W_h"].shape[0]
    grads = {k: np.zeros_like(v) for k, v in p.items()}
    tgt = np.asarray(target, dtype=np.float64)
    if loss_rows is None:
        dh = 2.0 * (h_last - tgt) / tgt.size
    else:
        rows = np.asarray(loss_rows)
        dh = np.zeros_like(h_last)
        dh[rows] = 2.0 * (h_last[rows] - tgt[rows]) / (rows.size * tgt.shape[1])
    dc = np.zeros_like(dh)
    for g, sv in zip(reversed(list(graphs)), reversed(saved)):
        x, h_prev = sv["x"], sv["h_prev"]
        if rnn == "gru":
            r, z, nn, ghn = sv["gates"]
            dn_pre = dh * (1.0 - z) * (1.0 - nn * nn)
            dz_pre = dh * (h_prev - nn) * z * (1.0 - z)
            dr_pre = dn_pre * ghn * r * (1.0 - r)
            dgi = np.concatenate([dr_pre, dz_pre, dn_pre], axis=1)
            dgh = np.concatenate([dr_pre, dz_pre, dn_pre * r], axis=1)
            dh_prev = dh * z + dgh @ p["W_h"].T
        else:
            i, f, gg, o = sv["gates"]
            tc = np.tanh(sv["c_new"])
            dcc = dc + dh * o * (1.0 - tc * tc)
            do_pre = dh * tc * o * (1.0 - o)
            di_pre = dcc * gg * i * (1.0 - i)
            df_pre = dcc * sv["c_prev"] * f * (1.0 - f)
            dg_pre = dcc * i * (1.0 - gg * gg)
            dgi = np.concatenate([di_pre, df_pre, dg_pre, do_pre], axis=1)
            dgh = dgi
            dh_prev = dgh @ p["W_h"].T
            dc = dcc * f
        grads["W_i"] += x.T @ dgi
        grads["W_h"] += h_prev.T @ dgh
        grads["b_i"] += dgi.sum(axis=0)
        grads["b_h"] += dgh.sum(axis=0)
        dhl = dgi @ p["W_i"].T
        for l in range(num_layers, 0, -1):
            dz = dhl * (sv["zs"][l - 1] > 0.0)
            grads[f"W{l}"] += sv["aggs"][l - 1].T @ dz
            grads[f"b{l}"] += dz.sum(axis=0)
            if l > 1:
                dagg = dz @ p[f"W{l}"].T
                dhl = aggregate_adjoint(g.row_ptr, g.col, dagg, mode, self_loop)
        dh = dh_prev
    return grads


# ----------------------------------------------------------------------------- the integrated model


def forward_window_integrated(
    graphs: Sequence[Graph],
    feats: Sequence[np.ndarray],
    params: Dict[str, np.ndarray],
    mode: str,
    self_loop: bool,
    rnn: str,
    target: Optional[np.ndarray] = None,
    keep: bool = False,
    loss_rows: Optional[np.ndarray] = None,
):
    """Forward over one window of the integrated model (Section 2.1: a GraphRNN replaces the matrix products of
    the recurrent gates by graph operations on x_t and h_{t-1}; Section 3.1, reuse across gates: the inputs are
    aggregated once and the hidden states once, and all gates share the two aggregates).  Per timestep
        ax = Agg(X_t; G_t),   ah = Agg(h_{t-1}; G_t),
        h_t = cell(x = ax, h = ah)  with the carry term taken from the un-aggregated state:
        GRU:  h_t = (1 - z) * n + z * h_{t-1};    LSTM:  c_t = f * c_{t-1} + i * g,  h_t = o * tanh(c_t).
    params: W_i [d0, K*H], W_h [H, K*H], b_i, b_h.  Zero initial state; loss = mean((h_last - target)^2), over the
    rows `loss_rows` of h_last and target only if given (a node mini-batch, Section 4.2)."""
    p = _f64(params)
    n = graphs[0].n
    hd = p["W_h"].shape[0]
    h = np.zeros((n, hd))
    c = np.zeros((n, hd))
    saved = []
    for g, x in zip(graphs, feats):
        _, ax = aggregate(g.row_ptr, g.col, np.asarray(x, dtype=np.float64), mode, self_loop)
        _, ah = aggregate(g.row_ptr, g.col, h, mode, self_loop)
        if rnn == "gru":
            h_cell, gates = gru_cell(ax, ah, p["W_i"], p["W_h"], p["b_i"], p["b_h"])
            z = gates[1]
            h_new = h_cell - z * ah + z * h  # the cell's carry z * (its h input) replaced by z * h_{t-1}
            c_new = c
        else:
            h_new, c_new, gates = lstm_cell(ax, ah, c, p["W_i"], p["W_h"], p["b_i"], p["b_h"])
        if keep:
            saved.append(dict(ax=ax, ah=ah, h_prev=h, c_prev=c, c_new=c_new, gates=gates))
        h, c = h_new, c_new
    loss = None
    if target is not None:
        diff = h - np.asarray(target, dtype=np.float64)
        loss = float(np.mean((diff if loss_rows is None else diff[np.asarray(loss_rows)]) ** 2))
    return loss, h, saved


def backward_window_integrated(
    graphs: Sequence[Graph],
    saved,
    h_last: np.ndarray,
    params: Dict[str, np.ndarray],
    mode: str,
    self_loop: bool,
    rnn: str,
    target: np.ndarray,
    loss_rows: Optional[np.ndarray] = None,
) -> Dict[str, np.ndarray]:
    """Back-propagation through time for forward_window_integrated (the same `loss_rows`).  The gradient reaches
    h_{t-1} over two paths: the carry term, and the aggregate ah through the adjoint of the aggregation."""
    p = _f64(params)
    grads = {k: np.zeros_like(v) for k, v in p.items()}
    tgt = np.asarray(target, dtype=np.float64)
    if loss_rows is None:
        dh = 2.0 * (h_last - tgt) / tgt.size
    else:
        rows = np.asarray(loss_rows)
        dh = np.zeros_like(h_last)
        dh[rows] = 2.0 * (h_last[rows] - tgt[rows]) / (rows.size * tgt.shape[1])
    dc = np.zeros_like(dh)
    for g, sv in zip(reversed(list(graphs)), reversed(saved)):
        ax, ah, h_prev = sv["ax"], sv["ah"], sv["h_prev"]
        if rnn == "gru":
            r, z, nn, ghn = sv["gates"]
            dn_pre = dh * (1.0 - z) * (1.0 - nn * nn)
            dz_pre = dh * (h_prev - nn) * z * (1.0 - z)
            dr_pre = dn_pre * ghn * r * (1.0 - r)
            dgi = np.concatenate([dr_pre, dz_pre, dn_pre], axis=1)
            dgh = np.concatenate([dr_pre, dz_pre, dn_pre * r], axis=1)
            carry = dh * z
        else:
            i, f, gg, o = sv["gates"]
            tc = np.tanh(sv["c_new"])
            dcc = dc + dh * o * (1.0 - tc * tc)
            do_pre = dh * tc * o * (1.0 - o)
            di_pre = dcc * gg * i * (1.0 - i)
            df_pre = dcc * sv["c_prev"] * f * (1.0 - f)
            dg_pre = dcc * i * (1.0 - gg * gg)
            dgi = np.concatenate([di_pre, df_pre, dg_pre, do_pre], axis=1)
            dgh = dgi
            carry = 0.0
            dc = dcc * f
        grads["W_i"] += ax.T @ dgi
        grads["W_h"] += ah.T @ dgh
        grads["b_i"] += dgi.sum(axis=0)
        grads["b_h"] += dgh.sum(axis=0)
        dah = dgh @ p["W_h"].T
        dh = carry + aggregate_adjoint(g.row_ptr, g.col, dah, mode, self_loop)
    return grads
