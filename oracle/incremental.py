"""Set-based transcription of the incremental aggregation rule (paper Section 3.2, Eq. 2).

TEST INFRASTRUCTURE, small graphs only (pure-Python loops over edge sets).  It exists to pin the
from-scratch reference in `oracle.dgnn` to the invariant "incremental equals full recompute", and
shares no code with the HIP library.

Eq. 2:  Agg_t = Agg_{t-1} - F_{t-1} * G-_t + F_t * G+_t, where the delta graphs hold
  * the deleted edges (G-) and the inserted edges (G+), and
  * for every node whose (scaled) feature row changed, its out-edges in the previous snapshot (G-)
    and its out-edges in the current snapshot (G+).
The unions are set unions: an edge that is both deleted and leaves a changed node counts once.
With a self-loop the implicit edge (v -> v) exists in every snapshot and is an out-edge of v.

Two algebraically equal rearrangements are also given; they use one feature matrix for the
structural terms and apply the row differences on one topology:
  form_prev_features:  S_t = S_{t-1} + sum_{E+} Y_{t-1}[u] - sum_{E-} Y_{t-1}[u] + sum_{(u->v) in E~_t} dY[u]
  form_cur_features:   S_t = S_{t-1} + sum_{E+} Y_t[u]     - sum_{E-} Y_t[u]     + sum_{(u->v) in E~_{t-1}} dY[u]
"""
from __future__ import annotations

from typing import Set, Tuple

import numpy as np

Edge = Tuple[int, int]  # (source, target)


def edge_set(src, dst) -> Set[Edge]:
    return {(int(u), int(v)) for u, v in zip(src, dst) if int(u) != int(v)}


def with_self_loops(edges: Set[Edge], n: int, self_loop: bool) -> Set[Edge]:
    return edges | {(v, v) for v in range(n)} if self_loop else set(edges)


def changed_rows(y_prev: np.ndarray, y_cur: np.ndarray) -> Set[int]:
    return {int(i) for i in np.nonzero(np.any(y_prev != y_cur, axis=1))[0]}


def delta_graphs(e_prev: Set[Edge], e_cur: Set[Edge], changed: Set[int], n: int, self_loop: bool):
    """(G-, G+) of Section 3.2, self-loops included as ordinary edges."""
    full_prev = with_self_loops(e_prev, n, self_loop)
    full_cur = with_self_loops(e_cur, n, self_loop)
    g_minus = (e_prev - e_cur) | {e for e in full_prev if e[0] in changed}
    g_plus = (e_cur - e_prev) | {e for e in full_cur if e[0] in changed}
    return g_minus, g_plus


def eq2_literal(s_prev, y_prev, y_cur, e_prev: Set[Edge], e_cur: Set[Edge], self_loop: bool) -> np.ndarray:
    """S_t from S_{t-1} exactly as Eq. 2 prints it."""
    n = s_prev.shape[0]
    g_minus, g_plus = delta_graphs(e_prev, e_cur, changed_rows(y_prev, y_cur), n, self_loop)
    s = np.array(s_prev, dtype=np.float64)
    for u, v in sorted(g_minus):
        s[v] -= y_prev[u]
    for u, v in sorted(g_plus):
        s[v] += y_cur[u]
    return s


def form_prev_features(s_prev, y_prev, y_cur, e_prev: Set[Edge], e_cur: Set[Edge], self_loop: bool) -> np.ndarray:
    n = s_prev.shape[0]
    changed = changed_rows(y_prev, y_cur)
    s = np.array(s_prev, dtype=np.float64)
    for u, v in sorted(e_cur - e_prev):
        s[v] += y_prev[u]
    for u, v in sorted(e_prev - e_cur):
        s[v] -= y_prev[u]
    for u, v in sorted(with_self_loops(e_cur, n, self_loop)):
        if u in changed:
            s[v] += y_cur[u] - y_prev[u]
    return s


def form_cur_features(s_prev, y_prev, y_cur, e_prev: Set[Edge], e_cur: Set[Edge], self_loop: bool) -> np.ndarray:
    n = s_prev.shape[0]
    changed = changed_rows(y_prev, y_cur)
    s = np.array(s_prev, dtype=np.float64)
    for u, v in sorted(e_cur - e_prev):
        s[v] += y_cur[u]
    for u, v in sorted(e_prev - e_cur):
        s[v] -= y_cur[u]
    for u, v in sorted(with_self_loops(e_prev, n, self_loop)):
        if u in changed:
            s[v] += y_cur[u] - y_prev[u]
    return s


def touched_rows(e_prev: Set[Edge], e_cur: Set[Edge], changed: Set[int], n: int, self_loop: bool) -> Set[int]:
    """Rows of S that may differ between t-1 and t; all other rows must stay bit-identical."""
    rows = {v for _, v in (e_prev ^ e_cur)}
    rows |= {v for u, v in with_self_loops(e_cur, n, self_loop) if u in changed}
    return rows
