"""Reference for the max / min neighbourhood aggregators (paper Section 3.2, the paragraph on aggregation
functions that cannot be updated by subtraction).

TEST INFRASTRUCTURE: see the package docstring for who may import this.  Plain loops over rows; small and
medium graphs only.  Shares no code with the HIP library.

Definition (from scratch).  For target v and feature j, over the sources u of the edges (u -> v) of the
snapshot, plus v itself with a self-loop:
    M[v, j] = max_u X[u, j]          (or min)
    C[v, j] = the source that attains it; among equal values the smallest source id
A target with no source at all (no in-edge, no self-loop) gets M = 0 and C = -1.

Incremental procedure (the paper's): the previous result is kept together with the ids of the edges that
produced it (here: the source id per (v, j), which names the edge (u -> v)).  An edge deletion is harmless unless
it removes such a contributing edge; when it does, the target is aggregated from scratch.  Otherwise the new
result is the old one combined with the values that arrive over inserted edges.  A source whose feature row
changed is a deletion of its old value (of its out-edges in the previous snapshot) plus an insertion of its new
value (over its out-edges in the current snapshot), as in Eq. 2.
"""
from __future__ import annotations

from typing import Set, Tuple

import numpy as np

__all__ = ["aggregate_minmax", "incremental_minmax_step"]


def _better(op: str, x: float, u: int, m: float, c: int) -> bool:
    if c < 0:
        return True
    if x != m:
        return x > m if op == "max" else x < m
    return u < c


def aggregate_minmax(row_ptr: np.ndarray, col: np.ndarray, x: np.ndarray, op: str, self_loop: bool) -> Tuple[np.ndarray, np.ndarray]:
    """(M, C) by the definition above.  x is used as given (any float dtype); M has x's dtype."""
    assert op in ("max", "min")
    n, d = x.shape
    m = np.zeros((n, d), dtype=x.dtype)
    c = np.full((n, d), -1, dtype=np.int32)
    for v in range(n):
        srcs = [int(u) for u in col[row_ptr[v]:row_ptr[v + 1]]]
        if self_loop:
            srcs.append(v)
        for u in srcs:
            for j in range(d):
                if _better(op, x[u, j], u, m[v, j], int(c[v, j])):
                    m[v, j] = x[u, j]
                    c[v, j] = u
    return m, c


def _row_from_scratch(v: int, row_ptr, col, x, op: str, self_loop: bool, m, c) -> None:
    d = x.shape[1]
    m[v, :] = 0
    c[v, :] = -1
    srcs = [int(u) for u in col[row_ptr[v]:row_ptr[v + 1]]]
    if self_loop:
        srcs.append(v)
    for u in srcs:
        for j in range(d):
            if _better(op, x[u, j], u, m[v, j], int(c[v, j])):
                m[v, j] = x[u, j]
                c[v, j] = u


def incremental_minmax_step(m_prev, c_prev, prev_ptr, prev_col, cur_ptr, cur_col, x_prev, x_cur, op: str, self_loop: bool,
                            arrivals_first: bool = False):
    """One snapshot step of the paper's procedure.  Returns (M, C, rows recomputed from scratch, rows touched).

    arrivals_first = False is the procedure as the paper words it: any lost contributing edge sends the target to
    the from-scratch path.  arrivals_first = True is the refinement the HIP kernel uses: the arriving values are
    combined first (inserted edges in ascending source order, then nothing else), and a lost source only forces
    the from-scratch path if it is still the recorded contributor afterwards -- a contributor that an arrival has
    already beaten (or tied with a smaller id) cannot matter any more.  Both give the from-scratch result."""
    n, d = x_cur.shape
    m, c = m_prev.copy(), c_prev.copy()
    changed: Set[int] = {int(i) for i in np.nonzero(np.any(x_prev != x_cur, axis=1))[0]}
    recomputed, touched = set(), set()
    for v in range(n):
        old = {int(u) for u in prev_col[prev_ptr[v]:prev_ptr[v + 1]]}
        new = {int(u) for u in cur_col[cur_ptr[v]:cur_ptr[v + 1]]}
        if self_loop:
            old.add(v)
            new.add(v)
        removed = (old - new) | (old & changed)        # contributions that no longer exist
        arrived = (new - old) | (new & changed)        # contributions that are new
        if not removed and not arrived:
            continue
        touched.add(v)
        if arrivals_first:
            # the kernel's order: values over inserted edges first, then the lost sources are looked up (deleted
            # edges, then changed sources, each changed source also contributing its new value as it is met)
            mv, cv = m[v].copy(), c[v].copy()
            for u in sorted(new - old):
                for j in range(d):
                    if _better(op, x_cur[u, j], u, mv[j], int(cv[j])):
                        mv[j], cv[j] = x_cur[u, j], u
            lost = any(int(cv[j]) in (old - new) for j in range(d))
            for u in sorted((new & changed) - {v}) + ([v] if v in (new & changed) else []):
                if u in old and any(int(cv[j]) == u for j in range(d)):
                    lost = True
                for j in range(d):
                    if _better(op, x_cur[u, j], u, mv[j], int(cv[j])):
                        mv[j], cv[j] = x_cur[u, j], u
            if lost:
                _row_from_scratch(v, cur_ptr, cur_col, x_cur, op, self_loop, m, c)
                recomputed.add(v)
            else:
                m[v], c[v] = mv, cv
            continue
        if any(int(c[v, j]) in removed for j in range(d)):
            _row_from_scratch(v, cur_ptr, cur_col, x_cur, op, self_loop, m, c)
            recomputed.add(v)
            continue
        for u in sorted(arrived):
            for j in range(d):
                if _better(op, x_cur[u, j], u, m[v, j], int(c[v, j])):
                    m[v, j] = x_cur[u, j]
                    c[v, j] = u
    return m, c, recomputed, touched
