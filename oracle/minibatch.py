"""Computational graphs of a node mini-batch over a snapshot sequence (paper Section 4.2, "Rethinking Mini-batch
Training": a set of nodes is selected, the computational graphs of those nodes are extracted from every snapshot
of the sequence, and that sequence of computational graphs is one sample).

TEST INFRASTRUCTURE: see the package docstring for who may import this.

Plain definitions, written with Python sets:
  F_0 = the batch;  F_k = F_{k-1} united with the sources of every edge, of any snapshot, whose target is in
  F_{k-1}  (k = 1 .. hops);  the sub-sequence keeps the nodes F_hops and, of every snapshot, the edges whose
  target is in F_{hops-1}.
A model of `hops` aggregation layers evaluated on the sub-sequence gives, on the batch rows, what it gives on the
whole graph: row v of layer l needs layer l-1 on v and on the sources of v's edges only.  (With the symmetric
normalisation the scale of a SOURCE is a degree too, so one more hop is needed for the same statement.)

The numbering of the sub-sequence: the batch nodes first, in the order given, then the nodes first reached in one
hop, in ascending order of their ids, then those first reached in two hops, and so on: F_k is the first |F_k| ids
for every k, and layer l of an L-layer model is needed on the first |F_{L-l}| rows only.

Pins (tests/test_oracle_minibatch.py): hand-worked chains and stars; the closure equals the breadth-first ball in
the union graph found by matrix powers of a dense adjacency; the model restricted to the sub-sequence reproduces
the full-graph model on the batch rows; batch losses and gradients over a partition add up to the full ones.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

__all__ = ["closure", "extract"]


def closure(edges: Sequence[Tuple[np.ndarray, np.ndarray]], batch: Sequence[int], hops: int) -> List[set]:
    """[F_0, F_1, ..., F_hops] for directed edge lists (src, dst) per snapshot; self-loops do not matter."""
    levels = [set(int(v) for v in batch)]
    for _ in range(hops):
        prev = levels[-1]
        nxt = set(prev)
        for src, dst in edges:
            for u, v in zip(np.asarray(src).tolist(), np.asarray(dst).tolist()):
                if v in prev:
                    nxt.add(u)
        levels.append(nxt)
    return levels


def extract(edges: Sequence[Tuple[np.ndarray, np.ndarray]], batch: Sequence[int], hops: int):
    """Returns (node_list, sub_edges, n_inner): node_list[new id] = old id (batch first, then by the number of hops
    at which a node is first reached, ascending ids within one number), sub_edges[t] = (src, dst) in new ids of the
    edges of snapshot t whose target lies in F_{hops-1}, in the order of the input list, and n_inner = |F_{hops-1}|."""
    batch = [int(v) for v in batch]
    if len(set(batch)) != len(batch):
        raise ValueError("batch nodes must be distinct")
    levels = closure(edges, batch, hops)
    inner = levels[hops - 1] if hops > 0 else set()
    rest = [v for k in range(1, hops + 1) for v in sorted(levels[k] - levels[k - 1])]
    node_list = np.array(batch + rest, dtype=np.int64)
    new_id = {old: i for i, old in enumerate(node_list.tolist())}
    sub = []
    for src, dst in edges:
        s_new, d_new = [], []
        for u, v in zip(np.asarray(src).tolist(), np.asarray(dst).tolist()):
            if v in inner:
                s_new.append(new_id[u])
                d_new.append(new_id[v])
        sub.append((np.array(s_new, dtype=np.int32), np.array(d_new, dtype=np.int32)))
    return node_list, sub, len(inner)
