"""Reference simulator of the aggregate cache's eviction policy (paper Section 3.3, "Eviction Policy":
score = future access count / size - imminence, plus expiration) and of the two classical policies the
paper compares it with (LRU and LFU, Section 5, "Effectiveness of Caching Policy").

TEST INFRASTRUCTURE: see the package docstring for who may import this.  Plain Python over dictionaries; it
shares no code with the HIP library's policy engine and never calls it.

The store (the semantics every policy shares)
---------------------------------------------
An entry has a key, a size, a remaining future access count F, an imminence I, the tick of its last use and
the number of uses since it entered.  A global tick advances by one on every `access` and `offer`.

access(key)  -> hit?   A present key is a hit: its last-use tick and use count are refreshed and F drops by
                       one (not below 0).  Under the score policy an entry whose F reaches 0 is expired: it
                       leaves at once, whatever its score (the paper's expiration rule).  An absent key is a
                       miss and changes nothing: the caller computes the aggregate and then offers it.
offer(key, size, F, I) -> admitted?, evicted keys
    score policy: an offer with F <= 0 is refused (it would expire immediately).  Otherwise, if room is short,
                  the entries are taken in ascending score F/S - I (ties: older last use, then smaller key) for as
                  long as room is short; the offer is admitted only if every one of them scores strictly below
                  the newcomer, else nothing is evicted and the offer is refused.
    LRU:          always admitted (if it fits the budget at all); victims by oldest last use.
    LFU:          always admitted; victims by fewest uses since entry, ties by oldest last use.
    keep-all:     no budget: everything is admitted, nothing leaves.
    An offer of a key that is already present only refreshes its F and I.
rescore(key, F, I)     Replaces F and I of a present key (no tick, no use): the caller's knowledge of the future
                       changed, e.g. the timestep that was using the aggregate is finished and its next use is a
                       sequence away.  An entry rescored to F <= 0 under the score policy expires.
Scores are compared exactly as rationals (integers cross-multiplied), never in floating point.

Where the paper is silent this file decides: the tie-breaks above, that a refused offer evicts nothing, that
F and I are integers supplied by the caller (the paper derives them from the position of the snapshot in the
sequence), and that LFU counts uses since entry (the count is lost on eviction).

Pins (tests/test_oracle_cache_policy.py): a textbook page-replacement string (LRU 12 faults, optimum 9), exhaustive
search for the optimal policy on small strings (no policy beats it; the score policy fed with true next-use distances
reaches it), closed forms for cyclic access, hand-worked LFU, exact score comparison, and the shape of the paper's
policy comparison on `encoder_decoder_flow`.  Parity unpinned: the hit rates the paper prints (52 % / 0 % at a 10 %
cache, 78 % plateau, 100 % at 60 %) - the model and the cache-size normalisation behind them are not given.

Access flows
------------
`sliding_window_flow`   the flow of the library's window driver: window q covers snapshots qS .. qS+L-1, looks
                        every one of them up in order, and after the window the aggregates it had to compute are
                        offered in snapshot order with F = number of later windows of the epoch that contain the
                        snapshot, I = L - S.
`encoder_decoder_flow`  the scenario the paper uses to define F and I: an LSTM-style encoder over sequence q and a
                        teacher-forced decoder over sequence q+1, K gates per cell, each gate reading the
                        aggregate of the input and then the aggregate of the hidden state; F and I by the
                        paper's formulas (its idx is 1-based).  Not part of the library's path; it exists to
                        compare the three policies on the access pattern the paper describes.
"""
from __future__ import annotations

from typing import Dict, Iterable, List, Sequence, Tuple

__all__ = ["CacheSim", "POLICIES", "sliding_window_flow", "sliding_window_future", "encoder_decoder_flow", "run_flow",
           "optimal_hits"]

POLICIES = ("keep_all", "score", "lru", "lfu")


class _Entry:
    __slots__ = ("size", "future", "imminence", "last_use", "uses")

    def __init__(self, size, future, imminence, tick):
        self.size, self.future, self.imminence, self.last_use, self.uses = size, future, imminence, tick, 1


def _score_less(a: _Entry, b: _Entry) -> bool:
    """F_a/S_a - I_a < F_b/S_b - I_b, exactly."""
    return a.future * b.size - a.imminence * a.size * b.size < b.future * a.size - b.imminence * a.size * b.size


class CacheSim:
    def __init__(self, policy: str, budget: int):
        assert policy in POLICIES
        self.policy, self.budget = policy, int(budget)
        self.entries: Dict[int, _Entry] = {}
        self.tick = 0
        self.used = 0
        self.peak_used = 0
        self.hits = self.misses = self.admitted = self.refused = self.evicted = self.expired = 0

    def __contains__(self, key: int) -> bool:
        return key in self.entries

    def _drop(self, key: int):
        self.used -= self.entries.pop(key).size

    def access(self, key: int) -> bool:
        self.tick += 1
        e = self.entries.get(key)
        if e is None:
            self.misses += 1
            return False
        self.hits += 1
        e.last_use = self.tick
        e.uses += 1
        e.future = max(e.future - 1, 0)
        if self.policy == "score" and e.future == 0:
            self._drop(key)
            self.expired += 1
        return True

    def rescore(self, key: int, future: int, imminence: int) -> None:
        e = self.entries.get(key)
        if e is None:
            return
        e.future, e.imminence = max(future, 0), imminence
        if self.policy == "score" and e.future == 0:
            self._drop(key)
            self.expired += 1

    def _victim_order(self, new: _Entry) -> List[int]:
        keys = list(self.entries)
        if self.policy == "lru":
            return sorted(keys, key=lambda k: (self.entries[k].last_use, k))
        if self.policy == "lfu":
            return sorted(keys, key=lambda k: (self.entries[k].uses, self.entries[k].last_use, k))
        # score: ascending F/S - I, exact; insertion sort by pairwise comparison keeps it obviously right
        order: List[int] = []
        for k in keys:
            e = self.entries[k]
            pos = len(order)
            for i, o in enumerate(order):
                eo = self.entries[o]
                if _score_less(e, eo) or (not _score_less(eo, e) and (e.last_use, k) < (eo.last_use, o)):
                    pos = i
                    break
            order.insert(pos, k)
        return order

    def offer(self, key: int, size: int, future: int, imminence: int) -> Tuple[bool, List[int]]:
        self.tick += 1
        assert size > 0
        if key in self.entries:
            e = self.entries[key]
            e.future, e.imminence = future, imminence
            return True, []
        new = _Entry(size, future, imminence, self.tick)
        if self.policy == "keep_all":
            self.entries[key] = new
            self.used += size
            self.peak_used = max(self.peak_used, self.used)
            self.admitted += 1
            return True, []
        if size > self.budget or (self.policy == "score" and future <= 0):
            self.refused += 1
            return False, []
        victims: List[int] = []
        freed = 0
        if self.used + size > self.budget:
            for k in self._victim_order(new):
                if self.used - freed + size <= self.budget:
                    break
                if self.policy == "score" and not _score_less(self.entries[k], new):
                    self.refused += 1
                    return False, []
                victims.append(k)
                freed += self.entries[k].size
        for k in victims:
            self._drop(k)
        self.evicted += len(victims)
        self.entries[key] = new
        self.used += size
        self.peak_used = max(self.peak_used, self.used)
        self.admitted += 1
        return True, victims


# ------------------------------------------------------------------------------------------------ flows
# A flow is a list of events: ("access", key), ("offer", key, size, F, I) or ("rescore", key, F, I).  `run_flow` makes an offer only when
# the latest access of that key was a miss (the aggregate had to be computed) and the key is still absent.


def sliding_window_future(t: int, q: int, T: int, L: int, stride: int) -> int:
    """Number of windows after window q (starts q*stride) of one epoch that contain snapshot t."""
    last = (T - L) // stride  # index of the last window
    count = 0
    for r in range(q + 1, last + 1):
        if r * stride <= t < r * stride + L:
            count += 1
    return count


def sliding_window_flow(T: int, L: int, stride: int, epochs: int = 1, size: int = 1):
    """Events of `epochs` passes of the window driver over T snapshots (Section 2.2: one window is one sample);
    every aggregate has the given size (the unit of the budget)."""
    events = []
    for _ in range(epochs):
        for q in range((T - L) // stride + 1):
            t0 = q * stride
            for t in range(t0, t0 + L):
                events.append(("access", t))
            for t in range(t0, t0 + L):
                events.append(("offer", t, size, sliding_window_future(t, q, T, L, stride), L - stride))
    return events


def encoder_decoder_flow(n_seq: int, L: int, stride: int, K: int, size: int = 1):
    """The paper's scenario (Section 3.3, eviction policy): per sequence q an encoder pass over snapshots
    qS .. qS+L-1, then a decoder pass over the next sequence's snapshots (teacher forcing).  At every timestep each
    of the K gates reads the aggregate of the input snapshot, then the aggregate of the hidden state.  Input
    aggregates are keyed by snapshot; hidden-state aggregates are unique to their timestep (key < 0).  Whenever
    gate g misses an aggregate it is computed and offered with the paper's F (which counts the accesses that
    remain after gate g); hidden-state aggregates belong to the local cache: F = K - g, I = 0.  While its timestep
    runs, an input aggregate is in local use as well (I = 0: the next gate reads it at once); when the timestep is
    finished it is rescored with the paper's global imminence (L - S from the encoder, L - 1 from the decoder).
    `size` is the size of every aggregate in the unit of the budget: with sizes counted in elements F/S is far
    below one unit of imminence, so imminence orders the entries and F/S breaks ties among equals."""
    events = []
    uniq = 0
    for q in range(n_seq):
        for part, base in (("enc", q * stride), ("dec", (q + 1) * stride)):
            for i in range(L):
                idx = i + 1  # the paper's idx is 1-based
                t = base + i
                uniq -= 1
                if part == "enc":
                    f_x = max(1, 2 * idx - 2 * stride + 1) * K
                    i_x = L - stride
                else:
                    f_x = max(2, 2 * idx - 2 * stride + 2) * K
                    i_x = L - 1
                for g in range(1, K + 1):
                    events.append(("access", t))
                    events.append(("offer", t, size, f_x - g, 0))
                    events.append(("access", uniq))
                    events.append(("offer", uniq, size, K - g, 0))
                events.append(("rescore", t, f_x - K, i_x))
    return events


def run_flow(sim: CacheSim, events: Iterable[Sequence]) -> List[bool]:
    """Feeds a flow to a simulator; returns hit/miss per access."""
    outcome: List[bool] = []
    missed = set()
    for ev in events:
        if ev[0] == "access":
            hit = sim.access(ev[1])
            outcome.append(hit)
            (missed.discard if hit else missed.add)(ev[1])
        elif ev[0] == "rescore":
            sim.rescore(ev[1], ev[2], ev[3])
        elif ev[1] in missed and ev[1] not in sim:
            sim.offer(ev[1], ev[2], ev[3], ev[4])
    return outcome


def optimal_hits(keys: Sequence[int], capacity: int) -> int:
    """Largest number of hits any demand policy with bypass can reach on a string of unit-size requests with
    `capacity` slots, by exhaustive search over every choice at every miss (tiny strings only).  Used to pin the
    simulator: no policy may beat it, and the textbook optimum (evict the key used farthest in the future) must
    equal it."""
    best = 0

    def go(i: int, held: frozenset, hits: int):
        nonlocal best
        if hits + (len(keys) - i) <= best:
            return
        if i == len(keys):
            best = max(best, hits)
            return
        k = keys[i]
        if k in held:
            go(i + 1, held, hits + 1)
            return
        go(i + 1, held, hits)  # bypass: do not keep it
        if len(held) < capacity:
            go(i + 1, held | {k}, hits)
        else:
            for v in held:
                go(i + 1, (held - {v}) | {k}, hits)

    go(0, frozenset(), 0)
    return best
