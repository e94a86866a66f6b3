"""The library's host-side cache-policy store (Section 3.3, eviction policy) against the reference simulator:
identical decisions, event by event, on random traces, on the window driver's flow and on the paper's
encoder-decoder scenario.  Runs without a GPU (the store never touches the device)."""
import random

import pytest

from oracle.cache_policy import CacheSim, encoder_decoder_flow, sliding_window_flow
from paper_2501_15348_amd import reinc

POLICIES = ("score", "lru", "lfu", "keep_all")


def replay_both(policy, budget, events):
    """Feeds the same events to both stores and compares every outcome."""
    ref = CacheSim(policy, budget)
    lib = reinc.PolicyStore(policy, budget)
    missed = set()
    for n, ev in enumerate(events):
        if ev[0] == "access":
            a, b = ref.access(ev[1]), lib.access(ev[1])
            assert a == b, (n, ev)
            (missed.discard if a else missed.add)(ev[1])
        elif ev[0] == "rescore":
            ref.rescore(ev[1], ev[2], ev[3])
            lib.rescore(ev[1], ev[2], ev[3])
        elif ev[0] == "offer_always" or (ev[1] in missed and ev[1] not in ref):
            (ok_a, gone_a), (ok_b, gone_b) = ref.offer(*ev[1:]), lib.offer(*ev[1:])
            assert ok_a == ok_b and sorted(gone_a) == sorted(gone_b), (n, ev, gone_a, gone_b)
        if n % 17 == 0:
            for k in list(ref.entries)[:4]:
                assert k in lib
    want = {k: getattr(ref, k) for k in reinc.POLICY_COUNTERS}
    assert lib.counters() == want
    lib.close()
    return ref


@pytest.mark.parametrize("policy", POLICIES)
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_traces(policy, seed):
    rng = random.Random(seed)
    events = []
    for _ in range(3000):
        k = rng.randrange(-20, 20)
        r = rng.random()
        if r < 0.55:
            events.append(("access", k))
        elif r < 0.9:
            events.append(("offer_always", k, rng.choice([1, 2, 3, 5, 1 << 20]), rng.randrange(0, 6), rng.randrange(0, 9)))
        else:
            events.append(("rescore", k, rng.randrange(0, 4), rng.randrange(0, 9)))
    ref = replay_both(policy, 9 if seed < 3 else (1 << 21) + 7, events)
    if policy != "keep_all":
        assert ref.evicted > 0


@pytest.mark.parametrize("policy", POLICIES)
@pytest.mark.parametrize("budget", [0, 1, 3, 7, 20])
def test_window_flow(policy, budget):
    replay_both(policy, budget, sliding_window_flow(24, 8, 1, epochs=2))
    replay_both(policy, budget, sliding_window_flow(24, 8, 3))


@pytest.mark.parametrize("policy", ["score", "lru", "lfu"])
@pytest.mark.parametrize("slots", [1, 2, 5, 9, 16])
def test_encoder_decoder_flow(policy, slots):
    size = 1 << 20
    replay_both(policy, slots * size, encoder_decoder_flow(12, 8, 1, 4, size))


def test_large_operands_stay_exact():
    # sizes, F and I just below the documented 2^40 limit: a score difference of one part in 2^39
    top = (1 << 40) - 1
    events = [("offer_always", 1, top, top, top), ("offer_always", 2, top, top - 1, top),
              ("offer_always", 3, top, top - 1, top), ("offer_always", 4, top, top, top - 1)]
    ref = replay_both("score", 2 * top, events)
    assert sorted(ref.entries) == [1, 4]


def test_bad_arguments_are_refused():
    import ctypes

    lib = reinc.load_library()
    h = ctypes.c_void_p()
    assert lib.reinc_policy_create(ctypes.byref(h), 9, 10) == -1
    assert lib.reinc_policy_create(ctypes.byref(h), 1, -1) == -1
    assert lib.reinc_policy_create(None, 1, 1) == -1
    store = reinc.PolicyStore("score", 4)
    with pytest.raises(reinc.ReincError):
        store.offer(1, 0, 1, 1)
    store.close()
