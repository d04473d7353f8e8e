"""Pins for the checker's computation-loading pipeline schedule (Sec. 4.2.2) and for the
replacement models of App. A when some tables are pinned.  Hand-worked cases, and properties any
correct schedule has."""
import numpy as np
import pytest

import oracle

MODELS = [oracle.LRUModel, oracle.FIFOModel, oracle.LFUModel]


def _warm(model, accesses):
    for t in accesses:
        model.access(t)
    return model


def test_lfu_without_pins_drops_the_table_it_has_just_inserted():
    # cache of 2 holding X (3 uses) and Y (2 uses); a query needs A and B, both new
    m = _warm(oracle.LFUModel(2), ["X", "X", "X", "Y", "Y"])
    assert m.access("A") == (False, "Y")            # Y has the smallest frequency
    assert m.access("B") == (False, "A")            # now A (frequency 1) has: the query lost A
    # the same with the query's tables pinned: B takes X's place, A and B are both cached
    m = _warm(oracle.LFUModel(2), ["X", "X", "X", "Y", "Y"])
    assert m.access("A", pinned={"A", "B"}) == (False, "Y")
    assert m.access("B", pinned={"A", "B"}) == (False, "X")
    assert set(m.items) == {"A", "B"}


def test_fifo_with_pins_skips_the_pinned_head():
    m = _warm(oracle.FIFOModel(3), [1, 2, 3])       # queue 1 2 3, head 1
    assert m.access(1, pinned={1, 4}) == (True, None)
    assert m.access(4, pinned={1, 4}) == (False, 2)     # head 1 is pinned: 2 goes
    assert m.items == [1, 3, 4]
    assert m.access(5) == (False, 1)                # nothing pinned: plain FIFO again


def test_lru_with_pins_takes_the_least_recent_unpinned():
    m = _warm(oracle.LRUModel(3), [1, 2, 3])        # front 3 2 1
    assert m.access(4, pinned={1}) == (False, 2)
    assert m.items == [4, 3, 1]


@pytest.mark.parametrize("cls", MODELS)
def test_everything_pinned_is_an_error(cls):
    m = _warm(cls(2), [1, 2])
    with pytest.raises((IndexError, ValueError)):
        m.access(3, pinned={1, 2, 3})


def test_plan_hand_worked():
    sets = [[0, 1], [1, 2], [3], [0, 3], [4, 5]]
    # C=4, b_c=2, b_m=2.  step 0 computes 0,1 (tables 0 1 2, asked for on demand); once stitched
    # they are released and requests 2,3 (tables 3 0) are prefetched.  step 1 computes 2,3, nothing
    # left to ask for; prefetches request 4.  step 2 computes 4.
    assert oracle.plan_pipeline(sets, 4, 2, 2) == [(0, 2, 0, 2, 2, 4), (2, 4, 4, 4, 4, 5), (4, 5, 5, 5, 5, 5)]
    # no overlap: every micro-batch is asked for on demand
    assert oracle.plan_pipeline(sets, 4, 2, 0) == [(0, 2, 0, 2, 2, 2), (2, 4, 2, 4, 4, 4), (4, 5, 4, 5, 5, 5)]
    # C=3, b_m=3: after step 0, requests 2,3 hold tables {3, 0}; request 4 would make 4 tables: stop
    assert oracle.plan_pipeline(sets, 3, 2, 3) == [(0, 2, 0, 2, 2, 4), (2, 4, 4, 4, 4, 5), (4, 5, 5, 5, 5, 5)]
    # b_m smaller than b_c: the second half of each micro-batch is asked for on demand
    assert oracle.plan_pipeline(sets, 4, 2, 1) == [(0, 2, 0, 2, 2, 3), (2, 4, 3, 4, 4, 5), (4, 5, 5, 5, 5, 5)]
    # C=2: requests 0,1 need three tables at once, so the first micro-batch is request 0 alone and
    # only request 1 can be prefetched behind it ({1 2}; request 2 would add table 3).  Request 1 is
    # then computed alone too (with request 2 it would need 1 2 3); behind it requests 2,3 (tables
    # 3 0) are prefetched and computed together; request 4 (4 5) follows.
    assert oracle.plan_pipeline(sets, 2, 2, 2) == [(0, 1, 0, 1, 1, 2), (1, 2, 2, 2, 2, 4), (2, 4, 4, 4, 4, 5),
                                                   (4, 5, 5, 5, 5, 5)]
    # C=3, b_c=3: requests 0,1 fit (0 1 2), request 2 (table 3) does not: cut short, and the prefetch
    # of up to three requests stops after 2,3 (tables 3 0; request 4 would add two more)
    assert oracle.plan_pipeline(sets, 3, 3, 3) == [(0, 2, 0, 2, 2, 4), (2, 4, 4, 4, 4, 5), (4, 5, 5, 5, 5, 5)]
    with pytest.raises(ValueError):
        oracle.plan_pipeline(sets, 1, 2, 2)             # request 0 alone needs two tables
    assert oracle.plan_pipeline([], 4, 2, 2) == []


def _random_sets(rng, n, n_tables, kmax):
    return [rng.choice(n_tables, size=int(rng.integers(1, kmax + 1)), replace=False).tolist() for _ in range(n)]


def test_plan_properties():
    rng = np.random.default_rng(5)
    n_cut = 0
    for trial in range(300):
        n = int(rng.integers(1, 40))
        sets = _random_sets(rng, n, 12, 4)
        b_c, b_m = int(rng.integers(1, 6)), int(rng.integers(0, 9))
        C = int(rng.integers(4, 14))
        steps = oracle.plan_pipeline(sets, C, b_c, b_m)
        asked, nxt = 0, 0
        uni = lambda a, b: set().union(*map(set, sets[a:b])) if b > a else set()
        for c0, c1, d0, d1, p0, p1 in steps:
            assert c0 == nxt and c0 < c1 <= min(n, c0 + b_c)   # in order, without gaps, at most b_c
            assert len(uni(c0, c1)) <= C                       # the micro-batch fits the cache
            if c1 < min(n, c0 + b_c):                          # cut short only for lack of room
                assert len(uni(c0, c1 + 1)) > C
                n_cut += 1
            assert d0 == asked and d1 == max(asked, c1) and p0 == d1 and p1 >= p0
            assert p1 <= max(c1 + b_m, p0)                     # never further ahead than b_m requests
            assert len(uni(c1, p1)) <= C                       # what stays pinned fits the cache
            if p1 < n and p1 < c1 + b_m:                       # stopped early only for lack of room
                assert len(uni(c1, p1 + 1)) > C
            asked, nxt = p1, c1
        assert nxt == n
    assert n_cut > 20


@pytest.mark.parametrize("cls", MODELS)
def test_simulated_pipeline_keeps_each_micro_batch_cached(cls):
    """The reason for the pins: when a micro-batch is stitched, all its tables are in the cache,
    under every rule, for any schedule."""
    rng = np.random.default_rng(9)
    for trial in range(60):
        n = int(rng.integers(1, 30))
        sets = _random_sets(rng, n, 10, 3)
        b_c, b_m = int(rng.integers(1, 4)), int(rng.integers(0, 7))
        C = int(rng.integers(3, 11))
        steps = oracle.plan_pipeline(sets, C, b_c, b_m)
        for k, (c0, c1, d0, d1, p0, p1) in enumerate(steps):
            # the schedule up to step k's demand loads, with its stitch and prefetch cut off
            part = list(steps[:k]) + [(c0, c0, d0, d1, d1, d1)]
            m = cls(C)
            oracle.simulate_pipeline(m, sets, part)
            need = set().union(*map(set, sets[c0:c1]))
            assert need <= set(m.items), (cls.__name__, trial, k)


@pytest.mark.parametrize("cls", MODELS)
def test_simulated_trace_visits_the_requests_in_order(cls):
    # a cache that holds every table never evicts, so the pins cannot matter and the trace is the
    # plain replay of the requests' tables in batch order, whatever b_c and b_m
    rng = np.random.default_rng(2)
    sets = _random_sets(rng, 25, 10, 3)
    flat = [t for q in sets for t in q]
    for b_c, b_m in ((1, 0), (2, 2), (3, 7), (4, 1)):
        steps = oracle.plan_pipeline(sets, 10, b_c, b_m)
        assert oracle.simulate_pipeline(cls(10), sets, steps) == oracle.replay(cls(10), flat)


def test_plan_with_the_computing_batch_kept_pinned():
    sets = [[0, 1], [1, 2], [3], [4], [5]]
    # C=4, b_c=2, b_m=2: while requests 0,1 (tables 0 1 2) are computed they stay pinned, so only
    # request 2 (table 3) can be prefetched; request 3 is then asked for on demand
    assert oracle.plan_pipeline(sets, 4, 2, 2, keep_pinned=True) == [(0, 2, 0, 2, 2, 3), (2, 4, 3, 4, 4, 5),
                                                                   (4, 5, 5, 5, 5, 5)]
    # without, the cache has room for requests 2 and 3 behind the stitch of 0 and 1
    assert oracle.plan_pipeline(sets, 4, 2, 2) == [(0, 2, 0, 2, 2, 4), (2, 4, 4, 4, 4, 5), (4, 5, 5, 5, 5, 5)]
    rng = np.random.default_rng(8)
    for trial in range(100):
        n = int(rng.integers(1, 30))
        s = _random_sets(rng, n, 10, 3)
        b_c, b_m, C = int(rng.integers(1, 4)), int(rng.integers(0, 6)), int(rng.integers(3, 11))
        steps = oracle.plan_pipeline(s, C, b_c, b_m, keep_pinned=True)
        uni = lambda a, b: set().union(*map(set, s[a:b])) if b > a else set()
        for c0, c1, d0, d1, p0, p1 in steps:
            assert len(uni(c0, p1)) <= C                       # computing batch and prefetch window together
            if p1 < n and p1 < c1 + b_m:
                assert len(uni(c0, p1 + 1)) > C
        for cls in MODELS:                                     # and the cache then really holds them all
            m = cls(C)
            oracle.simulate_pipeline(m, s, steps, keep_pinned=True)


def test_plan_with_tapering_tail():
    sets = [[i] for i in range(20)]
    # 20 requests, b_c = 8: 8, then half of what remains each time (12 -> 6, 6 -> 3, 3 -> 1), then singles
    steps = oracle.plan_pipeline(sets, 40, 8, 8, taper=True)
    assert [(s[0], s[1]) for s in steps] == [(0, 8), (8, 14), (14, 17), (17, 18), (18, 19), (19, 20)]
    # the copies stay b_m requests ahead of the computation, whatever the size of its micro-batches
    assert [(s[4], s[5]) for s in steps] == [(8, 16), (16, 20), (20, 20), (20, 20), (20, 20), (20, 20)]
    assert steps[0][2:4] == (0, 8) and all(s[2] == s[3] for s in steps[1:])       # nothing else on demand
    # a batch no longer than b_c still ends on a single request
    assert [(s[0], s[1]) for s in oracle.plan_pipeline(sets[:5], 40, 8, 8, taper=True)] == [(0, 2), (2, 3), (3, 4), (4, 5)]
