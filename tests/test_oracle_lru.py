"""Pins for the bucketed-LRU oracle: textbook page-replacement examples,
a set-level independent model, the closed form of the bounded timestamps, and
structural invariants."""
import numpy as np
import pytest

from oracle import lru

# The classic 20-reference string used in operating-systems textbooks to
# compare page-replacement policies with 3 frames: LRU takes 12 faults, the
# clairvoyant (Belady/OPT) policy 9.
REF = [7, 0, 1, 2, 0, 3, 0, 4, 2, 3, 0, 3, 2, 1, 2, 0, 1, 7, 0, 1]


def test_textbook_lru_and_opt_fault_counts():
    cache = lru.RowCache(3)
    faults = 0
    for step, p in enumerate(REF):
        _, misses, _ = lru.lru_step(cache, [p], step, 64)
        faults += len(misses)
        cache.check()
    assert faults == 12
    assert lru.belady_min_misses([[p] for p in REF], 3) == 9


def _model_step(last_access, pages, step, S):
    """Independent set-level model for step <= n-1 (timestamp == last access
    step): free room by dropping whole 'last accessed at step <= x' groups."""
    cur = set(pages)
    misses = [p for p in pages if p not in last_access]
    for p in pages:
        if p in last_access:
            last_access[p] = step
    free = S - len(last_access)
    net = max(0, len(misses) - free)
    if net > 0:
        others = sorted((t, p) for p, t in last_access.items() if p not in cur)
        x = others[net - 1][0]                      # time of the net-th oldest
        for t, p in others:
            if t <= x:
                del last_access[p]
    for p in misses:
        last_access[p] = step
    return len(misses)


@pytest.mark.parametrize("seed", range(5))
def test_resident_set_matches_independent_model(seed):
    rng = np.random.default_rng(seed)
    S, n, universe, k = 24, 64, 60, 6
    cache = lru.RowCache(S)
    model = {}
    hot = list(rng.choice(universe, size=12, replace=False))
    for step in range(50):
        pool = hot if rng.random() < 0.7 else list(range(universe))
        pages = sorted(set(int(x) for x in rng.choice(pool, size=k, replace=False)))
        slots, misses, hits = lru.lru_step(cache, pages, step, n)
        m = _model_step(model, pages, step, S)
        cache.check()
        assert len(misses) == m and hits == len(pages) - m
        assert set(cache.where) == set(model)
        assert all(cache.ts[cache.where[p]] == model[p] for p in model)
        # every selected page is resident, slots distinct and in range
        assert [cache.where[p] for p in pages] == slots
        assert len(set(slots)) == len(slots) and all(0 <= s < S for s in slots)
        assert [p for p, _ in misses] == sorted(p for p, _ in misses)


def test_bounded_timestamp_closed_form():
    """A page last accessed at step a has, at a later step s,
    ts = max(min(a, n-1) - max(0, s - max(a, n-1)), 0)."""
    n, S = 4, 64
    cache = lru.RowCache(S)
    last = {}
    rng = np.random.default_rng(0)
    for step in range(14):
        pages = sorted(set(int(x) for x in rng.choice(20, size=3, replace=False)))
        lru.lru_step(cache, pages, step, n)       # S is large: nothing is evicted
        for p in pages:
            last[p] = step
        for p, a in last.items():
            want = max(min(a, n - 1) - max(0, step - max(a, n - 1)), 0)
            assert cache.ts[cache.where[p]] == want, (p, a, step)


def test_admission_order_and_slot_reuse():
    cache = lru.RowCache(4)
    slots, misses, hits = lru.lru_step(cache, [10, 20, 30], 0, 64)
    assert slots == [0, 1, 2] and misses == [(10, 0), (20, 1), (30, 2)] and hits == 0
    slots, misses, hits = lru.lru_step(cache, [20, 40], 1, 64)
    assert slots == [1, 3] and misses == [(40, 3)] and hits == 1
    # full; need 2 slots: bucket ts=0 holds {10,30} -> both evicted, slots 0 and 2 reused in order
    slots, misses, hits = lru.lru_step(cache, [5, 20, 50], 2, 64)
    assert misses == [(5, 0), (50, 2)] and slots == [0, 1, 2] and hits == 1
    assert cache.page == [5, 20, 50, 40]


def test_whole_bucket_eviction_leaves_surplus_free_and_exact_mode_does_not():
    for exact, want_free in ((False, 2), (True, 0)):
        cache = lru.RowCache(4)
        lru.lru_step(cache, [1, 2, 3], 0, 64, evict_exact=exact)
        lru.lru_step(cache, [4], 1, 64, evict_exact=exact)
        # demand 1, no free slot: bucket 0 has three pages
        _, misses, _ = lru.lru_step(cache, [9], 2, 64, evict_exact=exact)
        assert misses == [(9, 0)]
        assert sum(1 for p in cache.page if p < 0) == want_free
        cache.check()


def test_exact_mode_never_misses_more_on_a_reuse_trace():
    rng = np.random.default_rng(5)
    tot = {}
    for exact in (False, True):
        cache = lru.RowCache(16)
        misses = 0
        r = np.random.default_rng(5)
        for step in range(60):
            pages = sorted(set(int(x) for x in r.choice(30, size=5, replace=False)))
            misses += len(lru.lru_step(cache, pages, step, 64, evict_exact=exact)[1])
        tot[exact] = misses
    assert tot[True] <= tot[False]


def test_selected_pages_are_never_evicted_and_budget_error():
    cache = lru.RowCache(3)
    lru.lru_step(cache, [1, 2, 3], 0, 64)
    slots, misses, hits = lru.lru_step(cache, [1, 2, 7], 1, 64)
    assert hits == 2 and misses == [(7, 2)]
    with pytest.raises(lru.BudgetExceeded):
        lru.lru_step(cache, [1, 2, 3, 4], 2, 64)


def test_belady_is_a_lower_bound_and_handles_batches():
    rng = np.random.default_rng(11)
    trace = [sorted(set(int(x) for x in rng.choice(25, size=4, replace=False))) for _ in range(40)]
    for exact in (False, True):
        cache = lru.RowCache(10)
        m = sum(len(lru.lru_step(cache, pg, s, 64, evict_exact=exact)[1]) for s, pg in enumerate(trace))
        assert lru.belady_min_misses(trace, 10) <= m
    # compulsory misses only when everything fits
    assert lru.belady_min_misses(trace, 25) == len({p for pg in trace for p in pg})


def test_reclaim_tail_evicts_only_tail_slots_and_growth_adds_empty_ones():
    cache = lru.RowCache(6)
    lru.lru_step(cache, [10, 11, 12, 13, 14], 0, 64)
    assert cache.page == [10, 11, 12, 13, 14, -1]
    lru.reclaim_tail(cache, 3)
    assert cache.page == [10, 11, 12] and set(cache.where) == {10, 11, 12}
    cache.check()
    slots, misses, hits = lru.lru_step(cache, [10, 13], 1, 64)        # 13 was evicted by the shrink
    assert hits == 1 and misses == [(13, 1)]          # bucket 0 held 11 and 12: both evicted, slot 2 left empty
    lru.reclaim_tail(cache, 5)
    assert cache.page[3:] == [-1, -1] and len(cache.ts) == 5
    slots, misses, _ = lru.lru_step(cache, [20, 21], 2, 64)
    assert [s for _, s in misses] == [2, 3]
    cache.check()
