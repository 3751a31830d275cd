"""Pins for the set-associative variant of the replacement oracle: the textbook
LRU example (one set), agreement with the bucketed oracle's exact mode when one
set spans all slots, an independent per-set model, structural invariants of the
placement, and statistical checks of the set hash."""
import numpy as np
import pytest

from oracle import lru

REF = [7, 0, 1, 2, 0, 3, 0, 4, 2, 3, 0, 3, 2, 1, 2, 0, 1, 7, 0, 1]


def test_one_set_is_textbook_lru():
    # a single set of 3 ways is a 3-frame LRU: 12 faults on the classic string
    cache = lru.RowCache(3)
    faults = 0
    for step, p in enumerate(REF):
        _, misses, _ = lru.setassoc_step(cache, [p], step, 64, row=5, ways=3)
        faults += len(misses)
        cache.check()
    assert faults == 12


@pytest.mark.parametrize("seed", range(4))
def test_one_set_over_all_slots_keeps_the_same_pages_as_the_exact_bucketed_policy(seed):
    # with one set as wide as the budget both policies evict the oldest pages.
    # Pages are requested in fixed groups of 4 and the budget is a multiple of 4,
    # so a step either hits a whole group or replaces one whole oldest group and
    # no choice among equal timestamps arises: same misses, same resident pages
    # (slot assignment differs: one ranks freed slots, the other fills victims)
    rng = np.random.default_rng(100 + seed)
    S, n, groups, g = 16, 64, 9, 4
    a, b = lru.RowCache(S), lru.RowCache(S)
    total = 0
    for step in range(60):
        grp = int(rng.integers(groups))
        pages = [grp * g + i for i in range(g)]
        _, ma, ha = lru.lru_step(a, pages, step, n, evict_exact=True)
        _, mb, hb = lru.setassoc_step(b, pages, step, n, row=0, ways=S)
        assert [p for p, _ in ma] == [p for p, _ in mb] and ha == hb
        assert set(a.where) == set(b.where)
        assert {p: a.ts[s] for p, s in a.where.items()} == {p: b.ts[s] for p, s in b.where.items()}
        total += len(ma)
    assert total > 5 * g                             # replacement happened, not only cold misses


class _SetModel:
    """Independent model for step <= n-1 (timestamp == last access step): per
    set a dict way -> (page, last access)."""

    def __init__(self, sets, ways, row):
        self.sets, self.ways, self.row = sets, ways, row
        self.tab = [dict() for _ in range(sets)]

    def resident(self):
        return {p for t in self.tab for (p, _) in t.values()}

    def step(self, pages, step):
        cur = set(pages)
        res = self.resident()
        for t in self.tab:
            for w, (p, _) in list(t.items()):
                if p in cur:
                    t[w] = (p, step)
        placed = []
        for p in pages:
            if p in res:
                continue
            s = lru.mix32(self.row, p) % self.sets
            hops = 0
            while len(self.tab[s]) == self.ways and all(q in cur for (q, _) in self.tab[s].values()):
                s = (s + 1) % self.sets
                hops += 1
                assert hops < self.sets
            t = self.tab[s]
            empty = [w for w in range(self.ways) if w not in t]
            if empty:
                w = empty[0]
            else:
                w = min((la, w) for w, (q, la) in t.items() if q not in cur)[1]
            t[w] = (p, step)
            placed.append((p, s * self.ways + w, hops))
        return placed


@pytest.mark.parametrize("seed,sets,k", [(0, 4, 6), (1, 3, 20), (2, 8, 20), (3, 2, 14)])
def test_matches_independent_set_model_with_overflow(seed, sets, k):
    rng = np.random.default_rng(seed)
    ways, n, universe, row = 8, 64, 20 * sets, 3 + seed
    cache = lru.RowCache(sets * ways + 3)            # 3 slots past the last whole set stay unused
    model = _SetModel(sets, ways, row)
    hot = list(rng.choice(universe, size=2 * k, replace=False))
    overflowed = 0
    for step in range(60):
        pool = hot if rng.random() < 0.6 else list(range(universe))
        pages = sorted(int(x) for x in rng.choice(pool, size=k, replace=False))
        slots, misses, hits = lru.setassoc_step(cache, pages, step, n, row)
        placed = model.step(pages, step)
        cache.check()
        assert misses == [(p, s) for p, s, _ in placed]
        assert hits + len(misses) == len(pages)
        assert set(cache.where) == model.resident()
        assert all(cache.where[p] == s for p, s in zip(pages, slots))
        assert all(p < 0 for p in cache.page[sets * ways:])
        overflowed += sum(1 for _, _, hops in placed if hops)
    if 5 * k >= 4 * sets * ways:
        assert overflowed > 0                        # the probing path is exercised


def test_selected_pages_survive_and_budget_errors():
    cache = lru.RowCache(16)
    pages = list(range(16))
    lru.setassoc_step(cache, pages, 0, 64, row=1)    # fills both sets whatever the hash says
    assert sorted(cache.where) == pages
    slots, misses, hits = lru.setassoc_step(cache, pages, 1, 64, row=1)
    assert hits == 16 and not misses
    with pytest.raises(lru.BudgetExceeded):
        lru.setassoc_step(cache, list(range(17)), 2, 64, row=1)
    with pytest.raises(lru.BudgetExceeded):
        lru.setassoc_step(lru.RowCache(7), [0], 0, 64, row=1)      # fewer slots than one set


def test_timestamp_floor_after_wraparound():
    # n = 4: from step 4 on, pages not selected lose one per step down to 0
    cache = lru.RowCache(8)
    lru.setassoc_step(cache, [1, 2], 0, 4, row=0)
    for step in range(1, 9):
        lru.setassoc_step(cache, [2], step, 4, row=0)
    assert cache.ts[cache.where[2]] == 3
    # page 1: timestamp 0 from step 0, stays at the floor
    assert cache.ts[cache.where[1]] == 0
    lru.setassoc_step(cache, [1, 2], 9, 4, row=0)
    lru.setassoc_step(cache, [2], 10, 4, row=0)
    lru.setassoc_step(cache, [2], 11, 4, row=0)
    assert cache.ts[cache.where[1]] == 1


def test_mix32_is_injective_per_row_and_spreads_pages_over_sets():
    pages = np.arange(1 << 16)
    h = np.array([lru.mix32(7, int(p)) for p in pages], dtype=np.uint64)
    assert len(np.unique(h)) == len(pages)           # every round of the finaliser is a bijection of 32-bit words
    for sets in (32, 61, 512):
        counts = np.bincount((h % sets).astype(np.int64), minlength=sets)
        expect = len(pages) / sets
        chi2 = float(((counts - expect) ** 2 / expect).sum())
        assert chi2 < sets + 6 * np.sqrt(2 * sets)   # within 6 sigma of a uniform spread
    # different rows send the same page to unrelated sets
    a = np.array([lru.mix32(0, int(p)) % 64 for p in range(4096)])
    b = np.array([lru.mix32(1, int(p)) % 64 for p in range(4096)])
    assert 0.005 < np.mean(a == b) < 0.03
