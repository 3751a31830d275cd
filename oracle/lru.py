"""Retrieve under an HBM budget: bucketed-LRU replacement (test infrastructure).

Step-by-step transcription of the four replacement steps of Section 5.3
("Bucketed LRU Replacement") for ONE row (one request, one KV head) that owns
``S`` HBM page slots:

1. classify the step's selected pages into hits and misses; the page demand is
   the number of missed pages;
2. timestamps live in [0, n-1]; selected pages take min(step, n-1); once
   step > n-1 every other resident page is demoted by one (not below 0);
3. histogram the evictable (resident, not selected) pages by timestamp, walk
   the buckets from oldest to newest to the smallest threshold x whose
   cumulative count covers the demand not already covered by empty slots, and
   evict the pages with timestamp <= x;
4. admit the misses into free slots and record the slot of every selected page.

Readings fixed where the paper is silent: steps are 0-based; selected pages are
never evicted; the whole bucket x is evicted (``evict_exact`` instead evicts
from bucket x only as many pages as still needed, lowest slot first); misses in
ascending page id take free slots in ascending slot index.
"""
from typing import Dict, List, Tuple


class BudgetExceeded(Exception):
    """The row's slot budget cannot hold the step's selected pages."""


class RowCache:
    """HBM slot table of one row: per slot the resident page (-1 = empty) and
    its timestamp; ``where`` is the forward map page -> slot."""

    def __init__(self, num_slots: int):
        self.page: List[int] = [-1] * num_slots
        self.ts: List[int] = [0] * num_slots
        self.where: Dict[int, int] = {}

    def check(self):
        seen = {}
        for s, p in enumerate(self.page):
            if p >= 0:
                assert p not in seen, "page resident twice"
                seen[p] = s
        assert seen == self.where, "forward and reverse tables disagree"


def reclaim_tail(cache: RowCache, keep: int) -> None:
    """Shrink (or grow) the row's budget to ``keep`` slots.  Buffer pages are
    reclaimed from the tail of the slot table (Section 5.3, buffer elasticity):
    pages resident in slots >= keep are evicted; growing appends empty slots."""
    S = len(cache.page)
    for s in range(keep, S):
        p = cache.page[s]
        if p >= 0:
            del cache.where[p]
    if keep <= S:
        del cache.page[keep:]
        del cache.ts[keep:]
    else:
        cache.page.extend([-1] * (keep - S))
        cache.ts.extend([0] * (keep - S))


def lru_step(cache: RowCache, pages: List[int], step: int, n: int,
             evict_exact: bool = False) -> Tuple[List[int], List[Tuple[int, int]], int]:
    """Apply one decode step.  ``pages`` = the selected logical pages, ascending.

    Returns ``(slots, misses, hits)``: the slot of every selected page in the
    order of ``pages``, the miss list ``[(page, slot)]`` ascending by page, and
    the hit count.  Mutates ``cache``."""
    S = len(cache.page)
    selected = set(pages)
    assert len(selected) == len(pages)
    if len(pages) > S:
        raise BudgetExceeded((len(pages), S))

    # 1. hit / miss classification
    misses = [p for p in pages if p not in cache.where]
    hits = len(pages) - len(misses)
    demand = len(misses)

    # 2. timestamp update
    ts_star = min(step, n - 1)
    for s in range(S):
        p = cache.page[s]
        if p < 0:
            continue
        if p in selected:
            cache.ts[s] = ts_star
        elif step > n - 1:
            cache.ts[s] = max(cache.ts[s] - 1, 0)

    # 3. eviction
    free = sum(1 for p in cache.page if p < 0)
    net = max(0, demand - free)
    if net > 0:
        hist = [0] * n
        for s in range(S):
            p = cache.page[s]
            if p >= 0 and p not in selected:
                hist[cache.ts[s]] += 1
        cum, x = 0, None
        for t in range(n):
            if cum + hist[t] >= net:
                x = t
                break
            cum += hist[t]
        if x is None:
            raise BudgetExceeded((len(pages), S))
        need_from_x = net - cum                       # only used by evict_exact
        for s in range(S):
            p = cache.page[s]
            if p < 0 or p in selected:
                continue
            t = cache.ts[s]
            evict = t <= x
            if evict_exact and t == x:
                evict = need_from_x > 0
                need_from_x -= 1 if evict else 0
            if evict:
                del cache.where[p]
                cache.page[s] = -1
                cache.ts[s] = 0

    # 4. admission
    free_slots = [s for s in range(S) if cache.page[s] < 0]
    miss_list = []
    for p, s in zip(misses, free_slots):
        cache.page[s] = p
        cache.ts[s] = ts_star
        cache.where[p] = s
        miss_list.append((p, s))
    assert len(miss_list) == demand
    slots = [cache.where[p] for p in pages]
    return slots, miss_list, hits


def belady_min_misses(trace: List[List[int]], num_slots: int) -> int:
    """Misses of the clairvoyant policy on a trace of per-step page sets (the
    paper's ideal envelope uses it to bound the miss ratio, Section 3.1).  A
    step's pages are all needed at once, so they are pinned during the step;
    on a miss with no empty slot the resident page whose next use is farthest
    away is evicted."""
    next_use = []
    last = {}
    for i in range(len(trace) - 1, -1, -1):
        nu = {}
        for p in trace[i]:
            nu[p] = last.get(p, float("inf"))
            last[p] = i
        next_use.append(nu)
    next_use.reverse()
    resident: Dict[int, float] = {}
    misses = 0
    for i, pages in enumerate(trace):
        cur = set(pages)
        for p in pages:
            if p in resident:
                resident[p] = next_use[i][p]
        for p in pages:
            if p in resident:
                continue
            misses += 1
            if len(resident) >= num_slots:
                victims = [r for r in resident if r not in cur]
                if not victims:
                    raise BudgetExceeded((len(cur), num_slots))
                far = max(victims, key=lambda r: (resident[r], r))
                del resident[far]
            resident[p] = next_use[i][p]
    return misses


# ---------------------------------------------------------------------------
# Second policy: set-associative placement (the "8-way buckets hashed on
# (request, page)" of the budget workload's description; the paper's own policy
# is lru_step above, Section 5.3).  Conventions of this build, stated in full:
# the row's S slots form S // ways sets of `ways` consecutive slots; a page's
# home set is mix32(row, page) mod sets; lookups go through the forward table,
# only placement is constrained.  Misses are handled one at a time in ascending
# page id: starting at the home set, skip (circularly) every set whose ways all
# hold pages selected in this step; in the first other set take the lowest empty
# way, else evict the non-selected way with the smallest timestamp (lowest way
# on ties).  Timestamps follow step 2 of the bucketed policy.
# ---------------------------------------------------------------------------
def mix32(row: int, page: int) -> int:
    """32-bit finaliser (xor-shift / multiply rounds of the MurmurHash3
    finaliser) of row * 0x9E3779B1 + page."""
    x = (row * 0x9E3779B1 + page) & 0xFFFFFFFF
    x ^= x >> 16
    x = (x * 0x85EBCA6B) & 0xFFFFFFFF
    x ^= x >> 13
    x = (x * 0xC2B2AE35) & 0xFFFFFFFF
    x ^= x >> 16
    return x


def setassoc_step(cache: RowCache, pages: List[int], step: int, n: int, row: int,
                  ways: int = 8) -> Tuple[List[int], List[Tuple[int, int]], int]:
    """One decode step of the set-associative policy; same interface as
    ``lru_step`` (slots beyond ``(S // ways) * ways`` are never used)."""
    S = len(cache.page)
    sets = S // ways
    selected = set(pages)
    assert len(selected) == len(pages)
    if sets < 1 or len(pages) > sets * ways:
        raise BudgetExceeded((len(pages), S))

    misses = [p for p in pages if p not in cache.where]
    hits = len(pages) - len(misses)

    ts_star = min(step, n - 1)
    for s in range(S):
        p = cache.page[s]
        if p < 0:
            continue
        if p in selected:
            cache.ts[s] = ts_star
        elif step > n - 1:
            cache.ts[s] = max(cache.ts[s] - 1, 0)

    miss_list = []
    for p in misses:
        st = mix32(row, p) % sets
        for _ in range(sets):
            base = st * ways
            if any(cache.page[base + w] not in selected for w in range(ways)):
                break
            st = (st + 1) % sets
        else:
            raise BudgetExceeded((len(pages), S))
        base = st * ways
        victim = None
        for w in range(ways):                          # lowest empty way
            if cache.page[base + w] < 0:
                victim = base + w
                break
        if victim is None:                             # oldest non-selected way, lowest way on ties
            best = None
            for w in range(ways):
                q = cache.page[base + w]
                if q in selected:
                    continue
                if best is None or cache.ts[base + w] < best:
                    best, victim = cache.ts[base + w], base + w
            del cache.where[cache.page[victim]]
        cache.page[victim] = p
        cache.ts[victim] = ts_star
        cache.where[p] = victim
        miss_list.append((p, victim))
    slots = [cache.where[p] for p in pages]
    return slots, miss_list, hits
