"""Pins for top-k selection: full sort on tiny inputs, tie rules, forced pages."""
import math

import numpy as np
import pytest

from oracle import select


def _brute(scores, P, forced, kprime):
    """Independent statement: repeatedly take the best remaining candidate,
    lowest index first among equals."""
    chosen = set(forced)
    cands = [i for i in range(P) if i not in chosen]
    taken = []
    for _ in range(min(kprime, len(cands))):
        best = None
        for i in cands:
            if i in taken:
                continue
            si = -math.inf if scores[i] != scores[i] else scores[i]
            if best is None:
                best = i
                continue
            sb = -math.inf if scores[best] != scores[best] else scores[best]
            if si > sb:
                best = i
        taken.append(best)
    return sorted(chosen | set(taken))


@pytest.mark.parametrize("seed", range(6))
def test_matches_repeated_argmax_with_many_ties(seed):
    rng = np.random.default_rng(seed)
    P = 40
    scores = rng.integers(-3, 4, size=P).astype(np.float64)      # heavy duplication
    got = select.select_topk(scores, P * 16, 16, 16, 12, True, 2, 3)
    forced = [0, 1, 37, 38, 39]
    assert got == _brute(scores, P, forced, 12 - 5)
    assert len(got) == 12 and got == sorted(got)


def test_all_equal_takes_lowest_indices():
    got = select.select_topk(np.zeros(20), 20 * 16, 16, 16, 5, True, 0, 0)
    assert got == [0, 1, 2, 3, 4]


def test_boundary_duplicates_take_lowest_index():
    s = np.array([5.0, 1.0, 3.0, 3.0, 3.0, 0.0, 3.0])
    assert select.select_topk(s, 7 * 16, 16, 16, 3, True, 0, 0) == [0, 2, 3]


def test_signed_zero_ties_and_neg_inf_and_nan():
    s = np.array([-0.0, 0.0, -math.inf, math.nan, -1.0])
    assert select.select_topk(s, 5 * 16, 16, 16, 1, True, 0, 0) == [0]
    assert select.select_topk(s, 5 * 16, 16, 16, 2, True, 0, 0) == [0, 1]
    assert select.select_topk(s, 5 * 16, 16, 16, 4, True, 0, 0) == [0, 1, 2, 4]
    assert select.select_topk(s, 5 * 16, 16, 16, 5, True, 0, 0) == [0, 1, 2, 3, 4]


def test_k_zero_and_k_larger_than_candidates():
    s = np.arange(6, dtype=np.float64)
    assert select.select_topk(s, 96, 16, 16, 0, True, 0, 0) == []
    assert select.select_topk(s, 96, 16, 16, 100, True, 1, 1) == [0, 1, 2, 3, 4, 5]
    # forced pages exceed the budget: forced still all present, no candidates
    assert select.select_topk(s, 96, 16, 16, 2, True, 2, 2) == [0, 1, 4, 5]
    assert select.select_topk(s, 0, 16, 16, 4, True, 1, 1) == []


def test_forced_pages_present_and_not_counted_twice():
    rng = np.random.default_rng(3)
    s = rng.standard_normal(2048)
    got = select.select_topk(s, 32768, 16, 16, 128, True, 4, 8)
    assert len(got) == 128
    assert set(range(4)) <= set(got) and set(range(2040, 2048)) <= set(got)
    rest = [p for p in got if 4 <= p < 2040]
    order = np.argsort(-s[4:2040], kind="stable")[:116] + 4
    assert sorted(order.tolist()) == rest


def test_overlapping_sink_and_recent_windows():
    s = np.zeros(3)
    assert select.forced_pages(40, 16, 2, 2) == [0, 1, 2]
    assert select.select_topk(s, 40, 16, 16, 3, True, 2, 2) == [0, 1, 2]


def test_ragged_context_last_page_is_recent():
    # 100 tokens -> 7 pages, last page holds 4 tokens
    assert select.forced_pages(100, 16, 1, 1) == [0, 6]
    s = np.array([0, 5, 1, 9, 2, 8, 0], dtype=np.float64)
    assert select.select_topk(s, 100, 16, 16, 4, True, 1, 1) == [0, 3, 5, 6]


def test_block_partitions_partial_cover_stays_candidate_and_budget_excludes_forced():
    # 128-token blocks = 8 pages; 4 sink pages cover half of block 0 -> candidate;
    # 64 recent pages cover the last 8 blocks entirely -> forced, not candidates.
    P = 32
    seq = P * 128
    assert select.forced_partitions(seq, 16, 128, 4, 64) == list(range(24, 32))
    s = np.zeros(P)
    s[0] = 10.0
    s[30] = 99.0                      # forced: its score must not consume budget
    s[5] = 7.0
    got = select.select_topk(s, seq, 16, 128, 2, False, 4, 64)
    assert got == [0, 5] + list(range(24, 32))
    # ragged: context ends inside a block; window covers block 31 wholly and
    # part of earlier ones
    seq2 = 31 * 128 + 40              # block 31 holds 40 tokens (3 pages)
    fp = select.forced_pages(seq2, 16, 0, 5)
    assert fp == [246, 247, 248, 249, 250]
    assert select.forced_partitions(seq2, 16, 128, 0, 5) == [31]


def test_token_partitions_forced_pages_force_their_tokens():
    seq = 70                           # 5 pages, last has 6 tokens
    f = select.forced_partitions(seq, 16, 1, 1, 1)
    assert f == list(range(16)) + list(range(64, 70))
    s = np.zeros(seq)
    s[40] = 3.0
    s[20] = 3.0
    s[21] = 2.0
    got = select.select_topk(s, seq, 16, 1, 24, True, 1, 1)
    assert got == sorted(f + [20, 40])


def test_pinned_partitions_always_participate():
    """Pinned (outlier) partitions are taken before every other candidate: an
    independent statement of the rule -- pinned candidates first, ascending id, then
    the best of the rest -- must agree with selecting on the pinned scores."""
    rng = np.random.default_rng(11)
    seq_len, tp, k = 16 * 60, 16, 12
    for trial in range(20):
        scores = np.round(rng.standard_normal(60) * 4) / 4
        pinned = sorted(set(int(x) for x in rng.integers(-3, 66, size=int(rng.integers(0, 9)))))
        sinks, recents = int(rng.integers(0, 3)), int(rng.integers(0, 4))
        got = select.select_topk(select.pin_scores(scores, seq_len, tp, pinned), seq_len, 16, tp, k, True, sinks, recents)
        forced = select.forced_partitions(seq_len, 16, tp, sinks, recents)
        kprime = max(k - len(forced), 0)
        pin_c = [p for p in pinned if 0 <= p < 60 and p not in forced][:kprime]
        rest = [p for p in range(60) if p not in forced and p not in pin_c]
        rest.sort(key=lambda p: (-scores[p], p))
        want = sorted(set(forced) | set(pin_c) | set(rest[:kprime - len(pin_c)]))
        assert got == want, trial
    # the input is left alone and out-of-row ids are ignored
    s = np.zeros(4)
    out = select.pin_scores(s, 64, 16, [1, 9, -1])
    assert s.tolist() == [0, 0, 0, 0] and out.tolist() == [0.0, math.inf, 0.0, 0.0]
