"""Pins for the variable-length-partition oracle: it must coincide with the
fixed-size oracle on uniform layouts, and match hand-worked ragged cases."""
import numpy as np
import pytest

from oracle import index, resolve, select, varpart


@pytest.mark.parametrize("seq_len,tp,sinks,recents,topk,incl", [(2000, 64, 3, 6, 9, True), (131 * 16 + 5, 128, 4, 11, 6, False),
                                                                 (700, 16, 2, 3, 24, True), (129, 128, 4, 11, 6, False)])
def test_uniform_layout_reproduces_fixed_size_oracle(seq_len, tp, sinks, recents, topk, incl):
    rng = np.random.default_rng(seq_len)
    first, toks = varpart.uniform_layout(seq_len, 16, tp)
    P = len(first)
    scores = np.round(rng.standard_normal(P) * 3) / 3
    assert varpart.forced_pages(first, toks, 16, sinks, recents) == select.forced_pages(seq_len, 16, sinks, recents)
    assert varpart.forced_partitions(first, toks, 16, sinks, recents) == \
        select.forced_partitions(seq_len, 16, tp, sinks, recents)
    sel_v = varpart.select_topk(scores, first, toks, 16, topk, incl, sinks, recents)
    assert sel_v == select.select_topk(scores, seq_len, 16, tp, topk, incl, sinks, recents)
    pages = -(-seq_len // 16)
    page_map = {(7, p): 1000 - p for p in range(pages)}
    assert varpart.resolve_slots(sel_v, first, toks, 16, sinks, recents, page_map, 7) == \
        resolve.resolve_slots(sel_v, seq_len, 16, tp, sinks, recents, page_map, 7)
    K = rng.standard_normal((pages * 16, 5))
    a = varpart.minmax_summaries(K, first, toks, 16)
    b = index.minmax_summaries(K, seq_len, tp)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    # one mean key per partition: the fixed-size representatives with a single sub-range
    assert np.array_equal(varpart.centroids(K, first, toks, 16), index.block_representatives(K, seq_len, tp, 1))


def test_hand_worked_ragged_layout():
    # partitions of 20, 16, 5, 40 and 33 tokens -> 2, 1, 1, 3, 3 pages
    toks = [20, 16, 5, 40, 33]
    first = [0, 2, 3, 4, 7]
    assert varpart.row_pages(first, toks, 16) == 10
    assert varpart.page_masks(first, toks, 0, 16) == [0xFFFF, 0xF]
    assert varpart.page_masks(first, toks, 2, 16) == [0x1F]
    assert varpart.page_masks(first, toks, 4, 16) == [0xFFFF, 0xFFFF, 0x1]
    # 3 sink pages cover partitions 0 and 1 wholly; 2 recent pages cover part of partition 4
    assert varpart.forced_pages(first, toks, 16, 3, 2) == [0, 1, 2, 8, 9]
    assert varpart.forced_partitions(first, toks, 16, 3, 2) == [0, 1]
    scores = np.array([9.0, 9.0, 1.0, 5.0, 0.0])
    sel = varpart.select_topk(scores, first, toks, 16, 3, True, 3, 2)        # 2 forced + the best candidate
    assert sel == [0, 1, 3]
    page_map = {(0, p): 50 + p for p in range(10)}
    pg, sl, mk = varpart.resolve_slots(sel, first, toks, 16, 3, 2, page_map, 0)
    assert pg == [0, 1, 2, 4, 5, 6, 8, 9]                                    # pages 8, 9 stand alone
    assert sl == [50, 51, 52, 54, 55, 56, 58, 59]
    assert mk == [0xFFFF, 0xF, 0xFFFF, 0xFFFF, 0xFFFF, 0xFF, 0xFFFF, 0x1]
    # brute-force min/max
    K = np.arange(160 * 2, dtype=np.float64).reshape(160, 2) * np.array([1.0, -1.0])
    mins, maxs = varpart.minmax_summaries(K, first, toks, 16)
    assert mins[2].tolist() == [96.0, -105.0] and maxs[2].tolist() == [104.0, -97.0]
    assert maxs[3][0] == (64 + 39) * 2 and mins[4][0] == 112 * 2


def test_centroids_by_hand():
    """The centroid is the arithmetic mean of the partition's own tokens (not of its pages'
    padding), stored with one bf16 rounding."""
    toks = [20, 16, 5, 40, 33]
    first = [0, 2, 3, 4, 7]
    K = np.arange(160 * 2, dtype=np.float64).reshape(160, 2) * np.array([1.0, -1.0])
    c = varpart.centroids(K, first, toks, 16)
    assert c.shape == (5, 1, 2)
    # partition 0: tokens 0..19, channel 0 holds 0, 2, .., 38 -> mean 19; channel 1 holds -1, -3, .., -39 -> -20
    assert c[0, 0].tolist() == [19.0, -20.0]
    # partition 2: 5 tokens from page 3 (token 48): 96..104 step 2 -> 100; -97..-105 -> -101
    assert c[2, 0].tolist() == [100.0, -101.0]
    # partition 4: 33 tokens from token 112: mean of 224..288 step 2 = 256; bf16 keeps it
    assert c[4, 0, 0] == 256.0
    # constant keys: the centroid is that key, whatever the partition sizes
    Kc = np.tile(np.array([[0.5, -3.0, 7.0]]), (160, 1))
    assert np.array_equal(varpart.centroids(Kc, first, toks, 16), np.tile(Kc[0], (5, 1, 1)))
    # one rounding to bf16 (8 significant bits): mean 1 + 2^-9 of two tokens rounds to 1
    Kr = np.zeros((160, 1))
    Kr[32] = 1.0
    Kr[33] = 1.0 + 2.0 ** -8
    assert varpart.centroids(Kr, [0, 2], [32, 2], 16)[1, 0, 0] == 1.0
