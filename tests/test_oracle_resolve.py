"""Pins for partition -> page -> slot resolution."""
import numpy as np
import pytest

from oracle import resolve
from paper_2604_26837_amd import synth


def test_page_token_mask():
    assert resolve.page_token_mask(0, 100, 16) == 0xFFFF
    assert resolve.page_token_mask(6, 100, 16) == 0b1111
    assert resolve.page_token_mask(7, 100, 16) == 0
    assert resolve.page_token_mask(5, 96, 16) == 0xFFFF


def test_page_partitions_dictionary_lookup_and_pool_round_trip():
    w = synth.config0().with_(seq_lens=(1000,), name="t")
    data = synth.generate(w, spare_slots=7)
    page_map = {}
    for h in range(w.num_kv_heads):
        for pg, s in enumerate(data.slot_of[0][h]):
            page_map[(h, pg)] = int(s)
    sel = [0, 3, 17, 62]
    for h in range(w.num_kv_heads):
        page_ids, slots, masks = resolve.resolve_slots(sel, 1000, 16, 16, 1, 1, page_map, h)
        assert page_ids == [0, 3, 17, 62]
        assert slots == [int(data.slot_of[0][h][p]) for p in page_ids]
        assert masks == [0xFFFF, 0xFFFF, 0xFFFF, (1 << (1000 - 62 * 16)) - 1]
        kb, vb = data.logical_kv_bits(0, h)
        for p, s in zip(page_ids, slots):
            assert np.array_equal(data.pool_bits[s, 0], kb[p * 16:(p + 1) * 16])
            assert np.array_equal(data.pool_bits[s, 1], vb[p * 16:(p + 1) * 16])
        assert sum(bin(m).count("1") for m in masks) == 16 * 3 + 8


def test_slots_are_a_permutation_not_identity():
    data = synth.generate(synth.config0())
    allslots = np.concatenate([s.reshape(-1) for s in data.slot_of])
    assert sorted(allslots.tolist()) == list(range(len(allslots)))
    assert not np.array_equal(allslots, np.arange(len(allslots)))


def test_block_partitions_expand_to_consecutive_pages_plus_forced():
    seq = 10 * 128 + 40                       # 83 pages; block 10 has 3 pages
    page_map = {(0, p): 1000 + p for p in range(83)}
    page_ids, slots, masks = resolve.resolve_slots([0, 4, 10], seq, 16, 128, 4, 2, page_map, 0)
    want = list(range(0, 8)) + list(range(32, 40)) + [80, 81, 82]
    assert page_ids == want                    # sinks 0..3 dedup with block 0; recents 81,82 with block 10
    assert slots == [1000 + p for p in want]
    assert masks[-1] == (1 << 8) - 1 and all(m == 0xFFFF for m in masks[:-1])
    # forced pages not inside any selected partition are still attended
    page_ids, _, _ = resolve.resolve_slots([4], seq, 16, 128, 4, 2, page_map, 0)
    assert page_ids == [0, 1, 2, 3] + list(range(32, 40)) + [81, 82]


def test_token_partitions_merge_bits_per_page():
    seq = 70
    page_map = {(3, p): 50 - p for p in range(5)}
    sel = [1, 5, 17, 18, 69]
    page_ids, slots, masks = resolve.resolve_slots(sel, seq, 16, 1, 0, 0, page_map, 3)
    assert page_ids == [0, 1, 4]
    assert slots == [50, 49, 46]
    assert masks == [(1 << 1) | (1 << 5), (1 << 1) | (1 << 2), 1 << 5]
    assert sum(bin(m).count("1") for m in masks) == len(sel)


def test_not_resident_raises():
    with pytest.raises(resolve.NotResident):
        resolve.resolve_slots([2], 64, 16, 16, 0, 0, {(0, 0): 1}, 0)
