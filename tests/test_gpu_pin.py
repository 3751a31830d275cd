"""Pinned (outlier) partitions on the GPU: the selection equals the oracle's on the
pinned scores, for page, block and long token rows; under a budget their pages stay
resident (selected in every step, so never evicted, and missed at most once)."""
import math

import numpy as np
import pytest
import torch

from oracle import select as oselect
from paper_2604_26837_amd import hier, runner, synth, tables

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _pins(w, rng, per_row, stride):
    pinned = np.full((w.rows, stride), -1, dtype=np.int32)
    npinned = np.zeros(w.rows, dtype=np.int32)
    for r in range(w.rows):
        P = w.partitions(r // w.num_kv_heads)
        n = int(rng.integers(0, per_row + 1))
        ids = rng.permutation(P)[:n].tolist() + [P + 5, -2][: max(0, min(2, stride - n))]   # two ids outside the row
        pinned[r, :len(ids)] = ids
        npinned[r] = len(ids)
    return pinned, npinned


@pytest.mark.parametrize("name", ["pages", "blocks", "long_token_rows"])
def test_selection_with_pinned_partitions(name):
    c0 = synth.config0().with_(num_q_heads=8, num_kv_heads=2)
    w = {
        "pages": c0.with_(seq_lens=(4096, 1000, 2049), topk=24, sink_pages=2, recent_pages=3, name="pin_pages"),
        "blocks": c0.with_(seq_lens=(64 * 50 + 17, 640), partition_tokens=64, topk=6, topk_includes_forced=False,
                           sink_pages=1, recent_pages=5, name="pin_blocks"),
        "long_token_rows": c0.with_(seq_lens=(20000, 17001), partition_tokens=1, score_kind=synth.SCORE_SKETCH,
                                    topk=300, sink_pages=1, recent_pages=1, name="pin_tokens"),
    }[name]
    data = synth.generate(w)
    natural = torch.from_numpy(data.pool_bits.view(np.int16).copy()).to(DEV).view(torch.bfloat16)
    layer = runner.LayerState.from_natural_pool(w, data.slot_of, natural)
    if w.score_kind == synth.SCORE_SKETCH:
        layer.set_channels(synth.sketch_channels(data))
    layer.build_summaries()
    sp = layer.spin
    rng = np.random.default_rng(5)
    pinned_np, npinned_np = _pins(w, rng, 10, 16)
    pinned, npinned = torch.from_numpy(pinned_np).to(DEV), torch.from_numpy(npinned_np).to(DEV)
    q = torch.from_numpy(data.q_bits.view(np.int16).copy()).to(DEV).view(torch.bfloat16)
    sp.score_partitions(w.batch, q, layer.summaries, layer.chan, layer.part_offsets, layer.seq_lens, layer.scores, layer.ws)
    torch.cuda.synchronize()
    plain = layer.scores.cpu().numpy().copy()
    sp.pin_partitions(w.batch, layer.scores, layer.part_offsets, pinned, npinned)
    sp.select_topk(w.batch, layer.scores, layer.part_offsets, layer.seq_lens, layer.sel, layer.nsel, layer.ws)
    sp.resolve_slots(w.batch, 0, layer.sel, layer.nsel, layer.seq_lens, layer.dir, layer.leaf_pool, layer.slots,
                     layer.page_ids, layer.valid_mask, layer.npages, layer.ws)
    sp.sparse_decode(w.batch, q, layer.kv_pool, layer.slots, layer.valid_mask, layer.npages, layer.out, layer.lse, layer.ws)
    torch.cuda.synchronize()
    assert layer.status() == 0
    got_scores = layer.scores.cpu().numpy()
    sel, nsel = layer.sel.cpu().numpy(), layer.nsel.cpu().numpy()
    for b in range(w.batch):
        for h in range(w.num_kv_heads):
            r = b * w.num_kv_heads + h
            base = tables.row_base(layer.part_offsets_np, b, h, w.num_kv_heads)
            P = w.partitions(b)
            ids = pinned_np[r, :npinned_np[r]].tolist()
            want_scores = oselect.pin_scores(plain[base:base + P], w.seq_lens[b], w.partition_tokens, ids)
            assert np.array_equal(got_scores[base:base + P].astype(np.float64), want_scores), (b, h)
            want = oselect.select_topk(want_scores, w.seq_lens[b], 16, w.partition_tokens, w.topk,
                                       w.topk_includes_forced, w.sink_pages, w.recent_pages)
            assert sel[r, :nsel[r]].tolist() == list(want), (b, h)
            forced = set(oselect.forced_partitions(w.seq_lens[b], 16, w.partition_tokens, w.sink_pages, w.recent_pages))
            inside = [p for p in ids if 0 <= p < P and p not in forced]
            kprime = max(w.topk - len(forced), 0) if w.topk_includes_forced else w.topk
            if len(inside) <= kprime:
                assert set(inside) <= set(want)
    assert bool(torch.isfinite(layer.out.float()).all())


def test_pinned_pages_stay_resident_under_a_budget():
    w = synth.config0().with_(seq_lens=(16 * 700, 16 * 420), num_q_heads=8, num_kv_heads=2, topk=24, sink_pages=2,
                              recent_pages=3, name="pin_budget")
    layer = hier.HierLayer(w, budget_frac=0.06, n_ts=8, copy_mode="gather", keep_natural=False)
    sp = layer.spin
    rng = np.random.default_rng(9)
    pinned_np, npinned_np = _pins(w, rng, 6, 8)
    pinned, npinned = torch.from_numpy(pinned_np).to(DEV), torch.from_numpy(npinned_np).to(DEV)
    q = layer.q0
    missed = [dict() for _ in range(w.rows)]
    for step in range(14):
        sp.score_partitions(w.batch, q, layer.summaries, None, layer.part_offsets, layer.seq_lens, layer.scores, layer.ws)
        sp.pin_partitions(w.batch, layer.scores, layer.part_offsets, pinned, npinned)
        sp.select_topk(w.batch, layer.scores, layer.part_offsets, layer.seq_lens, layer.sel, layer.nsel, layer.ws)
        sp.resolve_slots(w.batch, step, layer.sel, layer.nsel, layer.seq_lens, layer.dir, layer.leaf_pool, layer.slots,
                         layer.page_ids, layer.valid_mask, layer.npages, layer.ws, rev_table=layer.rev,
                         slot_base=layer.slot_base, miss_pages=layer.miss_pages, miss_slots=layer.miss_slots,
                         nmiss=layer.nmiss)
        sp.gather_misses(w.batch, layer.host_kv, layer.host_row_base_dev, layer.nmiss, layer.miss_pages,
                         layer.miss_slots, layer.kv_pool, layer.ws)
        sp.sparse_decode(w.batch, q, layer.kv_pool, layer.slots, layer.valid_mask, layer.npages, layer.out, layer.lse,
                         layer.ws)
        torch.cuda.synchronize()
        assert layer.status() == 0
        pages, npg = layer.page_ids.cpu().numpy(), layer.npages.cpu().numpy()
        mp, nm = layer.miss_pages.cpu().numpy(), layer.nmiss.cpu().numpy()
        for r in range(w.rows):
            P = w.partitions(r // w.num_kv_heads)
            ids = [p for p in pinned_np[r, :npinned_np[r]].tolist() if 0 <= p < P]
            assert set(ids) <= set(pages[r, :npg[r]].tolist()), (step, r)       # attended in every step
            for p in mp[r, :nm[r]].tolist():
                if p in ids:
                    missed[r][p] = missed[r].get(p, 0) + 1
        q_bits = q.view(torch.int16).cpu().numpy().view(np.uint16)
        q = torch.from_numpy(synth.next_query_ar1(q_bits, 0.5, w.seed + 900 + step).view(np.int16)).to(DEV).view(torch.bfloat16)
    for r in range(w.rows):
        assert all(c == 1 for c in missed[r].values()), (r, missed[r])           # fetched once, never evicted
