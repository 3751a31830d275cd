"""Stages 1 and 2 in one call must give exactly what the two stage calls give:
same score bits, same selection.  Rows of more than 16384 partitions take the path where
stage 1 counts the leading key bits for stage 2 (the histogram in the workspace must be
left cleared, so the calls are repeated and interleaved); every other shape
simply runs the two stages."""
import numpy as np
import pytest
import torch

from oracle import select as oselect
from paper_2604_26837_amd import runner, synth, tables

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _workloads():
    c0 = synth.config0()
    tok = dict(num_q_heads=8, num_kv_heads=2, partition_tokens=1, score_kind=synth.SCORE_SKETCH)
    return {
        # two-launch selection: histogram taken by stage 1
        "long_token_rows": c0.with_(seq_lens=(20000, 17001, 65536), topk=300, sink_pages=1, recent_pages=2,
                                    name="ss_long", **tok),
        "long_rows_no_forced": c0.with_(seq_lens=(40000, 16400), topk=1024, sink_pages=0, recent_pages=0,
                                        name="ss_long_nf", **tok),
        # one short request in a context sized for long rows; k' = 0 for the request that is all forced
        "long_context_short_rows": c0.with_(seq_lens=(100, 32, 17000), topk=40, sink_pages=1, recent_pages=1,
                                            name="ss_mixed", **tok),
        # long rows of page partitions: stage 1 of the other two score kinds counts the histogram too
        "long_page_rows_minmax": c0.with_(seq_lens=(16 * 17000 + 5, 300000, 900), num_q_heads=4, num_kv_heads=1,
                                          topk=200, sink_pages=3, recent_pages=6, name="ss_long_minmax"),
        "long_page_rows_repmax": c0.with_(seq_lens=(270000, 16 * 16385), num_q_heads=6, num_kv_heads=2,
                                          score_kind=synth.SCORE_REPMAX, reps_per_partition=2, topk=77,
                                          topk_includes_forced=False, sink_pages=2, recent_pages=0,
                                          name="ss_long_repmax"),
        # shapes where the combined call is the two launches
        "short_token_rows": c0.with_(seq_lens=(5000, 900), topk=64, sink_pages=1, recent_pages=1, name="ss_short", **tok),
        "pages_minmax": c0.with_(seq_lens=(4096, 1000, 2049), num_q_heads=8, num_kv_heads=2, topk=24, sink_pages=2,
                                 recent_pages=3, name="ss_pages"),
    }


@pytest.mark.parametrize("name", list(_workloads()))
def test_combined_call_equals_the_two_stage_calls(name):
    w = _workloads()[name]
    data = synth.generate(w)
    natural = torch.from_numpy(data.pool_bits.view(np.int16).copy()).to(DEV).view(torch.bfloat16)
    layer = runner.LayerState.from_natural_pool(w, data.slot_of, natural)
    if w.score_kind == synth.SCORE_SKETCH:
        layer.set_channels(synth.sketch_channels(data))
    layer.build_summaries()
    sp = layer.spin
    qs = [torch.from_numpy(synth.make_queries(w, 300 + i).view(np.int16)).to(DEV).view(torch.bfloat16) for i in range(3)]
    scores2, sel2, nsel2 = torch.zeros_like(layer.scores), torch.zeros_like(layer.sel), torch.zeros_like(layer.nsel)
    for rep in range(5):
        q = qs[rep % 3]
        # the two stage calls
        sp.score_partitions(w.batch, q, layer.summaries, layer.chan, layer.part_offsets, layer.seq_lens, layer.scores,
                            layer.ws)
        sp.select_topk(w.batch, layer.scores, layer.part_offsets, layer.seq_lens, layer.sel, layer.nsel, layer.ws)
        # the combined call, into its own buffers pre-filled with junk
        scores2.fill_(-7.0)
        sel2.fill_(-5)
        nsel2.fill_(-5)
        sp.score_select_topk(w.batch, q, layer.summaries, layer.chan, layer.part_offsets, layer.seq_lens, scores2,
                             sel2, nsel2, layer.ws)
        torch.cuda.synchronize()
        assert layer.status() == 0
        assert torch.equal(nsel2, layer.nsel), f"rep {rep}"
        assert torch.equal(sel2, layer.sel), f"rep {rep}"
        s1, s2 = layer.scores.cpu().numpy().view(np.uint32), scores2.cpu().numpy().view(np.uint32)
        for b in range(w.batch):
            for h in range(w.num_kv_heads):
                base = tables.row_base(layer.part_offsets_np, b, h, w.num_kv_heads)
                P = w.partitions(b)
                assert np.array_equal(s1[base:base + P], s2[base:base + P]), (rep, b, h)
    # and against the oracle's selection on the GPU's score bits
    sc = scores2.cpu().numpy()
    sel, nsel = sel2.cpu().numpy(), nsel2.cpu().numpy()
    for b in range(w.batch):
        for h in range(w.num_kv_heads):
            r = b * w.num_kv_heads + h
            base = tables.row_base(layer.part_offsets_np, b, h, w.num_kv_heads)
            want = oselect.select_topk(sc[base:base + w.partitions(b)].astype(np.float64), w.seq_lens[b], 16,
                                       w.partition_tokens, w.topk, w.topk_includes_forced, w.sink_pages,
                                       w.recent_pages)
            assert sel[r, :nsel[r]].tolist() == list(want), (b, h)


@pytest.mark.parametrize("name", ["long_token_rows", "long_page_rows_minmax", "long_page_rows_repmax"])
def test_combined_call_saves_the_histogram_launch(name):
    """For long rows the combined call issues no histogram launch over the score array (stage 1 has counted
    the bins), the separate stage 2 call issues one."""
    w = _workloads()[name]
    data = synth.generate(w)
    natural = torch.from_numpy(data.pool_bits.view(np.int16).copy()).to(DEV).view(torch.bfloat16)
    layer = runner.LayerState.from_natural_pool(w, data.slot_of, natural)
    if w.score_kind == synth.SCORE_SKETCH:
        layer.set_channels(synth.sketch_channels(data))
    layer.build_summaries()
    sp = layer.spin
    q = torch.from_numpy(synth.make_queries(w, 17).view(np.int16)).to(DEV).view(torch.bfloat16)
    sp.profile_enable(8)
    try:
        sp.score_select_topk(w.batch, q, layer.summaries, layer.chan, layer.part_offsets, layer.seq_lens, layer.scores,
                             layer.sel, layer.nsel, layer.ws)
        torch.cuda.synchronize()
        assert sp.profile_read("select_hist")[0] == 0 and sp.profile_read("score")[0] == 1
        assert sp.profile_read("select")[0] == 1
        sp.select_topk(w.batch, layer.scores, layer.part_offsets, layer.seq_lens, layer.sel, layer.nsel, layer.ws)
        torch.cuda.synchronize()
        assert sp.profile_read("select_hist")[0] == 1 and sp.profile_read("select")[0] == 1
    finally:
        sp.profile_enable(0)
    assert layer.status() == 0


def _heavy_ties(layer, w):
    """Scores that send a long row down the multi-pass fallback: a handful of distinct values."""
    rng = np.random.default_rng(11)
    vals = rng.choice(np.array([0.5, 0.5, 0.25, 1.0], dtype=np.float32), size=layer.scores.numel())
    return torch.from_numpy(vals).to(DEV)


@pytest.mark.parametrize("name", list(_workloads()))
def test_stages_1_to_3_in_one_call_equal_the_stage_calls(name):
    """spin_score_select_resolve (and spin_select_resolve on its own, also for long rows and for rows that take
    stage 2's multi-pass fallback) against the separate stage calls: every output identical."""
    w = _workloads()[name]
    data = synth.generate(w)
    natural = torch.from_numpy(data.pool_bits.view(np.int16).copy()).to(DEV).view(torch.bfloat16)
    layer = runner.LayerState.from_natural_pool(w, data.slot_of, natural)
    if w.score_kind == synth.SCORE_SKETCH:
        layer.set_channels(synth.sketch_channels(data))
    layer.build_summaries()
    sp = layer.spin
    qs = [torch.from_numpy(synth.make_queries(w, 400 + i).view(np.int16)).to(DEV).view(torch.bfloat16) for i in range(3)]
    names = ("scores", "sel", "nsel", "slots", "page_ids", "valid_mask", "npages")
    twin = {n: torch.zeros_like(getattr(layer, n)) for n in names}

    def stage_calls(q, scores=None):
        if scores is None:
            sp.score_partitions(w.batch, q, layer.summaries, layer.chan, layer.part_offsets, layer.seq_lens,
                                layer.scores, layer.ws)
            scores = layer.scores
        sp.select_topk(w.batch, scores, layer.part_offsets, layer.seq_lens, layer.sel, layer.nsel, layer.ws)
        sp.resolve_slots(w.batch, 0, layer.sel, layer.nsel, layer.seq_lens, layer.dir, layer.leaf_pool, layer.slots,
                         layer.page_ids, layer.valid_mask, layer.npages, layer.ws)

    def same(what, skip=()):
        torch.cuda.synchronize()
        assert layer.status() == 0
        rows_n = layer.npages.cpu().numpy()
        for n in names:
            if n in skip:
                continue
            a, b = getattr(layer, n), twin[n]
            if n in ("slots", "page_ids", "valid_mask"):       # entries past a row's page count are unspecified
                keep = torch.arange(a.shape[1], device=DEV)[None, :] < layer.npages[:, None]
                assert torch.equal(a[keep], b[keep]), f"{what}: {n}"
            elif n == "scores":
                s1, s2 = a.cpu().numpy().view(np.uint32), b.cpu().numpy().view(np.uint32)
                for bb in range(w.batch):
                    for h in range(w.num_kv_heads):
                        base = tables.row_base(layer.part_offsets_np, bb, h, w.num_kv_heads)
                        assert np.array_equal(s1[base:base + w.partitions(bb)], s2[base:base + w.partitions(bb)]), what
            else:
                assert torch.equal(a, b), f"{what}: {n}"
        assert rows_n.sum() > 0

    for rep in range(4):
        q = qs[rep % 3]
        stage_calls(q)
        for t in twin.values():
            t.fill_(-3)
        sp.score_select_resolve(w.batch, q, layer.summaries, layer.chan, layer.part_offsets, layer.seq_lens,
                                twin["scores"], twin["sel"], twin["nsel"], layer.dir, layer.leaf_pool, twin["slots"],
                                twin["page_ids"], twin["valid_mask"], twin["npages"], layer.ws)
        same(f"three stages, rep {rep}")
        for n in names[1:]:
            twin[n].fill_(-4)
        sp.select_resolve(w.batch, layer.scores, layer.part_offsets, layer.seq_lens, twin["sel"], twin["nsel"],
                          layer.dir, layer.leaf_pool, twin["slots"], twin["page_ids"], twin["valid_mask"],
                          twin["npages"], layer.ws)
        same(f"stages 2+3, rep {rep}", skip=("scores",))
    # heavy ties: the long rows leave the one-walk path inside the launch
    tied = _heavy_ties(layer, w)
    stage_calls(None, scores=tied)
    for n in names[1:]:
        twin[n].fill_(-6)
    sp.select_resolve(w.batch, tied, layer.part_offsets, layer.seq_lens, twin["sel"], twin["nsel"], layer.dir,
                      layer.leaf_pool, twin["slots"], twin["page_ids"], twin["valid_mask"], twin["npages"], layer.ws)
    same("heavy ties", skip=("scores",))
