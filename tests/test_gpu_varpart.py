"""GPU parity with variable-length partitions (Partition Offset + Meta-partition
tables): Index, scores, selection, slots/masks and attention against the
variable-length oracle, for the four-call step and the one-launch stage 2+3."""
import numpy as np
import pytest
import torch

from oracle import attend, bf16, score, varpart
from paper_2604_26837_amd import runner, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ATOL, RTOL = 2e-2, 1e-2


def _check(w, layouts, data, layer, three_launch):
    q = torch.from_numpy(data.q_bits.view(np.int16).copy()).to(DEV).view(torch.bfloat16)
    layer.build_summaries()
    (layer.step3 if three_launch else layer.step)(q)
    torch.cuda.synchronize()
    assert layer.status() == 0
    raw = layer.summaries.cpu().numpy().view(np.uint16)
    centroid = w.score_kind == synth.SCORE_REPMAX          # one mean key per partition instead of min / max
    kd = 128 if centroid else 256
    rows16 = raw.reshape(-1, kd // 8, 16, 8).transpose(0, 2, 1, 3).reshape(-1, kd)
    scores = layer.scores.cpu().numpy()
    sel, nsel = layer.sel.cpu().numpy(), layer.nsel.cpu().numpy()
    slots, npages = layer.slots.cpu().numpy(), layer.npages.cpu().numpy()
    page_ids = layer.page_ids.cpu().numpy()
    masks = layer.valid_mask.cpu().numpy().view(np.uint16)
    out = bf16.decode(layer.out.view(torch.int16).cpu().numpy().view(np.uint16))
    g = w.group
    r = 0
    for b in range(w.batch):
        for h in range(w.num_kv_heads):
            first, toks = layouts[b][h]
            P = len(first)
            kb, vb = data.logical_kv_bits(b, h)
            K = bf16.decode(kb)
            qh = bf16.decode(data.q_bits[b, h * g:(h + 1) * g])
            base = layer.row_base(b, h)
            got = bf16.decode(rows16[base: base + P])
            if centroid:
                cents = varpart.centroids(K, first, toks, 16)
                assert np.array_equal(got, cents[:, 0]), f"summaries row {r}"
                s64 = score.score_repmax(qh, cents)
                eps = 128 * 2.0 ** -24 * np.abs(qh[:, None] * cents[None, :, 0]).sum(-1).max()
            else:
                mins, maxs = varpart.minmax_summaries(K, first, toks, 16)
                assert np.array_equal(got, np.concatenate([maxs, mins], axis=1)), f"summaries row {r}"
                s64 = score.score_minmax(qh, mins, maxs)
                eps = 256 * 2.0 ** -24 * np.maximum(np.abs(qh[:, None] * mins[None]), np.abs(qh[:, None] * maxs[None])).sum(-1).max()
            s32 = scores[base: base + P]
            assert np.all(np.abs(s32.astype(np.float64) - s64) <= eps)
            want = varpart.select_topk(s32, first, toks, 16, w.topk, w.topk_includes_forced, w.sink_pages,
                                       w.recent_pages)
            assert sel[r, :nsel[r]].tolist() == want, f"selection row {r}"
            page_map = {(r, pg): int(s) for pg, s in enumerate(data.slot_of[b][h])}
            pg_w, sl_w, mk_w = varpart.resolve_slots(want, first, toks, 16, w.sink_pages, w.recent_pages, page_map, r)
            assert npages[r] == len(pg_w)
            assert page_ids[r, :npages[r]].tolist() == pg_w, f"pages row {r}"
            assert slots[r, :npages[r]].tolist() == sl_w
            assert masks[r, :npages[r]].tolist() == mk_w
            pages = bf16.decode(data.pool_bits[np.asarray(sl_w, dtype=np.int64)])
            ks, vs = attend.gather_tokens(pages[:, 0], pages[:, 1], mk_w)
            ref, _ = attend.attend(qh, ks, vs, layer.scale)
            o = out[b, h * g:(h + 1) * g]
            assert np.all(np.abs(o - ref) <= ATOL + RTOL * np.abs(ref)), f"attention row {r}"
            r += 1


@pytest.mark.parametrize("three_launch", [False, True])
@pytest.mark.parametrize("case", ["clusters", "mostly_single_pages", "forced_heavy", "cluster_centroids"])
def test_variable_length_partitions(case, three_launch):
    c0 = synth.config0().with_(num_q_heads=8, num_kv_heads=2)
    w, min_tok = {
        # clusters scored through their centroid (one mean key per partition)
        "cluster_centroids": (c0.with_(seq_lens=(16 * 300, 16 * 77, 16 * 1000), partition_tokens=96,
                                       score_kind=synth.SCORE_REPMAX, reps_per_partition=1, topk=12,
                                       topk_includes_forced=False, sink_pages=3, recent_pages=5,
                                       block_mean_std=0.5, name="v4"), 1),
        "clusters": (c0.with_(seq_lens=(16 * 300, 16 * 77, 16 * 1000), partition_tokens=80, topk=12,
                              topk_includes_forced=False, sink_pages=3, recent_pages=5, name="v1"), 1),
        "mostly_single_pages": (c0.with_(seq_lens=(16 * 500, 16 * 40), partition_tokens=32, topk=30,
                                         topk_includes_forced=True, sink_pages=4, recent_pages=8, name="v2"), 1),
        "forced_heavy": (c0.with_(seq_lens=(16 * 64, 16 * 9, 16 * 3), partition_tokens=128, topk=4,
                                  topk_includes_forced=True, sink_pages=6, recent_pages=7, name="v3"), 17),
    }[case]
    data = synth.generate(w, spare_slots=3)
    layouts = synth.variable_layouts(w, seed=w.seed + 77, min_tokens=min_tok)
    natural = torch.from_numpy(data.pool_bits.view(np.int16).copy()).to(DEV).view(torch.bfloat16)
    layer = runner.LayerState.from_natural_pool(w, data.slot_of, natural, layouts=layouts)
    _check(w, layouts, data, layer, three_launch)


@pytest.mark.parametrize("seed", range(16))
def test_variable_length_partitions_random(seed):
    """Randomly drawn cluster layouts, largest cluster size, summary kind (min / max keys or the
    centroid), heads, top-k and forced windows, through both launch shapes."""
    rng = np.random.default_rng(700 + seed)
    hkv = int(rng.choice([1, 2, 3]))
    g = int(rng.choice([1, 2, 4, 5, 8]))
    lens = tuple(16 * int(x) for x in rng.integers(2, 400, size=int(rng.integers(1, 4))))
    centroid = bool(rng.integers(0, 2))
    w = synth.config0().with_(seq_lens=lens, num_q_heads=g * hkv, num_kv_heads=hkv,
                              partition_tokens=16 * int(rng.integers(1, 10)),
                              score_kind=synth.SCORE_REPMAX if centroid else synth.SCORE_MINMAX,
                              reps_per_partition=1 if centroid else 4, topk=int(rng.integers(0, 30)),
                              topk_includes_forced=bool(rng.integers(0, 2)), sink_pages=int(rng.integers(0, 5)),
                              recent_pages=int(rng.integers(0, 7)), block_mean_std=0.5 if centroid else 0.0,
                              name=f"var_random{seed}")
    print(f"seed {seed}: lens {lens} largest {w.partition_tokens} centroid {centroid} group {g} kv {hkv} "
          f"topk {w.topk} incl {w.topk_includes_forced} sink {w.sink_pages} recent {w.recent_pages}", flush=True)
    data = synth.generate(w, spare_slots=3)
    layouts = synth.variable_layouts(w, seed=w.seed + seed, min_tokens=int(rng.integers(1, 17)))
    natural = torch.from_numpy(data.pool_bits.view(np.int16).copy()).to(DEV).view(torch.bfloat16)
    layer = runner.LayerState.from_natural_pool(w, data.slot_of, natural, layouts=layouts)
    _check(w, layouts, data, layer, three_launch=bool(seed % 2))


def test_uniform_tables_give_the_uniform_results():
    """Registering the tables of a uniform layout must not change any output bit."""
    w = synth.config0().with_(seq_lens=(2000, 4096), num_q_heads=8, num_kv_heads=2, partition_tokens=64, topk=9,
                              sink_pages=3, recent_pages=6, name="vu")
    data = synth.generate(w)
    natural = torch.from_numpy(data.pool_bits.view(np.int16).copy()).to(DEV).view(torch.bfloat16)
    q = torch.from_numpy(data.q_bits.view(np.int16).copy()).to(DEV).view(torch.bfloat16)
    ref = runner.LayerState.from_natural_pool(w, data.slot_of, natural)
    ref.build_summaries()
    ref.step(q)
    layouts = [[varpart.uniform_layout(w.seq_lens[b], 16, 64) for _ in range(w.num_kv_heads)] for b in range(w.batch)]
    var = runner.LayerState.from_natural_pool(w, data.slot_of, natural, layouts=layouts)
    var.build_summaries()
    var.step(q)
    torch.cuda.synchronize()
    assert var.status() == 0 and ref.status() == 0
    n = ref.npages.cpu().numpy()
    assert torch.equal(ref.sel[:, :ref.spin.sel_stride], var.sel[:, :ref.spin.sel_stride])
    assert torch.equal(ref.npages, var.npages)
    for r in range(w.rows):
        assert torch.equal(ref.slots[r, :n[r]], var.slots[r, :n[r]])
        assert torch.equal(ref.valid_mask[r, :n[r]], var.valid_mask[r, :n[r]])
    assert torch.equal(ref.out.view(torch.int16), var.out.view(torch.int16))
