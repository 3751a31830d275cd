"""spin_select_resolve_forced + spin_sparse_decode_rest: stages 2+3 whose launch also attends the row's sink and
recent pages, and the stage 4 that covers the rest of the page list and merges that partial.  Stages 2+3 must
give the bits of spin_select_resolve; the attention output is held to stage 4's tolerance against the oracle on
the GPU's own page list, and must be the same bits from run to run."""
import numpy as np
import pytest
import torch

from oracle import attend, bf16
from paper_2604_26837_amd import binding, runner, synth

pytestmark = pytest.mark.gpu
ATOL, RTOL = 2e-2, 1e-2


def _layer(w, **over):
    data = synth.generate(w, spare_slots=2)
    natural = torch.from_numpy(data.pool_bits.view(np.int16).copy()).to("cuda:0").view(torch.bfloat16)
    layer = runner.LayerState.from_natural_pool(w, data.slot_of, natural, **over)
    layer.build_summaries()
    q = torch.from_numpy(data.q_bits.view(np.int16).copy()).to("cuda:0").view(torch.bfloat16)
    return data, layer, q


def _oracle_out(w, data, layer):
    """fp64 attention per row over the page list, slots and masks the GPU produced."""
    slots, npages = layer.slots.cpu().numpy(), layer.npages.cpu().numpy()
    masks = layer.valid_mask.cpu().numpy().view(np.uint16)
    g = w.group
    ref = np.zeros((w.batch, w.num_q_heads, w.head_dim))
    lse = np.zeros((w.batch, w.num_q_heads))
    for r in range(w.rows):
        b, h = divmod(r, w.num_kv_heads)
        keep = [(int(s), int(m)) for s, m in zip(slots[r, :npages[r]], masks[r, :npages[r]]) if s >= 0]
        pages = bf16.decode(data.pool_bits[np.asarray([s for s, _ in keep], dtype=np.int64)]) if keep else \
            np.zeros((0, 2, 16, w.head_dim))
        ks, vs = attend.gather_tokens(pages[:, 0], pages[:, 1], [m for _, m in keep])
        o, l = attend.attend(bf16.decode(data.q_bits[b, h * g:(h + 1) * g]), ks, vs, layer.scale)
        ref[b, h * g:(h + 1) * g], lse[b, h * g:(h + 1) * g] = o, l
    return ref, lse


def _bits(t):
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


CASES = {
    # name: (workload, config overrides)
    "cfg0": (synth.config0(), {}),
    "ragged_4_sinks_8_recents": (synth.config0().with_(
        seq_lens=(4096, 1000, 2049, 40, 16 * 12, 5, 16 * 13 + 1, 3000), num_q_heads=8, num_kv_heads=2, topk=40,
        sink_pages=4, recent_pages=8, name="forced_ragged"), {}),
    "one_split": (synth.config0().with_(seq_lens=(4096, 700), topk=24, sink_pages=2, recent_pages=3,
                                        name="forced_1split"), dict(decode_splits=1)),
    "three_splits_group8": (synth.config0().with_(seq_lens=(3000, 4096, 17), num_q_heads=16, num_kv_heads=2, topk=50,
                                                  sink_pages=3, recent_pages=5, name="forced_g8"),
                            dict(decode_splits=3)),
    "group1_recent_only": (synth.config0().with_(seq_lens=(2500, 1300), num_q_heads=2, num_kv_heads=2, topk=20,
                                                 sink_pages=0, recent_pages=6, name="forced_g1"),
                           dict(decode_splits=2, decode_waves=4)),
    # partitions of several pages: the sink / recent pages need not line up with partitions, and there are enough
    # of them for several side workgroups per row
    "blocks_of_8_pages": (synth.config0().with_(seq_lens=(20000, 9000, 1500, 300, 16 * 70), num_q_heads=8, num_kv_heads=2,
                                                partition_tokens=128, score_kind=synth.SCORE_REPMAX, topk=8,
                                                topk_includes_forced=False, sink_pages=4, recent_pages=64,
                                                name="forced_blocks"), {}),
    "blocks_of_4_pages_minmax": (synth.config0().with_(seq_lens=(8000, 3001, 100), num_q_heads=8, num_kv_heads=2,
                                                       partition_tokens=64, topk=12, sink_pages=3, recent_pages=21,
                                                       name="forced_blocks4"), dict(decode_splits=2)),
    "many_recent_pages": (synth.config0().with_(seq_lens=(30000, 12000), num_q_heads=8, num_kv_heads=2, topk=300,
                                                sink_pages=16, recent_pages=200, name="forced_many"),
                          dict(decode_splits=3)),
    "rows_up_to_4096_pages": (synth.config0().with_(seq_lens=(65536, 40000), num_q_heads=8, num_kv_heads=2, topk=64,
                                                    sink_pages=8, recent_pages=56, name="forced_long"), {}),
}


def _random_case(seed):
    """A workload drawn at random among those the split supports: whole-page partitions of one size, at least
    one sink or recent page, ragged contexts from a few tokens to several leaves, random launch shape."""
    rng = np.random.default_rng(4200 + seed)
    kind = int(rng.choice([synth.SCORE_MINMAX, synth.SCORE_REPMAX]))
    reps = int(rng.choice([1, 2, 4])) if kind == synth.SCORE_REPMAX else 4
    tp = int(rng.choice([16, 16, 32, 64, 128]))
    g, hkv = int(rng.choice([1, 2, 4, 4, 5, 8])), int(rng.choice([1, 2, 3]))
    lens = []
    for _ in range(int(rng.integers(1, 5))):
        style = int(rng.integers(0, 4))
        lens.append(int({0: rng.integers(1, 60), 1: rng.integers(60, 900), 2: rng.integers(900, 12000),
                         3: 16 * rng.integers(1, 700)}[style]))
    sink, recent = int(rng.integers(0, 20)), int(rng.integers(0, 90))
    if sink + recent == 0:
        recent = 1
    w = synth.config0().with_(seq_lens=tuple(lens), num_q_heads=g * hkv, num_kv_heads=hkv, partition_tokens=tp,
                              score_kind=kind, reps_per_partition=reps, topk=int(rng.integers(1, 80)),
                              topk_includes_forced=bool(rng.integers(0, 2)), sink_pages=sink, recent_pages=recent,
                              name=f"forced_random{seed}")
    over = dict(decode_splits=int(rng.choice([0, 1, 2, 3, 5])), decode_waves=int(rng.choice([0, 2, 4, 8])),
                decode_depth=int(rng.choice([0, 2, 3])))
    return w, over


@pytest.mark.parametrize("name", list(CASES) + [f"random{i}" for i in range(24)])
def test_forced_pages_attended_beside_stages_2_and_3(name):
    w, over = CASES[name] if name in CASES else _random_case(int(name[6:]))
    data, layer, q = _layer(w, **over)
    assert layer.spin.forced_split_supported
    layer.step3(q)
    torch.cuda.synchronize()
    assert layer.status() == 0
    plain = dict(sel=layer.sel.clone(), nsel=layer.nsel.clone(), slots=layer.slots.clone(),
                 page_ids=layer.page_ids.clone(), mask=layer.valid_mask.clone(), npages=layer.npages.clone())
    plain_out = bf16.decode(_bits(layer.out))
    for t in (layer.sel, layer.slots, layer.page_ids):
        t.fill_(-7)
    layer.out.fill_(3.0)
    layer.step3f(q)
    torch.cuda.synchronize()
    assert layer.status() == 0
    # stages 2+3: the same bits as the plain launch
    for k, t in (("sel", layer.sel), ("nsel", layer.nsel), ("slots", layer.slots), ("page_ids", layer.page_ids),
                 ("mask", layer.valid_mask), ("npages", layer.npages)):
        assert torch.equal(t, plain[k]), k
    # stage 4 against the oracle on the GPU's own page list
    ref, lref = _oracle_out(w, data, layer)
    out = bf16.decode(_bits(layer.out))
    err = np.abs(out - ref)
    assert (err <= ATOL + RTOL * np.abs(ref)).all(), f"max err {err.max()}"
    assert (np.abs(out - plain_out) <= 2 * (ATOL + RTOL * np.abs(ref))).all()
    lse = layer.lse.cpu().numpy().astype(np.float64)
    fin = np.isfinite(lref)
    assert np.array_equal(np.isfinite(lse), fin) and np.allclose(lse[fin], lref[fin], rtol=2e-3, atol=2e-3)
    # the same bits from run to run, also after other work has used the workspace
    first = _bits(layer.out).copy()
    layer.step(q)
    for _ in range(3):
        layer.out.fill_(1.0)
        layer.step3f(q)
        torch.cuda.synchronize()
        assert np.array_equal(_bits(layer.out), first)


def test_forced_page_that_is_not_resident_is_reported_and_skipped():
    w = synth.config0().with_(seq_lens=(4096, 2000), topk=24, sink_pages=2, recent_pages=3, name="forced_missing")
    data, layer, q = _layer(w, decode_splits=2)
    # drop the mapping of sink page 1 of row 0 and of the last page of row 3
    d = layer.dir.cpu().numpy()
    leaf = layer.leaf_pool.cpu().numpy().copy()
    leaf[d[0, 0], 1] = -1
    last = w.pages(1) - 1
    leaf[d[3, last // w.leaf_entries], last % w.leaf_entries] = -1
    layer.leaf_pool.copy_(torch.from_numpy(leaf))
    layer.step3f(q)
    torch.cuda.synchronize()
    assert binding.STATUS_NAMES[layer.status()] == "SPIN_ERR_NOT_RESIDENT"
    slots, npages = layer.slots.cpu().numpy(), layer.npages.cpu().numpy()
    assert slots[0, 1] == -1 and slots[3, npages[3] - 1] == -1
    ref, _ = _oracle_out(w, data, layer)          # over the pages that are resident
    out = bf16.decode(_bits(layer.out))
    assert (np.abs(out - ref) <= ATOL + RTOL * np.abs(ref)).all()
