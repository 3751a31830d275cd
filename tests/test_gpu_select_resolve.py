"""The one-launch stage 2+3 call must reproduce spin_select_topk followed by
spin_resolve_slots bit for bit, and then the same attention output."""
import numpy as np
import pytest
import torch

from paper_2604_26837_amd import binding, runner, synth

pytestmark = pytest.mark.gpu


def _snapshot(layer):
    return [t.cpu().numpy().copy() for t in (layer.sel, layer.nsel, layer.slots, layer.page_ids, layer.valid_mask,
                                             layer.npages, layer.out.view(torch.int16))]


def _compare(layer, q):
    layer.step(q)
    torch.cuda.synchronize()
    assert layer.status() == 0
    ref = _snapshot(layer)
    for _ in range(2):
        for t in (layer.sel, layer.nsel, layer.slots, layer.page_ids, layer.valid_mask, layer.npages):
            t.fill_(-7)
        layer.out.fill_(3.0)
        layer.step3(q)
        torch.cuda.synchronize()
        assert layer.status() == 0
        for a, b in zip(ref, _snapshot(layer)):
            assert np.array_equal(a, b)


def _layer_from_host(w):
    data = synth.generate(w, spare_slots=2)
    natural = torch.from_numpy(data.pool_bits.view(np.int16).copy()).to("cuda:0").view(torch.bfloat16)
    layer = runner.LayerState.from_natural_pool(w, data.slot_of, natural)
    layer.build_summaries()
    q = torch.from_numpy(data.q_bits.view(np.int16).copy()).to("cuda:0").view(torch.bfloat16)
    return layer, q


@pytest.mark.parametrize("name", ["cfg0", "ragged", "empty_and_tiny", "blocks", "mm_blocks", "wide"])
def test_one_launch_equals_two_calls(name):
    c0 = synth.config0()
    w = {
        "cfg0": c0,
        "ragged": c0.with_(seq_lens=(700, 16, 333, 2049, 5), topk=24, sink_pages=2, recent_pages=3, name="r"),
        "empty_and_tiny": c0.with_(seq_lens=(0, 1, 4096, 0), topk=8, sink_pages=1, recent_pages=1, name="e"),
        "blocks": c0.with_(seq_lens=(131 * 16 + 5, 40 * 128, 129), partition_tokens=128,
                           score_kind=synth.SCORE_REPMAX, topk=6, topk_includes_forced=False, sink_pages=4,
                           recent_pages=11, block_mean_std=0.5, name="b"),
        "mm_blocks": c0.with_(seq_lens=(2000, 4096), partition_tokens=64, topk=9, sink_pages=3, recent_pages=6,
                              name="m"),
        "wide": c0.with_(seq_lens=(3000 * 16, 16 * 4000 + 7), num_q_heads=4, num_kv_heads=1, topk=128,
                         sink_pages=4, recent_pages=8, name="w"),     # 4096-partition rows: 512-thread variant
    }[name]
    layer, q = _layer_from_host(w)
    _compare(layer, q)


def test_headline_size_and_unsupported_shape():
    w = synth.config1()
    layer, _ = runner.build_device_layer(w)
    _compare(layer, layer.q0)
    # refused before anything is launched (the pointers are never used): rows beyond 131072 partitions, budget mode
    w2 = synth.config0().with_(seq_lens=(200000,), partition_tokens=1, score_kind=synth.SCORE_SKETCH, topk=16,
                               sink_pages=0, recent_pages=0, name="sk")
    sp = binding.Spin.for_workload(w2)
    assert sp.lib.spin_select_resolve(sp.h, 1, *([8] * 7), 1, *([8] * 6), 8, None) == -2
    assert sp.lib.spin_score_select_resolve(sp.h, 1, *([8] * 10), 1, *([8] * 6), 8, None) == -2
    sp3 = binding.Spin.for_workload(synth.config0(), lru_timestamps=64)
    assert sp3.lib.spin_select_resolve(sp3.h, 1, *([8] * 7), 1, *([8] * 6), 8, None) == -2
    assert sp3.lib.spin_score_select_resolve(sp3.h, 1, *([8] * 10), 1, *([8] * 6), 8, None) == -2


@pytest.mark.parametrize("seed", range(24))
def test_random_workloads_both_combined_calls(seed):
    """Random workloads (the draw of the stage tests): the stages 2+3 launch, the stages 1+2 call and the
    stages 1-3 call must each reproduce the separate stage calls bit for bit."""
    from test_gpu_stages import _random_workload
    w = _random_workload(200 + seed)
    print(f"seed {seed}: kind {w.score_kind} tp {w.partition_tokens} reps {w.reps_per_partition} group {w.group} "
          f"kv {w.num_kv_heads} lens {w.seq_lens} topk {w.topk}", flush=True)
    data = synth.generate(w, spare_slots=2)
    natural = torch.from_numpy(data.pool_bits.view(np.int16).copy()).to("cuda:0").view(torch.bfloat16)
    layer = runner.LayerState.from_natural_pool(w, data.slot_of, natural)
    if w.score_kind == synth.SCORE_SKETCH:
        layer.set_channels(synth.sketch_channels(data))
    layer.build_summaries()
    q = torch.from_numpy(data.q_bits.view(np.int16).copy()).to("cuda:0").view(torch.bfloat16)
    _compare(layer, q)                       # stages 2+3 in one launch (rows of at most 16384 partitions here)
    ref = _snapshot(layer)
    for t in (layer.sel, layer.nsel, layer.slots, layer.page_ids, layer.valid_mask, layer.npages):
        t.fill_(-7)
    layer.out.fill_(3.0)
    for step in (layer.step12, layer.step123):      # stages 1+2 in one call; stages 1-3 in one call
        for t in (layer.sel, layer.nsel, layer.slots, layer.page_ids, layer.valid_mask, layer.npages):
            t.fill_(-7)
        layer.out.fill_(3.0)
        step(q)
        torch.cuda.synchronize()
        assert layer.status() == 0
        for a, b in zip(ref, _snapshot(layer)):
            assert np.array_equal(a, b)
