"""The stage calls allocate nothing and record no memset, so a decode step can
be captured in a HIP graph.  The graph is replayed several times, with eager
work and synchronisations between replays, and every replay must reproduce the
eager result bit for bit."""
import numpy as np
import pytest
import torch

from paper_2604_26837_amd import hier, runner, synth

pytestmark = pytest.mark.gpu


def _workloads():
    c0 = synth.config0()
    return {
        # stages 2+3 in one launch
        "pages": (c0.with_(seq_lens=(4096, 1000, 2049), num_q_heads=8, num_kv_heads=2, topk=24, sink_pages=2,
                           recent_pages=3, name="graph"), "step3"),
        # the same with the sink / recent pages attended beside stages 2+3 (their partial travels through the workspace)
        "pages_forced_split": (c0.with_(seq_lens=(4096, 1000, 2049, 30), num_q_heads=8, num_kv_heads=2, topk=24,
                                        sink_pages=2, recent_pages=3, name="graph_forced"), "step3f"),
        # token partitions, rows long enough for the two-launch selection (its histogram lives in the
        # workspace and must be left cleared by every replay), partial page masks in the attention
        "long_token_rows": (c0.with_(seq_lens=(20000, 17001), num_q_heads=8, num_kv_heads=2, partition_tokens=1,
                                     score_kind=synth.SCORE_SKETCH, topk=300, sink_pages=1, recent_pages=1,
                                     name="graph_tokens"), "step"),
        # the same rows with stages 1+2 in one call: stage 1 fills the histogram stage 2 clears
        "long_token_rows_stage12_call": (c0.with_(seq_lens=(20000, 17001), num_q_heads=8, num_kv_heads=2,
                                                  partition_tokens=1, score_kind=synth.SCORE_SKETCH, topk=300,
                                                  sink_pages=1, recent_pages=1, name="graph_tokens12"), "step12"),
        # and with stages 1-3 in one call (the launch that finishes stage 2 resolves)
        "long_token_rows_stage123_call": (c0.with_(seq_lens=(20000, 17001), num_q_heads=8, num_kv_heads=2,
                                                   partition_tokens=1, score_kind=synth.SCORE_SKETCH, topk=300,
                                                   sink_pages=1, recent_pages=1, name="graph_tokens123"), "step123"),
    }


@pytest.mark.parametrize("name", list(_workloads()))
def test_step_replays_from_a_graph(name):
    w, how = _workloads()[name]
    data = synth.generate(w)
    natural = torch.from_numpy(data.pool_bits.view(np.int16).copy()).to("cuda:0").view(torch.bfloat16)
    layer = runner.LayerState.from_natural_pool(w, data.slot_of, natural, decode_splits=2)
    if w.score_kind == synth.SCORE_SKETCH:
        layer.set_channels(synth.sketch_channels(data))
    layer.build_summaries()
    layer.step3 = getattr(layer, how)              # the step as this workload runs it
    qs = [torch.from_numpy(synth.make_queries(w, 100 + i).view(np.int16)).to("cuda:0").view(torch.bfloat16)
          for i in range(3)]
    q_static = qs[0].clone()
    eager = []
    for q in qs:
        layer.step3(q)
        torch.cuda.synchronize()
        eager.append((layer.out.clone(), layer.sel.clone(), layer.slots.clone()))
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        layer.step3(q_static)                      # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(s)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        layer.step3(q_static)
    for rep in range(6):
        i = rep % 3
        q_static.copy_(qs[i])
        layer.out.fill_(9.0)                       # eager work between replays
        layer.sel.fill_(-3)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert layer.status() == 0
        assert torch.equal(layer.out.view(torch.int16), eager[i][0].view(torch.int16)), f"replay {rep}"
        assert torch.equal(layer.sel, eager[i][1]) and torch.equal(layer.slots, eager[i][2])


def test_budget_step_replays_with_the_workspace_step_counter():
    """A budget-mode step recorded once: the replacement policy must see step 0, 1, 2, ... on the
    replays (the workspace's counter), not the value present at capture.  A twin layer run eagerly
    with explicit steps gives the expected slots, misses and outputs, bit for bit; the timestamp
    range is short so that demotion (which depends on the step) happens within the trace."""
    w = synth.config4().with_(seq_lens=(16 * 700, 16 * 420), num_q_heads=8, num_kv_heads=2, topk=24, sink_pages=2,
                              recent_pages=3, name="graph_budget")
    mk = lambda: hier.HierLayer(w, budget_frac=0.06, n_ts=4, copy_mode="gather")
    ref, cap = mk(), mk()
    qs = [ref.q0]
    for s in range(9):
        bits = qs[-1].view(torch.int16).cpu().numpy().view(np.uint16)
        qs.append(torch.from_numpy(synth.next_query_ar1(bits, 0.7, w.seed + 50 + s).view(np.int16)).to("cuda:0")
                  .view(torch.bfloat16))
    eager = []
    for s, q in enumerate(qs):
        ref.step(q, s, count=False)
        torch.cuda.synchronize()
        assert ref.status() == 0
        eager.append(tuple(t.clone() for t in (ref.slots, ref.npages, ref.nmiss, ref.miss_pages, ref.miss_slots, ref.out)))
    q_static = qs[0].clone()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        cap.step(q_static, 12345, count=False, device_step=True)      # the step argument is not used
    for s, q in enumerate(qs):
        q_static.copy_(q)
        cap.out.fill_(3.0)                                             # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert cap.status() == 0
        got = (cap.slots, cap.npages, cap.nmiss, cap.miss_pages, cap.miss_slots)
        for a, b in zip(got, eager[s][:5]):
            assert torch.equal(a, b), f"replay {s}"
        assert torch.equal(cap.out.view(torch.int16), eager[s][5].view(torch.int16)), f"replay {s}"
    # the counter can be set: going back to step 0 semantics is not needed here, only that it reads back
    cap.spin.set_step(cap.ws, 7)
    torch.cuda.synchronize()
    assert int(cap.ws.view(torch.int32)[1].item()) == 7
