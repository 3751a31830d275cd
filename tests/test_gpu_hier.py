"""End-to-end budget mode on a small hierarchical workload: full KV in pinned
host memory, bucketed LRU (or the set-associative variant) on the device, misses copied in (both copiers), then
attention.  Every step is checked against the oracle: selection on the device's
fp32 scores, slots and miss list against the step-by-step LRU, and attention
against fp64 attention over the LOGICAL pages -- which only holds if every
missed page was copied into exactly the slot the LRU assigned."""
import numpy as np
import pytest
import torch

from oracle import attend, bf16, lru, select
from paper_2604_26837_amd import hier, synth

pytestmark = pytest.mark.gpu
ATOL, RTOL = 2e-2, 1e-2


def _small():
    return synth.config4().with_(seq_lens=(2048, 5000, 9001), num_q_heads=8, num_kv_heads=2, topk=24,
                                 sink_pages=2, recent_pages=3, name="hier_small")


# the last two cases: the request's pages scattered over the host pool behind a CPU page table
# (the case with overlap: attention over the hits runs beside the copy kernel, a second pass takes the misses)
@pytest.mark.parametrize("copy_mode,exact,policy,scatter,overlap", [
    ("memcpy", False, 0, False, False), ("gather", False, 0, False, False), ("gather", True, 0, False, False),
    ("gather", False, 1, False, False), ("gather", False, 0, True, False), ("memcpy", False, 0, True, False),
    ("gather", False, 0, False, True), ("gather", False, 1, True, True)])
def test_steps_match_oracle(copy_mode, exact, policy, scatter, overlap):
    w = _small()
    n_ts = 6                      # small range: demotion kicks in within the trace
    layer = hier.HierLayer(w, budget_frac=0.06, n_ts=n_ts, evict_exact=exact, copy_mode=copy_mode, keep_natural=True,
                           lru_policy=policy, scatter_host_pages=scatter, overlap_hits=overlap)
    rows, g = w.rows, w.group
    caches = [lru.RowCache(layer.budgets[r]) for r in range(rows)]
    nat = [n.view(torch.int16).numpy().view(np.uint16) for n in layer.natural]      # per request [slots][2][16][D]
    q = layer.q0
    trace = [[] for _ in range(rows)]
    for step in range(14):
        layer.step(q, step)
        torch.cuda.synchronize()
        assert layer.status() == 0
        scores = layer.scores.cpu().numpy()
        sel, nsel = layer.sel.cpu().numpy(), layer.nsel.cpu().numpy()
        slots, npages = layer.slots.cpu().numpy(), layer.npages.cpu().numpy()
        mp, ms, nm = layer.miss_pages.cpu().numpy(), layer.miss_slots.cpu().numpy(), layer.nmiss.cpu().numpy()
        out = bf16.decode(layer.out.view(torch.int16).cpu().numpy().view(np.uint16))
        q_bits = q.view(torch.int16).cpu().numpy().view(np.uint16)
        for r in range(rows):
            b, h = divmod(r, w.num_kv_heads)
            n, P = w.seq_lens[b], w.partitions(b)
            base = w.num_kv_heads * int(layer.part_offsets_np[b]) + h * int(layer.part_offsets_np[b + 1] - layer.part_offsets_np[b])
            want_sel = select.select_topk(scores[base:base + P], n, 16, 16, w.topk, True, w.sink_pages, w.recent_pages)
            assert sel[r, :nsel[r]].tolist() == want_sel
            trace[r].append(want_sel)
            if policy == 1:
                want_slots, want_miss, _ = lru.setassoc_step(caches[r], want_sel, step, n_ts, row=r)
            else:
                want_slots, want_miss, _ = lru.lru_step(caches[r], want_sel, step, n_ts, evict_exact=exact)
            sb = int(layer.slot_base_np[r])
            assert slots[r, :npages[r]].tolist() == [sb + s for s in want_slots], f"step {step} row {r}"
            assert mp[r, :nm[r]].tolist() == [p for p, _ in want_miss]
            assert ms[r, :nm[r]].tolist() == [sb + s for _, s in want_miss]
            if overlap:       # the masks of the two passes: every page in exactly one of them
                missed = {p for p, _ in want_miss}
                full = [(1 << min(16, n - 16 * p)) - 1 for p in want_sel]
                mh = layer.mask_hits.cpu().numpy().view(np.uint16)[r, :npages[r]].tolist()
                mm = layer.mask_misses.cpu().numpy().view(np.uint16)[r, :npages[r]].tolist()
                assert mh == [0 if p in missed else f for p, f in zip(want_sel, full)]
                assert mm == [f if p in missed else 0 for p, f in zip(want_sel, full)]
            # attention over the logical pages
            pages = bf16.decode(nat[b][layer.natural_slot_of[b][h][np.asarray(want_sel, dtype=np.int64)]])
            masks = [(1 << min(16, n - 16 * p)) - 1 for p in want_sel]
            ks, vs = attend.gather_tokens(pages[:, 0], pages[:, 1], masks)
            qh = bf16.decode(q_bits[b, h * g:(h + 1) * g])
            ref, _ = attend.attend(qh, ks, vs, layer.scale)
            o = out[b, h * g:(h + 1) * g]
            assert np.all(np.abs(o - ref) <= ATOL + RTOL * np.abs(ref)), f"step {step} row {r}: {np.abs(o - ref).max()}"
        q = torch.from_numpy(synth.next_query_ar1(q_bits, 0.9, w.seed + 5000 + step).view(np.int16)).to(q.device).view(torch.bfloat16)
    overall, warm = layer.hit_rates()
    # compulsory misses and the clairvoyant policy bound the measured misses from below
    compulsory = sum(len(set().union(*[set(x) for x in t])) for t in trace)
    belady = sum(lru.belady_min_misses(trace[r], layer.budgets[r]) for r in range(rows))
    assert compulsory <= belady <= layer.stats["misses"]
    assert 0.0 < warm < 1.0
    print(f"{copy_mode} exact={exact}: hit rate overall {overall:.3f}, after step 0 {warm:.3f}")


def _other_granularities():
    base = synth.config4().with_(num_q_heads=8, num_kv_heads=2)
    return {
        "blocks64": base.with_(seq_lens=(2048, 5000, 9001), partition_tokens=64, topk=5, sink_pages=2, recent_pages=3,
                               name="hier_b64"),
        "repmax128": base.with_(seq_lens=(6000, 128 * 40 + 9), partition_tokens=128, score_kind=synth.SCORE_REPMAX,
                                topk=3, topk_includes_forced=False, sink_pages=1, recent_pages=4, block_mean_std=0.5,
                                name="hier_rep"),
        "quarter_pages": base.with_(seq_lens=(3000, 1234), partition_tokens=4, topk=60, sink_pages=1, recent_pages=1,
                                    name="hier_q"),
    }


@pytest.mark.parametrize("policy", [0, 1])
@pytest.mark.parametrize("name", list(_other_granularities()))
def test_other_granularities_under_a_budget(name, policy):
    """Blocks, blocks with representative keys and sub-page partitions with the full KV on the
    host: selection on the device's scores, page list, masks, replacement state and miss list
    against the oracle, attention over the logical tokens (which needs every missed page copied
    into the slot the policy assigned, and for sub-page partitions the token-major slot layout
    to survive the trip through host memory)."""
    _check_hier_steps(_other_granularities()[name], policy, n_ts=5, budget_frac=0.05, steps=10, scatter=False)


@pytest.mark.parametrize("seed", range(12))
def test_random_workloads_under_a_budget(seed):
    """The whole path with the KV on the host for randomly drawn partition sizes, summary kinds, group
    sizes, contexts, top-k, windows, timestamp ranges, policies and host page placement."""
    rng = np.random.default_rng(8000 + seed)
    kind = int(rng.choice([synth.SCORE_MINMAX, synth.SCORE_MINMAX, synth.SCORE_REPMAX]))
    reps = int(rng.choice([1, 2, 4])) if kind == synth.SCORE_REPMAX else 4
    tps = [1, 2, 4, 8, 16, 16, 32, 64, 128] if kind == synth.SCORE_MINMAX else [t for t in (4, 8, 16, 32, 64, 128) if t % reps == 0]
    tp = int(rng.choice(tps))
    hkv, g = int(rng.choice([1, 2])), int(rng.choice([1, 2, 4, 5, 8]))
    lens = tuple(int(x) for x in rng.integers(300, 6000, size=int(rng.integers(1, 4))))
    max_parts = max(-(-n // tp) for n in lens)
    w = synth.config4().with_(seq_lens=lens, num_q_heads=g * hkv, num_kv_heads=hkv, partition_tokens=tp,
                              score_kind=kind, reps_per_partition=reps, topk=int(rng.integers(1, min(max_parts, 40) + 1)),
                              topk_includes_forced=bool(rng.integers(0, 2)), sink_pages=int(rng.integers(0, 3)),
                              recent_pages=int(rng.integers(1, 4)),
                              block_mean_std=0.5 if kind == synth.SCORE_REPMAX else 0.0, name=f"hier_random{seed}")
    policy, n_ts = int(rng.integers(0, 2)), int(rng.integers(2, 8))
    print(f"seed {seed}: kind {kind} reps {reps} tp {tp} group {g} kv {hkv} lens {lens} topk {w.topk} "
          f"incl {w.topk_includes_forced} sink {w.sink_pages} recent {w.recent_pages} policy {policy} n_ts {n_ts}", flush=True)
    _check_hier_steps(w, policy, n_ts, budget_frac=float(rng.uniform(0.02, 0.2)), steps=8, scatter=bool(rng.integers(0, 2)))


def _check_hier_steps(w, policy, n_ts, budget_frac, steps, scatter):
    from oracle import resolve as oresolve
    layer = hier.HierLayer(w, budget_frac=budget_frac, n_ts=n_ts, copy_mode="gather", keep_natural=True,
                           lru_policy=policy, scatter_host_pages=scatter)
    rows, g, tp = w.rows, w.group, w.partition_tokens
    caches = [lru.RowCache(layer.budgets[r]) for r in range(rows)]
    nat = [n.view(torch.int16).numpy().view(np.uint16) for n in layer.natural]
    q = layer.q0
    for step in range(steps):
        layer.step(q, step)
        torch.cuda.synchronize()
        assert layer.status() == 0, f"step {step}"
        scores = layer.scores.cpu().numpy()
        sel, nsel = layer.sel.cpu().numpy(), layer.nsel.cpu().numpy()
        slots, npages = layer.slots.cpu().numpy(), layer.npages.cpu().numpy()
        page_ids = layer.page_ids.cpu().numpy()
        masks = layer.valid_mask.cpu().numpy().view(np.uint16)
        ms, nm = layer.miss_slots.cpu().numpy(), layer.nmiss.cpu().numpy()
        out = bf16.decode(layer.out.view(torch.int16).cpu().numpy().view(np.uint16))
        q_bits = q.view(torch.int16).cpu().numpy().view(np.uint16)
        for r in range(rows):
            b, h = divmod(r, w.num_kv_heads)
            n, P = w.seq_lens[b], w.partitions(b)
            base = w.num_kv_heads * int(layer.part_offsets_np[b]) + h * int(layer.part_offsets_np[b + 1] - layer.part_offsets_np[b])
            want_sel = select.select_topk(scores[base:base + P], n, 16, tp, w.topk, w.topk_includes_forced,
                                          w.sink_pages, w.recent_pages)
            assert sel[r, :nsel[r]].tolist() == want_sel, f"step {step} row {r}"
            pm = oresolve.selected_pages(want_sel, n, 16, tp, w.sink_pages, w.recent_pages)
            pages = sorted(pm)
            if policy:
                want_slots, want_miss, _ = lru.setassoc_step(caches[r], pages, step, n_ts, row=r)
            else:
                want_slots, want_miss, _ = lru.lru_step(caches[r], pages, step, n_ts)
            sb = int(layer.slot_base_np[r])
            assert page_ids[r, :npages[r]].tolist() == pages
            assert masks[r, :npages[r]].tolist() == [pm[p] for p in pages]
            assert slots[r, :npages[r]].tolist() == [sb + s for s in want_slots], f"step {step} row {r}"
            assert ms[r, :nm[r]].tolist() == [sb + s for _, s in want_miss]
            pg = bf16.decode(nat[b][layer.natural_slot_of[b][h][np.asarray(pages, dtype=np.int64)]])
            ks, vs = attend.gather_tokens(pg[:, 0], pg[:, 1], [pm[p] for p in pages])
            ref, _ = attend.attend(bf16.decode(q_bits[b, h * g:(h + 1) * g]), ks, vs, layer.scale)
            o = out[b, h * g:(h + 1) * g]
            assert np.all(np.abs(o - ref) <= ATOL + RTOL * np.abs(ref)), f"step {step} row {r}: {np.abs(o - ref).max()}"
        q = torch.from_numpy(synth.next_query_ar1(q_bits, 0.9, w.seed + 6000 + step).view(np.int16)).to(q.device).view(torch.bfloat16)
    overall, warm = layer.hit_rates()
    assert 0.0 <= warm <= 1.0


def test_cpu_page_table_entries_out_of_range_are_reported_not_followed():
    """A CPU page table entry outside the host pool must raise the status word and skip
    the page (nothing is read out of bounds), in the copy kernel and in the host-driven copier."""
    w = _small()
    layer = hier.HierLayer(w, budget_frac=0.06, n_ts=6, copy_mode="gather", scatter_host_pages=True)
    pool_pages = layer.host_kv.shape[0]
    layer.cpu_table[:] = pool_pages + 5                       # every entry points past the pool
    layer.step(layer.q0, 0)
    torch.cuda.synchronize()
    assert layer.status() == -7                               # SPIN_ERR_SLOT_RANGE
    layer.spin.workspace_init(layer.ws)
    layer.cpu_table[:] = -1
    h = torch.zeros_like(layer.nmiss).cpu()
    h_pages, h_slots = layer.miss_pages.cpu(), layer.miss_slots.cpu()
    h.copy_(layer.nmiss)
    from paper_2604_26837_amd.binding import SpinError
    assert int(h.sum()) > 0                                   # step 0 is all misses
    with pytest.raises(SpinError):
        layer.spin.copy_misses_host(w.batch, layer.host_kv, layer.host_row_base, h, h_pages, h_slots, layer.kv_pool,
                                    layer.copy_stream)
