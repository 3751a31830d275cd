"""GPU parity of budget-mode resolve (bucketed LRU and the set-associative
variant) against the step-by-step oracle: slots of every selected page, the miss list, timestamps and the
forward/reverse tables, bit-exact, over multi-step traces."""
import numpy as np
import pytest
import torch

from oracle import lru
from paper_2604_26837_amd import binding, synth, tables

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


class Budget:
    """Device state of budget mode for a workload with page partitions; the
    selection of each step is fed in directly (stage 3b takes `sel` as input)."""

    def __init__(self, w, budgets, n_ts, evict_exact=False, policy=0, **cfg_over):
        self.w = w
        self.sp = binding.Spin.for_workload(w, lru_timestamps=n_ts, lru_evict_exact=int(evict_exact),
                                            lru_policy=policy, **cfg_over)
        sp = self.sp
        self.ws = sp.new_workspace(DEV)
        rows = w.rows
        self.budgets = budgets
        base = np.zeros(rows + 1, dtype=np.int32)
        base[1:] = np.cumsum(budgets)
        self.slot_base_np = base
        rng = np.stack([base[:-1], np.asarray(budgets, dtype=np.int32)], axis=1).astype(np.int32)
        self.slot_base = torch.from_numpy(np.ascontiguousarray(rng)).to(DEV)          # [rows][2] = {first, count}
        empty = [np.full((w.num_kv_heads, w.pages(b)), -1, dtype=np.int32) for b in range(w.batch)]
        d, l = tables.build_two_level(empty, sp.dir_stride, w.leaf_entries, allocate_all=True)
        self.dir = torch.from_numpy(d).to(DEV)
        self.leaf = torch.from_numpy(l).to(DEV)
        rev = np.zeros((int(base[-1]), 2), dtype=np.int32)
        rev[:, 0] = -1
        self.rev = torch.from_numpy(rev).to(DEV)
        self.seq_lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
        z = lambda *s, dt=torch.int32: torch.zeros(s, dtype=dt, device=DEV)
        self.sel = z(rows, sp.sel_stride)
        self.nsel = z(rows)
        self.slots, self.page_ids = z(rows, sp.page_stride), z(rows, sp.page_stride)
        self.mask = z(rows, sp.page_stride, dt=torch.int16)
        self.npages = z(rows)
        self.miss_pages, self.miss_slots = z(rows, sp.page_stride), z(rows, sp.page_stride)
        self.nmiss = z(rows)

    def step(self, step, selections):
        sp, w = self.sp, self.w
        sel = np.full((w.rows, sp.sel_stride), -1, dtype=np.int32)
        ns = np.zeros(w.rows, dtype=np.int32)
        for r, pages in enumerate(selections):
            sel[r, :len(pages)] = pages
            ns[r] = len(pages)
        self.sel.copy_(torch.from_numpy(sel))
        self.nsel.copy_(torch.from_numpy(ns))
        sp.resolve_slots(w.batch, step, self.sel, self.nsel, self.seq_lens, self.dir, self.leaf, self.slots,
                         self.page_ids, self.mask, self.npages, self.ws, rev_table=self.rev,
                         slot_base=self.slot_base, miss_pages=self.miss_pages, miss_slots=self.miss_slots,
                         nmiss=self.nmiss)
        torch.cuda.synchronize()
        return (self.slots.cpu().numpy(), self.npages.cpu().numpy(), self.miss_pages.cpu().numpy(),
                self.miss_slots.cpu().numpy(), self.nmiss.cpu().numpy())


def _trace(rng, rows, pages_per_row, k, steps, hot_frac=0.7):
    hot = [rng.choice(pages_per_row[r], size=min(3 * k, pages_per_row[r]), replace=False) for r in range(rows)]
    out = []
    for s in range(steps):
        cur = []
        for r in range(rows):
            kk = min(k, pages_per_row[r])
            nh = min(int(round(hot_frac * kk)), len(hot[r]))
            a = set(int(x) for x in rng.choice(hot[r], size=nh, replace=False))
            while len(a) < kk:
                a.add(int(rng.integers(0, pages_per_row[r])))
            cur.append(sorted(a))
        out.append(cur)
    return out


@pytest.mark.parametrize("n_ts,exact,budget_mult", [(64, False, 3.0), (64, True, 3.0), (4, False, 2.0),
                                                     (4, True, 1.2), (3, False, 1.0)])
def test_traces_match_oracle(n_ts, exact, budget_mult):
    k = 12
    w = synth.config0().with_(seq_lens=(1600, 700, 16 * 600 + 3), num_q_heads=4, num_kv_heads=2, topk=k,
                              sink_pages=0, recent_pages=0, name="lru")
    rows = w.rows
    pages_per_row = [w.pages(r // w.num_kv_heads) for r in range(rows)]
    rng = np.random.default_rng(n_ts * 7 + int(exact))
    budgets = [max(k, int(budget_mult * k) + r) for r in range(rows)]
    bd = Budget(w, budgets, n_ts, exact)
    caches = [lru.RowCache(budgets[r]) for r in range(rows)]
    trace = _trace(rng, rows, pages_per_row, k, 20)
    for step, selections in enumerate(trace):
        slots, npg, mpages, mslots, nmiss = bd.step(step, selections)
        assert bd.sp.poll_status(bd.ws) == 0
        rev = bd.rev.cpu().numpy()
        for r in range(rows):
            want_slots, want_miss, hits = lru.lru_step(caches[r], selections[r], step, n_ts, evict_exact=exact)
            base = int(bd.slot_base_np[r])
            assert npg[r] == len(selections[r])
            assert slots[r, :npg[r]].tolist() == [base + s for s in want_slots], f"step {step} row {r}"
            assert nmiss[r] == len(want_miss)
            assert mpages[r, :nmiss[r]].tolist() == [p for p, _ in want_miss]
            assert mslots[r, :nmiss[r]].tolist() == [base + s for _, s in want_miss]
            # reverse table: resident page and timestamp of every slot
            got_pages = rev[base:base + budgets[r], 0].tolist()
            assert got_pages == caches[r].page, f"step {step} row {r}"
            got_ts = [t if p >= 0 else 0 for p, t in zip(got_pages, rev[base:base + budgets[r], 1].tolist())]
            assert got_ts == [t if p >= 0 else 0 for p, t in zip(caches[r].page, caches[r].ts)]
        # forward table consistent with the reverse table
        leaf = bd.leaf.cpu().numpy()
        d = bd.dir.cpu().numpy()
        for r in range(rows):
            base = int(bd.slot_base_np[r])
            fwd = {}
            for ci in range(d.shape[1]):
                if d[r, ci] >= 0:
                    for i, s in enumerate(leaf[d[r, ci]]):
                        if s >= 0:
                            fwd[ci * w.leaf_entries + i] = int(s) - base
            assert fwd == caches[r].where


def test_budget_smaller_than_selection_is_reported():
    w = synth.config0().with_(seq_lens=(1600,), num_q_heads=4, num_kv_heads=2, topk=12, sink_pages=0,
                              recent_pages=0, name="lru_small")
    bd = Budget(w, [12, 5], 64)
    sel = [list(range(0, 24, 2)), list(range(1, 25, 2))]
    slots, npg, _, _, nmiss = bd.step(0, sel)
    assert bd.sp.poll_status(bd.ws) == -5
    assert npg[0] == 12 and npg[1] == 0 and nmiss[1] == 0
    assert (slots[1] == -1).all()


def test_large_row_many_slots():
    """A 256K-token row with a 4096-slot budget, 128 pages per step."""
    w = synth.config0().with_(seq_lens=(262144,), num_q_heads=4, num_kv_heads=1, topk=128, sink_pages=4,
                              recent_pages=8, name="lru_big")
    bd = Budget(w, [4096], 64)
    cache = lru.RowCache(4096)
    rng = np.random.default_rng(3)
    trace = _trace(rng, 1, [16384], 128, 40, hot_frac=0.8)
    for step, selections in enumerate(trace):
        slots, npg, mpages, mslots, nmiss = bd.step(step, selections)
        want_slots, want_miss, _ = lru.lru_step(cache, selections[0], step, 64)
        assert slots[0, :npg[0]].tolist() == want_slots
        assert mslots[0, :nmiss[0]].tolist() == [s for _, s in want_miss]
    assert bd.sp.poll_status(bd.ws) == 0


def _check_step(bd, caches, budgets, selections, step, n_ts, out):
    slots, npg, mpages, mslots, nmiss = out
    rev = bd.rev.cpu().numpy()
    hops = 0
    for r in range(bd.w.rows):
        want_slots, want_miss, hits = lru.setassoc_step(caches[r], selections[r], step, n_ts, row=r)
        base = int(bd.slot_base_np[r])
        sets = budgets[r] // 8
        hops += sum(1 for p, s in want_miss if s // 8 != lru.mix32(r, p) % sets)
        assert npg[r] == len(selections[r])
        assert slots[r, :npg[r]].tolist() == [base + s for s in want_slots], f"step {step} row {r}"
        assert nmiss[r] == len(want_miss)
        assert mpages[r, :nmiss[r]].tolist() == [p for p, _ in want_miss]
        assert mslots[r, :nmiss[r]].tolist() == [base + s for _, s in want_miss], f"step {step} row {r}"
        got_pages = rev[base:base + budgets[r], 0].tolist()
        assert got_pages == caches[r].page, f"step {step} row {r}"
        got_ts = [t if p >= 0 else 0 for p, t in zip(got_pages, rev[base:base + budgets[r], 1].tolist())]
        assert got_ts == [t if p >= 0 else 0 for p, t in zip(caches[r].page, caches[r].ts)]
    return hops


@pytest.mark.parametrize("n_ts,budget_mult,k", [(64, 3.0, 12), (4, 2.0, 12), (3, 1.0, 16), (64, 1.15, 28)])
def test_set_associative_traces_match_oracle(n_ts, budget_mult, k):
    w = synth.config0().with_(seq_lens=(1600, 700, 16 * 600 + 3), num_q_heads=4, num_kv_heads=2, topk=k,
                              sink_pages=0, recent_pages=0, name="lru_sa")
    rows = w.rows
    pages_per_row = [w.pages(r // w.num_kv_heads) for r in range(rows)]
    rng = np.random.default_rng(n_ts * 11 + k)
    # budgets that are not multiples of 8 leave up to 7 slots unused
    budgets = [max(8 * -(-k // 8), int(budget_mult * k) + r) for r in range(rows)]
    bd = Budget(w, budgets, n_ts, policy=1)
    caches = [lru.RowCache(budgets[r]) for r in range(rows)]
    trace = _trace(rng, rows, pages_per_row, k, 24)
    hops = 0
    for step, selections in enumerate(trace):
        out = bd.step(step, selections)
        assert bd.sp.poll_status(bd.ws) == 0
        hops += _check_step(bd, caches, budgets, selections, step, n_ts, out)
        leaf = bd.leaf.cpu().numpy()
        d = bd.dir.cpu().numpy()
        for r in range(rows):
            base = int(bd.slot_base_np[r])
            fwd = {}
            for ci in range(d.shape[1]):
                if d[r, ci] >= 0:
                    for i, s in enumerate(leaf[d[r, ci]]):
                        if s >= 0:
                            fwd[ci * w.leaf_entries + i] = int(s) - base
            assert fwd == caches[r].where
    if budget_mult < 1.5:
        assert hops > 0          # tight budgets reach the probing path (one lane walks the miss list)


def test_set_associative_large_row_and_errors():
    w = synth.config0().with_(seq_lens=(262144,), num_q_heads=4, num_kv_heads=1, topk=128, sink_pages=4,
                              recent_pages=8, name="lru_sa_big")
    bd = Budget(w, [4096], 64, policy=1)
    caches = [lru.RowCache(4096)]
    rng = np.random.default_rng(5)
    trace = _trace(rng, 1, [16384], 128, 30, hot_frac=0.8)
    for step, selections in enumerate(trace):
        out = bd.step(step, selections)
        _check_step(bd, caches, [4096], selections, step, 64, out)
    assert bd.sp.poll_status(bd.ws) == 0
    # fewer whole sets than the selection needs: reported, row emptied, tables untouched
    w2 = synth.config0().with_(seq_lens=(1600,), num_q_heads=4, num_kv_heads=2, topk=12, sink_pages=0,
                               recent_pages=0, name="lru_sa_small")
    bd2 = Budget(w2, [16, 15], 64, policy=1)
    sel = [list(range(0, 24, 2)), list(range(1, 25, 2))]
    slots, npg, _, _, nmiss = bd2.step(0, sel)
    assert bd2.sp.poll_status(bd2.ws) == -5
    assert npg[0] == 12 and npg[1] == 0 and nmiss[1] == 0
    assert (slots[1] == -1).all()
    assert (bd2.rev.cpu().numpy()[16:, 0] == -1).all()


# ---------------------------------------------------------------------------
# Budget mode for partitions other than one page each: the selection is first
# expanded to its page list (with masks), the replacement policy runs on pages.
# Oracle = the oracle's own expansion followed by the oracle's own policy.
# ---------------------------------------------------------------------------
def _granularity_workloads():
    c0 = synth.config0().with_(num_q_heads=4, num_kv_heads=2)
    return {
        "blocks128": c0.with_(seq_lens=(131 * 16 + 5, 40 * 128), partition_tokens=128, score_kind=synth.SCORE_REPMAX,
                              topk=4, topk_includes_forced=False, sink_pages=2, recent_pages=5, name="lru_blocks"),
        "blocks64": c0.with_(seq_lens=(3000, 1500), partition_tokens=64, topk=6, topk_includes_forced=True,
                             sink_pages=3, recent_pages=3, name="lru_b64"),
        "tokens": c0.with_(seq_lens=(2500, 900), partition_tokens=1, score_kind=synth.SCORE_SKETCH, topk=40,
                           sink_pages=1, recent_pages=2, name="lru_tokens"),
        "quarter_pages": c0.with_(seq_lens=(1000,), partition_tokens=4, topk=30, sink_pages=1, recent_pages=1,
                                  name="lru_q"),
    }


@pytest.mark.parametrize("policy", [0, 1])
@pytest.mark.parametrize("name", list(_granularity_workloads()))
def test_budget_mode_any_uniform_granularity(name, policy):
    _check_budget_steps(_granularity_workloads()[name], policy, n_ts=5, exact=False, seed=31 + policy, steps=16)


@pytest.mark.parametrize("policy,exact", [(0, False), (0, True), (1, False)])
def test_single_timestamp_value(policy, exact):
    """n = 1: every resident page carries timestamp 0, so the threshold bucket is always the only one
    (whole-bucket eviction empties everything not selected; the exact mode evicts by slot order)."""
    w = synth.config0().with_(seq_lens=(1500, 700), num_q_heads=2, num_kv_heads=2, topk=12, sink_pages=1,
                              recent_pages=2, name="lru_n1")
    _check_budget_steps(w, policy, n_ts=1, exact=exact, seed=5, steps=12)


def test_largest_timestamp_range_and_beyond():
    """n = 256 is the largest range the kernels take (the timestamp histogram lives in LDS); more is refused."""
    w = synth.config0().with_(seq_lens=(900,), num_q_heads=2, num_kv_heads=2, topk=10, name="lru_n256")
    _check_budget_steps(w, 0, n_ts=256, exact=False, seed=6, steps=10)
    with pytest.raises(binding.SpinError, match="UNSUPPORTED"):
        binding.Spin.for_workload(w, lru_timestamps=257)


@pytest.mark.parametrize("seed", range(24))
def test_budget_mode_random_workloads(seed):
    """Randomly drawn partition size, heads, ragged contexts, top-k, forced windows, timestamp range,
    policy and eviction mode: selection -> page list -> replacement against the oracle, step by step."""
    rng = np.random.default_rng(500 + seed)
    tp = int(rng.choice([1, 2, 4, 8, 16, 16, 16, 32, 64, 128]))
    hkv = int(rng.choice([1, 2, 3]))
    lens = tuple(int(x) for x in rng.integers(40, 4000, size=int(rng.integers(1, 4))))
    max_parts = max(-(-n // tp) for n in lens)
    topk = int(rng.integers(1, min(max(max_parts, 2), 48) + 1))
    policy = int(rng.integers(0, 2))
    w = synth.config0().with_(seq_lens=lens, num_q_heads=hkv, num_kv_heads=hkv, partition_tokens=tp, topk=topk,
                              topk_includes_forced=bool(rng.integers(0, 2)), sink_pages=int(rng.integers(0, 4)),
                              recent_pages=int(rng.integers(0, 5)), name=f"lru_random{seed}")
    n_ts = int(rng.integers(2, 9))
    exact = bool(rng.integers(0, 2)) and policy == 0
    print(f"seed {seed}: tp {tp} kv {hkv} lens {lens} topk {topk} policy {policy} n_ts {n_ts} exact {exact}", flush=True)
    _check_budget_steps(w, policy, n_ts, exact, seed=900 + seed, steps=int(rng.integers(8, 20)))


def _check_budget_steps(w, policy, n_ts, exact, seed, steps):
    from oracle import resolve as oresolve, select as oselect
    rows = w.rows
    probe = binding.Spin.for_workload(w, lru_timestamps=n_ts, lru_policy=policy)
    budgets = [probe.page_stride + 8 * (r % 3) + (0 if policy else r) for r in range(rows)]
    if policy:
        budgets = [8 * -(-b // 8) for b in budgets]
    bd = Budget(w, budgets, n_ts, evict_exact=exact, policy=policy)
    caches = [lru.RowCache(budgets[r]) for r in range(rows)]
    rng = np.random.default_rng(seed)
    for step in range(steps):
        selections, want_pages = [], []
        for r in range(rows):
            b = r // w.num_kv_heads
            n = w.seq_lens[b]
            P = w.partitions(b)
            scores = rng.standard_normal(P) + (np.arange(P) % 7 == step % 7) * 2.0   # drifting favourites
            sel = oselect.select_topk(scores, n, 16, w.partition_tokens, w.topk, w.topk_includes_forced,
                                      w.sink_pages, w.recent_pages)
            selections.append(sel)
            want_pages.append(oresolve.selected_pages(sel, n, 16, w.partition_tokens, w.sink_pages, w.recent_pages))
        slots, npg, mpages, mslots, nmiss = bd.step(step, selections)
        assert bd.sp.poll_status(bd.ws) == 0, f"step {step}"
        page_ids = bd.page_ids.cpu().numpy()
        masks = bd.mask.cpu().numpy().view(np.uint16)
        rev = bd.rev.cpu().numpy()
        for r in range(rows):
            pages = sorted(want_pages[r])
            if policy:
                want_slots, want_miss, _ = lru.setassoc_step(caches[r], pages, step, n_ts, row=r)
            else:
                want_slots, want_miss, _ = lru.lru_step(caches[r], pages, step, n_ts, evict_exact=exact)
            base = int(bd.slot_base_np[r])
            assert npg[r] == len(pages), f"step {step} row {r}"
            assert page_ids[r, :npg[r]].tolist() == pages
            assert masks[r, :npg[r]].tolist() == [want_pages[r][p] for p in pages]
            assert slots[r, :npg[r]].tolist() == [base + s for s in want_slots], f"step {step} row {r}"
            assert mpages[r, :nmiss[r]].tolist() == [p for p, _ in want_miss]
            assert mslots[r, :nmiss[r]].tolist() == [base + s for _, s in want_miss]
            assert rev[base:base + budgets[r], 0].tolist() == caches[r].page


def test_budget_mode_variable_length_partitions():
    from oracle import varpart
    w = synth.config0().with_(seq_lens=(4000, 2300), num_q_heads=4, num_kv_heads=2, partition_tokens=96, topk=7,
                              topk_includes_forced=True, sink_pages=2, recent_pages=3, name="lru_var")
    layouts = synth.variable_layouts(w, seed=77, min_tokens=5)
    rows, n_ts = w.rows, 4
    sp = binding.Spin.for_workload(w, lru_timestamps=n_ts, variable_partitions=1)
    budgets = [sp.page_stride + 3 * r for r in range(rows)]
    bd = Budget(w, budgets, n_ts, variable_partitions=1)
    offs = tables.part_offsets_from_counts([max(len(layouts[b][h][0]) for h in range(w.num_kv_heads))
                                            for b in range(w.batch)])
    count, first, toks = tables.partition_tables(layouts, offs, w.num_kv_heads)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)
    keep = [dev(offs), dev(count), dev(first), dev(toks)]
    bd.sp.set_partition_tables(*keep)
    caches = [lru.RowCache(budgets[r]) for r in range(rows)]
    rng = np.random.default_rng(9)
    for step in range(14):
        selections, wants = [], []
        for r in range(rows):
            b, h = divmod(r, w.num_kv_heads)
            fp, tk = layouts[b][h]
            scores = rng.standard_normal(len(fp))
            sel = varpart.select_topk(scores, fp, tk, 16, w.topk, True, w.sink_pages, w.recent_pages)
            selections.append(sel)
            pg, _, mk = varpart.resolve_slots(sel, fp, tk, 16, w.sink_pages, w.recent_pages,
                                              {(r, p): p for p in range(w.pages(b))}, r)
            wants.append((pg, mk))
        slots, npg, mpages, mslots, nmiss = bd.step(step, selections)
        assert bd.sp.poll_status(bd.ws) == 0, f"step {step}"
        page_ids = bd.page_ids.cpu().numpy()
        masks = bd.mask.cpu().numpy().view(np.uint16)
        for r in range(rows):
            pages, mk = wants[r]
            want_slots, want_miss, _ = lru.lru_step(caches[r], pages, step, n_ts)
            base = int(bd.slot_base_np[r])
            assert page_ids[r, :npg[r]].tolist() == pages, f"step {step} row {r}"
            assert masks[r, :npg[r]].tolist() == mk
            assert slots[r, :npg[r]].tolist() == [base + s for s in want_slots]
            assert mslots[r, :nmiss[r]].tolist() == [base + s for _, s in want_miss]
