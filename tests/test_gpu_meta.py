"""Metadata mechanisms around budget mode on the GPU: reclaiming slots from the
tail of a row's table against the oracle, and on-demand allocation of leaf
chunks from the bitmap-managed pool against a run with pre-allocated leaves."""
import numpy as np
import pytest
import torch

from oracle import lru
from paper_2604_26837_amd import synth

from test_gpu_lru import Budget, _trace, DEV

pytestmark = pytest.mark.gpu


def test_reclaim_tail_matches_oracle_over_a_trace():
    k = 10
    w = synth.config0().with_(seq_lens=(1600, 900), num_q_heads=4, num_kv_heads=2, topk=k, sink_pages=0,
                              recent_pages=0, name="reclaim")
    rows = w.rows
    cap = [40, 36, 44, 30]
    bd = Budget(w, cap, 64)
    caches = [lru.RowCache(c) for c in cap]
    rng = np.random.default_rng(4)
    trace = _trace(rng, rows, [w.pages(r // 2) for r in range(rows)], k, 24, hot_frac=0.6)
    plan = {6: [20, 36, 12, 30], 12: [40, 10, 44, 15], 18: [11, 36, 10, 30]}
    for step, selections in enumerate(trace):
        if step in plan:
            new = plan[step]
            bd.sp.reclaim_tail(w.batch, bd.slot_base, torch.tensor(new, dtype=torch.int32, device=DEV), bd.dir,
                               bd.leaf, bd.rev, bd.ws)
            for r in range(rows):
                lru.reclaim_tail(caches[r], new[r])
            rng_now = bd.slot_base.cpu().numpy()
            assert rng_now[:, 1].tolist() == new
        slots, npg, mpages, mslots, nmiss = bd.step(step, selections)
        assert bd.sp.poll_status(bd.ws) == 0
        rev = bd.rev.cpu().numpy()
        for r in range(rows):
            want_slots, want_miss, _ = lru.lru_step(caches[r], selections[r], step, 64)
            base = int(bd.slot_base_np[r])
            assert slots[r, :npg[r]].tolist() == [base + s for s in want_slots], f"step {step} row {r}"
            assert mslots[r, :nmiss[r]].tolist() == [base + s for _, s in want_miss]
            S = len(caches[r].page)
            assert rev[base:base + S, 0].tolist() == caches[r].page
            assert (rev[base + S: base + cap[r], 0] == -1).all()          # reclaimed slots are empty


@pytest.mark.parametrize("seed", range(12))
def test_reclaim_tail_random_plans(seed):
    """Random slot counts, selections, policies and shrink / grow plans: after every change the
    replacement state and every later step must equal the oracle's."""
    rng = np.random.default_rng(1200 + seed)
    policy = int(rng.integers(0, 2))
    k = int(rng.integers(4, 14))
    hkv = int(rng.choice([1, 2]))
    lens = tuple(int(x) for x in rng.integers(400, 2500, size=int(rng.integers(1, 3))))
    w = synth.config0().with_(seq_lens=lens, num_q_heads=hkv, num_kv_heads=hkv, topk=k, sink_pages=0, recent_pages=0,
                              name=f"reclaim_random{seed}")
    rows = w.rows
    unit = 8 if policy else 1
    cap = [unit * int(rng.integers(-(-2 * k // unit), -(-6 * k // unit) + 1)) for _ in range(rows)]
    n_ts = int(rng.integers(3, 9))
    bd = Budget(w, cap, n_ts, policy=policy)
    caches = [lru.RowCache(c) for c in cap]
    steps = 20
    trace = _trace(rng, rows, [w.pages(r // hkv) for r in range(rows)], k, steps, hot_frac=0.6)
    print(f"seed {seed}: policy {policy} k {k} kv {hkv} lens {lens} caps {cap} n_ts {n_ts}", flush=True)
    for step, selections in enumerate(trace):
        if step and rng.random() < 0.35:
            # a new count per row between "just enough for one step" and the full capacity
            new = [unit * int(rng.integers(-(-k // unit), cap[r] // unit + 1)) for r in range(rows)]
            bd.sp.reclaim_tail(w.batch, bd.slot_base, torch.tensor(new, dtype=torch.int32, device=DEV), bd.dir,
                               bd.leaf, bd.rev, bd.ws)
            for r in range(rows):
                lru.reclaim_tail(caches[r], new[r])
            assert bd.slot_base.cpu().numpy()[:, 1].tolist() == new
        slots, npg, mpages, mslots, nmiss = bd.step(step, selections)
        assert bd.sp.poll_status(bd.ws) == 0, f"step {step}"
        rev = bd.rev.cpu().numpy()
        for r in range(rows):
            if policy:
                want_slots, want_miss, _ = lru.setassoc_step(caches[r], selections[r], step, n_ts, row=r)
            else:
                want_slots, want_miss, _ = lru.lru_step(caches[r], selections[r], step, n_ts)
            base = int(bd.slot_base_np[r])
            assert slots[r, :npg[r]].tolist() == [base + s for s in want_slots], f"step {step} row {r}"
            assert mslots[r, :nmiss[r]].tolist() == [base + s for _, s in want_miss]
            S = len(caches[r].page)
            assert rev[base:base + S, 0].tolist() == caches[r].page
            assert (rev[base + S: base + cap[r], 0] == -1).all()


def test_leaves_allocated_on_demand_equal_preallocated_run():
    k = 16
    w = synth.config0().with_(seq_lens=(16 * 5000, 16 * 700, 16 * 2100), num_q_heads=4, num_kv_heads=2, topk=k,
                              sink_pages=2, recent_pages=3, leaf_entries=512, name="ondemand")
    rows = w.rows
    budgets = [64] * rows
    pre = Budget(w, budgets, 64)
    dyn = Budget(w, budgets, 64)
    chunks = 40                                       # fewer than the 2*(10+2+5)=34 ... enough for all ranges
    dyn.dir.fill_(-1)
    dyn.leaf = torch.full((chunks, w.leaf_entries), 12345, dtype=torch.int32, device=DEV)   # stale contents
    bitmap = torch.zeros((chunks + 31) // 32, dtype=torch.int32, device=DEV)
    rng = np.random.default_rng(9)
    # selections confined to a few ranges at first, so leaves appear gradually
    pages_per_row = [w.pages(r // 2) for r in range(rows)]
    trace = []
    for s in range(16):
        cur = []
        for r in range(rows):
            hi = min(pages_per_row[r], 600 + 450 * s)
            body = sorted(set(int(x) for x in rng.integers(2, max(hi - 3, 3), size=k - 5)))
            forced = [0, 1] + list(range(pages_per_row[r] - 3, pages_per_row[r]))
            cur.append(sorted(set(body + forced)))
        trace.append(cur)
    seen_chunks = 0
    for step, selections in enumerate(trace):
        a = pre.step(step, selections)
        # on-demand: upload the selection, allocate, then resolve
        sel = np.full((rows, dyn.sp.sel_stride), -1, dtype=np.int32)
        ns = np.zeros(rows, dtype=np.int32)
        for r, pg in enumerate(selections):
            sel[r, :len(pg)] = pg
            ns[r] = len(pg)
        dyn.sel.copy_(torch.from_numpy(sel))
        dyn.nsel.copy_(torch.from_numpy(ns))
        dyn.sp.alloc_leaves(w.batch, dyn.sel, dyn.nsel, dyn.seq_lens, dyn.dir, dyn.leaf, bitmap, dyn.ws)
        b = dyn.step(step, selections)
        assert dyn.sp.poll_status(dyn.ws) == 0
        for x, y in zip(a, b):
            assert np.array_equal(x, y), f"step {step}"
        d = dyn.dir.cpu().numpy()
        used = d[d >= 0]
        assert len(set(used.tolist())) == len(used)                       # no chunk handed out twice
        bits = int(sum(bin(int(v) & 0xFFFFFFFF).count("1") for v in bitmap.cpu().numpy()))
        assert bits == len(used) >= seen_chunks
        seen_chunks = len(used)
        # only ranges that were touched have leaves
        for r in range(rows):
            touched = {p // w.leaf_entries for t in trace[:step + 1] for p in t[r]}
            assert {ci for ci in range(d.shape[1]) if d[r, ci] >= 0} == touched
    assert 0 < seen_chunks <= 34
    dyn.sp.free_leaves(w.batch, dyn.dir, chunks, bitmap, dyn.ws)
    torch.cuda.synchronize()
    assert (bitmap.cpu().numpy() == 0).all() and (dyn.dir.cpu().numpy() == -1).all()


def test_leaf_pool_exhaustion_is_reported():
    w = synth.config0().with_(seq_lens=(16 * 3000,), num_q_heads=4, num_kv_heads=1, topk=8, sink_pages=0,
                              recent_pages=0, name="exhaust")
    bd = Budget(w, [32], 64)
    bd.dir.fill_(-1)
    bd.leaf = torch.full((2, 512), -1, dtype=torch.int32, device=DEV)
    bitmap = torch.zeros(1, dtype=torch.int32, device=DEV)
    sel = np.full((1, bd.sp.sel_stride), -1, dtype=np.int32)
    sel[0, :4] = [5, 600, 1200, 2500]                                     # four ranges, two chunks
    bd.sel.copy_(torch.from_numpy(sel))
    bd.nsel.fill_(4)
    bd.sp.alloc_leaves(1, bd.sel, bd.nsel, bd.seq_lens, bd.dir, bd.leaf, bitmap, bd.ws)
    assert bd.sp.poll_status(bd.ws) == -8
    assert (bd.dir.cpu().numpy() >= 0).sum() == 2 and int(bitmap.cpu().numpy()[0]) == 3
