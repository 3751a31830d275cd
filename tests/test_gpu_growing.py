"""Decode with a growing context under an HBM budget: every step appends one
token per request (decode-time Index), a page whose last token has just been
written is copied back to the pinned host copy (Offload's copy), and pages the
bucketed LRU evicted are fetched again later (Retrieve).  Each step is checked
against the oracle on the logical K/V the test keeps on the CPU: selection on
the device's fp32 scores, replacement state and miss list bit-exact, attention
over the logical pages.  Attention only matches if appended tokens survive the
round trip slot -> host page -> (eviction) -> another slot."""
import numpy as np
import pytest
import torch

from gpu_harness import bits_to_bf16
from oracle import attend, bf16, index, lru, select
from paper_2604_26837_amd import hier, synth

pytestmark = pytest.mark.gpu
ATOL, RTOL = 2e-2, 1e-2
DEV = "cuda:0"


@pytest.mark.parametrize("scatter", [False, True])
def test_append_offload_retrieve_over_many_steps(scatter):
    final = (1200, 2100)
    start = (1100, 2043)
    steps = 57                                     # crosses several page boundaries in both requests
    w = synth.config4().with_(seq_lens=final, num_q_heads=8, num_kv_heads=2, topk=16, sink_pages=1,
                              recent_pages=2, name="growing")
    n_ts = 5
    # scatter: the requests' pages lie anywhere in the host pool, found through the CPU page table
    layer = hier.HierLayer(w, budget_frac=0.02, n_ts=n_ts, copy_mode="gather", keep_natural=True,
                           scatter_host_pages=scatter)
    hpage = (lambda i: i) if layer.cpu_table is None else (lambda i: int(layer.cpu_table[i]))
    sp, hkv, g, rows = layer.spin, w.num_kv_heads, w.group, w.rows
    # logical K/V per row in token order (bf16 bits), the truth the appended tokens are taken from
    nat = [n.view(torch.int16).numpy().view(np.uint16) for n in layer.natural]
    logical = {}
    for r in range(rows):
        b, h = divmod(r, hkv)
        pg = nat[b][layer.natural_slot_of[b][h]]                       # [pages][2][16][D]
        logical[r] = (pg[:, 0].reshape(-1, w.head_dim).copy(), pg[:, 1].reshape(-1, w.head_dim).copy())
    # the host copy and the summaries beyond `start` are wiped: those tokens do not exist yet
    cur = list(start)
    for r in range(rows):
        b = r // hkv
        lo = int(layer.host_row_base_np[r])
        first_partial = cur[b] // 16
        for i in range(lo + first_partial, lo + w.pages(b)):
            layer.host_kv[hpage(i)].zero_()
        # tokens of the partial tail page that already exist stay; the rest of that page is zero
        if cur[b] % 16:
            k, v = logical[r]
            page = np.zeros((2, 16, w.head_dim), dtype=np.uint16)
            page[0, :cur[b] % 16] = k[first_partial * 16: cur[b]]
            page[1, :cur[b] % 16] = v[first_partial * 16: cur[b]]
            tmp = torch.zeros((1, 4096), dtype=torch.bfloat16, device=DEV)
            ids = torch.zeros(1, dtype=torch.int32, device=DEV)
            pk = bits_to_bf16(page)
            sp.pack_kv_pages(pk[0:1].contiguous(), pk[1:2].contiguous(), ids, tmp)
            torch.cuda.synchronize()
            layer.host_kv[hpage(lo + first_partial)].copy_(tmp[0].cpu())
    # summaries of the shorter contexts, built from a temporary all-resident copy of the host pages
    layer.seq_lens.copy_(torch.tensor(cur, dtype=torch.int32))
    layer.rebuild_summaries_from_host()
    caches = [lru.RowCache(layer.budgets[r]) for r in range(rows)]
    q = layer.q0
    one = torch.ones(rows, dtype=torch.int32, device=DEV)
    for step in range(steps):
        # the token at position cur[b] arrives; the step attends to cur[b] + 1 tokens
        k_new = np.stack([np.stack([logical[b * hkv + h][0][cur[b]] for h in range(hkv)]) for b in range(w.batch)])
        v_new = np.stack([np.stack([logical[b * hkv + h][1][cur[b]] for h in range(hkv)]) for b in range(w.batch)])
        k_dev = torch.from_numpy(k_new.view(np.int16)).to(DEV).view(torch.bfloat16)
        v_dev = torch.from_numpy(v_new.view(np.int16)).to(DEV).view(torch.bfloat16)
        done_pages = layer.step_append(q, step, k_dev, v_dev)
        torch.cuda.synchronize()
        assert layer.status() == 0, f"step {step}"
        new_len = [c + 1 for c in cur]
        scores = layer.scores.cpu().numpy()
        sel, nsel = layer.sel.cpu().numpy(), layer.nsel.cpu().numpy()
        slots, npages = layer.slots.cpu().numpy(), layer.npages.cpu().numpy()
        mp, ms, nm = layer.miss_pages.cpu().numpy(), layer.miss_slots.cpu().numpy(), layer.nmiss.cpu().numpy()
        out = bf16.decode(layer.out.view(torch.int16).cpu().numpy().view(np.uint16))
        q_bits = q.view(torch.int16).cpu().numpy().view(np.uint16)
        for r in range(rows):
            b, h = divmod(r, hkv)
            n, P = new_len[b], -(-new_len[b] // 16)
            base = layer.part_offsets_np[b] * hkv + h * int(layer.part_offsets_np[b + 1] - layer.part_offsets_np[b])
            want_sel = select.select_topk(scores[base:base + P], n, 16, 16, w.topk, True, w.sink_pages, w.recent_pages)
            assert sel[r, :nsel[r]].tolist() == want_sel, f"step {step} row {r}"
            want_slots, want_miss, _ = lru.lru_step(caches[r], want_sel, step, n_ts)
            sb = int(layer.slot_base_np[r])
            assert slots[r, :npages[r]].tolist() == [sb + s for s in want_slots], f"step {step} row {r}"
            assert mp[r, :nm[r]].tolist() == [p for p, _ in want_miss]
            assert ms[r, :nm[r]].tolist() == [sb + s for _, s in want_miss]
            k, v = logical[r]
            K = bf16.decode(k[:n]); V = bf16.decode(v[:n])
            toks = np.concatenate([np.arange(16 * p, min(16 * p + 16, n)) for p in want_sel])
            ref, _ = attend.attend(bf16.decode(q_bits[b, h * g:(h + 1) * g]), K[toks], V[toks], layer.scale)
            o = out[b, h * g:(h + 1) * g]
            assert np.all(np.abs(o - ref) <= ATOL + RTOL * np.abs(ref)), f"step {step} row {r}: {np.abs(o - ref).max()}"
        assert done_pages == sum(1 for b in range(w.batch) if new_len[b] % 16 == 0) * hkv
        cur = new_len
        q = torch.from_numpy(synth.next_query_ar1(q_bits, 0.9, w.seed + 9000 + step).view(np.int16)).to(DEV).view(torch.bfloat16)
    # summaries after all appends: exactly those of the grown contexts
    raw = layer.summaries.cpu().numpy().view(np.uint16).reshape(-1, 32, 16, 8).transpose(0, 2, 1, 3).reshape(-1, 256)
    for r in range(rows):
        b, h = divmod(r, hkv)
        base = layer.part_offsets_np[b] * hkv + h * int(layer.part_offsets_np[b + 1] - layer.part_offsets_np[b])
        mins, maxs = index.minmax_summaries(bf16.decode(logical[r][0][:cur[b]]), cur[b], 16)
        want = np.concatenate([maxs, mins], axis=1)
        got = bf16.decode(raw[base: base + want.shape[0]])
        assert np.array_equal(got, want), f"row {r}"
    # every page completed during the run sits in the host copy exactly as packing it would write it
    checked = 0
    for r in range(rows):
        b = r // hkv
        lo = int(layer.host_row_base_np[r])
        k, v = logical[r]
        for pg in range(start[b] // 16, cur[b] // 16):
            page = np.stack([k[16 * pg: 16 * pg + 16], v[16 * pg: 16 * pg + 16]])
            pk = bits_to_bf16(page)
            tmp = torch.zeros((1, 4096), dtype=torch.bfloat16, device=DEV)
            sp.pack_kv_pages(pk[0:1].contiguous(), pk[1:2].contiguous(), torch.zeros(1, dtype=torch.int32, device=DEV), tmp)
            torch.cuda.synchronize()
            assert torch.equal(tmp[0].cpu().view(torch.int16), layer.host_kv[hpage(lo + pg)].view(torch.int16)), (r, pg)
            checked += 1
    assert checked >= 3 * rows
    overall, warm = layer.hit_rates()
    assert 0.0 < warm < 1.0                       # pages were evicted and fetched again during the run
