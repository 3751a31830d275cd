"""Device-side guards of the C ABI: inputs the kernels' own range checks turn into a status word and a
defined output, and the documented behaviour for summary values outside the supported range."""
import numpy as np
import pytest
import torch

from oracle import attend, bf16, index, score
from paper_2604_26837_amd import binding, synth

pytestmark = pytest.mark.gpu
ATOL, RTOL = 2e-2, 1e-2


def _resolve(dw, sel_np, nsel_np):
    from gpu_harness import DEV, alloc_step_buffers
    if not hasattr(dw, "summaries"):
        alloc_step_buffers(dw)
    dw.sel.copy_(torch.from_numpy(sel_np).to(DEV))
    dw.nsel.copy_(torch.from_numpy(nsel_np).to(DEV))
    dw.spin.resolve_slots(dw.w.batch, 0, dw.sel, dw.nsel, dw.seq_lens, dw.dir, dw.leaf_pool, dw.slots, dw.page_ids,
                          dw.valid_mask, dw.npages, dw.ws)
    torch.cuda.synchronize()


@pytest.mark.parametrize("tp", [16, 64])
def test_selection_entry_outside_the_row_leaves_no_stale_page(tp):
    """An entry of `sel` that names no partition of the row: its output position must hold no page (not what an
    earlier step left there), SPIN_ERR_INVALID is reported, and attention covers exactly the valid entries."""
    from gpu_harness import DeviceWorkload, bf16_to_bits
    w = synth.config0().with_(seq_lens=(4096,), partition_tokens=tp, topk=12, sink_pages=0, recent_pages=0,
                              score_kind=synth.SCORE_REPMAX if tp > 16 else synth.SCORE_MINMAX, name="poison")
    dw = DeviceWorkload(synth.generate(w))
    sp, m, P = dw.spin, tp // 16, w.partitions(0)
    good = np.full((w.rows, sp.sel_stride), -1, dtype=np.int32)
    good[:, :12] = np.arange(3, 3 + 2 * 12, 2, dtype=np.int32)[None, :]
    nsel = np.full(w.rows, 12, dtype=np.int32)
    _resolve(dw, good, nsel)                                      # a valid step first: fills every position
    dw.check_ok()
    first = dw.page_ids.cpu().numpy().copy()
    bad = good.copy()
    bad[0, 5] = P + 7                                             # beyond the row's partitions
    bad[1, 2] = -4
    _resolve(dw, bad, nsel)
    assert binding.STATUS_NAMES[dw.spin.poll_status(dw.ws)] == "SPIN_ERR_INVALID"
    slots, pages = dw.slots.cpu().numpy(), dw.page_ids.cpu().numpy()
    masks, npages = dw.valid_mask.cpu().numpy().view(np.uint16), dw.npages.cpu().numpy()
    for r, i in ((0, 5), (1, 2)):
        lo, hi = i * m, (i + 1) * m
        assert (slots[r, lo:hi] == -1).all() and (pages[r, lo:hi] == -1).all() and (masks[r, lo:hi] == 0).all()
        keep = np.r_[0:lo, hi:12 * m]
        assert np.array_equal(pages[r, keep], first[r, keep])     # the valid entries are where they were
    assert (npages == 12 * m).all()
    # stage 4 skips the empty positions: attention over the valid entries only
    dw.spin.workspace_init(dw.ws)
    dw.spin.sparse_decode(w.batch, dw.q, dw.kv_pool, dw.slots, dw.valid_mask, dw.npages, dw.out, dw.lse, dw.ws)
    torch.cuda.synchronize()
    out = bf16.decode(bf16_to_bits(dw.out))
    g = w.group
    for r in range(w.rows):
        valid = [int(p) for p in pages[r, :npages[r]] if p >= 0]
        pg = bf16.decode(dw.data.pool_bits[np.asarray([dw.page_map[(r, p)] for p in valid], dtype=np.int64)])
        ks, vs = attend.gather_tokens(pg[:, 0], pg[:, 1], [0xFFFF] * len(valid))
        ref, _ = attend.attend(bf16.decode(dw.data.q_bits[0, r * g:(r + 1) * g]), ks, vs, dw.scale)
        assert np.all(np.abs(out[0, r * g:(r + 1) * g] - ref) <= ATOL + RTOL * np.abs(ref))


@pytest.mark.parametrize("with_table", [False, True])
def test_copy_kernel_refuses_host_pages_outside_the_registered_pool(with_table):
    """Retrieve / Offload copies: a page list entry that leads outside the pinned host pool is skipped and
    reported, in both directions, with the identity mapping (pool size registered) and with a CPU page table."""
    from gpu_harness import DEV
    w = synth.config0().with_(seq_lens=(1024,), name="host_bounds")
    sp = binding.Spin.for_workload(w, lru_timestamps=8)
    ws = sp.new_workspace(DEV)
    rows, stride, host_pages = w.rows, sp.page_stride, 40
    host = torch.empty((host_pages, 4096), dtype=torch.bfloat16, pin_memory=True)
    gen = torch.Generator().manual_seed(11)
    host.view(torch.int16).copy_(torch.randint(-30000, 30000, (host_pages, 4096), generator=gen, dtype=torch.int16))
    table = None
    if with_table:
        table = torch.arange(host_pages - 1, -1, -1, dtype=torch.int32).pin_memory()      # reversed pool
        table[7] = host_pages + 3                                                        # a bad physical page
        sp.set_host_page_table(table, host_pages)
    else:
        sp.set_host_page_table(None, host_pages)
    pool = torch.zeros((16, 4096), dtype=torch.bfloat16, device=DEV)
    row_base = torch.tensor([0, 20], dtype=torch.int64, device=DEV)
    count = torch.tensor([3, 3], dtype=torch.int32, device=DEV)
    pages = torch.zeros((rows, stride), dtype=torch.int32, device=DEV)
    slots = torch.zeros((rows, stride), dtype=torch.int32, device=DEV)
    # row 1's last entry: offset 20 + 25 = 45 lies outside a pool (or table) of 40; with the table, row 0's entry 7
    pages[0, :3] = torch.tensor([1, 7, 9], dtype=torch.int32)
    pages[1, :3] = torch.tensor([0, 2, 25], dtype=torch.int32)
    slots[0, :3] = torch.tensor([0, 1, 2], dtype=torch.int32)
    slots[1, :3] = torch.tensor([3, 4, 5], dtype=torch.int32)
    sp.gather_misses(w.batch, host, row_base, count, pages, slots, pool, ws)
    torch.cuda.synchronize()
    assert binding.STATUS_NAMES[sp.poll_status(ws)] == "SPIN_ERR_SLOT_RANGE"
    phys = (lambda o: int(table[o])) if with_table else (lambda o: o)
    want = {0: phys(1), 2: phys(9), 3: phys(20), 4: phys(22)}
    if not with_table:
        want[1] = 7
    got = pool.view(torch.int16).cpu()
    for s in range(6):
        if s in want:
            assert torch.equal(got[s], host.view(torch.int16)[want[s]]), s
        else:
            assert int(got[s].abs().sum()) == 0, s              # the refused page's slot is untouched
    # the other direction: nothing is written outside the pool, the valid pages arrive
    sp.workspace_init(ws)
    before = host.clone()
    pool.view(torch.int16).add_(1)
    sp.offload_pages(w.batch, pool, host, row_base, count, pages, slots, ws)
    torch.cuda.synchronize()
    assert binding.STATUS_NAMES[sp.poll_status(ws)] == "SPIN_ERR_SLOT_RANGE"
    after = host.view(torch.int16)
    touched = set(want.values())
    for hp in range(host_pages):
        if hp in touched:
            src = [s for s, p in want.items() if p == hp][0]
            assert torch.equal(after[hp], pool.view(torch.int16).cpu()[src])
        else:
            assert torch.equal(after[hp], before.view(torch.int16)[hp])


def test_infinite_summary_value_gives_the_documented_scores():
    """Summaries must be finite.  The documented behaviour when one is not: the kernel pairs max[d] with
    max(q, 0) and min[d] with min(q, 0), so an infinite max[d] met by a non-positive q[d] makes that head's sum
    0 x inf = NaN (the definition gives a finite term there).  The maximum over the group's heads drops NaN
    operands: the partition scores as the best of the other heads, -inf if every head's sum is NaN.  Stage 2
    ranks it accordingly and the other partitions are unaffected."""
    from gpu_harness import DeviceWorkload, build_summaries, run_step
    w = synth.config0().with_(sink_pages=0, recent_pages=0, name="inf_summary")
    data = synth.generate(w)
    d, p_inf = 37, 100
    g = w.group
    for h in range(w.num_kv_heads):
        data.q_bits[0, h * g:(h + 1) * g, d] |= 0x8000                        # every head: q[d] <= 0 ...
        data.pool_bits[data.slot_of[0][h][p_inf], 0, 3, d] = 0x7F80           # +inf key element in partition 100
    data.q_bits[0, g + 2, d] &= 0x7FFF                                        # ... but one head of KV head 1: q[d] > 0
    assert bf16.decode(data.q_bits[0, g + 2, d:d + 1])[0] > 0
    dw = DeviceWorkload(data)
    build_summaries(dw)
    run_step(dw)
    torch.cuda.synchronize()
    dw.check_ok()
    scores = dw.scores.cpu().numpy()
    sel, nsel = dw.sel.cpu().numpy(), dw.nsel.cpu().numpy()
    for h in range(w.num_kv_heads):
        kb, _ = data.logical_kv_bits(0, h)
        K = bf16.decode(kb)
        q = bf16.decode(data.q_bits[0, h * g:(h + 1) * g])
        mins, maxs = index.minmax_summaries(K, w.seq_lens[0], 16)
        assert np.isposinf(maxs[p_inf, d])
        s64 = score.score_minmax(q, mins, maxs)
        base = dw.row_base(0, h)
        got = scores[base:base + w.partitions(0)]
        if h == 0:
            assert np.isfinite(s64[p_inf])                 # the definition: q * min wins for a negative q
            assert np.isneginf(got[p_inf])                 # the kernel: every head's sum is NaN, none is left
            assert p_inf not in sel[h, :nsel[h]].tolist()
        else:
            assert np.isposinf(s64[p_inf]) and np.isposinf(got[p_inf])       # the head with q[d] > 0 decides
            assert p_inf in sel[h, :nsel[h]].tolist()
        assert nsel[h] == w.topk
        others = np.arange(w.partitions(0)) != p_inf
        eps = 256 * 2.0 ** -24 * np.maximum(np.abs(q[:, None] * mins[None]), np.abs(q[:, None] * maxs[None]))[:, others].sum(-1).max()
        assert np.all(np.abs(got[others] - s64[others]) <= eps)
