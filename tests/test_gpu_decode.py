"""GPU parity of spin_sparse_decode against the fp64 oracle: attention
restricted to a given page list (the selected set is an input of this stage).
Tolerance: |gpu - ref| <= 2e-2 + 1e-2 |ref| elementwise on the bf16 output."""
import math

import numpy as np
import pytest
import torch

from oracle import attend, bf16
from paper_2604_26837_amd import synth

pytestmark = pytest.mark.gpu

ATOL, RTOL = 2e-2, 1e-2


def _oracle_rows(dw, page_lists, mask_lists):
    """fp64 attention per row over the given logical pages and token masks."""
    w, data = dw.w, dw.data
    g = w.group
    outs, lses = [], []
    r = 0
    for b in range(w.batch):
        for h in range(w.num_kv_heads):
            slots = [dw.page_map[(r, p)] for p in page_lists[r]]
            pages = bf16.decode(data.pool_bits[np.asarray(slots, dtype=np.int64)]) if slots else \
                np.zeros((0, 2, 16, w.head_dim))
            K_S, V_S = attend.gather_tokens(pages[:, 0], pages[:, 1], mask_lists[r])
            q = bf16.decode(data.q_bits[b, h * g:(h + 1) * g])
            o, l = attend.attend(q, K_S, V_S, dw.scale)
            outs.append(o)
            lses.append(l)
            r += 1
    return np.stack(outs), np.stack(lses)     # [rows][G][D], [rows][G]


def _run_decode(dw, page_lists, mask_lists):
    from gpu_harness import DEV, bf16_to_bits
    w, sp = dw.w, dw.spin
    rows = w.rows
    slots = np.full((rows, sp.page_stride), -1, dtype=np.int32)
    masks = np.zeros((rows, sp.page_stride), dtype=np.uint16)
    npg = np.zeros(rows, dtype=np.int32)
    for r in range(rows):
        n = len(page_lists[r])
        assert n <= sp.page_stride
        slots[r, :n] = [dw.page_map[(r, p)] for p in page_lists[r]]
        masks[r, :n] = mask_lists[r]
        npg[r] = n
    d_slots = torch.from_numpy(slots).to(DEV)
    d_masks = torch.from_numpy(masks.view(np.int16)).to(DEV)
    d_np = torch.from_numpy(npg).to(DEV)
    out = torch.full((w.batch, w.num_q_heads, w.head_dim), 7.0, dtype=torch.bfloat16, device=DEV)
    lse = torch.full((w.batch, w.num_q_heads), 7.0, dtype=torch.float32, device=DEV)
    sp.sparse_decode(w.batch, dw.q, dw.kv_pool, d_slots, d_masks, d_np, out, lse, dw.ws)
    torch.cuda.synchronize()
    dw.check_ok()
    got = bf16.decode(bf16_to_bits(out)).reshape(w.batch, w.num_kv_heads, w.group, w.head_dim)
    got = got.reshape(rows, w.group, w.head_dim)
    return got, lse.cpu().numpy().astype(np.float64).reshape(rows, w.group)


def _compare(got, ref, lse_got, lse_ref):
    err = np.abs(got - ref)
    bound = ATOL + RTOL * np.abs(ref)
    assert (err <= bound).all(), f"max err {err.max():.4g}, worst excess {(err - bound).max():.4g}"
    fin = np.isfinite(lse_ref)
    assert np.array_equal(np.isfinite(lse_got), fin)
    assert np.allclose(lse_got[fin], lse_ref[fin], rtol=2e-3, atol=2e-3)
    return err.max()


def _random_selection(w, rng, npages_per_row, ragged_masks=False):
    page_lists, mask_lists = [], []
    for b in range(w.batch):
        pages = w.pages(b)
        for h in range(w.num_kv_heads):
            n = min(npages_per_row, pages)
            pl = sorted(int(x) for x in rng.choice(pages, size=n, replace=False))
            ml = []
            for p in pl:
                full = (1 << min(16, w.seq_lens[b] - 16 * p)) - 1
                ml.append(int(full & int(rng.integers(1, 1 << 16))) if ragged_masks else full)
            page_lists.append(pl)
            mask_lists.append(ml)
    return page_lists, mask_lists


@pytest.mark.parametrize("splits", [0, 1, 3])
def test_config0_random_page_lists(splits):
    from gpu_harness import DeviceWorkload
    w = synth.config0()
    dw = DeviceWorkload(synth.generate(w), decode_splits=splits)
    rng = np.random.default_rng(5)
    pl, ml = _random_selection(w, rng, 32)
    ref, lref = _oracle_rows(dw, pl, ml)
    got, lgot = _run_decode(dw, pl, ml)
    _compare(got, ref, lgot, lref)


def test_all_tokens_is_dense_attention():
    from gpu_harness import DeviceWorkload
    w = synth.config0().with_(seq_lens=(1000,), topk=64, name="dense1000")
    dw = DeviceWorkload(synth.generate(w))
    pages = w.pages(0)
    pl = [list(range(pages))] * w.rows
    ml = [[0xFFFF] * (pages - 1) + [(1 << (1000 - 16 * (pages - 1))) - 1]] * w.rows
    ref, lref = _oracle_rows(dw, pl, ml)
    got, lgot = _run_decode(dw, pl, ml)
    _compare(got, ref, lgot, lref)


def test_ragged_batch_token_masks_and_empty_rows():
    from gpu_harness import DeviceWorkload
    w = synth.config0().with_(seq_lens=(700, 16, 333, 2049), num_q_heads=8, num_kv_heads=2, topk=40,
                              name="ragged")
    dw = DeviceWorkload(synth.generate(w, spare_slots=5), decode_splits=4)
    rng = np.random.default_rng(8)
    pl, ml = _random_selection(w, rng, 40, ragged_masks=True)
    pl[3], ml[3] = [], []                       # a row with nothing selected
    ml[4] = [0] * len(pl[4])                    # a row whose every token is masked off
    pl[1], ml[1] = pl[1][:1], [1 << 9]          # a single token
    ref, lref = _oracle_rows(dw, pl, ml)
    got, lgot = _run_decode(dw, pl, ml)
    _compare(got, ref, lgot, lref)
    assert (got[3] == 0).all() and (got[4] == 0).all()


def test_group_sizes_and_page_order_invariance():
    from gpu_harness import DeviceWorkload
    for hq, hkv in ((4, 4), (16, 2), (32, 2)):
        w = synth.config0().with_(seq_lens=(512, 512), num_q_heads=hq, num_kv_heads=hkv, topk=16,
                                  name=f"g{hq // hkv}")
        dw = DeviceWorkload(synth.generate(w), decode_splits=2)
        rng = np.random.default_rng(hq)
        pl, ml = _random_selection(w, rng, 16)
        ref, lref = _oracle_rows(dw, pl, ml)
        got, lgot = _run_decode(dw, pl, ml)
        _compare(got, ref, lgot, lref)
        pl2 = [list(reversed(p)) for p in pl]
        ml2 = [list(reversed(m)) for m in ml]
        got2, _ = _run_decode(dw, pl2, ml2)
        _compare(got2, ref, lgot, lref)


def test_slot_out_of_range_is_reported_not_read():
    from gpu_harness import DEV, DeviceWorkload
    from paper_2604_26837_amd import binding
    w = synth.config0().with_(seq_lens=(256,), topk=4, name="badslot")
    dw = DeviceWorkload(synth.generate(w))
    sp = dw.spin
    slots = torch.full((w.rows, sp.page_stride), dw.pool_slots + 3, dtype=torch.int32, device=DEV)
    masks = torch.full((w.rows, sp.page_stride), -1, dtype=torch.int16, device=DEV)
    npg = torch.full((w.rows,), 2, dtype=torch.int32, device=DEV)
    out = torch.zeros((w.batch, w.num_q_heads, w.head_dim), dtype=torch.bfloat16, device=DEV)
    sp.sparse_decode(w.batch, dw.q, dw.kv_pool, slots, masks, npg, out, None, dw.ws)
    assert sp.poll_status(dw.ws) == -7
    assert (out == 0).all()
    sp.workspace_init(dw.ws)
    assert sp.poll_status(dw.ws) == 0


def test_run_to_run_bits_identical():
    from gpu_harness import DEV, DeviceWorkload, bf16_to_bits
    w = synth.config0()
    dw = DeviceWorkload(synth.generate(w), decode_splits=4)
    rng = np.random.default_rng(1)
    pl, ml = _random_selection(w, rng, 32)
    a, _ = _run_decode(dw, pl, ml)
    b, _ = _run_decode(dw, pl, ml)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("splits,npages,sparse", [(1, 600, True), (1, 600, False), (2, 200, True), (4, 37, True)])
def test_token_partitions_gathered_tiles(splits, npages, sparse):
    """Slots of token partitions are token-major and attention gathers attended tokens into
    tiles of 16: page lists long enough that a wavefront walks more than 64 pages, masks with
    one or two tokens, empty masks in between, and full pages."""
    from gpu_harness import DeviceWorkload
    w = synth.config0().with_(seq_lens=(16 * 640 + 5, 4000), num_q_heads=8, num_kv_heads=2, partition_tokens=1,
                              score_kind=synth.SCORE_SKETCH, topk=16 * 640, sink_pages=0, recent_pages=0,
                              name="tok_tiles")
    dw = DeviceWorkload(synth.generate(w), decode_splits=splits)
    rng = np.random.default_rng(17 + splits)
    pl, ml = _random_selection(w, rng, npages, ragged_masks=True)
    if sparse:
        for r in range(w.rows):
            for i in range(len(ml[r])):
                kind = rng.integers(0, 4)
                full = ml[r][i]
                if kind == 0:
                    ml[r][i] = 0                                    # page listed, nothing attended
                elif kind in (1, 2):
                    bits = [t for t in range(16) if (full >> t) & 1]
                    keep = rng.choice(bits, size=min(len(bits), int(kind)), replace=False) if bits else []
                    ml[r][i] = int(sum(1 << int(t) for t in keep))
    ref, lref = _oracle_rows(dw, pl, ml)
    got, lgot = _run_decode(dw, pl, ml)
    _compare(got, ref, lgot, lref)
    got2, lgot2 = _run_decode(dw, pl, ml)
    assert np.array_equal(got, got2) and np.array_equal(lgot, lgot2)      # same bits run to run
    # no attended token at all in a row: zeros and -inf
    ml0 = [[0] * len(m) for m in ml]
    got0, lgot0 = _run_decode(dw, pl, ml0)
    assert (got0 == 0).all() and np.isneginf(lgot0).all()


@pytest.mark.parametrize("seed", range(24))
def test_random_launch_shapes_and_page_lists(seed):
    """Randomly drawn group size, heads, contexts, page-list lengths (some rows empty), token masks,
    split-K factor, wavefronts per workgroup and page buffers, for whole-page and token-major slots."""
    from gpu_harness import DeviceWorkload
    rng = np.random.default_rng(300 + seed)
    g = int(rng.choice([1, 2, 3, 4, 4, 5, 8, 12, 16]))
    hkv = int(rng.choice([1, 2, 3]))
    lens = tuple(int(x) for x in rng.integers(1, 5000, size=int(rng.integers(1, 4))))
    token_major = bool(rng.integers(0, 3) == 0)               # partitions smaller than a page: gathered tiles
    w = synth.config0().with_(seq_lens=lens, num_q_heads=g * hkv, num_kv_heads=hkv, topk=int(rng.integers(8, 200)),
                              partition_tokens=4 if token_major else 16, name=f"decode_random{seed}")
    over = dict(decode_splits=int(rng.choice([0, 1, 2, 3, 5, 8])), decode_waves=int(rng.choice([0, 2, 4, 8])),
                decode_depth=int(rng.choice([0, 2, 3, 4])))
    print(f"seed {seed}: group {g} kv {hkv} lens {lens} token-major {token_major} {over}", flush=True)
    dw = DeviceWorkload(synth.generate(w), **over)
    stride = dw.spin.page_stride
    page_lists, mask_lists = [], []
    for b in range(w.batch):
        pages = w.pages(b)
        for h in range(hkv):
            n = int(rng.choice([0, 1, min(pages, stride), rng.integers(0, min(pages, stride) + 1)]))
            pl = sorted(int(x) for x in rng.choice(pages, size=n, replace=False))
            ml = []
            for p in pl:
                full = (1 << min(16, w.seq_lens[b] - 16 * p)) - 1
                style = rng.integers(0, 3)
                ml.append(full if style == 0 else int(full & int(rng.integers(0, 1 << 16))) if style == 1
                          else int(full & (1 << int(rng.integers(0, 16)))))
            page_lists.append(pl)
            mask_lists.append(ml)
    ref, lref = _oracle_rows(dw, page_lists, mask_lists)
    got, lgot = _run_decode(dw, page_lists, mask_lists)
    # rows that attend to no token at all: zeros, lse = -inf
    _compare(got, np.nan_to_num(ref), lgot, lref)


@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 8), (3, 4), (2, 2)])
def test_two_pass_attention_over_a_split_page_list(splits, waves):
    """spin_sparse_decode_begin + spin_sparse_decode_finish over any two-way split of the token masks (a page in
    one pass, the other, both in part, or neither) equal attention over the union: oracle tolerance, and the
    same bits from run to run."""
    from gpu_harness import DEV, DeviceWorkload, bf16_to_bits
    w = synth.config0().with_(seq_lens=(700, 16, 333, 2049), num_q_heads=8, num_kv_heads=2, topk=40, name="two_pass")
    dw = DeviceWorkload(synth.generate(w, spare_slots=5), decode_splits=splits, decode_waves=waves)
    sp = dw.spin
    rng = np.random.default_rng(21 + splits)
    pl, ml = _random_selection(w, rng, 40, ragged_masks=True)
    rows = w.rows
    slots = np.full((rows, sp.page_stride), -1, dtype=np.int32)
    ma = np.zeros((rows, sp.page_stride), dtype=np.uint16)
    mb = np.zeros((rows, sp.page_stride), dtype=np.uint16)
    npg = np.zeros(rows, dtype=np.int32)
    for r in range(rows):
        n = len(pl[r])
        slots[r, :n] = [dw.page_map[(r, p)] for p in pl[r]]
        npg[r] = n
        for i, m in enumerate(ml[r]):
            kind = int(rng.integers(0, 4))
            a = {0: m, 1: 0, 2: m & int(rng.integers(0, 1 << 16)), 3: 0}[kind]
            ma[r, i], mb[r, i] = a, (m & ~a) & 0xFFFF
            if kind == 3:
                ml[r][i] = 0            # attended in neither pass
                mb[r, i] = 0
    if rows > 1:
        ma[1, :] = 0                    # a row whose first pass is empty, and one whose second pass is
        mb[1, :npg[1]] = ml[1]
        mb[rows - 1, :] = 0
        ma[rows - 1, :npg[rows - 1]] = ml[rows - 1]
    d_slots = torch.from_numpy(slots).to(DEV)
    d_a, d_b = torch.from_numpy(ma.view(np.int16)).to(DEV), torch.from_numpy(mb.view(np.int16)).to(DEV)
    d_np = torch.from_numpy(npg).to(DEV)
    ref, lref = _oracle_rows(dw, pl, ml)
    bits = []
    for _ in range(3):
        out = torch.full((w.batch, w.num_q_heads, w.head_dim), 7.0, dtype=torch.bfloat16, device=DEV)
        lse = torch.full((w.batch, w.num_q_heads), 7.0, dtype=torch.float32, device=DEV)
        sp.sparse_decode_begin(w.batch, dw.q, dw.kv_pool, d_slots, d_a, d_np, dw.ws)
        sp.sparse_decode_finish(w.batch, dw.q, dw.kv_pool, d_slots, d_b, d_np, out, lse, dw.ws)
        torch.cuda.synchronize()
        dw.check_ok()
        bits.append(bf16_to_bits(out).copy())
    assert np.array_equal(bits[0], bits[1]) and np.array_equal(bits[0], bits[2])
    got = bf16.decode(bits[0]).reshape(rows, w.group, w.head_dim)
    _compare(got, ref, lse.cpu().numpy().astype(np.float64).reshape(rows, w.group), lref)
