"""spin_sparse_decode_static (stage 4 with its split-K scratch in the library's own device array, for callers
that cannot allocate) against spin_sparse_decode: the same kernels run, so the output bits must be equal; the
first call is also held to the oracle's tolerance.  Two calls in a row share the array, the second one on a
smaller batch with shorter page lists."""
import numpy as np
import pytest
import torch

from paper_2604_26837_amd import binding, synth

pytestmark = pytest.mark.gpu


def _device_lists(dw, page_lists, mask_lists, rows):
    from gpu_harness import DEV
    sp = dw.spin
    slots = np.full((rows, sp.page_stride), -1, dtype=np.int32)
    masks = np.zeros((rows, sp.page_stride), dtype=np.uint16)
    npg = np.zeros(rows, dtype=np.int32)
    for r in range(rows):
        n = len(page_lists[r])
        slots[r, :n] = [dw.page_map[(r, p)] for p in page_lists[r]]
        masks[r, :n] = mask_lists[r]
        npg[r] = n
    return (torch.from_numpy(slots).to(DEV), torch.from_numpy(masks.view(np.int16)).to(DEV),
            torch.from_numpy(npg).to(DEV))


def _both(dw, batch, lists):
    """(workspace entry point, static entry point) outputs as raw bits, lse as float bits."""
    from gpu_harness import DEV, bf16_to_bits
    w, sp = dw.w, dw.spin
    d_slots, d_masks, d_np = lists
    res = []
    for static in (False, True):
        out = torch.full((batch, w.num_q_heads, w.head_dim), 7.0, dtype=torch.bfloat16, device=DEV)
        lse = torch.full((batch, w.num_q_heads), 7.0, dtype=torch.float32, device=DEV)
        if static:
            status = torch.zeros(1, dtype=torch.int32, device=DEV)
            sp.sparse_decode_static(batch, dw.q, dw.kv_pool, d_slots, d_masks, d_np, out, lse, status)
            torch.cuda.synchronize()
            assert int(status.item()) == 0
        else:
            sp.sparse_decode(batch, dw.q, dw.kv_pool, d_slots, d_masks, d_np, out, lse, dw.ws)
            torch.cuda.synchronize()
            dw.check_ok()
        res.append((bf16_to_bits(out), lse.cpu().numpy().view(np.uint32)))
    return res


@pytest.mark.parametrize("partition_tokens,splits", [(16, 3), (16, 1), (1, 2)])
def test_static_scratch_matches_workspace_entry_point(partition_tokens, splits):
    from gpu_harness import DeviceWorkload
    from test_gpu_decode import _compare, _oracle_rows, _random_selection
    from oracle import bf16
    w = synth.config0().with_(seq_lens=(700, 2049, 333, 1500), num_q_heads=8, num_kv_heads=2, topk=48,
                              partition_tokens=partition_tokens, name="static_scratch")
    if partition_tokens == 1:
        w = w.with_(score_kind=1, topk=640)
    dw = DeviceWorkload(synth.generate(w, spare_slots=3), decode_splits=splits)
    assert dw.spin.decode_splits == splits
    rng = np.random.default_rng(77)

    # first call: the whole batch, long page lists, ragged token masks
    pl, ml = _random_selection(w, rng, 40, ragged_masks=True)
    (o_ws, l_ws), (o_st, l_st) = _both(dw, w.batch, _device_lists(dw, pl, ml, w.rows))
    assert np.array_equal(o_ws, o_st) and np.array_equal(l_ws, l_st)
    ref, lref = _oracle_rows(dw, pl, ml)
    got = bf16.decode(o_st).reshape(w.rows, w.group, w.head_dim)
    _compare(got, ref, l_st.view(np.float32).astype(np.float64).reshape(w.rows, w.group), lref)

    # second call right after it: fewer requests, fewer pages; the array still holds the first call's partials
    small_rows = 2 * w.num_kv_heads
    pl2, ml2 = _random_selection(w, rng, 9, ragged_masks=True)
    pl2, ml2 = pl2[:small_rows], ml2[:small_rows]
    (o_ws2, l_ws2), (o_st2, l_st2) = _both(dw, 2, _device_lists(dw, pl2, ml2, small_rows))
    assert np.array_equal(o_ws2, o_st2) and np.array_equal(l_ws2, l_st2)
    # the smaller batch against the oracle as well (rows of the first two requests)
    ref2, lref2 = _oracle_rows(dw, pl2 + [[]] * (w.rows - small_rows), ml2 + [[]] * (w.rows - small_rows))
    got2 = bf16.decode(o_st2).reshape(small_rows, w.group, w.head_dim)
    _compare(got2, ref2[:small_rows], l_st2.view(np.float32).astype(np.float64).reshape(small_rows, w.group),
             lref2[:small_rows])


def test_static_scratch_reports_a_slot_outside_the_pool():
    from gpu_harness import DEV, DeviceWorkload
    from test_gpu_decode import _random_selection
    w = synth.config0()
    dw = DeviceWorkload(synth.generate(w), decode_splits=2)
    rng = np.random.default_rng(3)
    pl, ml = _random_selection(w, rng, 16)
    d_slots, d_masks, d_np = _device_lists(dw, pl, ml, w.rows)
    d_slots[0, 3] = dw.pool_slots + 5      # the kernel's own range check skips the page and raises the status
    out = torch.zeros((w.batch, w.num_q_heads, w.head_dim), dtype=torch.bfloat16, device=DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    dw.spin.sparse_decode_static(w.batch, dw.q, dw.kv_pool, d_slots, d_masks, d_np, out, None, status)
    torch.cuda.synchronize()
    assert binding.STATUS_NAMES[int(status.item())] == "SPIN_ERR_SLOT_RANGE"
    assert torch.isfinite(out.float()).all()
