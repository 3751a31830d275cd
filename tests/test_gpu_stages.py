"""GPU parity of Index, stage 1 (score), stage 2 (select) and stage 3 (resolve)
against the oracle, stage by stage and end to end.

Bars: summaries, selected ids, page ids, slots and masks bit-exact.  Scores are
fp32 matrix-core sums of exact bf16 products compared with the fp64 oracle
within the first-order summation bound K * 2^-24 * sum|terms|.  Where fp32
scores decide the top-k, the oracle takes the decision on the same fp32 score
bits (copied back); against fp64 scores the selection must agree outside the
rounding band around the k-th score.
"""
import math

import numpy as np
import pytest
import torch

from oracle import attend, bf16, index, resolve, score, select
from paper_2604_26837_amd import synth

pytestmark = pytest.mark.gpu

ATOL, RTOL = 2e-2, 1e-2


def _workloads():
    c0 = synth.config0()
    return {
        "cfg0": c0,
        "ragged_pages": c0.with_(seq_lens=(700, 16, 333, 2049, 5), topk=24, sink_pages=2, recent_pages=3,
                                 planted_frac=0.02, name="ragged_pages"),
        "blocks": c0.with_(seq_lens=(131 * 16 + 5, 40 * 128, 129), partition_tokens=128,
                           score_kind=synth.SCORE_REPMAX, topk=6, topk_includes_forced=False,
                           sink_pages=4, recent_pages=11, block_mean_std=0.5, name="blocks"),
        "tokens": c0.with_(seq_lens=(3000, 777), partition_tokens=1, score_kind=synth.SCORE_SKETCH,
                           topk=200, sink_pages=1, recent_pages=2, planted_frac=0.01, name="tokens"),
        "minmax_blocks": c0.with_(seq_lens=(2000, 4096), partition_tokens=64, topk=9,
                                  topk_includes_forced=True, sink_pages=3, recent_pages=6, name="mm_blocks"),
        "minmax_quarter": c0.with_(seq_lens=(500,), partition_tokens=4, topk=50, sink_pages=1,
                                   recent_pages=1, name="mm_quarter"),
        # representatives that cover half a page each (the Index kernel for whole-page sub-ranges does not apply)
        "blocks_small": c0.with_(seq_lens=(70 * 32 + 9, 32 * 16), partition_tokens=32, score_kind=synth.SCORE_REPMAX,
                                 topk=7, topk_includes_forced=False, sink_pages=2, recent_pages=3, block_mean_std=0.5,
                                 name="blocks_small"),
        # one mean key per partition (a landmark per page, a centroid per block) and two representatives
        "mean_pages": c0.with_(seq_lens=(3000, 16 * 130 + 5), score_kind=synth.SCORE_REPMAX, reps_per_partition=1,
                               topk=24, sink_pages=2, recent_pages=3, block_mean_std=0.5, name="mean_pages"),
        "mean_blocks": c0.with_(seq_lens=(64 * 50 + 17, 640), partition_tokens=64, score_kind=synth.SCORE_REPMAX,
                                reps_per_partition=1, topk=6, topk_includes_forced=False, sink_pages=1,
                                recent_pages=5, block_mean_std=0.5, name="mean_blocks"),
        "two_reps_blocks": c0.with_(seq_lens=(64 * 41 + 33,), partition_tokens=64, score_kind=synth.SCORE_REPMAX,
                                    reps_per_partition=2, topk=6, topk_includes_forced=False, sink_pages=1,
                                    recent_pages=2, block_mean_std=0.5, name="two_reps_blocks"),
        "mean_quarter_pages": c0.with_(seq_lens=(777,), partition_tokens=4, score_kind=synth.SCORE_REPMAX,
                                       reps_per_partition=1, topk=40, sink_pages=1, recent_pages=1,
                                       block_mean_std=0.5, name="mean_quarter_pages"),
        # partitions of 32 pages: more pages per wavefront than the Index kernels look up at once
        "minmax_big_blocks": c0.with_(seq_lens=(512 * 9 + 300, 512 * 2 + 5), partition_tokens=512, topk=3,
                                      topk_includes_forced=False, sink_pages=1, recent_pages=2, name="mm_big_blocks"),
        "mean_big_blocks": c0.with_(seq_lens=(512 * 7 + 130,), partition_tokens=512, score_kind=synth.SCORE_REPMAX,
                                    reps_per_partition=1, topk=2, topk_includes_forced=False, sink_pages=1,
                                    recent_pages=2, block_mean_std=0.5, name="mean_big_blocks"),
        # a ragged last partition whose trailing representatives are empty (they repeat representative 0)
        "four_reps_ragged": c0.with_(seq_lens=(128 * 6 + 20, 128 * 3 + 70), partition_tokens=128,
                                     score_kind=synth.SCORE_REPMAX, reps_per_partition=4, topk=3,
                                     topk_includes_forced=False, sink_pages=1, recent_pages=2, block_mean_std=0.5,
                                     name="four_reps_ragged"),
        # group sizes other than 4: one head, a group that is no power of two, more than one lane quarter
        "g1_pages": c0.with_(seq_lens=(900, 333), num_q_heads=2, num_kv_heads=2, topk=12, sink_pages=1,
                             recent_pages=1, name="g1_pages"),
        "g3_pages": c0.with_(seq_lens=(900,), num_q_heads=6, num_kv_heads=2, topk=12, name="g3_pages"),
        "g8_blocks": c0.with_(seq_lens=(40 * 128 + 77,), num_q_heads=16, num_kv_heads=2, partition_tokens=128,
                              score_kind=synth.SCORE_REPMAX, topk=5, topk_includes_forced=False, sink_pages=2,
                              recent_pages=4, block_mean_std=0.5, name="g8_blocks"),
        "g16_tokens": c0.with_(seq_lens=(2500,), num_q_heads=32, num_kv_heads=2, partition_tokens=1,
                               score_kind=synth.SCORE_SKETCH, topk=150, planted_frac=0.01, name="g16_tokens"),
        # token partitions: the four-tile sketch kernel with fewer than four heads and a ragged tile tail,
        # the one-tile kernel for groups of five and eight heads
        "g1_tokens": c0.with_(seq_lens=(2500 + 16 * 5, 33), num_q_heads=2, num_kv_heads=2, partition_tokens=1,
                              score_kind=synth.SCORE_SKETCH, topk=90, name="g1_tokens"),
        "g3_tokens": c0.with_(seq_lens=(16 * 4 * 9 + 16 * 3 - 5,), num_q_heads=6, num_kv_heads=2, partition_tokens=1,
                              score_kind=synth.SCORE_SKETCH, topk=60, sink_pages=1, recent_pages=1, name="g3_tokens"),
        "g5_tokens": c0.with_(seq_lens=(1999,), num_q_heads=10, num_kv_heads=2, partition_tokens=1,
                              score_kind=synth.SCORE_SKETCH, topk=70, name="g5_tokens"),
        "g8_tokens": c0.with_(seq_lens=(1200, 640), num_q_heads=16, num_kv_heads=2, partition_tokens=1,
                              score_kind=synth.SCORE_SKETCH, topk=70, sink_pages=1, name="g8_tokens"),
        "g12_pages": c0.with_(seq_lens=(1500,), num_q_heads=24, num_kv_heads=2, topk=20, sink_pages=1,
                              recent_pages=2, name="g12_pages"),
    }


def _oracle_row_inputs(dw, b, h, chan):
    w = dw.w
    g = w.group
    kb, vb = dw.data.logical_kv_bits(b, h)
    K = bf16.decode(kb)
    q = bf16.decode(dw.data.q_bits[b, h * g:(h + 1) * g])
    n = w.seq_lens[b]
    if w.score_kind == synth.SCORE_MINMAX:
        mins, maxs = index.minmax_summaries(K, n, w.partition_tokens)
        summ = (mins, maxs)
        rows = np.concatenate([maxs, mins], axis=1)
        s = score.score_minmax(q, mins, maxs)
        sabs = np.maximum(np.abs(q[:, None, :] * mins[None]), np.abs(q[:, None, :] * maxs[None])).sum(-1).max()
        kterms = 256
    elif w.score_kind == synth.SCORE_REPMAX:
        reps = index.block_representatives(K, n, w.partition_tokens, w.reps_per_partition)
        summ = reps
        rows = reps.reshape(-1, w.head_dim)
        s = score.score_repmax(q, reps)
        sabs = np.abs(np.einsum("prd,gd->prgd", reps, q)).sum(-1).max() if len(reps) else 0.0
        kterms = 128
    else:
        sk = index.key_sketch(K, n, chan[h])
        summ = sk
        rows = sk
        s = score.score_sketch(q, sk, chan[h])
        sabs = np.abs(sk[:, None, :] * q[None][:, :, chan[h]]).sum(-1).max() if len(sk) else 0.0
        kterms = 16
    return q, K, bf16.decode(vb), summ, rows, s, kterms * 2.0 ** -24 * sabs


def _kd_kc(w):
    return {synth.SCORE_MINMAX: (256, 8), synth.SCORE_REPMAX: (128, 8), synth.SCORE_SKETCH: (16, 4)}[w.score_kind]


@pytest.mark.parametrize("name", list(_workloads()))
def test_stage_by_stage(name):
    _check_workload(_workloads()[name], name)


def test_million_token_context():
    """One request of a million tokens (62 500 pages: 123 leaf chunks per row, the two-launch stage 2)
    through every stage against the oracle."""
    w = synth.config0().with_(seq_lens=(1_000_000 - 7,), num_q_heads=4, num_kv_heads=1, topk=256, sink_pages=4,
                              recent_pages=8, name="million")
    _check_workload(w, w.name)


def test_many_short_requests():
    """A large batch of short ragged requests: 1200 rows, most of them smaller than one summary tile."""
    rng = np.random.default_rng(3)
    lens = tuple(int(x) for x in rng.integers(1, 400, size=300))
    w = synth.config0().with_(seq_lens=lens, num_q_heads=8, num_kv_heads=4, topk=6, sink_pages=1, recent_pages=1,
                              name="many_rows")
    _check_workload(w, w.name)


def _random_workload(seed):
    """A valid workload drawn at random: score kind, partition size, group size, heads, ragged
    contexts (down to a single token), top-k (down to 0, up to beyond the row) and forced windows."""
    rng = np.random.default_rng(1000 + seed)
    kind = int(rng.choice([synth.SCORE_MINMAX, synth.SCORE_SKETCH, synth.SCORE_REPMAX]))
    reps = 4
    if kind == synth.SCORE_SKETCH:
        tp = 1
    elif kind == synth.SCORE_MINMAX:
        tp = int(rng.choice([1, 2, 4, 8, 16, 16, 32, 64, 128]))
    else:
        reps = int(rng.choice([1, 2, 4]))
        tp = int(rng.choice([t for t in (4, 8, 16, 16, 32, 64, 128) if t % reps == 0]))
    g = int(rng.choice([1, 2, 3, 4, 4, 5, 8, 16]))
    hkv = int(rng.choice([1, 2, 3]))
    batch = int(rng.integers(1, 4))
    lens = []
    for _ in range(batch):
        style = rng.integers(0, 4)
        lens.append(int({0: rng.integers(1, 40), 1: rng.integers(40, 700), 2: rng.integers(700, 3000),
                         3: 16 * rng.integers(1, 120)}[int(style)]))
    max_parts = max(-(-n // tp) for n in lens)
    topk = int(rng.choice([0, 1, 2, rng.integers(3, 40), rng.integers(3, max(max_parts, 4) + 20)]))
    c0 = synth.config0()
    return c0.with_(seq_lens=tuple(lens), num_q_heads=g * hkv, num_kv_heads=hkv, partition_tokens=tp, score_kind=kind,
                    reps_per_partition=reps, topk=topk, topk_includes_forced=bool(rng.integers(0, 2)),
                    sink_pages=int(rng.integers(0, 4)), recent_pages=int(rng.integers(0, 5)),
                    block_mean_std=0.5 if kind == synth.SCORE_REPMAX else 0.0, seed=c0.seed + 17 * seed,
                    name=f"random{seed}")


@pytest.mark.parametrize("seed", range(64))
def test_random_workloads_stage_by_stage(seed):
    w = _random_workload(seed)
    print(f"seed {seed}: kind {w.score_kind} tp {w.partition_tokens} reps {w.reps_per_partition} group {w.group} "
          f"kv {w.num_kv_heads} lens {w.seq_lens} topk {w.topk} incl {w.topk_includes_forced} "
          f"sink {w.sink_pages} recent {w.recent_pages}", flush=True)
    _check_workload(w, w.name)


@pytest.mark.parametrize("seed", range(32))
def test_random_workloads_with_random_launch_knobs(seed):
    """The same draw with the launch-shape knobs of stages 1 and 4 drawn as well: results may not
    depend on them beyond the tolerances."""
    w = _random_workload(100 + seed)
    rng = np.random.default_rng(77 + seed)
    over = dict(score_waves=int(rng.choice([0, 1, 2, 4, 8])), score_tiles_per_wg=int(rng.choice([0, 1, 2, 3, 4, 8, 16, 64])),
                decode_splits=int(rng.choice([0, 1, 2, 3, 7])), decode_waves=int(rng.choice([0, 2, 4, 8])),
                decode_depth=int(rng.choice([0, 2, 3, 4])))
    print(f"seed {seed}: kind {w.score_kind} tp {w.partition_tokens} reps {w.reps_per_partition} group {w.group} "
          f"kv {w.num_kv_heads} lens {w.seq_lens} topk {w.topk} {over}", flush=True)
    _check_workload(w, w.name, **over)


def _check_workload(w, name, **cfg_over):
    from gpu_harness import DeviceWorkload, bf16_to_bits, build_summaries, run_step, unpack_summary_rows
    data = synth.generate(w, spare_slots=3)
    dw = DeviceWorkload(data, **cfg_over)
    sp = dw.spin
    chan = synth.sketch_channels(data) if w.score_kind == synth.SCORE_SKETCH else None
    build_summaries(dw, chan)
    run_step(dw)
    torch.cuda.synchronize()
    dw.check_ok()

    kd, kc = _kd_kc(w)
    summ_rows = unpack_summary_rows(dw.summaries, kd, kc)
    scores = dw.scores.cpu().numpy()
    sel = dw.sel.cpu().numpy()
    nsel = dw.nsel.cpu().numpy()
    slots = dw.slots.cpu().numpy()
    page_ids = dw.page_ids.cpu().numpy()
    masks = dw.valid_mask.cpu().numpy().view(np.uint16)
    npages = dw.npages.cpu().numpy()
    out = bf16.decode(bf16_to_bits(dw.out))
    lse = dw.lse.cpu().numpy()
    rpp = w.reps_per_partition if w.score_kind == synth.SCORE_REPMAX else 1
    band_rows = 0

    r = 0
    for b in range(w.batch):
        n = w.seq_lens[b]
        P = w.partitions(b)
        for h in range(w.num_kv_heads):
            q, K, V, summ, ref_rows, s64, eps = _oracle_row_inputs(dw, b, h, chan)
            base = dw.row_base(b, h)
            # --- Index: stored summaries bit-exact
            got_rows = bf16.decode(summ_rows[base * rpp: base * rpp + ref_rows.shape[0]])
            assert np.array_equal(got_rows, ref_rows), f"summaries differ row {r}"
            # --- stage 1: scores within the fp32 summation bound
            s32 = scores[base: base + P].astype(np.float64)
            assert np.all(np.abs(s32 - s64) <= eps + 1e-30), f"score err {np.abs(s32 - s64).max()} > {eps}"
            # --- stage 2 (i): decision taken on the same fp32 bits
            want = select.select_topk(scores[base: base + P], n, 16, w.partition_tokens, w.topk,
                                      w.topk_includes_forced, w.sink_pages, w.recent_pages)
            got = sel[r, :nsel[r]].tolist()
            assert got == want, f"sel differs row {r}"
            assert (sel[r, nsel[r]:] == -1).all()
            # --- stage 2 (ii): against fp64 scores, outside the rounding band
            want64 = select.select_topk(s64, n, 16, w.partition_tokens, w.topk, w.topk_includes_forced,
                                        w.sink_pages, w.recent_pages)
            if want64 != got:
                band_rows += 1
                forced = set(select.forced_partitions(n, 16, w.partition_tokens, w.sink_pages, w.recent_pages))
                cand_sel = [p for p in want64 if p not in forced]
                tau = min(s64[p] for p in cand_sel)
                assert len(got) == len(want64)
                for p in set(got) ^ set(want64):
                    assert abs(s64[p] - tau) <= 2 * eps, "selection differs outside the rounding band"
            # --- stage 3: dictionary lookup on the GPU's own selection
            pg_w, sl_w, mk_w = resolve.resolve_slots(got, n, 16, w.partition_tokens, w.sink_pages,
                                                     w.recent_pages, dw.page_map, r)
            assert npages[r] == len(pg_w)
            assert page_ids[r, :npages[r]].tolist() == pg_w
            assert slots[r, :npages[r]].tolist() == sl_w
            assert masks[r, :npages[r]].tolist() == mk_w
            assert (slots[r, npages[r]:] == -1).all()
            # --- stage 4: attention restricted to the GPU's own page list
            pages = bf16.decode(data.pool_bits[np.asarray(sl_w, dtype=np.int64)]) if sl_w else \
                np.zeros((0, 2, 16, w.head_dim))
            K_S, V_S = attend.gather_tokens(pages[:, 0], pages[:, 1], mk_w)
            ref, lref = attend.attend(q, K_S, V_S, dw.scale)
            g = w.group
            o = out[b, h * g:(h + 1) * g]
            assert np.all(np.abs(o - ref) <= ATOL + RTOL * np.abs(ref)), f"attention err {np.abs(o - ref).max()}"
            if np.isfinite(lref).all():
                assert np.allclose(lse[b, h * g:(h + 1) * g], lref, rtol=2e-3, atol=2e-3)
            r += 1
    print(f"{name}: rows inside the rounding band: {band_rows}/{w.rows}")


def test_quest_bound_holds_for_gpu_scores():
    from gpu_harness import DeviceWorkload, build_summaries, run_step
    w = synth.config0()
    dw = DeviceWorkload(synth.generate(w))
    build_summaries(dw)
    run_step(dw)
    scores = dw.scores.cpu().numpy().astype(np.float64)
    for h in range(w.num_kv_heads):
        q, K, V, summ, rows, s64, eps = _oracle_row_inputs(dw, 0, h, None)
        true_max = (q @ K[:4096].T).reshape(w.group, 256, 16).max(axis=2).max(axis=0)
        base = dw.row_base(0, h)
        assert np.all(scores[base: base + 256] >= true_max - eps)


def _select_only(w, score_rows):
    """Run stage 2 alone on hand-made score rows (one per KV row)."""
    from gpu_harness import DEV, DeviceWorkload, alloc_step_buffers
    from paper_2604_26837_amd import binding, tables
    sp = binding.Spin.for_workload(w)
    ws = sp.new_workspace(DEV)
    po = tables.part_offsets(w.seq_lens, w.partition_tokens)
    buf = np.zeros(int(po[-1]) * w.num_kv_heads, dtype=np.float32)
    r = 0
    for b in range(w.batch):
        for h in range(w.num_kv_heads):
            base = tables.row_base(po, b, h, w.num_kv_heads)
            buf[base: base + len(score_rows[r])] = score_rows[r]
            r += 1
    d_scores = torch.from_numpy(buf).to(DEV)
    sel = torch.zeros((w.rows, sp.sel_stride), dtype=torch.int32, device=DEV)
    nsel = torch.zeros(w.rows, dtype=torch.int32, device=DEV)
    sp.select_topk(w.batch, d_scores, torch.from_numpy(po).to(DEV),
                   torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV), sel, nsel, ws)
    torch.cuda.synchronize()
    assert sp.poll_status(ws) == 0
    sel, nsel = sel.cpu().numpy(), nsel.cpu().numpy()
    return [sel[r, :nsel[r]].tolist() for r in range(w.rows)], sel


def _check_select(w, score_rows):
    got, raw = _select_only(w, score_rows)
    r = 0
    for b in range(w.batch):
        for h in range(w.num_kv_heads):
            want = select.select_topk(score_rows[r], w.seq_lens[b], 16, w.partition_tokens, w.topk,
                                      w.topk_includes_forced, w.sink_pages, w.recent_pages)
            assert got[r] == want, f"row {r}"
            assert (raw[r, len(want):] == -1).all()
            r += 1


def test_select_adversarial_ties_and_specials():
    base = synth.config0().with_(num_q_heads=4, num_kv_heads=1)
    rng = np.random.default_rng(0)
    P = 300
    w = base.with_(seq_lens=(P * 16,) * 8, topk=40, sink_pages=2, recent_pages=3, name="adv")
    rows = [
        np.zeros(P, dtype=np.float32),                                           # all equal
        rng.integers(-2, 3, size=P).astype(np.float32),                          # heavy ties
        np.where(rng.random(P) < 0.5, 0.0, -0.0).astype(np.float32),              # signed zeros
        np.where(rng.random(P) < 0.3, -np.inf, rng.standard_normal(P)).astype(np.float32),
        np.where(rng.random(P) < 0.9, np.nan, rng.standard_normal(P)).astype(np.float32),   # mostly NaN
        np.full(P, np.inf, dtype=np.float32),
        (rng.standard_normal(P) * 1e-38).astype(np.float32),                     # subnormals
        np.concatenate([np.full(150, 3.0), np.full(150, 3.0000002)]).astype(np.float32),
    ]
    _check_select(w, rows)


def test_select_k_extremes():
    base = synth.config0().with_(num_q_heads=4, num_kv_heads=1)
    rng = np.random.default_rng(1)
    for topk, sinks, recents, seq in [(0, 0, 0, 800), (0, 2, 2, 800), (1000, 1, 1, 800), (3, 4, 4, 800),
                                      (5, 0, 0, 7), (5, 3, 3, 40), (50, 0, 0, 50 * 16)]:
        w = base.with_(seq_lens=(seq, 1, seq + 9), topk=topk, sink_pages=sinks, recent_pages=recents, name="kx")
        rows = [rng.standard_normal(w.partitions(b)).astype(np.float32) for b in range(w.batch)]
        _check_select(w, rows)


def test_select_large_rows_token_partitions():
    base = synth.config0().with_(num_q_heads=4, num_kv_heads=1)
    rng = np.random.default_rng(2)
    w = base.with_(seq_lens=(65536, 40000), partition_tokens=1, topk=1024, sink_pages=0, recent_pages=0,
                   score_kind=synth.SCORE_SKETCH, name="big_tokens")
    rows = [np.round(rng.standard_normal(n) * 50).astype(np.float32) / 50 for n in w.seq_lens]  # many ties
    _check_select(w, rows)
    w2 = base.with_(seq_lens=(262144,), topk=128, sink_pages=4, recent_pages=8, name="big_pages")
    _check_select(w2, [rng.standard_normal(16384).astype(np.float32)])


def test_select_wide_dynamic_range_rows():
    """Rows whose k'-th candidate lies many exponents below the largest score (the first radix
    digit cannot be settled from the highest few digits), on every register variant's row size."""
    base = synth.config0().with_(num_q_heads=4, num_kv_heads=1)
    rng = np.random.default_rng(21)
    for n, tp, topk in [(65536, 1, 1024), (12000, 1, 900), (3000 * 16, 16, 200), (300 * 16, 16, 64)]:
        w = base.with_(seq_lens=(n,) * 5, partition_tokens=tp, topk=topk, sink_pages=1, recent_pages=1,
                       score_kind=synth.SCORE_SKETCH if tp == 1 else synth.SCORE_MINMAX, name="wide")
        P = w.partitions(0)
        spread = (rng.choice([-1.0, 1.0], size=P) * np.exp2(rng.uniform(-100, 100, size=P))).astype(np.float32)
        few_huge = rng.standard_normal(P).astype(np.float32)
        few_huge[rng.choice(P, size=topk // 3, replace=False)] = 1e30      # k' reaches far below the top digit
        negative = -np.exp2(rng.uniform(-20, 60, size=P)).astype(np.float32)
        one_spike = np.full(P, 1e-20, dtype=np.float32)
        one_spike[P // 2] = 3e38
        exact_top8 = np.exp2(rng.integers(0, 16, size=P).astype(np.float64) * 2.0).astype(np.float32)  # 8 digits
        _check_select(w, [spread, few_huge, negative, one_spike, exact_top8])
        # several candidates share the threshold key while its leading-bits bin stays small
        tied = (np.round(rng.standard_normal(P) * 4 * 64) / 64).astype(np.float32)
        tied_neg = (-np.abs(tied) - 1.0).astype(np.float32)
        smooth = (rng.standard_normal(P) * 4).astype(np.float32)
        _check_select(w, [tied, tied_neg, smooth, -smooth, tied])
        # subnormals, signed zeros, infinities and NaN among smooth scores
        specials = (rng.standard_normal(P) * 1e-39).astype(np.float32)
        mixed = smooth.copy()
        idx = rng.choice(P, size=P // 8, replace=False)
        mixed[idx] = rng.choice(np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1e-40, -1e-40], dtype=np.float32),
                                size=idx.size)
        mostly_minus_inf = np.where(rng.random(P) < 0.995, -np.inf, smooth).astype(np.float32)
        _check_select(w, [specials, mixed, mostly_minus_inf, np.abs(specials), mixed])


def test_select_rows_beyond_the_register_variants():
    """Rows of more than 65536 partitions: the long-row kernels, their fall-back that re-reads the
    scores per pass, and that kernel on its own for rows beyond 131072 partitions."""
    base = synth.config0().with_(num_q_heads=4, num_kv_heads=1)
    rng = np.random.default_rng(12)
    w = base.with_(seq_lens=(100000, 70001), partition_tokens=1, topk=500, sink_pages=1, recent_pages=2,
                   score_kind=synth.SCORE_SKETCH, name="huge_tokens")
    rows = [np.round(rng.standard_normal(n) * 20).astype(np.float32) / 20 for n in w.seq_lens]
    _check_select(w, rows)
    # smooth scores: the threshold bin is small, so the long-row kernels do not fall back
    _check_select(w, [(rng.standard_normal(n) * 3).astype(np.float32) for n in w.seq_lens])
    _check_select(w, [(np.round(rng.standard_normal(n) * 3 * 128) / 128).astype(np.float32) for n in w.seq_lens])
    # past the long-row kernels' range (131072 partitions): every pass re-reads the scores
    w3 = base.with_(seq_lens=(140000,), partition_tokens=1, topk=700, sink_pages=2, recent_pages=1,
                    score_kind=synth.SCORE_SKETCH, name="huge_tokens2")
    _check_select(w3, [rng.standard_normal(140000).astype(np.float32)])


@pytest.mark.parametrize("seed", range(24))
def test_select_random_rows(seed):
    """Row length drawn log-uniformly from 1 to 150000 partitions (every kernel variant and the
    two-launch path), random k, windows and score distributions with ties and special values."""
    rng = np.random.default_rng(4000 + seed)
    tp = int(rng.choice([1, 16]))
    P0 = int(np.exp(rng.uniform(0, np.log(150000))))
    lens = tuple(max(1, int(P0 * f)) * tp - int(rng.integers(0, tp)) for f in (1.0, rng.uniform(0.01, 1.0), 0.5))
    lens = tuple(max(n, 1) for n in lens)
    topk = int(rng.choice([0, 1, rng.integers(1, 64), rng.integers(1, 2000)]))
    w = synth.config0().with_(num_q_heads=4, num_kv_heads=1, seq_lens=lens, partition_tokens=tp, topk=topk,
                              topk_includes_forced=bool(rng.integers(0, 2)), sink_pages=int(rng.integers(0, 5)),
                              recent_pages=int(rng.integers(0, 9)),
                              score_kind=synth.SCORE_SKETCH if tp == 1 else synth.SCORE_MINMAX, name=f"selrand{seed}")
    print(f"seed {seed}: tp {tp} lens {lens} topk {topk} incl {w.topk_includes_forced} sink {w.sink_pages} "
          f"recent {w.recent_pages}", flush=True)

    def scores(P):
        kind = int(rng.integers(0, 6))
        x = rng.standard_normal(P)
        if kind == 0:
            out = x * 3
        elif kind == 1:
            out = np.round(x * 8) / 8                                          # heavy ties
        elif kind == 2:
            out = rng.choice([-1.0, 1.0], size=P) * np.exp2(rng.uniform(-60, 60, size=P))
        elif kind == 3:
            out = x.copy()
            idx = rng.choice(P, size=max(P // 6, 1), replace=False)
            out[idx] = rng.choice(np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1e-40]), size=idx.size)
        elif kind == 4:
            out = np.full(P, float(rng.integers(-3, 4)))                        # all equal
        else:
            out = 100.0 + x * 1e-3                                             # equal leading bits
        return out.astype(np.float32)

    _check_select(w, [scores(w.partitions(b)) for b in range(w.batch)])


@pytest.mark.parametrize("name", ["ragged_pages", "minmax_blocks", "mean_pages", "mean_blocks", "two_reps_blocks",
                                  "mean_quarter_pages", "tokens", "g8_blocks"])
def test_index_with_pages_that_are_not_resident(name):
    """Index over a row with holes (no slot, a slot number outside the pool): the fault is reported and every
    summary row that does not touch a missing page is still exactly the oracle's (the kernels look the
    slots of several pages up at once and keep the next page in flight: a hole must not shift that)."""
    from gpu_harness import DeviceWorkload, build_summaries, unpack_summary_rows
    w = _workloads()[name]
    data = synth.generate(w, spare_slots=3)
    dw = DeviceWorkload(data)
    chan = synth.sketch_channels(data) if w.score_kind == synth.SCORE_SKETCH else None
    rng = np.random.default_rng(5)
    dirs = dw.dir.cpu().numpy()
    holes = {}
    r = 0
    for b in range(w.batch):
        pages = (w.seq_lens[b] + 15) // 16
        for h in range(w.num_kv_heads):
            pick = sorted(set([0, pages - 1, pages // 2] + rng.integers(0, pages, size=3).tolist()))
            if (b + h) % 2:
                pick = pick[1:-1]                                     # rows whose first and last page stay
            holes[(b, h)] = pick
            for i, pg in enumerate(pick):
                chunk = int(dirs[r, pg // w.leaf_entries])
                dw.leaf_pool[chunk, pg % w.leaf_entries] = -1 if i % 2 == 0 else dw.pool_slots + 7 * i
            r += 1
    build_summaries(dw, chan)
    torch.cuda.synchronize()
    assert dw.spin.poll_status(dw.ws) == -6
    kd, kc = _kd_kc(w)
    summ_rows = unpack_summary_rows(dw.summaries, kd, kc)
    rpp = w.reps_per_partition if w.score_kind == synth.SCORE_REPMAX else 1
    tp = w.partition_tokens
    compared = 0
    for b in range(w.batch):
        for h in range(w.num_kv_heads):
            _, _, _, _, ref_rows, _, _ = _oracle_row_inputs(dw, b, h, chan)
            base = dw.row_base(b, h)
            got_rows = bf16.decode(summ_rows[base * rpp: base * rpp + ref_rows.shape[0]])
            touched = np.zeros(ref_rows.shape[0], dtype=bool)
            for pg in holes[(b, h)]:
                for p in range(16 * pg // tp, min((16 * pg + 15) // tp + 1, ref_rows.shape[0] // rpp)):
                    touched[p * rpp:(p + 1) * rpp] = True
            compared += int((~touched).sum())
            assert np.array_equal(got_rows[~touched], ref_rows[~touched]), f"{name}: rows away from the holes differ ({b}, {h})"
    assert compared > 0


def test_resolve_reports_missing_leaf_and_missing_slot():
    from gpu_harness import DEV, DeviceWorkload, build_summaries, run_step
    w = synth.config0().with_(seq_lens=(4096,), name="holes")
    data = synth.generate(w)
    dw = DeviceWorkload(data)
    build_summaries(dw)
    run_step(dw)
    dw.check_ok()
    sel0 = dw.sel.cpu().numpy()[0]
    # knock out the slot of one selected page
    victim = int(sel0[5])
    chunk = int(dw.dir.cpu().numpy()[0, victim // 512])
    dw.leaf_pool[chunk, victim % 512] = -1
    run_step(dw)
    assert dw.spin.poll_status(dw.ws) == -6
    slots = dw.slots.cpu().numpy()[0]
    assert slots[5] == -1 and (slots[:5] >= 0).all()
    assert dw.valid_mask.cpu().numpy()[0, 5] == 0
    dw.spin.workspace_init(dw.ws)
    # missing leaf
    dw.dir[0, 0] = -1
    run_step(dw)
    assert dw.spin.poll_status(dw.ws) == -6
