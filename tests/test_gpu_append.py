"""Decode-time Index: appending tokens one at a time must leave the pool and the
summaries exactly as packing / building them for the longer context would
(bit-exact against the oracle's summaries of the grown context), and a decode
step afterwards must match the oracle."""
import numpy as np
import pytest
import torch

from oracle import bf16, index
from paper_2604_26837_amd import runner, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
KD_KC = {synth.SCORE_MINMAX: (256, 8), synth.SCORE_REPMAX: (128, 8), synth.SCORE_SKETCH: (16, 4)}


def _summary_rows(layer, kd, kc):
    raw = layer.summaries.cpu().numpy().view(np.uint16)
    return raw.reshape(-1, kd // kc, 16, kc).transpose(0, 2, 1, 3).reshape(-1, kd)


def _oracle_rows(w, K, n, chan_h):
    if w.score_kind == synth.SCORE_MINMAX:
        mins, maxs = index.minmax_summaries(K, n, w.partition_tokens)
        return np.concatenate([maxs, mins], axis=1)
    if w.score_kind == synth.SCORE_REPMAX:
        return index.block_representatives(K, n, w.partition_tokens, w.reps_per_partition).reshape(-1, w.head_dim)
    return index.key_sketch(K, n, chan_h)


@pytest.mark.parametrize("kind", ["minmax_page", "minmax_block", "repmax", "sketch", "mean_page", "two_reps_block"])
def test_append_tokens(kind):
    c0 = synth.config0().with_(num_q_heads=8, num_kv_heads=2)
    final = (500, 128 * 3 + 37, 70)
    start = (455, 128 * 3 - 10, 16)
    w = {
        "minmax_page": c0.with_(seq_lens=final, topk=8, sink_pages=1, recent_pages=1, name="a1"),
        "minmax_block": c0.with_(seq_lens=final, partition_tokens=64, topk=3, sink_pages=1, recent_pages=1, name="a2"),
        "repmax": c0.with_(seq_lens=final, partition_tokens=128, score_kind=synth.SCORE_REPMAX, topk=2,
                           topk_includes_forced=False, sink_pages=1, recent_pages=2, block_mean_std=0.5, name="a3"),
        "mean_page": c0.with_(seq_lens=final, score_kind=synth.SCORE_REPMAX, reps_per_partition=1, topk=8,
                              sink_pages=1, recent_pages=1, block_mean_std=0.5, name="a5"),
        "two_reps_block": c0.with_(seq_lens=final, partition_tokens=64, score_kind=synth.SCORE_REPMAX,
                                   reps_per_partition=2, topk=3, topk_includes_forced=False, sink_pages=1,
                                   recent_pages=1, block_mean_std=0.5, name="a6"),
        "sketch": c0.with_(seq_lens=final, partition_tokens=1, score_kind=synth.SCORE_SKETCH, topk=40,
                           sink_pages=0, recent_pages=0, name="a4"),
    }[kind]
    _check_append(w, start)


@pytest.mark.parametrize("seed", range(16))
def test_append_random_workloads(seed):
    """Summary kind, partition size (down to single tokens: token-major slots), representative count,
    heads and the appended stretch drawn at random."""
    rng = np.random.default_rng(600 + seed)
    kind = int(rng.choice([synth.SCORE_MINMAX, synth.SCORE_REPMAX, synth.SCORE_SKETCH]))
    reps = int(rng.choice([1, 2, 4])) if kind == synth.SCORE_REPMAX else 4
    if kind == synth.SCORE_SKETCH:
        tp = 1
    elif kind == synth.SCORE_MINMAX:
        tp = int(rng.choice([1, 2, 4, 8, 16, 32, 64, 128]))
    else:
        tp = int(rng.choice([t for t in (4, 8, 16, 32, 64, 128) if t % reps == 0]))
    hkv, g = int(rng.choice([1, 2, 3])), int(rng.choice([1, 2, 4, 5]))
    final = tuple(int(x) for x in rng.integers(20, 700, size=int(rng.integers(1, 4))))
    start = tuple(max(1, f - int(rng.integers(1, 90))) for f in final)
    w = synth.config0().with_(seq_lens=final, num_q_heads=g * hkv, num_kv_heads=hkv, partition_tokens=tp,
                              score_kind=kind, reps_per_partition=reps, topk=int(rng.integers(1, 30)),
                              topk_includes_forced=bool(rng.integers(0, 2)), sink_pages=int(rng.integers(0, 3)),
                              recent_pages=int(rng.integers(0, 3)),
                              block_mean_std=0.5 if kind == synth.SCORE_REPMAX else 0.0, name=f"append_random{seed}")
    print(f"seed {seed}: kind {kind} reps {reps} tp {tp} group {g} kv {hkv} final {final} start {start}", flush=True)
    _check_append(w, start)


def _check_append(w, start):
    final = w.seq_lens
    data = synth.generate(w)
    truth = torch.from_numpy(data.pool_bits.view(np.int16).copy()).to(DEV).view(torch.bfloat16)
    # the layer starts from a pool whose tokens in [start, final) hold junk
    junk = truth.clone()
    for b in range(w.batch):
        for h in range(w.num_kv_heads):
            for t in range(start[b], final[b]):
                junk[int(data.slot_of[b][h][t // 16]), :, t % 16] = 777.0
    layer = runner.LayerState.from_natural_pool(w, data.slot_of, junk)
    ref = runner.LayerState.from_natural_pool(w, data.slot_of, truth)
    chan = synth.sketch_channels(data) if w.score_kind == synth.SCORE_SKETCH else None
    if chan is not None:
        layer.set_channels(chan)
    cur = list(start)
    layer.seq_lens.copy_(torch.tensor(cur, dtype=torch.int32))
    layer.build_summaries()
    kd, kc = KD_KC[w.score_kind]
    rpp = w.reps_per_partition if w.score_kind == synth.SCORE_REPMAX else 1
    nat = data.pool_bits
    step = 0
    while any(c < f for c, f in zip(cur, final)):
        k_new = np.zeros((w.batch, w.num_kv_heads, w.head_dim), dtype=np.uint16)
        v_new = np.zeros_like(k_new)
        active = [c < f for c, f in zip(cur, final)]
        for b in range(w.batch):
            t = min(cur[b], final[b] - 1)
            for h in range(w.num_kv_heads):
                s = int(data.slot_of[b][h][t // 16])
                k_new[b, h], v_new[b, h] = nat[s, 0, t % 16], nat[s, 1, t % 16]
        # requests that are complete re-append their last token at the same position: a no-op rewrite
        lens = torch.tensor([min(c, f - 1) for c, f in zip(cur, final)], dtype=torch.int32, device=DEV)
        layer.spin.append_kv(w.batch, torch.from_numpy(k_new.view(np.int16)).to(DEV).view(torch.bfloat16),
                             torch.from_numpy(v_new.view(np.int16)).to(DEV).view(torch.bfloat16), lens, layer.kv_pool,
                             layer.dir, layer.leaf_pool, layer.part_offsets, layer.chan, layer.summaries, layer.ws)
        cur = [min(c + 1, f) for c, f in zip(cur, final)]
        step += 1
        if step % 13 == 0 or not any(c < f for c, f in zip(cur, final)):
            torch.cuda.synchronize()
            assert layer.status() == 0
            rows = _summary_rows(layer, kd, kc)
            for b in range(w.batch):
                for h in range(w.num_kv_heads):
                    kb, _ = data.logical_kv_bits(b, h)
                    want = _oracle_rows(w, bf16.decode(kb), cur[b], chan[h] if chan is not None else None)
                    base = layer.row_base(b, h) * rpp
                    got = bf16.decode(rows[base: base + want.shape[0]])
                    assert np.array_equal(got, want), f"step {step} request {b} head {h}"
    assert torch.equal(layer.kv_pool.view(torch.int16), ref.kv_pool.view(torch.int16))
    # a decode step on the grown context agrees with a layer built from scratch
    layer.seq_lens.copy_(torch.tensor(final, dtype=torch.int32))
    if chan is not None:
        ref.set_channels(chan)
    ref.build_summaries()
    q = torch.from_numpy(data.q_bits.view(np.int16).copy()).to(DEV).view(torch.bfloat16)
    layer.step(q)
    ref.step(q)
    torch.cuda.synchronize()
    assert layer.status() == 0 and ref.status() == 0
    assert torch.equal(layer.sel, ref.sel) and torch.equal(layer.out.view(torch.int16), ref.out.view(torch.int16))


def test_append_without_slot_or_room_is_reported():
    w = synth.config0().with_(seq_lens=(64,), num_q_heads=8, num_kv_heads=2, topk=4, name="full")
    data = synth.generate(w)
    natural = torch.from_numpy(data.pool_bits.view(np.int16).copy()).to(DEV).view(torch.bfloat16)
    layer = runner.LayerState.from_natural_pool(w, data.slot_of, natural)
    layer.build_summaries()
    z = torch.zeros((1, 2, 128), dtype=torch.bfloat16, device=DEV)
    before = layer.kv_pool.clone()
    layer.spin.append_kv(1, z, z, layer.seq_lens, layer.kv_pool, layer.dir, layer.leaf_pool, layer.part_offsets,
                         None, layer.summaries, layer.ws)     # position 64: page 4 has no slot, partition 4 no room
    assert layer.status() in (-1, -6)
    assert torch.equal(before.view(torch.int16), layer.kv_pool.view(torch.int16))
