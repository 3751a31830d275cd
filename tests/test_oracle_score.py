"""Pins for Index summaries and the three score functions: brute force in pure
Python, the Quest upper-bound property, and special cases that reduce to an
exact q.k."""
import numpy as np
import pytest

from oracle import bf16, index, score
from paper_2604_26837_amd import synth


def _row(seed, tokens, D=8, G=2):
    rng = np.random.default_rng(seed)
    K = bf16.decode(synth.f32_to_bf16_bits(rng.standard_normal((tokens, D)).astype(np.float32)))
    q = bf16.decode(synth.f32_to_bf16_bits(rng.standard_normal((G, D)).astype(np.float32)))
    return q, K


def _brute_minmax(q, K, seq_len, T):
    P = -(-seq_len // T)
    out = []
    for p in range(P):
        toks = range(p * T, min((p + 1) * T, seq_len))
        best = None
        for g in range(q.shape[0]):
            tot = 0.0
            for d in range(q.shape[1]):
                lo = min(K[t][d] for t in toks)
                hi = max(K[t][d] for t in toks)
                tot += max(q[g][d] * lo, q[g][d] * hi)
            best = tot if best is None else max(best, tot)
        out.append(best)
    return np.array(out)


@pytest.mark.parametrize("seq_len,T", [(64, 16), (61, 16), (7, 4), (33, 1)])
def test_minmax_matches_pure_python_brute_force(seq_len, T):
    q, K = _row(1, 80)
    K[seq_len:] = 1e6          # filler beyond the context must never be seen
    mins, maxs = index.minmax_summaries(K, seq_len, T)
    got = score.score_minmax(q, mins, maxs)
    ref = _brute_minmax(q, K, seq_len, T)
    assert got.shape == ref.shape
    assert np.allclose(got, ref, rtol=1e-14, atol=1e-14)


def test_minmax_summaries_bracket_and_are_attained():
    q, K = _row(2, 96, D=16)
    seq_len, T = 90, 16
    mins, maxs = index.minmax_summaries(K, seq_len, T)
    for p in range(mins.shape[0]):
        blk = K[p * T:min((p + 1) * T, seq_len)]
        assert (mins[p] <= blk).all() and (blk <= maxs[p]).all()
        for d in range(K.shape[1]):
            assert mins[p, d] in blk[:, d] and maxs[p, d] in blk[:, d]


def test_quest_bound_on_config0_every_partition():
    """sum_d max(q*min, q*max) >= q.k for every key of the partition, per head."""
    w = synth.config0()
    data = synth.generate(w)
    g = w.group
    for h in range(w.num_kv_heads):
        kb, _ = data.logical_kv_bits(0, h)
        K = bf16.decode(kb)
        q = bf16.decode(data.q_bits[0, h * g:(h + 1) * g])
        mins, maxs = index.minmax_summaries(K, w.seq_lens[0], w.partition_tokens)
        per_head = np.maximum(q[:, None, :] * mins[None], q[:, None, :] * maxs[None]).sum(-1)  # [G][P]
        true = (q @ K.T).reshape(g, -1, w.partition_tokens).max(axis=2)                          # [G][P]
        assert (per_head >= true - 1e-12).all()
        s = score.score_minmax(q, mins, maxs)
        assert np.allclose(s, per_head.max(axis=0), rtol=0, atol=1e-12)
        # the bound is not vacuous: it is within a modest factor for N(0,1) data
        assert (s > true.max(axis=0)).all()


def test_minmax_single_token_partition_is_exact_dot():
    q, K = _row(3, 40, D=32, G=4)
    mins, maxs = index.minmax_summaries(K, 40, 1)
    assert np.array_equal(mins, K) and np.array_equal(maxs, K)
    s = score.score_minmax(q, mins, maxs)
    assert np.allclose(s, (q @ K.T).max(axis=0), rtol=1e-14, atol=1e-14)


def test_minmax_sign_handling():
    # one channel, hand-computed: q>0 picks max, q<0 picks min
    q = np.array([[2.0, -3.0]])
    mins = np.array([[-1.0, -5.0]])
    maxs = np.array([[4.0, 0.5]])
    assert score.score_minmax(q, mins, maxs)[0] == 2.0 * 4.0 + (-3.0) * (-5.0)
    # group reduction is a max over heads, not a sum or a mean
    q2 = np.array([[2.0, -3.0], [-1.0, 1.0]])
    assert score.score_minmax(q2, mins, maxs)[0] == 23.0
    q3 = np.array([[-1.0, 1.0], [0.0, 0.0]])
    assert score.score_minmax(q3, mins, maxs)[0] == 1.5


def test_sketch_full_channels_is_exact_and_topk_matches_true_logits():
    q, K = _row(4, 200, D=16, G=4)
    chan = np.arange(16)
    sk = index.key_sketch(K, 200, chan)
    s = score.score_sketch(q, sk, chan)
    ref = (q @ K.T).max(axis=0)
    assert np.allclose(s, ref, rtol=1e-14, atol=1e-14)
    assert set(np.argsort(-s, kind="stable")[:10]) == set(np.argsort(-ref, kind="stable")[:10])


def test_sketch_subset_brute_force():
    q, K = _row(5, 50, D=12, G=3)
    chan = [1, 4, 7, 11]
    s = score.score_sketch(q, index.key_sketch(K, 47, chan), chan)
    assert s.shape == (47,)
    for t in range(47):
        ref = max(sum(q[g][c] * K[t][c] for c in chan) for g in range(3))
        assert abs(s[t] - ref) < 1e-13


def test_repmax_constant_blocks_reduce_to_dot():
    rng = np.random.default_rng(6)
    D, T, P = 8, 16, 5
    centers = bf16.decode(synth.f32_to_bf16_bits(rng.standard_normal((P, D)).astype(np.float32)))
    K = np.repeat(centers, T, axis=0)
    q = rng.standard_normal((2, D))
    reps = index.block_representatives(K, P * T, T, 4)
    assert np.array_equal(reps, np.repeat(centers[:, None, :], 4, axis=1))
    s = score.score_repmax(q, reps)
    assert np.allclose(s, (q @ centers.T).max(axis=0), rtol=1e-14, atol=1e-14)


@pytest.mark.parametrize("R", [1, 2, 4])
def test_repmax_brute_force_and_ragged_tail(R):
    """R = 4: quarter means; R = 2: half means; R = 1: the mean key of the whole partition (a landmark)."""
    q, K = _row(7, 64, D=8, G=2)
    seq_len, T = 37, 16                # last block has 5 tokens: with R = 4 its quarters 2, 3 are empty
    K[seq_len:] = 1e6
    reps = index.block_representatives(K, seq_len, T, R)
    assert reps.shape == (3, R, 8)
    sub = T // R
    # sub-range means rounded to bf16, written out by hand
    for p in range(3):
        for r in range(R):
            t0, t1 = p * T + r * sub, min(p * T + r * sub + sub, seq_len)
            if t1 > t0:
                mean = sum(K[t] for t in range(t0, t1)) / (t1 - t0)
                assert np.array_equal(reps[p, r], bf16.decode(bf16.encode_rne(mean)))
            else:
                assert np.array_equal(reps[p, r], reps[p, 0])
    s = score.score_repmax(q, reps)
    for p in range(3):
        ref = max(float(q[g] @ reps[p, r]) for g in range(2) for r in range(R))
        assert abs(s[p] - ref) < 1e-13
