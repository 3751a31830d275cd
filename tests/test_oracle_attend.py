"""Pins for attention over a selected set: textbook dense attention, closed
forms, the split/merge identity and structural invariants."""
import math

import numpy as np
from scipy.special import softmax

from oracle import attend


def _rand(seed, n=37, G=3, D=8):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((G, D)), rng.standard_normal((n, D)), rng.standard_normal((n, D))


def test_equals_textbook_dense_attention_when_all_tokens_selected():
    q, K, V = _rand(0)
    scale = 1 / math.sqrt(8)
    out, lse = attend.attend(q, K, V, scale)
    ref = softmax(scale * q @ K.T, axis=1) @ V
    assert np.allclose(out, ref, rtol=1e-13, atol=1e-13)
    assert np.allclose(lse, np.log(np.exp(scale * q @ K.T).sum(axis=1)), rtol=1e-13)


def test_pure_python_brute_force():
    q, K, V = _rand(1, n=5, G=2, D=3)
    out, _ = attend.attend(q, K, V, 0.7)
    for g in range(2):
        logits = [0.7 * sum(q[g][d] * K[t][d] for d in range(3)) for t in range(5)]
        z = sum(math.exp(x) for x in logits)
        for d in range(3):
            ref = sum(math.exp(logits[t]) / z * V[t][d] for t in range(5))
            assert abs(out[g][d] - ref) < 1e-13


def test_equal_keys_give_mean_value_and_huge_logit_picks_its_value():
    q, K, V = _rand(2)
    Keq = np.repeat(K[:1], K.shape[0], axis=0)
    out, _ = attend.attend(q, Keq, V, 0.3)
    assert np.allclose(out, np.repeat(V.mean(axis=0)[None], 3, axis=0), rtol=1e-13, atol=1e-13)
    K2 = K.copy()
    K2[11] = 1e3 * q[0]
    out, _ = attend.attend(q[:1], K2, V, 1.0)
    assert np.allclose(out[0], V[11], atol=1e-12)


def test_scale_is_applied_to_logits():
    q, K, V = _rand(3)
    a, _ = attend.attend(q, K, V, 0.5)
    b, _ = attend.attend(0.5 * q, K, V, 1.0)
    c, _ = attend.attend(q, K, V, 1.0)
    assert np.allclose(a, b, rtol=1e-13, atol=1e-13) and not np.allclose(a, c)


def test_split_merge_identity():
    q, K, V = _rand(4, n=50)
    scale = 0.35
    full, _ = attend.attend(q, K, V, scale)
    parts = []
    for lo, hi in [(0, 7), (7, 8), (8, 33), (33, 50)]:
        logits = scale * q @ K[lo:hi].T
        m = logits.max(axis=1)
        w = np.exp(logits - m[:, None])
        parts.append((m, w.sum(axis=1), w @ V[lo:hi]))
    assert np.allclose(attend.merge_partials(parts), full, rtol=1e-13, atol=1e-14)


def test_permutation_invariance_and_convexity():
    q, K, V = _rand(5)
    out, _ = attend.attend(q, K, V, 0.4)
    perm = np.random.default_rng(9).permutation(K.shape[0])
    out2, _ = attend.attend(q, K[perm], V[perm], 0.4)
    assert np.allclose(out, out2, rtol=1e-13, atol=1e-14)
    assert (out <= V.max(axis=0) + 1e-12).all() and (out >= V.min(axis=0) - 1e-12).all()


def test_gather_respects_masks_and_empty_selection():
    Kp = np.arange(2 * 4 * 2, dtype=np.float64).reshape(2, 4, 2)
    Vp = -Kp
    ks, vs = attend.gather_tokens(Kp, Vp, [0b0101, 0b1000])
    assert np.array_equal(ks, np.stack([Kp[0, 0], Kp[0, 2], Kp[1, 3]]))
    assert np.array_equal(vs, -ks)
    out, lse = attend.attend(np.ones((2, 2)), *attend.gather_tokens(Kp, Vp, [0, 0]), 1.0)
    assert (out == 0).all() and np.isneginf(lse).all()
