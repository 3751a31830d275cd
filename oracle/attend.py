"""Attention over the selected KV (test infrastructure).

Given the selected set, attention is the textbook definition (Section 4.1,
Attention: the output is computed from the selected KV tokens with standard
attention): for every query head g of the KV head's group

    out_g = sum_t softmax_t(scale * q_g . k_t) * v_t,   t over the selected tokens.

At decode there is no causal mask: the current token's K/V already sits in the
cache.  An empty selection gives a zero output and lse = -inf.
"""
import numpy as np


def attend(q: np.ndarray, K_S: np.ndarray, V_S: np.ndarray, scale: float):
    """q ``[G][D]``, K_S/V_S ``[n][D]`` float64 -> (out ``[G][D]``, lse ``[G]``)."""
    G, D = q.shape
    if K_S.shape[0] == 0:
        return np.zeros((G, D)), np.full(G, -np.inf)
    logits = scale * (q @ K_S.T)                         # [G][n]
    m = logits.max(axis=1, keepdims=True)
    w = np.exp(logits - m)
    l = w.sum(axis=1, keepdims=True)
    out = (w @ V_S) / l
    return out, (m + np.log(l)).reshape(G)


def gather_tokens(K_pages: np.ndarray, V_pages: np.ndarray, masks):
    """Flatten resolved pages ``[n_pages][page][D]`` to the attended tokens, in
    page order then token order, keeping only tokens whose mask bit is set."""
    ks, vs = [], []
    for i, m in enumerate(masks):
        for t in range(K_pages.shape[1]):
            if (int(m) >> t) & 1:
                ks.append(K_pages[i, t])
                vs.append(V_pages[i, t])
    D = K_pages.shape[2]
    if not ks:
        return np.zeros((0, D)), np.zeros((0, D))
    return np.stack(ks), np.stack(vs)


def merge_partials(parts):
    """Combine online-softmax partial results ``(m [G], l [G], acc [G][D])`` of
    disjoint token subsets into the attention output over their union.  Used
    only to pin the split/merge identity the GPU path relies on."""
    m = np.max(np.stack([p[0] for p in parts]), axis=0)
    l = sum(p[1] * np.exp(p[0] - m) for p in parts)
    acc = sum(p[2] * np.exp(p[0] - m)[:, None] for p in parts)
    return acc / l[:, None]
