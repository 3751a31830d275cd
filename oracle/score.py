"""Select, scoring half: one scalar per partition (test infrastructure).

Select scores the summaries of all partitions against the current query
(Section 4.1, Select; Table 1, ``score(roped_q, k_sums)``).  The paper leaves
the score function to the algorithm; the three below are the ones the
workloads define.  A KV head serves a group of G query heads and pages are
head-wise per KV head (Section 5.2), so the group's scores are reduced to one
per KV head by a maximum.

``q`` is the group's queries ``[G][D]`` float64.
"""
import numpy as np


def score_minmax(q: np.ndarray, mins: np.ndarray, maxs: np.ndarray) -> np.ndarray:
    """s_p = max_g sum_d max(q[g,d]*min[p,d], q[g,d]*max[p,d]).

    The inner sum is an upper bound of q_g . k over every key k of the
    partition, because min <= k <= max holds per channel."""
    P = mins.shape[0]
    s = np.empty(P)
    for p in range(P):
        per_head = np.maximum(q * mins[p][None, :], q * maxs[p][None, :]).sum(axis=1)
        s[p] = per_head.max()
    return s


def score_sketch(q: np.ndarray, sketch: np.ndarray, channels) -> np.ndarray:
    """s_t = max_g sum_c q[g, channels[c]] * sketch[t, c] (exact q.k on the
    sketched channels)."""
    qc = q[:, np.asarray(channels, dtype=np.int64)]          # [G][C]
    return (sketch @ qc.T).max(axis=1)


def score_repmax(q: np.ndarray, reps: np.ndarray) -> np.ndarray:
    """s_p = max_g max_r q[g] . rep[p, r]."""
    dots = np.einsum("prd,gd->prg", reps, q)
    return dots.max(axis=(1, 2))
