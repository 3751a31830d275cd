"""Index: per-partition summaries kept in HBM for Select (test infrastructure).

The paper's pipeline builds, at Index time, one summary per partition that
Select later scores against the query (Section 4.1, Index and Offload; Table 1,
"k_sums"; Section 2.2, the "auxiliary sketch" pattern).  The three summary
kinds below are the ones the synthetic workloads use.

All functions take the decoded keys of ONE row (one request, one KV head) in
logical token order, ``K[tokens][D]`` float64, and the row's context length;
only tokens ``< seq_len`` take part.
"""
import numpy as np

from . import bf16


def num_partitions(seq_len: int, partition_tokens: int) -> int:
    return -(-seq_len // partition_tokens)


def minmax_summaries(K: np.ndarray, seq_len: int, partition_tokens: int):
    """Elementwise minimum and maximum key of every partition (Quest-style
    metadata).  Returns ``(mins, maxs)``, each ``[P][D]``.  Values are a subset
    of the stored bf16 keys, hence exactly representable."""
    P = num_partitions(seq_len, partition_tokens)
    D = K.shape[1]
    mins = np.empty((P, D))
    maxs = np.empty((P, D))
    for p in range(P):
        t0 = p * partition_tokens
        t1 = min(t0 + partition_tokens, seq_len)
        mins[p] = K[t0:t1].min(axis=0)
        maxs[p] = K[t0:t1].max(axis=0)
    return mins, maxs


def block_representatives(K: np.ndarray, seq_len: int, partition_tokens: int, reps: int):
    """``reps`` representative keys per partition: the mean key of each of its
    ``reps`` equal sub-ranges, rounded to bf16 for storage.  A sub-range of a
    ragged last partition that holds no valid token repeats the partition's
    first representative, so it never changes a maximum over representatives.
    Returns the stored values as float64 ``[P][reps][D]``."""
    P = num_partitions(seq_len, partition_tokens)
    D = K.shape[1]
    sub = partition_tokens // reps
    out = np.empty((P, reps, D))
    for p in range(P):
        for r in range(reps):
            t0 = p * partition_tokens + r * sub
            t1 = min(t0 + sub, seq_len)
            if t1 > t0:
                mean = K[t0:t1].sum(axis=0) / float(t1 - t0)
                out[p, r] = bf16.decode(bf16.encode_rne(mean))
            else:
                out[p, r] = out[p, 0]
    return out


def key_sketch(K: np.ndarray, seq_len: int, channels) -> np.ndarray:
    """Token-granularity summary: the stored key restricted to ``channels``.
    Returns ``[seq_len][C]``."""
    return K[:seq_len][:, np.asarray(channels, dtype=np.int64)]
