"""Select, top-k half (test infrastructure).

Keeps the k most critical partitions of a row (Table 1, ``-> topk``;
Section 4.2: Select "simply implements top-k scoring").  Pages that must
always take part -- the first ``sink_pages`` pages and the last
``recent_pages`` pages of the context -- are never candidates and are always
attended (Section 4.2: the recent window is filtered out of the candidates and
always participates in attention).

Conventions fixed here: ties go to the lower partition id; +0.0 and -0.0 tie;
NaN ranks below everything; the result is ascending by partition id.
"""
import math
from typing import List


def forced_pages(seq_len: int, page_tokens: int, sink_pages: int, recent_pages: int) -> List[int]:
    """Ascending ids of the pages that always participate."""
    pages = -(-seq_len // page_tokens)
    s = set(range(0, min(sink_pages, pages)))
    s |= set(range(max(pages - recent_pages, 0), pages))
    return sorted(s)


def partition_pages(p: int, seq_len: int, page_tokens: int, partition_tokens: int) -> List[int]:
    """Logical pages that hold at least one valid token of partition ``p``."""
    t0 = p * partition_tokens
    t1 = min(t0 + partition_tokens, seq_len)
    if t1 <= t0:
        return []
    return list(range(t0 // page_tokens, (t1 - 1) // page_tokens + 1))


def forced_partitions(seq_len, page_tokens, partition_tokens, sink_pages, recent_pages) -> List[int]:
    """Partitions all of whose pages are forced pages: they are not candidates
    and are always part of the selection."""
    fp = set(forced_pages(seq_len, page_tokens, sink_pages, recent_pages))
    if not fp:
        return []
    P = -(-seq_len // partition_tokens)
    out = []
    for p in range(P):
        pg = partition_pages(p, seq_len, page_tokens, partition_tokens)
        if pg and all(x in fp for x in pg):
            out.append(p)
    return out


def select_topk(scores, seq_len: int, page_tokens: int, partition_tokens: int, topk: int,
                topk_includes_forced: bool, sink_pages: int, recent_pages: int) -> List[int]:
    """Forced partitions plus the k' best-scoring candidates, ascending.

    k' = topk - (number of forced partitions) when the budget includes them,
    else topk; never negative; all candidates are taken when fewer exist."""
    P = -(-seq_len // partition_tokens)
    assert len(scores) >= P
    forced = forced_partitions(seq_len, page_tokens, partition_tokens, sink_pages, recent_pages)
    fset = set(forced)
    kprime = topk - len(forced) if topk_includes_forced else topk
    kprime = max(kprime, 0)

    def rank_key(i):
        s = float(scores[i])
        if s != s:
            s = -math.inf
        return (-s, i)          # -0.0 == 0.0 compares equal, so signed zeros tie

    cands = [p for p in range(P) if p not in fset]
    best = sorted(cands, key=rank_key)[:kprime]
    return sorted(fset | set(best))


def pin_scores(scores, seq_len: int, partition_tokens: int, pinned):
    """Outlier partitions that, like the recent window, always participate in
    attention (Section 4.2): a pinned partition ranks above every finite score,
    i.e. as a score of +inf.  Returns a copy of ``scores`` (float64); ids outside
    the row's partitions are ignored."""
    import numpy as np
    P = -(-seq_len // partition_tokens)
    out = np.array(scores, dtype=np.float64, copy=True)
    for p in pinned:
        if 0 <= p < P:
            out[p] = math.inf
    return out
