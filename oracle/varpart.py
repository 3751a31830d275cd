"""Variable-length partitions (test infrastructure).

A partition is a contiguous group of tokens of any size -- a block, a cluster
or a single token (Section 4.1) -- that owns whole pages: the Partition Offset
table says where its page list starts and the Meta-partition table how many
tokens it holds, from which its page count follows (Section 5.2).  Only the last
page of a partition may be partly filled.

A row's layout is two lists: ``first_page[p]`` and ``tokens[p]``; partitions
ascend and follow one another without gaps.  The functions below restate Index
(min/max), the forced-partition rule, top-k selection and slot resolution for
such a layout; with a uniform layout they coincide with the fixed-size versions.
"""
import math
from typing import Dict, List, Tuple

import numpy as np


def npages(tokens: int, page_tokens: int) -> int:
    return -(-tokens // page_tokens)


def uniform_layout(seq_len: int, page_tokens: int, partition_tokens: int):
    """The layout that cutting a context every ``partition_tokens`` tokens gives
    (partition_tokens a multiple of page_tokens)."""
    assert partition_tokens % page_tokens == 0
    P = -(-seq_len // partition_tokens)
    first = [p * partition_tokens // page_tokens for p in range(P)]
    toks = [min(partition_tokens, seq_len - p * partition_tokens) for p in range(P)]
    return first, toks


def row_pages(first_page: List[int], tokens: List[int], page_tokens: int) -> int:
    return first_page[-1] + npages(tokens[-1], page_tokens) if first_page else 0


def partition_page_list(first_page, tokens, p, page_tokens) -> List[int]:
    return list(range(first_page[p], first_page[p] + npages(tokens[p], page_tokens)))


def page_masks(first_page, tokens, p, page_tokens) -> List[int]:
    """Token mask of every page of partition p."""
    out = []
    for k in range(npages(tokens[p], page_tokens)):
        n = min(max(tokens[p] - page_tokens * k, 0), page_tokens)
        out.append((1 << n) - 1)
    return out


def minmax_summaries(K_pages: np.ndarray, first_page, tokens, page_tokens: int):
    """``K_pages`` = the row's keys in page order ``[pages * page_tokens][D]``.
    Elementwise min and max over each partition's tokens."""
    P, D = len(first_page), K_pages.shape[1]
    mins, maxs = np.empty((P, D)), np.empty((P, D))
    for p in range(P):
        t0 = first_page[p] * page_tokens
        blk = K_pages[t0: t0 + tokens[p]]
        mins[p], maxs[p] = blk.min(axis=0), blk.max(axis=0)
    return mins, maxs


def centroids(K_pages: np.ndarray, first_page, tokens, page_tokens: int):
    """One representative key per partition: the mean key of its tokens (a
    cluster's centroid, a block's landmark; Section 4.1, Index), rounded to bf16
    for storage.  Returns the stored values as float64 ``[P][1][D]``, the shape
    the representative-key score takes."""
    from . import bf16
    P, D = len(first_page), K_pages.shape[1]
    out = np.empty((P, 1, D))
    for p in range(P):
        t0 = first_page[p] * page_tokens
        blk = K_pages[t0: t0 + tokens[p]]
        out[p, 0] = bf16.decode(bf16.encode_rne(blk.sum(axis=0) / float(tokens[p])))
    return out


def forced_pages(first_page, tokens, page_tokens, sink_pages, recent_pages) -> List[int]:
    pages = row_pages(first_page, tokens, page_tokens)
    s = set(range(0, min(sink_pages, pages)))
    s |= set(range(max(pages - recent_pages, 0), pages))
    return sorted(s)


def forced_partitions(first_page, tokens, page_tokens, sink_pages, recent_pages) -> List[int]:
    fp = set(forced_pages(first_page, tokens, page_tokens, sink_pages, recent_pages))
    return [p for p in range(len(first_page))
            if all(x in fp for x in partition_page_list(first_page, tokens, p, page_tokens))] if fp else []


def select_topk(scores, first_page, tokens, page_tokens, topk, topk_includes_forced, sink_pages,
                recent_pages) -> List[int]:
    P = len(first_page)
    forced = forced_partitions(first_page, tokens, page_tokens, sink_pages, recent_pages)
    fset = set(forced)
    kprime = max(topk - len(forced) if topk_includes_forced else topk, 0)

    def rank_key(i):
        s = float(scores[i])
        if s != s:
            s = -math.inf
        return (-s, i)

    best = sorted((p for p in range(P) if p not in fset), key=rank_key)[:kprime]
    return sorted(fset | set(best))


def resolve_slots(sel, first_page, tokens, page_tokens, sink_pages, recent_pages,
                  page_map: Dict[Tuple[int, int], int], row: int):
    """(page_ids, slots, masks), ascending by page; forced pages outside every
    selected partition are attended too, with the mask of the partition they lie in."""
    masks: Dict[int, int] = {}
    owner = {}
    for p in range(len(first_page)):
        for pg, m in zip(partition_page_list(first_page, tokens, p, page_tokens),
                         page_masks(first_page, tokens, p, page_tokens)):
            owner[pg] = m
    for pg in forced_pages(first_page, tokens, page_tokens, sink_pages, recent_pages):
        masks[pg] = owner[pg]
    for p in sel:
        for pg, m in zip(partition_page_list(first_page, tokens, p, page_tokens),
                         page_masks(first_page, tokens, p, page_tokens)):
            masks[pg] = m
    page_ids = sorted(masks)
    slots = [page_map[(row, pg)] for pg in page_ids]
    return page_ids, slots, [masks[pg] for pg in page_ids]
