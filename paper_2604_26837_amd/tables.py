"""Host-side set-up of the metadata the device stages read.

The page map is two-level (Section 5.4): a small per-row directory whose
entries point at fixed-size leaf chunks that are handed out only for page
ranges that actually hold pages, so metadata grows with the mapped pages and
not with the worst-case context.  This module only builds those arrays from a
logical->slot map and computes the padded partition offsets; the walk itself
runs on the device.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

PART_ALIGN = 16


def cdiv(a: int, b: int) -> int:
    return -(-a // b)


def part_offsets(seq_lens: Sequence[int], partition_tokens: int) -> np.ndarray:
    """Prefix sum of per-request partition counts rounded up to PART_ALIGN."""
    out = np.zeros(len(seq_lens) + 1, dtype=np.int32)
    for b, n in enumerate(seq_lens):
        p = cdiv(n, partition_tokens)
        out[b + 1] = out[b] + cdiv(p, PART_ALIGN) * PART_ALIGN
    return out


def part_offsets_from_counts(max_parts_per_request: Sequence[int]) -> np.ndarray:
    """Padded offsets when every request brings its own partition count (the
    largest over its KV heads)."""
    out = np.zeros(len(max_parts_per_request) + 1, dtype=np.int32)
    for b, p in enumerate(max_parts_per_request):
        out[b + 1] = out[b] + cdiv(p, PART_ALIGN) * PART_ALIGN
    return out


def partition_tables(layouts, offsets: np.ndarray, num_kv_heads: int):
    """Flattens per-row ``(first_page, tokens)`` lists into the three device
    tables of variable-length partitions, indexed like the score array."""
    rows = len(layouts) * num_kv_heads
    total = int(offsets[-1]) * num_kv_heads
    count = np.zeros(rows, dtype=np.int32)
    first = np.zeros(total, dtype=np.int32)
    toks = np.zeros(total, dtype=np.int32)
    for b, per_head in enumerate(layouts):
        for h, (fp, tk) in enumerate(per_head):
            base = row_base(offsets, b, h, num_kv_heads)
            count[b * num_kv_heads + h] = len(fp)
            first[base: base + len(fp)] = fp
            toks[base: base + len(tk)] = tk
    return count, first, toks


def row_base(offsets: np.ndarray, b: int, h: int, num_kv_heads: int) -> int:
    """First entry of row (b, h) in the scores / summary-row arrays."""
    pp = int(offsets[b + 1] - offsets[b])
    return num_kv_heads * int(offsets[b]) + h * pp


def build_two_level(slot_of: List[np.ndarray], dir_stride: int, leaf_entries: int,
                    allocate_all: bool = False) -> Tuple[np.ndarray, np.ndarray]:
    """``slot_of[b]`` = int32 ``[H_kv][pages_b]`` (-1 = page not resident).

    Returns ``(dir [rows][dir_stride], leaf_pool [chunks][leaf_entries])``.  A
    leaf chunk is allocated for a 512-page range of a row only if that range
    holds at least one resident page (``allocate_all``: for every range inside
    the row's context, as budget mode needs, where any page may be admitted
    later); everything else stays -1."""
    rows = sum(s.shape[0] for s in slot_of)
    directory = np.full((rows, dir_stride), -1, dtype=np.int32)
    leaves = []
    r = 0
    for s in slot_of:
        for h in range(s.shape[0]):
            pages = s.shape[1]
            for ci in range(cdiv(pages, leaf_entries)):
                seg = s[h, ci * leaf_entries:(ci + 1) * leaf_entries]
                if allocate_all or (seg >= 0).any():
                    leaf = np.full(leaf_entries, -1, dtype=np.int32)
                    leaf[:len(seg)] = seg
                    directory[r, ci] = len(leaves)
                    leaves.append(leaf)
            r += 1
    if not leaves:
        leaves.append(np.full(leaf_entries, -1, dtype=np.int32))
    return directory, np.stack(leaves)
