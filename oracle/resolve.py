"""Retrieve, lookup half: selected partitions -> HBM page slots (test
infrastructure).

Follows the lookup path of Retrieve (Section 5.2, steps 1-2): each selected
partition is expanded to its pages (its page count follows from its token
count) and every page is looked up in the GPU page map.  The oracle's page map
is a plain dictionary ``{(row, page): slot}``.

Output per row, ascending by logical page id: page ids, slots and a validity
mask per page (bit t set = token t of the page is attended).  For partitions
of at least a page every valid token of the page is attended; for token
partitions only the selected tokens are.  Forced pages (sinks, recent window)
are attended whole.
"""
from typing import Dict, List, Tuple

from .select import forced_pages


class NotResident(Exception):
    """A selected page has no HBM slot (all-resident mode treats that as an error)."""


def page_token_mask(page: int, seq_len: int, page_tokens: int) -> int:
    """Bit mask of the tokens of ``page`` that lie inside the context."""
    n = min(max(seq_len - page * page_tokens, 0), page_tokens)
    return (1 << n) - 1


def selected_pages(sel: List[int], seq_len: int, page_tokens: int, partition_tokens: int,
                   sink_pages: int, recent_pages: int) -> Dict[int, int]:
    """``{page: token mask}`` for a row's selection, forced pages included."""
    masks: Dict[int, int] = {}
    for pg in forced_pages(seq_len, page_tokens, sink_pages, recent_pages):
        masks[pg] = page_token_mask(pg, seq_len, page_tokens)
    for p in sel:
        t0 = p * partition_tokens
        t1 = min(t0 + partition_tokens, seq_len)
        for t in range(t0, t1):
            pg = t // page_tokens
            if partition_tokens >= page_tokens:
                masks[pg] = page_token_mask(pg, seq_len, page_tokens)
            else:
                masks[pg] = masks.get(pg, 0) | (1 << (t % page_tokens))
    return masks


def resolve_slots(sel: List[int], seq_len: int, page_tokens: int, partition_tokens: int,
                  sink_pages: int, recent_pages: int, page_map: Dict[Tuple[int, int], int],
                  row: int) -> Tuple[List[int], List[int], List[int]]:
    """Returns ``(page_ids, slots, masks)``, ascending by page id."""
    masks = selected_pages(sel, seq_len, page_tokens, partition_tokens, sink_pages, recent_pages)
    page_ids = sorted(masks)
    slots = []
    for pg in page_ids:
        slot = page_map.get((row, pg), -1)
        if slot < 0:
            raise NotResident((row, pg))
        slots.append(slot)
    return page_ids, slots, [masks[pg] for pg in page_ids]
