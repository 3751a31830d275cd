"""One decode step of one row, end to end, out of the oracle's stages (test
infrastructure): index (summaries) is an input; score -> select -> resolve ->
attend follow the decode half of the paper's five-operation pipeline
(Section 4.1: Select, Retrieve, Attention)."""
import numpy as np

from . import attend as _attend
from . import bf16, resolve, score, select

SCORE_MINMAX, SCORE_SKETCH, SCORE_REPMAX = 0, 1, 2


def score_row(kind, q, summaries, channels=None):
    if kind == SCORE_MINMAX:
        return score.score_minmax(q, summaries[0], summaries[1])
    if kind == SCORE_SKETCH:
        return score.score_sketch(q, summaries, channels)
    if kind == SCORE_REPMAX:
        return score.score_repmax(q, summaries)
    raise ValueError(kind)


def decode_row(q, summaries, kind, seq_len, page_tokens, partition_tokens, topk,
               topk_includes_forced, sink_pages, recent_pages, page_map, row,
               pool_bits, scale, channels=None):
    """Returns dict with scores, sel, page_ids, slots, masks, out, lse."""
    s = score_row(kind, q, summaries, channels)
    sel = select.select_topk(s, seq_len, page_tokens, partition_tokens, topk,
                             topk_includes_forced, sink_pages, recent_pages)
    page_ids, slots, masks = resolve.resolve_slots(sel, seq_len, page_tokens, partition_tokens,
                                                   sink_pages, recent_pages, page_map, row)
    pages = bf16.decode(pool_bits[np.asarray(slots, dtype=np.int64)]) if slots else \
        np.zeros((0, 2, page_tokens, q.shape[1]))
    K_S, V_S = _attend.gather_tokens(pages[:, 0], pages[:, 1], masks)
    out, lse = _attend.attend(q, K_S, V_S, scale)
    return dict(scores=s, sel=sel, page_ids=page_ids, slots=slots, masks=masks, out=out, lse=lse)
