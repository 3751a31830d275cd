"""Device-side state of one attention layer and the four-call decode step.

Pure orchestration: allocates torch tensors for the buffers the C ABI wants,
uploads tables, and issues ``score -> select -> resolve -> decode`` on the
current stream.  Every computation happens inside libspin.so.
"""
from __future__ import annotations

import math
from typing import List, Optional

import numpy as np
import torch

from . import binding, synth, tables


class LayerState:
    def __init__(self, w: synth.Workload, slot_of: List[np.ndarray], kv_pool: torch.Tensor,
                 device: str = "cuda:0", layouts=None, **cfg_over):
        """``layouts`` (optional): per request, per KV head, a pair of lists
        ``(first_page, tokens)`` describing variable-length partitions; the
        workload's ``partition_tokens`` is then the largest partition allowed."""
        self.w = w
        self.device = device
        self.layouts_none = layouts is None
        if layouts is not None:
            cfg_over = dict(cfg_over, variable_partitions=1)
        self.spin = binding.Spin.for_workload(w, **cfg_over)
        self.ws = self.spin.new_workspace(device)
        self.kv_pool = kv_pool
        self.pool_slots = kv_pool.numel() * kv_pool.element_size() // 8192
        self.slot_of = slot_of
        sp = self.spin
        rows = w.rows
        self.seq_lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=device)
        if layouts is None:
            self.part_offsets_np = tables.part_offsets(w.seq_lens, w.partition_tokens)
        else:
            self.part_offsets_np = tables.part_offsets_from_counts(
                [max(len(fp) for fp, _ in layouts[b]) for b in range(w.batch)])
        self.part_offsets = torch.from_numpy(self.part_offsets_np).to(device)
        if layouts is not None:
            cnt, first, toks = tables.partition_tables(layouts, self.part_offsets_np, w.num_kv_heads)
            self.part_count = torch.from_numpy(cnt).to(device)
            self.part_first_page = torch.from_numpy(first).to(device)
            self.part_tokens = torch.from_numpy(toks).to(device)
            self.spin.set_partition_tables(self.part_offsets, self.part_count, self.part_first_page,
                                           self.part_tokens)
        d, l = tables.build_two_level(slot_of, sp.dir_stride, w.leaf_entries)
        self.dir = torch.from_numpy(d).to(device)
        self.leaf_pool = torch.from_numpy(l).to(device)
        padded = int(self.part_offsets_np[-1])
        self.summaries = torch.zeros(sp.summary_bytes(padded), dtype=torch.uint8, device=device)
        self.scores = torch.zeros(padded * w.num_kv_heads, dtype=torch.float32, device=device)
        self.sel = torch.zeros((rows, sp.sel_stride), dtype=torch.int32, device=device)
        self.nsel = torch.zeros(rows, dtype=torch.int32, device=device)
        self.slots = torch.zeros((rows, sp.page_stride), dtype=torch.int32, device=device)
        self.page_ids = torch.zeros((rows, sp.page_stride), dtype=torch.int32, device=device)
        self.valid_mask = torch.zeros((rows, sp.page_stride), dtype=torch.int16, device=device)
        self.npages = torch.zeros(rows, dtype=torch.int32, device=device)
        self.out = torch.zeros((w.batch, w.num_q_heads, w.head_dim), dtype=torch.bfloat16, device=device)
        self.lse = torch.zeros((w.batch, w.num_q_heads), dtype=torch.float32, device=device)
        self.chan: Optional[torch.Tensor] = None
        self.scale = 1.0 / math.sqrt(w.head_dim)

    # ------------------------------------------------------------------
    @classmethod
    def from_natural_pool(cls, w, slot_of, natural_pool: torch.Tensor, device="cuda:0", layouts=None, **cfg_over):
        """``natural_pool``: bf16 ``[slots][2][16][128]`` in plain token-major
        order; it is re-written into the library's slot layout by the pack kernel."""
        nslots = natural_pool.shape[0]
        kv_pool = torch.empty((nslots, 4096), dtype=torch.bfloat16, device=device)
        self = cls(w, slot_of, kv_pool, device=device, layouts=layouts, **cfg_over)
        chunk = 32768
        for s0 in range(0, nslots, chunk):
            s1 = min(nslots, s0 + chunk)
            ids = torch.arange(s0, s1, dtype=torch.int32, device=device)
            self.spin.pack_kv_pages(natural_pool[s0:s1, 0].contiguous(), natural_pool[s0:s1, 1].contiguous(),
                                    ids, kv_pool)
        return self

    def set_channels(self, chan_np):
        self.chan = torch.from_numpy(np.ascontiguousarray(chan_np, dtype=np.int32)).to(self.device)

    def build_summaries(self, summaries: Optional[torch.Tensor] = None):
        self.spin.build_summaries(self.w.batch, self.kv_pool, self.dir, self.leaf_pool, self.part_offsets,
                                  self.seq_lens, self.chan, self.summaries if summaries is None else summaries,
                                  self.ws)

    def step(self, q: torch.Tensor, summaries: Optional[torch.Tensor] = None):
        """One decode step of the layer: the four stage calls, back to back."""
        sp, w = self.spin, self.w
        summ = self.summaries if summaries is None else summaries
        sp.score_partitions(w.batch, q, summ, self.chan, self.part_offsets, self.seq_lens, self.scores, self.ws)
        sp.select_topk(w.batch, self.scores, self.part_offsets, self.seq_lens, self.sel, self.nsel, self.ws)
        sp.resolve_slots(w.batch, 0, self.sel, self.nsel, self.seq_lens, self.dir, self.leaf_pool, self.slots,
                         self.page_ids, self.valid_mask, self.npages, self.ws)
        sp.sparse_decode(w.batch, q, self.kv_pool, self.slots, self.valid_mask, self.npages, self.out, self.lse,
                         self.ws)

    def step12(self, q: torch.Tensor, summaries: Optional[torch.Tensor] = None):
        """The step with stages 1 and 2 in one call (same results as :meth:`step`)."""
        sp, w = self.spin, self.w
        summ = self.summaries if summaries is None else summaries
        sp.score_select_topk(w.batch, q, summ, self.chan, self.part_offsets, self.seq_lens, self.scores, self.sel,
                             self.nsel, self.ws)
        sp.resolve_slots(w.batch, 0, self.sel, self.nsel, self.seq_lens, self.dir, self.leaf_pool, self.slots,
                         self.page_ids, self.valid_mask, self.npages, self.ws)
        sp.sparse_decode(w.batch, q, self.kv_pool, self.slots, self.valid_mask, self.npages, self.out, self.lse,
                         self.ws)

    def step3(self, q: torch.Tensor, summaries: Optional[torch.Tensor] = None):
        """The same step in three launches: stages 2 and 3 share one."""
        sp, w = self.spin, self.w
        summ = self.summaries if summaries is None else summaries
        sp.score_partitions(w.batch, q, summ, self.chan, self.part_offsets, self.seq_lens, self.scores, self.ws)
        sp.select_resolve(w.batch, self.scores, self.part_offsets, self.seq_lens, self.sel, self.nsel, self.dir,
                          self.leaf_pool, self.slots, self.page_ids, self.valid_mask, self.npages, self.ws)
        sp.sparse_decode(w.batch, q, self.kv_pool, self.slots, self.valid_mask, self.npages, self.out, self.lse,
                         self.ws)

    def step123(self, q: torch.Tensor, summaries: Optional[torch.Tensor] = None):
        """The step in three launches for rows of any supported length: stages 1-3 in one call
        (two launches), then attention (same results as :meth:`step`)."""
        sp, w = self.spin, self.w
        summ = self.summaries if summaries is None else summaries
        sp.score_select_resolve(w.batch, q, summ, self.chan, self.part_offsets, self.seq_lens, self.scores, self.sel,
                                self.nsel, self.dir, self.leaf_pool, self.slots, self.page_ids, self.valid_mask,
                                self.npages, self.ws)
        sp.sparse_decode(w.batch, q, self.kv_pool, self.slots, self.valid_mask, self.npages, self.out, self.lse,
                         self.ws)

    def step3f(self, q: torch.Tensor, summaries: Optional[torch.Tensor] = None):
        """Three launches, and the launch of stages 2+3 also attends the sink / recent pages on the compute
        units it leaves idle; stage 4 covers the rest of the page list and merges that partial."""
        sp, w = self.spin, self.w
        summ = self.summaries if summaries is None else summaries
        sp.score_partitions(w.batch, q, summ, self.chan, self.part_offsets, self.seq_lens, self.scores, self.ws)
        sp.select_resolve_forced(w.batch, self.scores, self.part_offsets, self.seq_lens, self.sel, self.nsel, self.dir,
                                 self.leaf_pool, self.slots, self.page_ids, self.valid_mask, self.npages, q,
                                 self.kv_pool, self.ws)
        sp.sparse_decode_rest(w.batch, q, self.kv_pool, self.slots, self.valid_mask, self.npages, self.out, self.lse,
                              self.ws)

    def step_fused(self, q: torch.Tensor, summaries: Optional[torch.Tensor] = None):
        """The step in the fewest launches the row length allows (what ``bench.py`` times): stages 2+3 in one
        launch for rows of at most 16384 partitions (with the sink / recent pages attended beside them where
        that applies), stages 1-3 in one call for longer ones."""
        if self.spin.forced_split_supported and self.layouts_none:
            self.step3f(q, summaries)
        elif max(self.w.partitions(b) for b in range(self.w.batch)) <= 16384:
            self.step3(q, summaries)
        else:
            self.step123(q, summaries)

    def row_base(self, b: int, h: int) -> int:
        return tables.row_base(self.part_offsets_np, b, h, self.w.num_kv_heads)

    def status(self) -> int:
        return self.spin.poll_status(self.ws)


def build_device_layer(w: synth.Workload, device: str = "cuda:0", keep_natural: bool = False, **cfg_over):
    """Generate a workload directly in HBM, pack it and build its summaries.

    Returns ``(layer, natural_pool or None)``; the natural (token-major) pool is
    only kept when a caller wants to hand sampled rows to a checker."""
    dd = synth.generate_on_device(w, device=device)
    layer = LayerState.from_natural_pool(w, dd.slot_of, dd.pool, device=device, **cfg_over)
    layer.q0 = dd.q
    if w.score_kind == synth.SCORE_SKETCH:
        layer.set_channels(synth.sketch_channels_on_device(dd))
    layer.build_summaries()
    torch.cuda.synchronize()
    natural = dd.pool if keep_natural else None
    return layer, natural
