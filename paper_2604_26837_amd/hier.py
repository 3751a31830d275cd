"""Hierarchical-KV layer: the full KV of every request lives in pinned host
memory, each (request, KV head) row owns a fixed budget of HBM slots, and a
decode step is score -> select -> resolve under the budget (bucketed LRU) ->
copy of the missed pages -> attention.  Orchestration only; the compute is in
libspin.so."""
from __future__ import annotations

import math
from typing import List, Optional

import numpy as np
import torch

from . import binding, runner, synth, tables


def request_workload(w: synth.Workload, b: int) -> synth.Workload:
    """The single-request workload request ``b`` of ``w`` is generated from."""
    return w.with_(seq_lens=(w.seq_lens[b],), seed=w.seed * 100 + b, name=f"{w.name}_req{b}")


class HierLayer:
    def __init__(self, w: synth.Workload, budget_frac: float = 0.25, n_ts: int = 64, evict_exact: bool = False,
                 device: str = "cuda:0", copy_mode: str = "memcpy", keep_natural: bool = False,
                 scatter_host_pages: bool = False, overlap_hits: bool = False, **cfg_over):
        """``overlap_hits`` (copy kernel only): attention over the pages that hit runs while the copy kernel brings
        the missed pages in on a side stream; a second pass attends the missed pages and completes the result."""
        # any uniform partition size; scores that need no per-head channel table
        assert w.score_kind in (synth.SCORE_MINMAX, synth.SCORE_REPMAX)
        assert copy_mode in ("memcpy", "gather")
        assert not overlap_hits or (copy_mode == "gather" and w.partition_tokens >= 16)
        self.w, self.device, self.copy_mode, self.overlap_hits = w, device, copy_mode, overlap_hits
        self.spin = binding.Spin.for_workload(w, lru_timestamps=n_ts, lru_evict_exact=int(evict_exact), **cfg_over)
        sp = self.spin
        self.ws = sp.new_workspace(device)
        rows, hkv = w.rows, w.num_kv_heads
        # slot budget per row: a fraction of the request's pages, never below one step's selection
        self.budgets = [max(int(math.ceil(budget_frac * w.pages(r // hkv))), sp.page_stride) for r in range(rows)]
        if cfg_over.get("lru_policy", 0) == 1:       # whole 8-way sets
            self.budgets = [8 * -(-x // 8) for x in self.budgets]
        base = np.zeros(rows + 1, dtype=np.int64)
        base[1:] = np.cumsum(self.budgets)
        self.pool_slots = int(base[-1])
        self.slot_base_np = base.astype(np.int32)
        rng = np.stack([self.slot_base_np[:-1], np.asarray(self.budgets, dtype=np.int32)], axis=1)
        self.slot_base = torch.from_numpy(np.ascontiguousarray(rng, dtype=np.int32)).to(device)   # [rows][2]
        self.kv_pool = torch.zeros((self.pool_slots, 4096), dtype=torch.bfloat16, device=device)
        # host side: all pages of all rows, in slot layout, row after row
        hrb = np.zeros(rows + 1, dtype=np.int64)
        hrb[1:] = np.cumsum([w.pages(r // hkv) for r in range(rows)])
        self.host_row_base_np = hrb
        self.host_row_base = torch.from_numpy(hrb[:-1].copy())                  # host int64 [rows]
        self.host_row_base_dev = self.host_row_base.to(device)
        # the host pool; with scatter_host_pages a request's pages lie anywhere in a somewhat larger pool and a
        # CPU page table (offset in the row's page list -> physical host page) says where
        n_host = int(hrb[-1])
        self.cpu_table = None
        if scatter_host_pages:
            pool_pages = n_host + max(n_host // 16, 3)
            perm = np.random.Generator(np.random.PCG64(w.seed + 4242)).permutation(pool_pages)[:n_host]
            self.cpu_table = torch.from_numpy(perm.astype(np.int32)).pin_memory()
            self.spin.set_host_page_table(self.cpu_table, pool_pages)
            n_host = pool_pages
        else:
            self.spin.set_host_page_table(None, n_host)      # identity mapping, bounded by the pool's size
        self.host_kv = torch.empty((n_host, 4096), dtype=torch.bfloat16, pin_memory=True)
        # metadata: leaves for every page range inside a row's context, nothing resident yet
        empty = [np.full((hkv, w.pages(b)), -1, dtype=np.int32) for b in range(w.batch)]
        d, l = tables.build_two_level(empty, sp.dir_stride, w.leaf_entries, allocate_all=True)
        self.dir = torch.from_numpy(d).to(device)
        self.leaf_pool = torch.from_numpy(l).to(device)
        rev = np.zeros((self.pool_slots, 2), dtype=np.int32)
        rev[:, 0] = -1
        self.rev = torch.from_numpy(rev).to(device)
        self.seq_lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=device)
        self.part_offsets_np = tables.part_offsets(w.seq_lens, w.partition_tokens)
        self.part_offsets = torch.from_numpy(self.part_offsets_np).to(device)
        padded = int(self.part_offsets_np[-1])
        self.summaries = torch.zeros(sp.summary_bytes(padded), dtype=torch.uint8, device=device)
        self.summary_bytes_per_partition = sp.summary_bytes(16) // (16 * hkv)   # per KV head
        self.scores = torch.zeros(padded * hkv, dtype=torch.float32, device=device)
        z = lambda *s, dt=torch.int32: torch.zeros(s, dtype=dt, device=device)
        self.sel, self.nsel = z(rows, sp.sel_stride), z(rows)
        self.slots, self.page_ids = z(rows, sp.page_stride), z(rows, sp.page_stride)
        self.valid_mask, self.npages = z(rows, sp.page_stride, dt=torch.int16), z(rows)
        self.miss_pages, self.miss_slots, self.nmiss = z(rows, sp.page_stride), z(rows, sp.page_stride), z(rows)
        self.mask_hits, self.mask_misses = z(rows, sp.page_stride, dt=torch.int16), z(rows, sp.page_stride, dt=torch.int16)
        self.out = torch.zeros((w.batch, w.num_q_heads, w.head_dim), dtype=torch.bfloat16, device=device)
        self.lse = torch.zeros((w.batch, w.num_q_heads), dtype=torch.float32, device=device)
        hp = lambda *s: torch.zeros(s, dtype=torch.int32, pin_memory=True)
        self.h_nmiss, self.h_miss_pages, self.h_miss_slots = hp(rows), hp(rows, sp.page_stride), hp(rows, sp.page_stride)
        self.copy_stream = torch.cuda.Stream(device=device)
        self.scale = 1.0 / math.sqrt(w.head_dim)
        self.natural: List[Optional[torch.Tensor]] = []
        self.natural_slot_of: List[np.ndarray] = []
        self.stats = dict(steps=0, selected=0, misses=0, misses_after_first=0, selected_after_first=0)
        self._materialise(keep_natural)

    # ------------------------------------------------------------------
    def _materialise(self, keep_natural: bool):
        """Generate every request in HBM, build its summaries there, and move its
        packed pages to pinned host memory (the prefill-side Index and Offload)."""
        w, hkv = self.w, self.w.num_kv_heads
        qs = []
        for b in range(w.batch):
            wb = request_workload(w, b)
            tmp, natural = runner.build_device_layer(wb, device=self.device, keep_natural=True)
            qs.append(tmp.q0)
            pp = int(self.part_offsets_np[b + 1] - self.part_offsets_np[b])
            spb = self.summary_bytes_per_partition
            off = hkv * int(self.part_offsets_np[b]) * spb
            self.summaries[off: off + hkv * pp * spb] = tmp.summaries[: hkv * pp * spb]
            for h in range(hkv):
                r = b * hkv + h
                slots = torch.from_numpy(tmp.slot_of[0][h].astype(np.int64)).to(self.device)
                lo, hi = int(self.host_row_base_np[r]), int(self.host_row_base_np[r + 1])
                if self.cpu_table is None:
                    self.host_kv[lo:hi].copy_(tmp.kv_pool[slots])
                else:
                    self.host_kv[self.cpu_table[lo:hi].long()] = tmp.kv_pool[slots].cpu()
            if keep_natural:
                self.natural.append(natural.cpu())
                self.natural_slot_of.append(tmp.slot_of[0])
            del tmp, natural
        self.q0 = torch.cat(qs, dim=0).contiguous()
        torch.cuda.synchronize()

    # ------------------------------------------------------------------
    def step(self, q: torch.Tensor, step: int, summaries: Optional[torch.Tensor] = None, count: bool = True,
             device_step: bool = False):
        """``device_step``: the replacement policy reads the step from the workspace's own counter and the
        counter is advanced after the step (what a step recorded in a HIP graph needs; ``step`` is ignored)."""
        sp, w = self.spin, self.w
        summ = self.summaries if summaries is None else summaries
        sp.score_partitions(w.batch, q, summ, None, self.part_offsets, self.seq_lens, self.scores, self.ws)
        sp.select_topk(w.batch, self.scores, self.part_offsets, self.seq_lens, self.sel, self.nsel, self.ws)
        sp.resolve_slots(w.batch, sp.STEP_FROM_WORKSPACE if device_step else step, self.sel, self.nsel, self.seq_lens, self.dir, self.leaf_pool, self.slots,
                         self.page_ids, self.valid_mask, self.npages, self.ws, rev_table=self.rev,
                         slot_base=self.slot_base, miss_pages=self.miss_pages, miss_slots=self.miss_slots,
                         nmiss=self.nmiss)
        main = torch.cuda.current_stream()
        if self.copy_mode == "memcpy":
            self.h_nmiss.copy_(self.nmiss, non_blocking=True)
            self.h_miss_pages.copy_(self.miss_pages, non_blocking=True)
            self.h_miss_slots.copy_(self.miss_slots, non_blocking=True)
            main.synchronize()                       # the host needs the miss list
            copied = sp.copy_misses_host(w.batch, self.host_kv, self.host_row_base, self.h_nmiss,
                                         self.h_miss_pages, self.h_miss_slots, self.kv_pool, self.copy_stream)
            ev = torch.cuda.Event()
            ev.record(self.copy_stream)
            main.wait_event(ev)
        elif self.overlap_hits:
            # the copy kernel on the side stream, attention over the hits beside it, then the missed pages
            sp.split_hits_misses(w.batch, self.page_ids, self.valid_mask, self.npages, self.miss_pages, self.nmiss,
                                 self.mask_hits, self.mask_misses)
            resolved = torch.cuda.Event()
            resolved.record(main)
            with torch.cuda.stream(self.copy_stream):
                self.copy_stream.wait_event(resolved)
                sp.gather_misses(w.batch, self.host_kv, self.host_row_base_dev, self.nmiss, self.miss_pages,
                                 self.miss_slots, self.kv_pool, self.ws)
                fetched = torch.cuda.Event()
                fetched.record(self.copy_stream)
            sp.sparse_decode_begin(w.batch, q, self.kv_pool, self.slots, self.mask_hits, self.npages, self.ws)
            main.wait_event(fetched)
            sp.sparse_decode_finish(w.batch, q, self.kv_pool, self.slots, self.mask_misses, self.npages, self.out,
                                    self.lse, self.ws)
            copied = None
        else:
            sp.gather_misses(w.batch, self.host_kv, self.host_row_base_dev, self.nmiss, self.miss_pages,
                             self.miss_slots, self.kv_pool, self.ws)
            copied = None
        if not self.overlap_hits:
            sp.sparse_decode(w.batch, q, self.kv_pool, self.slots, self.valid_mask, self.npages, self.out, self.lse,
                             self.ws)
        if device_step:
            sp.advance_step(self.ws)
        if count:
            if copied is None:
                copied = int(self.nmiss.sum().item())
            selected = int(self.npages.sum().item())
            st = self.stats
            st["steps"] += 1
            st["selected"] += selected
            st["misses"] += copied
            if step > 0:
                st["selected_after_first"] += selected
                st["misses_after_first"] += copied
        return copied

    # ------------------------------------------------------------------
    def rebuild_summaries_from_host(self):
        """Index over the host copy for the current ``seq_lens`` (shorter than the
        lengths the layer was sized for): each request's pages are staged in a
        temporary all-resident pool and summarised there."""
        sp, w, hkv = self.spin, self.w, self.w.num_kv_heads
        lens = self.seq_lens.cpu().tolist()
        self.summaries.zero_()
        for b in range(w.batch):
            pages_b = w.pages(b)
            tmp = torch.empty((hkv * pages_b, 4096), dtype=torch.bfloat16, device=self.device)
            slot_of = np.empty((hkv, pages_b), dtype=np.int32)
            for h in range(hkv):
                r = b * hkv + h
                lo = int(self.host_row_base_np[r])
                src = (self.host_kv[lo:lo + pages_b] if self.cpu_table is None
                       else self.host_kv[self.cpu_table[lo:lo + pages_b].long()])
                tmp[h * pages_b:(h + 1) * pages_b].copy_(src)
                slot_of[h] = np.arange(h * pages_b, (h + 1) * pages_b, dtype=np.int32)
            d, l = tables.build_two_level([slot_of], sp.dir_stride, w.leaf_entries)
            pp = int(self.part_offsets_np[b + 1] - self.part_offsets_np[b])
            po = torch.tensor([0, pp], dtype=torch.int32, device=self.device)
            sl = torch.tensor([lens[b]], dtype=torch.int32, device=self.device)
            spb = self.summary_bytes_per_partition
            off = hkv * int(self.part_offsets_np[b]) * spb
            part = self.summaries[off: off + hkv * pp * spb]
            sp.build_summaries(1, tmp, torch.from_numpy(d).to(self.device), torch.from_numpy(l).to(self.device), po, sl,
                               None, part, self.ws)
            torch.cuda.synchronize()
            del tmp

    def step_append(self, q: torch.Tensor, step: int, k_new: torch.Tensor, v_new: torch.Tensor) -> int:
        """One decode step in which every request grows by one token: the stages run for
        the new lengths (the tail partition is forced, so its summary need not hold the
        new token yet), misses are fetched, the token is appended to its now resident page
        (decode-time Index), attention runs, and a page that the token completed is copied
        back to the host (Offload's copy) so that a later eviction loses nothing.
        ``seq_lens`` holds the lengths before the call and is incremented.  Returns the
        number of pages written back.  Needs recent_pages >= 1."""
        sp, w, hkv = self.spin, self.w, self.w.num_kv_heads
        assert w.recent_pages >= 1 and self.copy_mode == "gather" and w.partition_tokens == 16
        before = self.seq_lens.clone()
        after = before + 1
        sp.score_partitions(w.batch, q, self.summaries, None, self.part_offsets, after, self.scores, self.ws)
        sp.select_topk(w.batch, self.scores, self.part_offsets, after, self.sel, self.nsel, self.ws)
        sp.resolve_slots(w.batch, step, self.sel, self.nsel, after, self.dir, self.leaf_pool, self.slots,
                         self.page_ids, self.valid_mask, self.npages, self.ws, rev_table=self.rev,
                         slot_base=self.slot_base, miss_pages=self.miss_pages, miss_slots=self.miss_slots,
                         nmiss=self.nmiss)
        sp.gather_misses(w.batch, self.host_kv, self.host_row_base_dev, self.nmiss, self.miss_pages,
                         self.miss_slots, self.kv_pool, self.ws)
        sp.append_kv(w.batch, k_new, v_new, before, self.kv_pool, self.dir, self.leaf_pool, self.part_offsets, None,
                     self.summaries, self.ws)
        sp.sparse_decode(w.batch, q, self.kv_pool, self.slots, self.valid_mask, self.npages, self.out, self.lse,
                         self.ws)
        # the tail page is the last entry of every row's ascending page list
        last = (self.npages - 1).clamp(min=0).long().unsqueeze(1)
        off_pages = torch.full_like(self.page_ids, -1)
        off_slots = torch.full_like(self.slots, -1)
        off_pages[:, 0:1] = torch.gather(self.page_ids, 1, last)
        off_slots[:, 0:1] = torch.gather(self.slots, 1, last)
        complete = ((after % 16) == 0).to(torch.int32).repeat_interleave(hkv)
        sp.offload_pages(w.batch, self.kv_pool, self.host_kv, self.host_row_base_dev, complete, off_pages, off_slots,
                         self.ws)
        self.seq_lens.copy_(after)
        copied = int(self.nmiss.sum().item())
        selected = int(self.npages.sum().item())
        st = self.stats
        st["steps"] += 1
        st["selected"] += selected
        st["misses"] += copied
        if step > 0:
            st["selected_after_first"] += selected
            st["misses_after_first"] += copied
        return int(complete.sum().item())

    def hit_rates(self):
        st = self.stats
        overall = 1.0 - st["misses"] / max(st["selected"], 1)
        warm = 1.0 - st["misses_after_first"] / max(st["selected_after_first"], 1)
        return overall, warm

    def status(self) -> int:
        return self.spin.poll_status(self.ws)
