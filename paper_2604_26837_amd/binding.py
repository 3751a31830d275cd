"""ctypes binding of ``libspin.so``: same names as the C ABI, argument
marshalling only.  torch supplies device memory and the current stream."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

from . import build as _build

_LIB: Optional[C.CDLL] = None

SPIN_OK = 0
STATUS_NAMES = {0: "SPIN_OK", -1: "SPIN_ERR_INVALID", -2: "SPIN_ERR_UNSUPPORTED", -3: "SPIN_ERR_WORKSPACE",
                -4: "SPIN_ERR_HIP", -5: "SPIN_ERR_BUDGET", -6: "SPIN_ERR_NOT_RESIDENT",
                -7: "SPIN_ERR_SLOT_RANGE", -8: "SPIN_ERR_LEAF_POOL", -9: "SPIN_ERR_STATIC_LIMIT"}

EXPORTS = [
    "spin_create", "spin_destroy", "spin_status_string", "spin_workspace_bytes", "spin_sel_stride",
    "spin_page_stride", "spin_dir_stride", "spin_decode_splits", "spin_summary_bytes",
    "spin_workspace_init", "spin_poll_status", "spin_profile_enable", "spin_profile_read", "spin_pack_kv_pages", "spin_build_summaries",
    "spin_score_partitions", "spin_select_topk", "spin_resolve_slots", "spin_sparse_decode",
    "spin_copy_misses_host", "spin_gather_misses", "spin_select_resolve", "spin_append_kv", "spin_reclaim_tail", "spin_alloc_leaves", "spin_free_leaves",
    "spin_set_partition_tables", "spin_probe_stream_read", "spin_offload_pages", "spin_score_select_topk", "spin_score_select_resolve", "spin_pin_partitions",
    "spin_set_host_page_table", "spin_set_step", "spin_advance_step", "spin_sparse_decode_static",
    "spin_select_resolve_forced", "spin_sparse_decode_rest", "spin_split_hits_misses", "spin_sparse_decode_begin",
    "spin_sparse_decode_finish",
]


class SpinConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "max_batch", "num_q_heads", "num_kv_heads", "head_dim", "page_tokens", "partition_tokens",
        "score_kind", "sketch_channels", "reps_per_partition", "topk", "topk_includes_forced",
        "sink_pages", "recent_pages", "max_context", "leaf_entries", "lru_timestamps",
        "lru_evict_exact", "lru_policy", "decode_splits", "decode_waves", "decode_depth", "score_tiles_per_wg",
        "score_waves", "variable_partitions")] + [("softmax_scale", C.c_float)]


class SpinError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {STATUS_NAMES.get(code, code)}")


def load_library() -> C.CDLL:
    """Load the in-tree library; there is no fallback if it is missing."""
    global _LIB
    if _LIB is not None:
        return _LIB
    if not os.path.exists(_build.LIB_PATH):
        raise RuntimeError(f"{_build.LIB_PATH} is not built: run `python -m paper_2604_26837_amd.build` "
                           "(the HIP library is required; there is no CPU fallback)")
    lib = C.CDLL(_build.LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.spin_create.argtypes = [C.POINTER(SpinConfig), C.POINTER(vp)]
    lib.spin_destroy.argtypes = [vp]
    lib.spin_destroy.restype = None
    lib.spin_status_string.argtypes = [C.c_int]
    lib.spin_status_string.restype = C.c_char_p
    lib.spin_workspace_bytes.argtypes = [vp]
    lib.spin_workspace_bytes.restype = C.c_size_t
    for n in ("spin_sel_stride", "spin_page_stride", "spin_dir_stride", "spin_decode_splits"):
        getattr(lib, n).argtypes = [vp]
        getattr(lib, n).restype = i32
    lib.spin_summary_bytes.argtypes = [vp, i64]
    lib.spin_summary_bytes.restype = C.c_size_t
    lib.spin_workspace_init.argtypes = [vp, vp, vp]
    lib.spin_poll_status.argtypes = [vp, vp, vp]
    lib.spin_profile_enable.argtypes = [vp, i32]
    lib.spin_profile_read.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(C.c_float), C.POINTER(C.c_float)]
    lib.spin_pack_kv_pages.argtypes = [vp, i64, vp, vp, vp, vp, i64, vp]
    lib.spin_build_summaries.argtypes = [vp, i32, vp, i64, vp, vp, i64, vp, vp, vp, vp, vp, vp]
    lib.spin_score_partitions.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.spin_select_topk.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.spin_score_select_topk.argtypes = [vp, i32] + [vp] * 10
    lib.spin_score_select_resolve.argtypes = [vp, i32] + [vp] * 10 + [i64] + [vp] * 6
    lib.spin_pin_partitions.argtypes = [vp, i32, vp, vp, vp, vp, i32, vp]
    lib.spin_set_host_page_table.argtypes = [vp, vp, i64, i64]
    lib.spin_set_step.argtypes = [vp, vp, i32, vp]
    lib.spin_advance_step.argtypes = [vp, vp, vp]
    lib.spin_resolve_slots.argtypes = [vp, i32, i32] + [vp] * 5 + [i64] + [vp] * 11
    lib.spin_sparse_decode.argtypes = [vp, i32, vp, vp, i64, vp, vp, vp, vp, vp, vp, vp]
    lib.spin_sparse_decode_static.argtypes = [vp, i32, vp, vp, i64, vp, vp, vp, vp, vp, vp, vp]
    lib.spin_select_resolve_forced.argtypes = [vp, i32] + [vp] * 7 + [i64] + [vp] * 6 + [i64, vp, vp]
    lib.spin_split_hits_misses.argtypes = [vp, i32] + [vp] * 8
    lib.spin_sparse_decode_begin.argtypes = [vp, i32, vp, vp, i64, vp, vp, vp, vp, vp]
    lib.spin_sparse_decode_finish.argtypes = [vp, i32, vp, vp, i64, vp, vp, vp, vp, vp, vp, vp]
    lib.spin_sparse_decode_rest.argtypes = [vp, i32, vp, vp, i64, vp, vp, vp, vp, vp, vp, vp]
    lib.spin_probe_stream_read.argtypes = [vp, vp, C.c_size_t, vp, vp]
    lib.spin_set_partition_tables.argtypes = [vp, vp, vp, vp, vp]
    lib.spin_reclaim_tail.argtypes = [vp, i32, vp, vp, vp, vp, i64, vp, vp, vp]
    lib.spin_alloc_leaves.argtypes = [vp, i32, vp, vp, vp, vp, vp, i64, vp, vp, vp]
    lib.spin_free_leaves.argtypes = [vp, i32, vp, i64, vp, vp, vp]
    lib.spin_append_kv.argtypes = [vp, i32, vp, vp, vp, vp, i64, vp, vp, i64, vp, vp, vp, vp, vp]
    lib.spin_select_resolve.argtypes = [vp, i32] + [vp] * 7 + [i64] + [vp] * 6
    lib.spin_copy_misses_host.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, i64, vp, C.POINTER(i64)]
    lib.spin_gather_misses.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, i64, vp, vp]
    lib.spin_offload_pages.argtypes = [vp, i32, vp, i64, vp, vp, vp, vp, vp, vp, vp]
    _LIB = lib
    return lib


def _ptr(t: Optional[torch.Tensor], dtype=None, name="tensor") -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class Spin:
    """Owns one ``spin_ctx``; methods mirror the C entry points one to one."""

    def __init__(self, **cfg):
        self.lib = load_library()
        c = SpinConfig()
        defaults = dict(head_dim=128, page_tokens=16, partition_tokens=16, score_kind=0, sketch_channels=16,
                        reps_per_partition=4, topk_includes_forced=1, sink_pages=0, recent_pages=0,
                        leaf_entries=512, lru_timestamps=0, lru_evict_exact=0, lru_policy=0, decode_splits=0, decode_waves=0, decode_depth=0, score_tiles_per_wg=0, score_waves=0, variable_partitions=0,
                        softmax_scale=0.0)
        defaults.update(cfg)
        for k, v in defaults.items():
            if not hasattr(c, k):
                raise TypeError(f"unknown config field {k}")
            setattr(c, k, v)
        self.cfg = c
        h = C.c_void_p()
        st = self.lib.spin_create(C.byref(c), C.byref(h))
        if st != SPIN_OK:
            raise SpinError(st, "spin_create")
        self.h = h
        self.sel_stride = self.lib.spin_sel_stride(h)
        self.page_stride = self.lib.spin_page_stride(h)
        self.dir_stride = self.lib.spin_dir_stride(h)
        self.decode_splits = self.lib.spin_decode_splits(h)
        self.workspace_bytes = self.lib.spin_workspace_bytes(h)

    @classmethod
    def for_workload(cls, w, **over):
        cfg = dict(max_batch=w.batch, num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads,
                   head_dim=w.head_dim, page_tokens=w.page_tokens, partition_tokens=w.partition_tokens,
                   score_kind=w.score_kind, sketch_channels=w.sketch_channels,
                   reps_per_partition=w.reps_per_partition, topk=w.topk,
                   topk_includes_forced=int(w.topk_includes_forced), sink_pages=w.sink_pages,
                   recent_pages=w.recent_pages, max_context=max(max(w.seq_lens), 1),
                   leaf_entries=w.leaf_entries)
        cfg.update(over)
        return cls(**cfg)

    def __del__(self):
        try:
            if getattr(self, "h", None):
                self.lib.spin_destroy(self.h)
                self.h = None
        except Exception:
            pass

    def _check(self, st: int, where: str):
        if st != SPIN_OK:
            raise SpinError(st, where)

    # -- plumbing ---------------------------------------------------------
    def new_workspace(self, device="cuda:0") -> torch.Tensor:
        ws = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=device)
        self.workspace_init(ws)
        return ws

    def workspace_init(self, ws):
        self._check(self.lib.spin_workspace_init(self.h, _ptr(ws), _stream()), "spin_workspace_init")

    def poll_status(self, ws) -> int:
        return self.lib.spin_poll_status(self.h, _ptr(ws), _stream())

    def summary_bytes(self, padded_partitions: int) -> int:
        return self.lib.spin_summary_bytes(self.h, padded_partitions)

    KERNEL_IDS = dict(score=0, select=1, resolve=2, decode=3, merge=4, index=5, pack=6, gather=7, probe=8, select_hist=9, offload=10, append=11,
                      meta=12)

    def profile_enable(self, capacity: int):
        self._check(self.lib.spin_profile_enable(self.h, capacity), "spin_profile_enable")

    def profile_read(self, which: str):
        """(count, mean_us, min_us) of the timed launches of one kernel."""
        n, mean, mn = C.c_int32(), C.c_float(), C.c_float()
        self._check(self.lib.spin_profile_read(self.h, self.KERNEL_IDS[which], C.byref(n), C.byref(mean),
                                               C.byref(mn)), "spin_profile_read")
        return n.value, mean.value, mn.value

    # -- set-up calls -----------------------------------------------------
    def pack_kv_pages(self, src_k, src_v, slots, kv_pool):
        n = src_k.shape[0]
        pool_slots = kv_pool.numel() * kv_pool.element_size() // 8192
        self._check(self.lib.spin_pack_kv_pages(
            self.h, n, _ptr(src_k, torch.bfloat16, "src_k"), _ptr(src_v, torch.bfloat16, "src_v"),
            _ptr(slots, torch.int32, "slots"), _ptr(kv_pool, None, "kv_pool"), pool_slots, _stream()),
            "spin_pack_kv_pages")

    def build_summaries(self, batch, kv_pool, dir_, leaf_pool, part_offsets, seq_lens, chan_idx, summaries, ws):
        pool_slots = kv_pool.numel() * kv_pool.element_size() // 8192
        self._check(self.lib.spin_build_summaries(
            self.h, batch, _ptr(kv_pool), pool_slots, _ptr(dir_, torch.int32, "dir"),
            _ptr(leaf_pool, torch.int32, "leaf_pool"), leaf_pool.shape[0],
            _ptr(part_offsets, torch.int32, "part_offsets"), _ptr(seq_lens, torch.int32, "seq_lens"),
            _ptr(chan_idx, torch.int32, "chan_idx"), _ptr(summaries), _ptr(ws), _stream()),
            "spin_build_summaries")

    def append_kv(self, batch, k_new, v_new, seq_lens, kv_pool, dir_, leaf_pool, part_offsets, chan_idx,
                  summaries, ws):
        pool_slots = kv_pool.numel() * kv_pool.element_size() // 8192
        self._check(self.lib.spin_append_kv(
            self.h, batch, _ptr(k_new, torch.bfloat16, "k_new"), _ptr(v_new, torch.bfloat16, "v_new"),
            _ptr(seq_lens, torch.int32, "seq_lens"), _ptr(kv_pool), pool_slots, _ptr(dir_, torch.int32, "dir"),
            _ptr(leaf_pool, torch.int32, "leaf_pool"), leaf_pool.shape[0],
            _ptr(part_offsets, torch.int32, "part_offsets"), _ptr(chan_idx, torch.int32, "chan_idx"),
            _ptr(summaries), _ptr(ws), _stream()), "spin_append_kv")

    def probe_stream_read(self, buf, nbytes, ws):
        self._check(self.lib.spin_probe_stream_read(self.h, _ptr(buf), nbytes, _ptr(ws), _stream()),
                    "spin_probe_stream_read")

    def set_partition_tables(self, part_offsets=None, part_count=None, part_first_page=None, part_tokens=None):
        """Registers (or, with no arguments, clears) the variable-length partition tables.  The
        tensors are kept alive by this object because the library stores their addresses."""
        self._var_tables = (part_offsets, part_count, part_first_page, part_tokens)
        self._check(self.lib.spin_set_partition_tables(
            self.h, _ptr(part_offsets, torch.int32, "part_offsets"), _ptr(part_count, torch.int32, "part_count"),
            _ptr(part_first_page, torch.int32, "part_first_page"), _ptr(part_tokens, torch.int32, "part_tokens")),
            "spin_set_partition_tables")

    def set_host_page_table(self, cpu_pages=None, host_pages=0):
        """cpu_pages: pinned int32 CPU tensor (kept alive here: the library stores its address)."""
        self._cpu_table = cpu_pages
        if cpu_pages is None:
            self._check(self.lib.spin_set_host_page_table(self.h, None, 0, host_pages), "spin_set_host_page_table")
            return
        if not cpu_pages.is_pinned() or cpu_pages.dtype != torch.int32 or not cpu_pages.is_contiguous():
            raise ValueError("cpu_pages must be a contiguous pinned int32 host tensor")
        self._check(self.lib.spin_set_host_page_table(self.h, cpu_pages.data_ptr(), cpu_pages.numel(), host_pages),
                    "spin_set_host_page_table")

    STEP_FROM_WORKSPACE = -1

    def set_step(self, ws, step: int):
        self._check(self.lib.spin_set_step(self.h, _ptr(ws), step, _stream()), "spin_set_step")

    def advance_step(self, ws):
        self._check(self.lib.spin_advance_step(self.h, _ptr(ws), _stream()), "spin_advance_step")

    def reclaim_tail(self, batch, slot_range, new_count, dir_, leaf_pool, rev_table, ws):
        self._check(self.lib.spin_reclaim_tail(
            self.h, batch, _ptr(slot_range, torch.int32, "slot_range"), _ptr(new_count, torch.int32, "new_count"),
            _ptr(dir_, torch.int32, "dir"), _ptr(leaf_pool, torch.int32, "leaf_pool"), leaf_pool.shape[0],
            _ptr(rev_table, torch.int32, "rev_table"), _ptr(ws), _stream()), "spin_reclaim_tail")

    def alloc_leaves(self, batch, sel, nsel, seq_lens, dir_, leaf_pool, leaf_bitmap, ws):
        self._check(self.lib.spin_alloc_leaves(
            self.h, batch, _ptr(sel, torch.int32, "sel"), _ptr(nsel, torch.int32, "nsel"),
            _ptr(seq_lens, torch.int32, "seq_lens"), _ptr(dir_, torch.int32, "dir"),
            _ptr(leaf_pool, torch.int32, "leaf_pool"), leaf_pool.shape[0],
            _ptr(leaf_bitmap, torch.int32, "leaf_bitmap"), _ptr(ws), _stream()), "spin_alloc_leaves")

    def free_leaves(self, batch, dir_, leaf_chunks, leaf_bitmap, ws):
        self._check(self.lib.spin_free_leaves(
            self.h, batch, _ptr(dir_, torch.int32, "dir"), leaf_chunks, _ptr(leaf_bitmap, torch.int32, "leaf_bitmap"),
            _ptr(ws), _stream()), "spin_free_leaves")

    # -- the four stages --------------------------------------------------
    def score_partitions(self, batch, q, summaries, chan_idx, part_offsets, seq_lens, scores, ws):
        self._check(self.lib.spin_score_partitions(
            self.h, batch, _ptr(q, torch.bfloat16, "q"), _ptr(summaries), _ptr(chan_idx, torch.int32, "chan_idx"),
            _ptr(part_offsets, torch.int32, "part_offsets"), _ptr(seq_lens, torch.int32, "seq_lens"),
            _ptr(scores, torch.float32, "scores"), _ptr(ws), _stream()), "spin_score_partitions")

    def select_topk(self, batch, scores, part_offsets, seq_lens, sel, nsel, ws):
        self._check(self.lib.spin_select_topk(
            self.h, batch, _ptr(scores, torch.float32, "scores"), _ptr(part_offsets, torch.int32, "part_offsets"),
            _ptr(seq_lens, torch.int32, "seq_lens"), _ptr(sel, torch.int32, "sel"),
            _ptr(nsel, torch.int32, "nsel"), _ptr(ws), _stream()), "spin_select_topk")

    def pin_partitions(self, batch, scores, part_offsets, pinned, npinned):
        self._check(self.lib.spin_pin_partitions(
            self.h, batch, _ptr(scores, torch.float32, "scores"), _ptr(part_offsets, torch.int32, "part_offsets"),
            _ptr(pinned, torch.int32, "pinned"), _ptr(npinned, torch.int32, "npinned"), pinned.shape[1], _stream()),
            "spin_pin_partitions")

    def score_select_topk(self, batch, q, summaries, chan_idx, part_offsets, seq_lens, scores, sel, nsel, ws):
        self._check(self.lib.spin_score_select_topk(
            self.h, batch, _ptr(q, torch.bfloat16, "q"), _ptr(summaries), _ptr(chan_idx, torch.int32, "chan_idx"),
            _ptr(part_offsets, torch.int32, "part_offsets"), _ptr(seq_lens, torch.int32, "seq_lens"),
            _ptr(scores, torch.float32, "scores"), _ptr(sel, torch.int32, "sel"), _ptr(nsel, torch.int32, "nsel"),
            _ptr(ws), _stream()), "spin_score_select_topk")

    def resolve_slots(self, batch, step, sel, nsel, seq_lens, dir_, leaf_pool, slots, page_ids, valid_mask,
                      npages, ws, rev_table=None, slot_base=None, miss_pages=None, miss_slots=None, nmiss=None):
        self._check(self.lib.spin_resolve_slots(
            self.h, batch, step, _ptr(sel, torch.int32, "sel"), _ptr(nsel, torch.int32, "nsel"),
            _ptr(seq_lens, torch.int32, "seq_lens"), _ptr(dir_, torch.int32, "dir"),
            _ptr(leaf_pool, torch.int32, "leaf_pool"), leaf_pool.shape[0],
            _ptr(rev_table, torch.int32, "rev_table"), _ptr(slot_base, torch.int32, "slot_base"),
            _ptr(slots, torch.int32, "slots"), _ptr(page_ids, torch.int32, "page_ids"),
            _ptr(valid_mask, torch.int16, "valid_mask"), _ptr(npages, torch.int32, "npages"),
            _ptr(miss_pages, torch.int32, "miss_pages"), _ptr(miss_slots, torch.int32, "miss_slots"),
            _ptr(nmiss, torch.int32, "nmiss"), _ptr(ws), _stream()), "spin_resolve_slots")

    def select_resolve(self, batch, scores, part_offsets, seq_lens, sel, nsel, dir_, leaf_pool, slots, page_ids,
                       valid_mask, npages, ws):
        self._check(self.lib.spin_select_resolve(
            self.h, batch, _ptr(scores, torch.float32, "scores"), _ptr(part_offsets, torch.int32, "part_offsets"),
            _ptr(seq_lens, torch.int32, "seq_lens"), _ptr(sel, torch.int32, "sel"), _ptr(nsel, torch.int32, "nsel"),
            _ptr(dir_, torch.int32, "dir"), _ptr(leaf_pool, torch.int32, "leaf_pool"), leaf_pool.shape[0],
            _ptr(slots, torch.int32, "slots"), _ptr(page_ids, torch.int32, "page_ids"),
            _ptr(valid_mask, torch.int16, "valid_mask"), _ptr(npages, torch.int32, "npages"), _ptr(ws), _stream()),
            "spin_select_resolve")

    def score_select_resolve(self, batch, q, summaries, chan_idx, part_offsets, seq_lens, scores, sel, nsel, dir_,
                             leaf_pool, slots, page_ids, valid_mask, npages, ws):
        self._check(self.lib.spin_score_select_resolve(
            self.h, batch, _ptr(q, torch.bfloat16, "q"), _ptr(summaries), _ptr(chan_idx, torch.int32, "chan_idx"),
            _ptr(part_offsets, torch.int32, "part_offsets"), _ptr(seq_lens, torch.int32, "seq_lens"),
            _ptr(scores, torch.float32, "scores"), _ptr(sel, torch.int32, "sel"), _ptr(nsel, torch.int32, "nsel"),
            _ptr(dir_, torch.int32, "dir"), _ptr(leaf_pool, torch.int32, "leaf_pool"), leaf_pool.shape[0],
            _ptr(slots, torch.int32, "slots"), _ptr(page_ids, torch.int32, "page_ids"),
            _ptr(valid_mask, torch.int16, "valid_mask"), _ptr(npages, torch.int32, "npages"), _ptr(ws), _stream()),
            "spin_score_select_resolve")

    def copy_misses_host(self, batch, host_kv, host_row_base, nmiss, miss_pages, miss_slots, kv_pool,
                         copy_stream) -> int:
        """All list arguments are HOST (pinned) tensors; returns the pages copied."""
        pool_slots = kv_pool.numel() * kv_pool.element_size() // 8192
        n = C.c_int64(0)
        for t, dt in ((host_row_base, torch.int64), (nmiss, torch.int32), (miss_pages, torch.int32),
                      (miss_slots, torch.int32)):
            if t.is_cuda or not t.is_contiguous() or t.dtype != dt:
                raise ValueError("host lists must be contiguous CPU tensors of the documented dtype")
        self._check(self.lib.spin_copy_misses_host(
            self.h, batch, host_kv.data_ptr(), host_row_base.data_ptr(), nmiss.data_ptr(), miss_pages.data_ptr(),
            miss_slots.data_ptr(), _ptr(kv_pool), pool_slots, copy_stream.cuda_stream, C.byref(n)),
            "spin_copy_misses_host")
        return n.value

    def gather_misses(self, batch, host_kv, row_base, nmiss, miss_pages, miss_slots, kv_pool, ws):
        """host_kv: pinned CPU tensor (read by the kernel); the lists are DEVICE tensors."""
        pool_slots = kv_pool.numel() * kv_pool.element_size() // 8192
        if not host_kv.is_pinned():
            raise ValueError("host_kv must be pinned host memory")
        self._check(self.lib.spin_gather_misses(
            self.h, batch, host_kv.data_ptr(), _ptr(row_base, torch.int64, "row_base"),
            _ptr(nmiss, torch.int32, "nmiss"), _ptr(miss_pages, torch.int32, "miss_pages"),
            _ptr(miss_slots, torch.int32, "miss_slots"), _ptr(kv_pool), pool_slots, _ptr(ws), _stream()),
            "spin_gather_misses")

    def offload_pages(self, batch, kv_pool, host_kv, row_base, count, pages, slots, ws):
        """host_kv: pinned CPU tensor (written by the kernel); the lists are DEVICE tensors."""
        pool_slots = kv_pool.numel() * kv_pool.element_size() // 8192
        if not host_kv.is_pinned():
            raise ValueError("host_kv must be pinned host memory")
        self._check(self.lib.spin_offload_pages(
            self.h, batch, _ptr(kv_pool), pool_slots, host_kv.data_ptr(), _ptr(row_base, torch.int64, "row_base"),
            _ptr(count, torch.int32, "count"), _ptr(pages, torch.int32, "pages"),
            _ptr(slots, torch.int32, "slots"), _ptr(ws), _stream()), "spin_offload_pages")

    def sparse_decode(self, batch, q, kv_pool, slots, valid_mask, npages, out, lse, ws):
        pool_slots = kv_pool.numel() * kv_pool.element_size() // 8192
        self._check(self.lib.spin_sparse_decode(
            self.h, batch, _ptr(q, torch.bfloat16, "q"), _ptr(kv_pool), pool_slots,
            _ptr(slots, torch.int32, "slots"), _ptr(valid_mask, torch.int16, "valid_mask"),
            _ptr(npages, torch.int32, "npages"), _ptr(out, torch.bfloat16, "out"),
            _ptr(lse, torch.float32, "lse"), _ptr(ws), _stream()), "spin_sparse_decode")

    def sparse_decode_static(self, batch, q, kv_pool, slots, valid_mask, npages, out, lse, status=None):
        """Stage 4 with the split-K scratch in the library's own device array (no workspace argument)."""
        pool_slots = kv_pool.numel() * kv_pool.element_size() // 8192
        self._check(self.lib.spin_sparse_decode_static(
            self.h, batch, _ptr(q, torch.bfloat16, "q"), _ptr(kv_pool), pool_slots,
            _ptr(slots, torch.int32, "slots"), _ptr(valid_mask, torch.int16, "valid_mask"),
            _ptr(npages, torch.int32, "npages"), _ptr(out, torch.bfloat16, "out"),
            _ptr(lse, torch.float32, "lse"), _ptr(status, torch.int32, "status"), _stream()),
            "spin_sparse_decode_static")

    def select_resolve_forced(self, batch, scores, part_offsets, seq_lens, sel, nsel, dir_, leaf_pool, slots, page_ids,
                              valid_mask, npages, q, kv_pool, ws):
        pool_slots = kv_pool.numel() * kv_pool.element_size() // 8192
        self._check(self.lib.spin_select_resolve_forced(
            self.h, batch, _ptr(scores, torch.float32, "scores"), _ptr(part_offsets, torch.int32, "part_offsets"),
            _ptr(seq_lens, torch.int32, "seq_lens"), _ptr(sel, torch.int32, "sel"), _ptr(nsel, torch.int32, "nsel"),
            _ptr(dir_, torch.int32, "dir"), _ptr(leaf_pool, torch.int32, "leaf_pool"), leaf_pool.shape[0],
            _ptr(slots, torch.int32, "slots"), _ptr(page_ids, torch.int32, "page_ids"),
            _ptr(valid_mask, torch.int16, "valid_mask"), _ptr(npages, torch.int32, "npages"),
            _ptr(q, torch.bfloat16, "q"), _ptr(kv_pool), pool_slots, _ptr(ws), _stream()),
            "spin_select_resolve_forced")

    def sparse_decode_rest(self, batch, q, kv_pool, slots, valid_mask, npages, out, lse, ws):
        pool_slots = kv_pool.numel() * kv_pool.element_size() // 8192
        self._check(self.lib.spin_sparse_decode_rest(
            self.h, batch, _ptr(q, torch.bfloat16, "q"), _ptr(kv_pool), pool_slots,
            _ptr(slots, torch.int32, "slots"), _ptr(valid_mask, torch.int16, "valid_mask"),
            _ptr(npages, torch.int32, "npages"), _ptr(out, torch.bfloat16, "out"),
            _ptr(lse, torch.float32, "lse"), _ptr(ws), _stream()), "spin_sparse_decode_rest")

    def split_hits_misses(self, batch, page_ids, valid_mask, npages, miss_pages, nmiss, mask_hits, mask_misses):
        self._check(self.lib.spin_split_hits_misses(
            self.h, batch, _ptr(page_ids, torch.int32, "page_ids"), _ptr(valid_mask, torch.int16, "valid_mask"),
            _ptr(npages, torch.int32, "npages"), _ptr(miss_pages, torch.int32, "miss_pages"),
            _ptr(nmiss, torch.int32, "nmiss"), _ptr(mask_hits, torch.int16, "mask_hits"),
            _ptr(mask_misses, torch.int16, "mask_misses"), _stream()), "spin_split_hits_misses")

    def sparse_decode_begin(self, batch, q, kv_pool, slots, valid_mask, npages, ws):
        pool_slots = kv_pool.numel() * kv_pool.element_size() // 8192
        self._check(self.lib.spin_sparse_decode_begin(
            self.h, batch, _ptr(q, torch.bfloat16, "q"), _ptr(kv_pool), pool_slots, _ptr(slots, torch.int32, "slots"),
            _ptr(valid_mask, torch.int16, "valid_mask"), _ptr(npages, torch.int32, "npages"), _ptr(ws), _stream()),
            "spin_sparse_decode_begin")

    def sparse_decode_finish(self, batch, q, kv_pool, slots, valid_mask, npages, out, lse, ws):
        pool_slots = kv_pool.numel() * kv_pool.element_size() // 8192
        self._check(self.lib.spin_sparse_decode_finish(
            self.h, batch, _ptr(q, torch.bfloat16, "q"), _ptr(kv_pool), pool_slots, _ptr(slots, torch.int32, "slots"),
            _ptr(valid_mask, torch.int16, "valid_mask"), _ptr(npages, torch.int32, "npages"),
            _ptr(out, torch.bfloat16, "out"), _ptr(lse, torch.float32, "lse"), _ptr(ws), _stream()),
            "spin_sparse_decode_finish")

    @property
    def forced_split_supported(self) -> bool:
        """Whether spin_select_resolve_forced / spin_sparse_decode_rest apply to this context (the library
        decides; this mirrors its documented conditions so that a caller can choose its step up front)."""
        c = self.cfg
        parts = -(-c.max_context // max(c.partition_tokens, 1))
        return (c.lru_timestamps == 0 and c.partition_tokens >= 16 and not c.variable_partitions and parts <= 4096
                and 1 <= c.sink_pages + c.recent_pages <= 1024)
