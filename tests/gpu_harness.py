"""Device-side set-up shared by the GPU tests: uploads a synthetic workload,
packs the pool into the library's slot layout and builds the two-level tables.
Only plumbing lives here; the compute under test is in libspin.so."""
from __future__ import annotations

import math

import numpy as np
import torch

from paper_2604_26837_amd import binding, synth, tables

DEV = "cuda:0"


def bits_to_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16).copy()).to(DEV).view(torch.bfloat16)


def bf16_to_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


class DeviceWorkload:
    def __init__(self, data: synth.SynthData, **cfg_over):
        w = data.workload
        self.data, self.w = data, w
        self.spin = binding.Spin.for_workload(w, **cfg_over)
        self.ws = self.spin.new_workspace(DEV)
        nslots = data.pool_bits.shape[0]
        self.pool_slots = nslots
        natural = bits_to_bf16(data.pool_bits)                      # [slots][2][16][128]
        self.kv_pool = torch.zeros((nslots, 4096), dtype=torch.bfloat16, device=DEV)
        all_slots = torch.arange(nslots, dtype=torch.int32, device=DEV)
        self.spin.pack_kv_pages(natural[:, 0].contiguous(), natural[:, 1].contiguous(), all_slots, self.kv_pool)
        self.q = bits_to_bf16(data.q_bits)
        self.seq_lens = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
        self.part_offsets_np = tables.part_offsets(w.seq_lens, w.partition_tokens)
        self.part_offsets = torch.from_numpy(self.part_offsets_np).to(DEV)
        d, l = tables.build_two_level(data.slot_of, self.spin.dir_stride, w.leaf_entries)
        self.dir = torch.from_numpy(d).to(DEV)
        self.leaf_pool = torch.from_numpy(l).to(DEV)
        self.page_map = {}
        r = 0
        for b in range(w.batch):
            for h in range(w.num_kv_heads):
                for pg, s in enumerate(data.slot_of[b][h]):
                    self.page_map[(r, pg)] = int(s)
                r += 1
        self.scale = 1.0 / math.sqrt(w.head_dim)

    def row_base(self, b, h):
        return tables.row_base(self.part_offsets_np, b, h, self.w.num_kv_heads)

    def check_ok(self):
        st = self.spin.poll_status(self.ws)
        assert st == 0, binding.STATUS_NAMES.get(st, st)


# ---------------------------------------------------------------------------
# running the stages
# ---------------------------------------------------------------------------
def alloc_step_buffers(dw: "DeviceWorkload"):
    sp, w = dw.spin, dw.w
    rows = w.rows
    padded = int(dw.part_offsets_np[-1])
    dw.summaries = torch.zeros(sp.summary_bytes(padded), dtype=torch.uint8, device=DEV)
    dw.scores = torch.zeros(padded * w.num_kv_heads, dtype=torch.float32, device=DEV)
    dw.sel = torch.zeros((rows, sp.sel_stride), dtype=torch.int32, device=DEV)
    dw.nsel = torch.zeros(rows, dtype=torch.int32, device=DEV)
    dw.slots = torch.zeros((rows, sp.page_stride), dtype=torch.int32, device=DEV)
    dw.page_ids = torch.zeros((rows, sp.page_stride), dtype=torch.int32, device=DEV)
    dw.valid_mask = torch.zeros((rows, sp.page_stride), dtype=torch.int16, device=DEV)
    dw.npages = torch.zeros(rows, dtype=torch.int32, device=DEV)
    dw.out = torch.zeros((w.batch, w.num_q_heads, w.head_dim), dtype=torch.bfloat16, device=DEV)
    dw.lse = torch.zeros((w.batch, w.num_q_heads), dtype=torch.float32, device=DEV)
    dw.chan = None


def build_summaries(dw: "DeviceWorkload", chan_np=None):
    if not hasattr(dw, "summaries"):
        alloc_step_buffers(dw)
    if chan_np is not None:
        dw.chan = torch.from_numpy(np.ascontiguousarray(chan_np, dtype=np.int32)).to(DEV)
    dw.spin.build_summaries(dw.w.batch, dw.kv_pool, dw.dir, dw.leaf_pool, dw.part_offsets, dw.seq_lens,
                            dw.chan, dw.summaries, dw.ws)


def run_step(dw: "DeviceWorkload", q=None):
    """score -> select -> resolve -> decode on the current stream."""
    sp, w = dw.spin, dw.w
    q = dw.q if q is None else q
    sp.score_partitions(w.batch, q, dw.summaries, dw.chan, dw.part_offsets, dw.seq_lens, dw.scores, dw.ws)
    sp.select_topk(w.batch, dw.scores, dw.part_offsets, dw.seq_lens, dw.sel, dw.nsel, dw.ws)
    sp.resolve_slots(w.batch, 0, dw.sel, dw.nsel, dw.seq_lens, dw.dir, dw.leaf_pool, dw.slots, dw.page_ids,
                     dw.valid_mask, dw.npages, dw.ws)
    sp.sparse_decode(w.batch, q, dw.kv_pool, dw.slots, dw.valid_mask, dw.npages, dw.out, dw.lse, dw.ws)


def unpack_summary_rows(raw_u8: torch.Tensor, kd: int, kc: int) -> np.ndarray:
    """Undo the tile layout [KD/KC chunks][16 rows][KC]: returns uint16 [rows][kd]."""
    bits = raw_u8.cpu().numpy().view(np.uint16)
    tiles = bits.reshape(-1, kd // kc, 16, kc)
    return tiles.transpose(0, 2, 1, 3).reshape(-1, kd)
