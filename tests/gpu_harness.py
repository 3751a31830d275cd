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
