"""Seeded synthetic inputs for the sparse-decode hot path.

This module only draws random numbers, rounds them to bf16 and lays them out
in pages.  It holds none of the method's arithmetic (no scoring, no selection,
no table walk, no attention): the CPU oracle and the HIP path each bring their
own.  Both consume what is produced here, so a mistake here cannot hide a
disagreement between them.

The inputs stand in for the long-context serving requests the paper evaluates
on (Table 2: 16K-120K token inputs; GQA models with 8 KV heads and head
dimension 128; Table 3: retrieval budgets of a few percent of the context).
Only those shapes are taken; no dataset item or model weight is involved.

Layout produced (identical for the numpy and the torch/device generators):

* ``q_bits``      uint16 ``[B][H_q][D]``             bf16 bit patterns
* ``pool_bits``   uint16 ``[slots][2][page][D]``      K page then V page, one
                  head-wise physical page per slot (Section 5.2, head-wise
                  physical pages; the page is the unit of transfer)
* ``slot_of[b]``  int32  ``[H_kv][pages_b]``          logical page -> slot, a
                  seeded permutation so physical order != logical order
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 20260427

SCORE_MINMAX = 0
SCORE_SKETCH = 1
SCORE_REPMAX = 2


# --------------------------------------------------------------------------
# bf16 <-> fp32 bit conversion (dtype plumbing, round-to-nearest-even)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (nearest, ties to even); return uint16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = u + np.uint32(0x7FFF) + lsb
    out = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32)


# --------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    """Shape and policy parameters of one synthetic workload."""

    name: str
    seq_lens: Tuple[int, ...]            # context length per request (tokens)
    num_q_heads: int = 32
    num_kv_heads: int = 8
    head_dim: int = 128
    page_tokens: int = 16
    partition_tokens: int = 16           # 1, 16 or a multiple of 16
    score_kind: int = SCORE_MINMAX
    sketch_channels: int = 16
    reps_per_partition: int = 4
    topk: int = 128                      # partitions (tokens if partition_tokens == 1)
    topk_includes_forced: bool = True
    sink_pages: int = 0
    recent_pages: int = 0
    leaf_entries: int = 512
    planted_frac: float = 0.0            # fraction of tokens per KV head aligned to q
    planted_sigma: float = 3.0
    block_mean_std: float = 0.0          # >0: per-partition Gaussian mixture
    seed: int = BASE_SEED

    @property
    def batch(self) -> int:
        return len(self.seq_lens)

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    @property
    def rows(self) -> int:
        return self.batch * self.num_kv_heads

    def pages(self, b: int) -> int:
        return -(-self.seq_lens[b] // self.page_tokens)

    def partitions(self, b: int) -> int:
        return -(-self.seq_lens[b] // self.partition_tokens)

    @property
    def total_pages_per_head(self) -> int:
        return sum(self.pages(b) for b in range(self.batch))

    @property
    def total_slots(self) -> int:
        return self.total_pages_per_head * self.num_kv_heads

    def with_(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


def config0() -> Workload:
    """Tiny single-layer case: 1 request, 8q/2kv heads, 4096 tokens, k=32 pages
    including page 0 and the last page."""
    return Workload(name="cfg0_tiny_b1_ctx4k", seq_lens=(4096,), num_q_heads=8, num_kv_heads=2,
                    topk=32, topk_includes_forced=True, sink_pages=1, recent_pages=1,
                    seed=BASE_SEED + 0)


def config1() -> Workload:
    """Headline: Llama-3-8B-shaped layer, batch 16 x 32768 tokens, 128 of 2048
    pages per KV head including 4 sink and 8 recent pages, 2 % planted keys."""
    return Workload(name="cfg1_llama3_8b_b16_ctx32k", seq_lens=(32768,) * 16,
                    topk=128, topk_includes_forced=True, sink_pages=4, recent_pages=8,
                    planted_frac=0.02, seed=BASE_SEED + 1)


def config2() -> Workload:
    """Token-granularity partitions scored on a 16-channel key sketch."""
    return Workload(name="cfg2_token_sketch_b8_ctx64k", seq_lens=(65536,) * 8,
                    partition_tokens=1, score_kind=SCORE_SKETCH, topk=1024,
                    topk_includes_forced=True, sink_pages=0, recent_pages=0,
                    planted_frac=0.01, seed=BASE_SEED + 2)


def config3() -> Workload:
    """128-token blocks with 4 representative keys; 32 blocks plus 4 sink pages
    and a 1024-token (64-page) local window."""
    return Workload(name="cfg3_block_repmax_b4_ctx128k", seq_lens=(131072,) * 4,
                    partition_tokens=128, score_kind=SCORE_REPMAX, topk=32,
                    topk_includes_forced=False, sink_pages=4, recent_pages=64,
                    block_mean_std=0.5, seed=BASE_SEED + 3)


def config4_seq_lens(batch: int = 32, seed: int = BASE_SEED + 4) -> Tuple[int, ...]:
    """Lognormal contexts, median 48K, clipped to [16K, 256K], multiples of 16."""
    rng = np.random.Generator(np.random.PCG64(seed))
    z = rng.standard_normal(batch)
    n = np.exp(np.log(49152.0) + 0.7 * z)
    n = np.clip(np.round(n / 16.0) * 16.0, 16384, 262144).astype(np.int64)
    return tuple(int(v) for v in n)


def config4() -> Workload:
    """Hierarchical budget: 32 ragged requests, page partitions, min/max score."""
    return Workload(name="cfg4_budget_b32_lognormal", seq_lens=config4_seq_lens(),
                    topk=128, topk_includes_forced=True, sink_pages=4, recent_pages=8,
                    planted_frac=0.02, seed=BASE_SEED + 4)


CONFIGS = {0: config0, 1: config1, 2: config2, 3: config3, 4: config4}


# --------------------------------------------------------------------------
# host (numpy) generator: sizes the oracle finishes in seconds
# --------------------------------------------------------------------------
@dataclass
class SynthData:
    workload: Workload
    q_bits: np.ndarray                   # uint16 [B][Hq][D]
    pool_bits: np.ndarray                # uint16 [slots][2][page][D]
    slot_of: List[np.ndarray]            # per request int32 [Hkv][pages_b]
    planted: List[np.ndarray] = field(default_factory=list)  # per row: token ids

    def logical_kv_bits(self, b: int, h: int) -> Tuple[np.ndarray, np.ndarray]:
        """K and V bit patterns of row (b, h) in logical token order,
        ``[pages_b * page][D]`` (the tail beyond seq_len is filler)."""
        s = self.slot_of[b][h]
        pages = self.pool_bits[s]                      # [pages][2][page][D]
        d = self.workload.head_dim
        return pages[:, 0].reshape(-1, d), pages[:, 1].reshape(-1, d)


def make_queries(w: Workload, seed: int) -> np.ndarray:
    """A fresh query set ``[B][Hq][D]`` (bf16 bits), i.i.d. N(0,1)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    q = rng.standard_normal((w.batch, w.num_q_heads, w.head_dim), dtype=np.float32)
    return f32_to_bf16_bits(q)


def next_query_ar1(q_bits: np.ndarray, rho: float, seed: int) -> np.ndarray:
    """AR(1) query drift: q' = rho q + sqrt(1 - rho^2) eps, rounded to bf16."""
    rng = np.random.Generator(np.random.PCG64(seed))
    q = bf16_bits_to_f32(q_bits)
    eps = rng.standard_normal(q.shape, dtype=np.float32)
    return f32_to_bf16_bits(np.float32(rho) * q + np.float32(np.sqrt(1.0 - rho * rho)) * eps)


def generate(w: Workload, seed: Optional[int] = None, spare_slots: int = 0) -> SynthData:
    """Generate q, the paged KV pool and the logical->physical page map.

    K, V and q are drawn in fp32 and stored as bf16.  With ``planted_frac`` a
    seeded subset of each KV head's tokens gets ``planted_sigma`` times the unit
    vector of one (seeded) query head of its group added to its key before
    rounding.  With ``block_mean_std`` every partition gets its own Gaussian
    mean for K and for V (independent per channel).
    """
    seed = w.seed if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed))
    d, pt, g = w.head_dim, w.page_tokens, w.group
    q_bits = f32_to_bf16_bits(rng.standard_normal((w.batch, w.num_q_heads, d), dtype=np.float32))
    q32 = bf16_bits_to_f32(q_bits)

    nslots = w.total_slots + spare_slots
    perm = rng.permutation(nslots).astype(np.int32)
    pool = np.zeros((nslots, 2, pt, d), dtype=np.uint16)
    if spare_slots:
        # spare slots hold filler so that a wrong slot id reads plausible data
        spare = perm[w.total_slots:]
        pool[spare] = f32_to_bf16_bits(
            rng.standard_normal((len(spare), 2, pt, d), dtype=np.float32))

    slot_of: List[np.ndarray] = []
    planted: List[np.ndarray] = []
    cursor = 0
    for b in range(w.batch):
        n, pages = w.seq_lens[b], w.pages(b)
        s = perm[cursor:cursor + w.num_kv_heads * pages].reshape(w.num_kv_heads, pages)
        cursor += w.num_kv_heads * pages
        slot_of.append(s)
        for h in range(w.num_kv_heads):
            ntok = pages * pt
            k = rng.standard_normal((ntok, d), dtype=np.float32)
            v = rng.standard_normal((ntok, d), dtype=np.float32)
            if w.block_mean_std > 0.0:
                tp = max(w.partition_tokens, 1)
                nblk = -(-ntok // tp)
                km = rng.standard_normal((nblk, d), dtype=np.float32) * np.float32(w.block_mean_std)
                vm = rng.standard_normal((nblk, d), dtype=np.float32) * np.float32(w.block_mean_std)
                k += np.repeat(km, tp, axis=0)[:ntok]
                v += np.repeat(vm, tp, axis=0)[:ntok]
            if w.planted_frac > 0.0 and n > 0:
                cnt = int(round(w.planted_frac * n))
                toks = np.sort(rng.choice(n, size=cnt, replace=False))
                heads = rng.integers(0, g, size=cnt)
                qg = q32[b, h * g + heads]                                  # [cnt][D]
                qhat = qg / np.linalg.norm(qg.astype(np.float64), axis=1, keepdims=True).astype(np.float32)
                k[toks] += np.float32(w.planted_sigma) * qhat
                planted.append(toks.astype(np.int32))
            else:
                planted.append(np.zeros(0, dtype=np.int32))
            pool[s[h], 0] = f32_to_bf16_bits(k).reshape(pages, pt, d)
            pool[s[h], 1] = f32_to_bf16_bits(v).reshape(pages, pt, d)
    return SynthData(workload=w, q_bits=q_bits, pool_bits=pool, slot_of=slot_of, planted=planted)


def variable_layouts(w: Workload, seed: int, min_tokens: int = 1):
    """Seeded variable-length partition layouts: for every (request, KV head) row,
    partition sizes drawn uniformly from [min_tokens, partition_tokens] until the
    row's pages are used up (the last one is cut to fit).  Returns, per request,
    per head, ``(first_page, tokens)`` lists.  Partitions own whole pages."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for b in range(w.batch):
        pages = w.pages(b)
        per_head = []
        for _ in range(w.num_kv_heads):
            first, toks, pg = [], [], 0
            while pg < pages:
                t = int(rng.integers(min_tokens, w.partition_tokens + 1))
                t = min(t, (pages - pg) * w.page_tokens)
                first.append(pg)
                toks.append(t)
                pg += -(-t // w.page_tokens)
            per_head.append((first, toks))
        out.append(per_head)
    return out


def sketch_channels(data: SynthData) -> np.ndarray:
    """Per KV head, the ``sketch_channels`` channels with the largest mean |K|
    over all requests and valid tokens (ties -> lowest channel), ascending.
    This fixes an input of the workload ("fixed from the seed"); it is not part
    of the decode path."""
    w = data.workload
    acc = np.zeros((w.num_kv_heads, w.head_dim), dtype=np.float64)
    cnt = 0
    for b in range(w.batch):
        n = w.seq_lens[b]
        for h in range(w.num_kv_heads):
            kb, _ = data.logical_kv_bits(b, h)
            acc[h] += np.abs(bf16_bits_to_f32(kb[:n]).astype(np.float64)).sum(axis=0)
        cnt += n
    acc /= max(cnt, 1)
    out = np.zeros((w.num_kv_heads, w.sketch_channels), dtype=np.int32)
    for h in range(w.num_kv_heads):
        order = sorted(range(w.head_dim), key=lambda c: (-acc[h, c], c))
        out[h] = np.sort(np.array(order[: w.sketch_channels], dtype=np.int32))
    return out


# --------------------------------------------------------------------------
# device (torch) generator: full-size pools that never exist on the host
# --------------------------------------------------------------------------
@dataclass
class DeviceData:
    workload: Workload
    q: "object"                           # torch bf16 [B][Hq][D] on device
    pool: "object"                        # torch bf16 [slots][2][page][D] on device
    slot_of: List[np.ndarray]             # host int32 [Hkv][pages_b] per request


def generate_on_device(w: Workload, device: str = "cuda:0", seed: Optional[int] = None,
                       chunk_slots: int = 32768) -> DeviceData:
    """Same recipe as :func:`generate`, drawn with torch's device generator so a
    multi-GiB pool is filled in HBM directly.  Because K/V are i.i.d. the pool
    is filled slot by slot; planted keys are rewritten in place afterwards."""
    import torch

    seed = w.seed if seed is None else seed
    d, pt, g = w.head_dim, w.page_tokens, w.group
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    rng = np.random.Generator(np.random.PCG64(seed))

    q = torch.randn((w.batch, w.num_q_heads, d), generator=gen, device=device,
                    dtype=torch.float32).to(torch.bfloat16)
    nslots = w.total_slots
    perm = rng.permutation(nslots).astype(np.int32)
    slot_of: List[np.ndarray] = []
    cursor = 0
    for b in range(w.batch):
        pages = w.pages(b)
        slot_of.append(perm[cursor:cursor + w.num_kv_heads * pages].reshape(w.num_kv_heads, pages))
        cursor += w.num_kv_heads * pages

    pool = torch.empty((nslots, 2, pt, d), device=device, dtype=torch.bfloat16)
    if w.block_mean_std > 0.0:
        # per-partition Gaussian mixture: filled row by row in logical order
        tp = max(w.partition_tokens, 1)
        for b in range(w.batch):
            pages = w.pages(b)
            ntok = pages * pt
            nblk = -(-ntok // tp)
            for h in range(w.num_kv_heads):
                kv = torch.randn((2, ntok, d), generator=gen, device=device, dtype=torch.float32)
                means = torch.randn((2, nblk, d), generator=gen, device=device,
                                    dtype=torch.float32) * w.block_mean_std
                kv += means.repeat_interleave(tp, dim=1)[:, :ntok]
                slots = torch.from_numpy(slot_of[b][h].astype(np.int64)).to(device)
                pool[slots] = kv.to(torch.bfloat16).reshape(2, pages, pt, d).transpose(0, 1)
    else:
        for s0 in range(0, nslots, chunk_slots):
            s1 = min(nslots, s0 + chunk_slots)
            pool[s0:s1] = torch.randn((s1 - s0, 2, pt, d), generator=gen, device=device,
                                      dtype=torch.float32).to(torch.bfloat16)

    if w.planted_frac > 0.0:
        qf = q.to(torch.float32)
        qhat = qf / qf.norm(dim=-1, keepdim=True)
        for b in range(w.batch):
            n = w.seq_lens[b]
            cnt = int(round(w.planted_frac * n))
            if cnt == 0:
                continue
            for h in range(w.num_kv_heads):
                toks = np.sort(rng.choice(n, size=cnt, replace=False))
                heads = rng.integers(0, g, size=cnt)
                slots = torch.from_numpy(slot_of[b][h][toks // pt].astype(np.int64)).to(device)
                tin = torch.from_numpy((toks % pt).astype(np.int64)).to(device)
                hq = torch.from_numpy((h * g + heads).astype(np.int64)).to(device)
                base = torch.randn((cnt, d), generator=gen, device=device, dtype=torch.float32)
                pool[slots, 0, tin] = (base + w.planted_sigma * qhat[b, hq]).to(torch.bfloat16)
    return DeviceData(workload=w, q=q, pool=pool, slot_of=slot_of)


def sketch_channels_on_device(dd: DeviceData) -> np.ndarray:
    """Device-side twin of :func:`sketch_channels` for pools that live in HBM."""
    import torch

    w = dd.workload
    acc = torch.zeros((w.num_kv_heads, w.head_dim), dtype=torch.float64, device=dd.pool.device)
    cnt = 0
    for b in range(w.batch):
        n = w.seq_lens[b]
        for h in range(w.num_kv_heads):
            slots = torch.from_numpy(dd.slot_of[b][h].astype(np.int64)).to(dd.pool.device)
            k = dd.pool[slots, 0].reshape(-1, w.head_dim)[:n]
            acc[h] += k.to(torch.float64).abs().sum(dim=0)
        cnt += n
    acc = (acc / max(cnt, 1)).cpu().numpy()
    out = np.zeros((w.num_kv_heads, w.sketch_channels), dtype=np.int32)
    for h in range(w.num_kv_heads):
        order = sorted(range(w.head_dim), key=lambda c: (-acc[h, c], c))
        out[h] = np.sort(np.array(order[: w.sketch_channels], dtype=np.int32))
    return out


def make_queries_on_device(w: Workload, seed: int, device: str = "cuda:0"):
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    return torch.randn((w.batch, w.num_q_heads, w.head_dim), generator=gen, device=device,
                       dtype=torch.float32).to(torch.bfloat16)
