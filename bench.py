#!/usr/bin/env python3
"""Benchmark of the sparse-decode hot path on one MI355X.

One "step" = one pass of the whole path (score -> select -> resolve -> attend)
for one layer over one batch of synthetic input, resident in HBM.  Prints ONE
JSON line.  `roofline` is about the attention kernel: the bytes its launch moves (512 B per token it
attends) over its mean duration, taken from HIP events on the launch stream, against 8 TB/s.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0
METRIC = "sparse decode µs/layer + attended-KV HBM GB/s (% peak) at 32K ctx"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--query-sets", type=int, default=8, help="distinct query sets cycled through")
    ap.add_argument("--layers", type=int, default=4,
                    help="distinct copies of the summary array cycled through (keeps the last-level cache "
                         "from serving stage 1, as the other layers of a model would)")
    ap.add_argument("--cpu-rows", type=int, default=32, help="rows of the workload timed on the CPU oracle")
    ap.add_argument("--cpu-reps", type=int, default=8)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--workload", default="cfg1", choices=["cfg1", "cfg2", "cfg3", "cfg4", "setup", "cfg1_mean", "attention_sweep"],
                    help="cfg1: the headline all-resident layer (the metric's workload); cfg2: token partitions scored "
                         "on a key sketch; cfg3: 128-token blocks with representative keys; cfg4: hierarchical HBM "
                         "budget, 64 decode steps; cfg1_mean: cfg1's shape with one mean key per page as the summary; setup: the layout, Index, append, copy and metadata kernels at "
                         "cfg1's shape; attention_sweep: stage 4 alone at cfg1's shape with 32 ... 128 pages per row")
    ap.add_argument("--copy-mode", default="both", choices=["memcpy", "gather", "both"])
    ap.add_argument("--budget-frac", type=float, default=0.25)
    ap.add_argument("--four-calls", action="store_true",
                    help="time the four separate stage calls as the step (default: stages 2+3 share one launch)")
    ap.add_argument("--decode-splits", type=int, default=0, help="split-K factor of the attention kernel (0: library default)")
    ap.add_argument("--decode-waves", type=int, default=0, help="wavefronts per attention workgroup (0: library default)")
    ap.add_argument("--decode-depth", type=int, default=0, help="page buffers per attention wavefront (0: library default)")
    ap.add_argument("--score-waves", type=int, default=0, help="wavefronts per stage-1 workgroup (0: library default)")
    ap.add_argument("--score-tiles", type=int, default=0, help="summary tiles per stage-1 workgroup (0: library default)")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the step")
    ap.add_argument("--no-other-form", action="store_true",
                    help="skip the pass that times the other launch form of the step (under a profiler: every launch of "
                         "a kernel then belongs to the timed form)")
    ap.add_argument("--print-source-hash", action="store_true",
                    help="print the hash of the library's sources that counter summaries under profiles/ record, and exit")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="do not bracket kernels with HIP events during the timed region")
    return ap.parse_args()


def source_hash():
    """sha256 over the library's sources (csrc/* and include/spin.h, sorted by name): what a counter summary
    under profiles/ must have been taken from for its figures to describe the library that runs now."""
    import glob
    import hashlib
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(ROOT, "paper_2604_26837_amd", "csrc", "*"))) + \
        [os.path.join(ROOT, "include", "spin.h")]
    for f in files:
        h.update(os.path.basename(f).encode() + b"\0")
        h.update(open(f, "rb").read())
    return h.hexdigest()


def read_traffic(path, kernel):
    """(HBM bytes per launch of the attention kernel, note) from the committed counter summary.  The figure is
    a recorded one (an earlier rocprofv3 session), so it is only passed on when the summary names the same
    kernel instantiation and the same source hash as the library in the tree; otherwise (None, reason)."""
    name = os.path.relpath(path, ROOT)
    try:
        txt = open(path).read()
    except OSError:
        return None, f"{name} not found"
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", txt, re.M)
    k = re.search(r"^traffic_kernel:\s*(.+?)\s*$", txt, re.M)
    hs = re.search(r"^csrc_sha256:\s*([0-9a-f]+)", txt, re.M)
    if not m:
        return None, f"{name} holds no traffic_bytes_per_launch"
    if not k or not hs:
        return None, f"{name} does not say which kernel and sources it was taken from"
    if k.group(1).replace(" ", "") != kernel.replace(" ", ""):
        return None, f"{name} was taken from {k.group(1)}, this run launches {kernel}"
    if hs.group(1) != source_hash():
        return None, f"{name} was taken from other sources (csrc_sha256 differs): regenerate it"
    return float(m.group(1)), f"recorded in {name} (rocprofv3 FETCH_SIZE + WRITE_SIZE, same kernel and sources)"


def _oracle_worker(conn):
    """Child process of the all-cores leg: receives rows of the workload, then runs the oracle's decode step
    over them when told to and reports the time it took.  Single-threaded numpy; no GPU, no torch."""
    for v in ("OMP_NUM_THREADS", "OPENBLAS_NUM_THREADS", "MKL_NUM_THREADS"):
        os.environ[v] = "1"
    from oracle import step as ostep
    try:
        from threadpoolctl import threadpool_limits
        threadpool_limits(limits=1)
    except Exception:
        pass
    rows = []
    while True:
        msg = conn.recv()
        if msg[0] == "row":
            rows.append(msg[1])
        elif msg[0] == "run":
            t0 = time.perf_counter()
            for _ in range(msg[1]):
                for a in rows:
                    ostep.decode_row(*a[:-1], channels=a[-1])
            conn.send(time.perf_counter() - t0)
        else:
            return


class OraclePool:
    """Worker processes for the all-cores leg of `cpu_baseline`.  They are forked before the first GPU call of
    this program (a process that has initialised the GPU must not be forked), sit idle during the GPU part and
    hold nothing but the interpreter."""

    def __init__(self):
        import multiprocessing as mp
        try:
            avail = len(os.sched_getaffinity(0))
        except AttributeError:
            avail = os.cpu_count() or 1
        self.n = max(1, min(avail, 16))          # the GPU machine's CPU share for one GPU is 16
        ctx = mp.get_context("fork")
        self.conns, self.procs = [], []
        for _ in range(self.n):
            a, b = ctx.Pipe()
            p = ctx.Process(target=_oracle_worker, args=(b,), daemon=True)
            p.start()
            b.close()
            self.conns.append(a)
            self.procs.append(p)

    def run(self, row_args, reps):
        """Deals the rows round-robin, then times `reps` passes of all workers over their rows (wall clock of
        the parent from the start signal to the last report)."""
        used = min(self.n, len(row_args))
        for i, a in enumerate(row_args):
            self.conns[i % used].send(("row", a))
        t0 = time.perf_counter()
        for c in self.conns[:used]:
            c.send(("run", reps))
        busy = [c.recv() for c in self.conns[:used]]
        wall = time.perf_counter() - t0
        return wall / reps, used, max(busy) / reps

    def close(self):
        for c in self.conns:
            try:
                c.send(("quit",))
            except Exception:
                pass
        for p in self.procs:
            p.join(timeout=5)


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_oracle_leg(layer, natural, q_bits, rows, reps, pool=None):
    """Times the fp64 oracle (as it stands) on `rows` rows of the same workload, on one core and, with `pool`,
    fanned out over the host's cores; the caller checks the GPU's output for those rows against the results."""
    import numpy as np
    import torch
    from oracle import bf16, index, step as ostep

    try:
        from threadpoolctl import threadpool_limits
        limiter = threadpool_limits(limits=1)
    except Exception:
        limiter = None
    w = layer.w
    g = w.group
    stride = max(1, w.rows // rows)
    picked = list(range(0, w.rows, stride))[:rows]
    chan_all = layer.chan.cpu().numpy() if layer.chan is not None else None
    prepared = []
    for r in picked:
        b, h = divmod(r, w.num_kv_heads)
        slots = torch.from_numpy(layer.slot_of[b][h].astype(np.int64)).to(natural.device)
        pages = natural[slots].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)  # [pages][2][16][128]
        K = bf16.decode(pages[:, 0].reshape(-1, w.head_dim))
        chan = None
        if w.score_kind == ostep.SCORE_MINMAX:
            summ = index.minmax_summaries(K, w.seq_lens[b], w.partition_tokens)
        elif w.score_kind == ostep.SCORE_REPMAX:
            summ = index.block_representatives(K, w.seq_lens[b], w.partition_tokens, w.reps_per_partition)
        else:
            chan = chan_all[h]
            summ = index.key_sketch(K, w.seq_lens[b], chan)
        page_map = {(r, pg): pg for pg in range(pages.shape[0])}      # local pool: slot == logical page
        q = bf16.decode(q_bits[b, h * g:(h + 1) * g])
        prepared.append((r, b, h, q, summ, page_map, pages, chan))

    def row_args(p):
        r, b, h, q, summ, page_map, pages, chan = p
        return (q, summ, w.score_kind, w.seq_lens[b], w.page_tokens, w.partition_tokens, w.topk,
                w.topk_includes_forced, w.sink_pages, w.recent_pages, page_map, r, pages, layer.scale, chan)

    t0 = time.perf_counter()
    results = None
    for _ in range(reps):
        results = [ostep.decode_row(*a[:-1], channels=a[-1]) for a in map(row_args, prepared)]
    dt = (time.perf_counter() - t0) / reps
    if limiter is not None:
        limiter.restore_original_limits() if hasattr(limiter, "restore_original_limits") else None
    scale = w.rows / len(picked)
    us_per_layer = dt * 1e6 * scale
    all_cores = None
    if pool is not None:
        wall, used, busiest = pool.run([row_args(p) for p in prepared], reps)
        all_cores = dict(value=round(wall * 1e6 * scale, 1), unit="us/layer", cores=used,
                         busiest_worker_us=round(busiest * 1e6, 1))
    return picked, prepared, results, us_per_layer, all_cores


def run_cfg4(args):
    """Hierarchical budget workload: 32 ragged requests, full KV in pinned host
    memory, 25 % of each request's pages as HBM slots, 64 decode steps with AR(1)
    query drift; reports LRU hit rate and step latency for each copier."""
    import numpy as np
    import torch
    from paper_2604_26837_amd import hier, synth

    dev = "cuda:0"
    w = synth.config4()
    steps = 64
    results = {}
    modes = ["memcpy", "gather"] if args.copy_mode == "both" else [args.copy_mode]
    # the paper's bucketed policy (whole buckets, then exact), then the 8-way set-associative variant
    # (and, with the copy kernel, the step whose attention over the hits runs beside the copy)
    for exact, policy, overlap in ((False, 0, False), (False, 0, True), (True, 0, False), (False, 1, False)):
        for mode in modes:
            if (exact or policy or overlap) and mode != modes[-1]:
                continue
            if overlap and mode != "gather":
                continue
            layer = hier.HierLayer(w, budget_frac=args.budget_frac, n_ts=64, evict_exact=exact, copy_mode=mode,
                                   overlap_hits=overlap, lru_policy=policy, decode_splits=args.decode_splits,
                                   decode_waves=args.decode_waves, decode_depth=args.decode_depth)
            q = layer.q0
            lat, persist, prev = [], [], None
            layer.spin.profile_enable(steps)          # kernels bracketed by HIP events on the launch stream
            trace = [[] for _ in range(w.rows)] if (mode == modes[-1] and not exact and not policy and not overlap
                                                     and not args.no_cpu) else None
            for s in range(steps):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                layer.step(q, s)
                torch.cuda.synchronize()
                lat.append((time.perf_counter() - t0) * 1e6)
                sel = layer.page_ids.cpu().numpy()
                npg = layer.npages.cpu().numpy()
                cur = [set(sel[r, :npg[r]].tolist()) for r in range(w.rows)]
                if prev is not None:
                    persist.append(np.mean([len(a & b) / max(len(a), 1) for a, b in zip(cur, prev)]))
                prev = cur
                if trace is not None:
                    for r in range(w.rows):
                        trace[r].append(sorted(cur[r]))
                q_bits = q.view(torch.int16).cpu().numpy().view(np.uint16)
                q = torch.from_numpy(synth.next_query_ar1(q_bits, 0.9, w.seed + 7000 + s).view(np.int16)).to(dev).view(torch.bfloat16)
            assert layer.status() == 0, "device fault in the budget workload"
            kern = {}
            for name in ("score", "select", "resolve", "gather", "decode"):
                n, mean, mn = layer.spin.profile_read(name)
                if n:
                    kern[name] = dict(mean_us=round(mean, 1), min_us=round(mn, 1))
            layer.spin.profile_enable(0)
            overall, warm = layer.hit_rates()
            lat_w = sorted(lat[1:])
            key = f"{mode}{'_overlap_hits' if overlap else ''}{'_evict_exact' if exact else ''}{'_set_assoc8' if policy else ''}"
            results[key] = dict(hit_rate=round(overall, 4), hit_rate_after_step0=round(warm, 4),
                                misses_per_step=round(layer.stats["misses_after_first"] / (steps - 1), 1),
                                selected_per_step=round(layer.stats["selected"] / steps, 1),
                                step_us_median=round(lat_w[len(lat_w) // 2], 1), step_us_p90=round(lat_w[int(0.9 * len(lat_w))], 1),
                                first_step_us=round(lat[0], 1), topk_persistence=round(float(np.mean(persist)), 4),
                                kernel_us=kern, pool_gib=round(layer.pool_slots * 8192 / 2**30, 2),
                                host_kv_gib=round(layer.host_kv.numel() * 2 / 2**30, 2))
            # the paper's envelope for this step (Eq. 3 with T_MLP = 0): summary and attended bytes over the
            # HBM peak plus the missed pages over the host link's raw rate (PCIe Gen5 x16, 64 GB/s)
            summary_bytes = int(layer.summaries.numel())
            attended_bytes = layer.stats["selected"] / steps * 8192
            miss_bytes = results[key]["misses_per_step"] * 8192
            results[key]["eq3_ideal_us"] = round((summary_bytes + attended_bytes) / PEAK_HBM_GBPS / 1e3
                                                 + miss_bytes / 64.0 / 1e3, 1)
            if trace is not None:
                from oracle import lru as olru
                rows_b = list(range(0, w.rows, 8))          # one KV head per request: 32 rows
                bel = sum(olru.belady_min_misses(trace[r], layer.budgets[r]) for r in rows_b)
                tot = sum(len(t) for r in rows_b for t in trace[r])
                results[key]["belady_hit_rate_bound_32_rows"] = round(1.0 - bel / tot, 4)
            del layer
            torch.cuda.empty_cache()
    best = min((v["step_us_median"], k) for k, v in results.items())
    line = {"metric": "cfg4 decode step latency (us) with bucketed-LRU HBM budget + LRU hit rate",
            "value": best[0], "unit": "us/step", "n_gpus": 1, "steps": steps, "warmup": 0,
            "ms_per_step": round(best[0] / 1e3, 4), "higher_is_better": False, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": w.name, "batch": w.batch, "contexts_min_median_max": [min(w.seq_lens), int(np.median(w.seq_lens)), max(w.seq_lens)],
                       "budget_frac": args.budget_frac, "lru_timestamps": 64, "best": best[1]},
            "variants": results,
            "paper_context": "bucketed LRU: +49 % decode throughput over keeping only the last step's pages "
                             "(Qwen3-14B, 32K ctx, A100); hit ratio saturates at buffering:mandatory = 4x"}
    print(json.dumps(line))


def run_setup(args):
    """The kernels around the decode step at the headline workload's shape: the
    layout and Index passes of set-up, the decode-time append, the copy kernel in
    both directions over the host link, and the metadata mechanisms.  Every figure
    is the kernel's own duration (HIP events on the launch stream)."""
    import numpy as np
    import torch
    from paper_2604_26837_amd import binding, runner, synth, tables

    dev = "cuda:0"
    w = synth.config1()
    dd = synth.generate_on_device(w, device=dev)
    layer = runner.LayerState.from_natural_pool(w, dd.slot_of, dd.pool, device=dev)
    sp, rows, hkv = layer.spin, w.rows, w.num_kv_heads
    out = {}

    def timed(spx, kid, n, fn):
        spx.profile_enable(n)
        for i in range(n):
            fn(i)
        torch.cuda.synchronize()
        cnt, mean, mn = spx.profile_read(kid)
        spx.profile_enable(0)
        assert cnt == n, (kid, cnt, n)
        return mean, mn

    def entry(mean, mn, nbytes=None, what=None):
        e = dict(mean_us=round(mean, 2), min_us=round(mn, 2))
        if nbytes:
            e.update(bytes=int(nbytes), gbps=round(nbytes / mean / 1e3, 1), counts=what)
        return e

    # --- layout pass: token-major pages -> slot layout, 32768 pages per launch
    k_all, v_all = dd.pool[:, 0].contiguous(), dd.pool[:, 1].contiguous()
    ids = torch.arange(layer.pool_slots, dtype=torch.int32, device=dev)
    chunk = 32768
    nchunk = layer.pool_slots // chunk
    def pack(i):
        s0 = (i % nchunk) * chunk
        sp.pack_kv_pages(k_all[s0:s0 + chunk], v_all[s0:s0 + chunk], ids[s0:s0 + chunk], layer.kv_pool)
    mean, mn = timed(sp, "pack", 16, pack)
    out["pack_32768_pages"] = entry(mean, mn, chunk * 8192 * 2, "bytes read + written")
    del k_all, v_all

    # --- Index: min/max summaries of every page from the keys in the pool
    mean, mn = timed(sp, "index", 8, lambda i: layer.build_summaries())
    index_bytes = layer.pool_slots * 4096 + layer.summaries.numel()      # K tiles read + summaries written
    out["index_minmax_all_pages"] = entry(mean, mn, index_bytes, "K tiles read + summaries written")
    index_us = mean

    # --- copy kernel over the host link, both directions: 64 pages of every row (64 MiB)
    per_row = 64
    host = torch.empty((rows * per_row, 4096), dtype=torch.bfloat16, pin_memory=True)
    row_base = (torch.arange(rows, dtype=torch.int64) * per_row).to(dev)
    count = torch.full((rows,), per_row, dtype=torch.int32, device=dev)
    pages = torch.zeros((rows, sp.page_stride), dtype=torch.int32, device=dev)
    pages[:, :per_row] = torch.arange(per_row, dtype=torch.int32, device=dev)[None, :]
    slots = torch.zeros((rows, sp.page_stride), dtype=torch.int32, device=dev)
    g = torch.Generator(device="cpu")
    g.manual_seed(w.seed)
    slots[:, :per_row] = torch.randperm(layer.pool_slots, generator=g)[:rows * per_row].to(torch.int32).reshape(rows, per_row).to(dev)
    before = layer.kv_pool[slots[:, :per_row].reshape(-1).long()].clone()
    mean, mn = timed(sp, "offload", 8, lambda i: sp.offload_pages(w.batch, layer.kv_pool, host, row_base, count, pages,
                                                                  slots, layer.ws))
    out["offload_8192_pages_to_host"] = entry(mean, mn, rows * per_row * 8192, "page bytes over the host link")
    mean, mn = timed(sp, "gather", 8, lambda i: sp.gather_misses(w.batch, host, row_base, count, pages, slots,
                                                                 layer.kv_pool, layer.ws))
    out["gather_8192_pages_from_host"] = entry(mean, mn, rows * per_row * 8192, "page bytes over the host link")
    assert torch.equal(layer.kv_pool[slots[:, :per_row].reshape(-1).long()], before), "offload + gather round trip"
    del before

    # --- a real selection for the metadata kernels
    layer.step(dd.q)
    torch.cuda.synchronize()
    assert layer.status() == 0

    # --- budget mode at 512 slots per row: resolve under the budget, shrink to half, grow back
    cfg = dict(lru_timestamps=64)
    spb, spb_untimed = binding.Spin.for_workload(w, **cfg), binding.Spin.for_workload(w, **cfg)
    wsb = spb.new_workspace(dev)
    S = 512
    rng_np = np.stack([np.arange(rows, dtype=np.int32) * S, np.full(rows, S, dtype=np.int32)], axis=1)
    slot_range = torch.from_numpy(np.ascontiguousarray(rng_np)).to(dev)
    empty = [np.full((hkv, w.pages(b)), -1, dtype=np.int32) for b in range(w.batch)]
    d, l = tables.build_two_level(empty, spb.dir_stride, w.leaf_entries, allocate_all=True)
    dir_b, leaf_b = torch.from_numpy(d).to(dev), torch.from_numpy(l).to(dev)
    rev = torch.zeros((rows * S, 2), dtype=torch.int32, device=dev)
    rev[:, 0] = -1
    z = lambda *sh, dt=torch.int32: torch.zeros(sh, dtype=dt, device=dev)
    b_slots, b_pages, b_mask, b_np = z(rows, spb.page_stride), z(rows, spb.page_stride), z(rows, spb.page_stride, dt=torch.int16), z(rows)
    m_pages, m_slots, m_n = z(rows, spb.page_stride), z(rows, spb.page_stride), z(rows)
    qsets = [dd.q] + [synth.make_queries_on_device(w, w.seed + 1000 + i, dev) for i in range(1, 8)]
    sels = []
    for q in qsets:
        layer.step(q)
        sels.append((layer.sel.clone(), layer.nsel.clone()))
    half, full = torch.full((rows,), S // 2, dtype=torch.int32, device=dev), torch.full((rows,), S, dtype=torch.int32, device=dev)
    def budget_step(i, spx):
        sel, nsel = sels[i % len(sels)]
        spx.resolve_slots(w.batch, i, sel, nsel, layer.seq_lens, dir_b, leaf_b, b_slots, b_pages, b_mask, b_np, wsb,
                          rev_table=rev, slot_base=slot_range, miss_pages=m_pages, miss_slots=m_slots, nmiss=m_n)
    def shrink_cycle(i):
        budget_step(i, spb_untimed)
        spb.reclaim_tail(w.batch, slot_range, half, dir_b, leaf_b, rev, wsb)          # timed: evicts the tail's pages
        spb_untimed.reclaim_tail(w.batch, slot_range, full, dir_b, leaf_b, rev, wsb)  # grow back
    mean, mn = timed(spb, "meta", 16, shrink_cycle)
    out["reclaim_tail_512_to_256_slots_per_row"] = entry(mean, mn)
    mean, mn = timed(spb, "resolve", 16, lambda i: budget_step(100 + i, spb))
    out["resolve_under_budget_512_slots_per_row"] = entry(mean, mn)
    assert spb.poll_status(wsb) == 0

    # --- leaf chunks on demand: every row's selection touches up to 4 page ranges; a pool with
    # twice the chunks needed, and the worst case of a pool that ends exactly full
    sel0, nsel0 = sels[0]
    for label, chunks in (("pool_2x", rows * 8), ("pool_exact", rows * 4)):
        dir_d = torch.full_like(dir_b, -1)
        leaf_d = torch.zeros((chunks, w.leaf_entries), dtype=torch.int32, device=dev)
        bitmap = torch.zeros((chunks + 31) // 32, dtype=torch.int32, device=dev)
        def alloc_cycle(i):
            spb.alloc_leaves(w.batch, sel0, nsel0, layer.seq_lens, dir_d, leaf_d, bitmap, wsb)       # timed
            spb_untimed.free_leaves(w.batch, dir_d, chunks, bitmap, wsb)
        mean, mn = timed(spb, "meta", 16, alloc_cycle)
        out[f"alloc_leaves_from_empty_directory_{label}"] = entry(mean, mn)
        def free_cycle(i):
            spb_untimed.alloc_leaves(w.batch, sel0, nsel0, layer.seq_lens, dir_d, leaf_d, bitmap, wsb)
            spb.free_leaves(w.batch, dir_d, chunks, bitmap, wsb)                                     # timed
        mean, mn = timed(spb, "meta", 16, free_cycle)
        out[f"free_leaves_{label}"] = entry(mean, mn)
        assert spb.poll_status(wsb) == 0 and int(bitmap.abs().sum().item()) == 0

    # --- decode-time Index: one token per request appended to its slot and its page's summary
    k_new = torch.randn((w.batch, hkv, w.head_dim), device=dev).to(torch.bfloat16)
    v_new = torch.randn((w.batch, hkv, w.head_dim), device=dev).to(torch.bfloat16)
    n_app = 32
    lens = [torch.full((w.batch,), w.seq_lens[0] - 40 + i, dtype=torch.int32, device=dev) for i in range(n_app)]
    mean, mn = timed(sp, "append", n_app, lambda i: sp.append_kv(w.batch, k_new, v_new, lens[i], layer.kv_pool, layer.dir,
                                                                  layer.leaf_pool, layer.part_offsets, None,
                                                                  layer.summaries, layer.ws))
    out["append_one_token_per_request"] = entry(mean, mn)
    assert layer.status() == 0

    ach = index_bytes / index_us / 1e3
    line = {"metric": "set-up and maintenance kernels at the headline workload's shape (kernel us per launch)",
            "value": round(index_us, 2), "unit": "us (Index over all pages)", "n_gpus": 1, "steps": 8, "warmup": 0,
            "ms_per_step": round(index_us / 1e3, 4), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
            "dtype": "bf16", "data": "synthetic",
            "config": {"workload": w.name + "_setup", "batch": w.batch, "context": w.seq_lens[0], "kv_heads": hkv,
                       "pool_slots": layer.pool_slots},
            "kernels": out,
            "roofline": dict(bound="hbm", kernel="spin_index_minmax_pages_kernel", achieved=round(ach, 1),
                             peak=PEAK_HBM_GBPS, unit="GB/s", frac=round(ach / PEAK_HBM_GBPS, 4), traffic=None,
                             algorithmic_bytes=int(index_bytes), mean_us=round(index_us, 2)),
            "cpu_baseline": None}
    print(json.dumps(line))


def run_attention_sweep(args):
    """Stage 4 alone at the headline workload's shape, page lists of 32 ... 128 random resident pages per row:
    the kernel's own duration (HIP events on the launch stream) against the pages per row, and the straight
    line through it: a fixed part per launch and a rate for the bytes."""
    import numpy as np
    import torch
    from paper_2604_26837_amd import binding, synth

    dev = "cuda:0"
    w = synth.config1()
    rows, nslots, pages_per_row = w.rows, w.total_slots, w.pages(0)
    pool = torch.empty((nslots, 4096), dtype=torch.bfloat16, device=dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)
    for s0 in range(0, nslots, 32768):
        n = min(32768, nslots - s0)
        pool[s0:s0 + n] = torch.randn((n, 4096), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    q = torch.randn((w.batch, w.num_q_heads, w.head_dim), generator=gen, device=dev).to(torch.bfloat16)
    rng = np.random.default_rng(w.seed)
    perm = rng.permutation(nslots).astype(np.int32)          # physical order differs from logical order
    sp = binding.Spin.for_workload(w, decode_splits=args.decode_splits, decode_waves=args.decode_waves,
                                   decode_depth=args.decode_depth)
    width = sp.page_stride
    lists = []
    for _ in range(args.query_sets):                          # distinct page lists, so that no cache serves the pages
        sl = np.empty((rows, width), dtype=np.int32)
        for r in range(rows):
            sl[r] = perm[r * pages_per_row + np.sort(rng.choice(pages_per_row, size=width, replace=False))]
        lists.append(torch.from_numpy(sl).to(dev))
    ws = sp.new_workspace(dev)
    masks = torch.full((rows, width), -1, dtype=torch.int16, device=dev)
    out = torch.zeros((w.batch, w.num_q_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
    points = []
    for npr in (32, 48, 64, 80, 96, 104, 112, 116, 120, 124, 128):
        if npr > width:
            continue
        npg = torch.full((rows,), npr, dtype=torch.int32, device=dev)
        for i in range(args.warmup):
            sp.sparse_decode(w.batch, q, pool, lists[i % len(lists)], masks, npg, out, None, ws)
        torch.cuda.synchronize()
        sp.profile_enable(args.steps)
        for i in range(args.steps):
            sp.sparse_decode(w.batch, q, pool, lists[i % len(lists)], masks, npg, out, None, ws)
        torch.cuda.synchronize()
        n, mean, mn = sp.profile_read("decode")
        sp.profile_enable(0)
        nbytes = rows * npr * 8192
        points.append(dict(pages_per_row=npr, bytes=nbytes, mean_us=round(mean, 2), min_us=round(mn, 2),
                           gbps=round(nbytes / mean / 1e3, 1), pct_peak=round(nbytes / mean / 1e3 / 80.0, 1)))
    assert sp.poll_status(ws) == 0, "device fault during the sweep"
    x = np.array([p["bytes"] for p in points], dtype=np.float64)
    y = np.array([p["mean_us"] for p in points], dtype=np.float64)
    slope, fixed = np.polyfit(x, y, 1)                        # us per byte, us
    resid = y - (fixed + slope * x)
    print(json.dumps({
        "metric": "stage-4 kernel duration against the pages per row (cfg1's shape: 128 rows, 8 KiB pages, random slots)",
        "unit": "us", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "cfg1_attention_pages_per_row_sweep", "rows": rows, "decode_splits": sp.decode_splits,
                   "decode_waves": args.decode_waves or 8},
        "points": points,
        "fit": {"fixed_us_per_launch": round(float(fixed), 2), "marginal_gbps": round(1e-3 / float(slope), 0),
                "max_abs_residual_us": round(float(np.abs(resid).max()), 2)}}))


def main():
    args = parse_args()
    if args.print_source_hash:
        print(source_hash())
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (every stage is independent per (request, KV head) "
              "row and no collective is involved); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    # the all-cores leg of the CPU baseline runs in worker processes; they are created here, before anything
    # touches the GPU (only the workloads that have a CPU leg need them)
    pool = None
    if not args.no_cpu and args.workload in ("cfg1", "cfg2", "cfg3", "cfg1_mean"):
        pool = OraclePool()

    import numpy as np
    import torch
    from paper_2604_26837_amd import build as _build
    if not os.path.exists(_build.LIB_PATH):
        _build.build_library()
    from paper_2604_26837_amd import runner, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.workload == "cfg4":
        run_cfg4(args)
        return
    if args.workload == "setup":
        run_setup(args)
        return
    if args.workload == "attention_sweep":
        run_attention_sweep(args)
        return
    if args.workload == "cfg1_mean":
        # the headline shape scored the way the paper's page-partition algorithm does: one mean key
        # (landmark) per page instead of its min / max keys
        w = synth.config1().with_(score_kind=synth.SCORE_REPMAX, reps_per_partition=1, name="cfg1_mean_landmarks")
    else:
        w = {"cfg1": synth.config1, "cfg2": synth.config2, "cfg3": synth.config3}[args.workload]()
    layer, natural = runner.build_device_layer(w, device=dev, keep_natural=not args.no_cpu,
                                               decode_splits=args.decode_splits, decode_waves=args.decode_waves,
                                               decode_depth=args.decode_depth, score_waves=args.score_waves,
                                               score_tiles_per_wg=args.score_tiles)
    # rows of at most 16384 partitions: stage 2 is one launch, which also resolves
    one_launch_23 = max(w.partitions(b) for b in range(w.batch)) <= 16384
    # longer rows: stages 1-3 in one call (stage 1 takes stage 2's histogram along, stage 2's last launch resolves)
    fused_12 = not one_launch_23 and not args.four_calls
    sp = layer.spin

    # distinct query sets (seeds base+1000+i) and distinct summary copies
    qsets = [layer.q0] + [synth.make_queries_on_device(w, w.seed + 1000 + i, dev) for i in range(1, args.query_sets)]
    summ_copies = [layer.summaries] + [layer.summaries.clone() for _ in range(1, args.layers)]
    torch.cuda.synchronize()

    def run_four(i):
        layer.step(qsets[i % len(qsets)], summ_copies[i % len(summ_copies)])

    # the step as timed: three launches whatever the row length (score, select+resolve, attention; for long
    # rows stages 1-3 are one call), same results bit for bit; the four separate calls are timed beside it
    def run_fused(i):
        layer.step_fused(qsets[i % len(qsets)], summ_copies[i % len(summ_copies)])

    run_three = run_12 = run_fused
    run = run_four if args.four_calls else run_fused

    for i in range(args.warmup):
        run(i)
    torch.cuda.synchronize()
    assert layer.status() == 0, "device fault during warm-up"

    # --- timed region: exactly K steps of the decode step as `run` issues it (by default the three-launch form:
    # score, select+resolve in one launch, attention; --four-calls times the four separate stage calls instead;
    # `step_launches` in the output says which, and the other form is timed right after for reference)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        run(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    us_per_step = dt * 1e6 / args.steps
    assert layer.status() == 0, "device fault during the timed region"
    # mean of three more runs of the same K steps, as a steadier figure beside `value` (which stays the first run)
    more = []
    for _ in range(3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            run(i)
        torch.cuda.synchronize()
        more.append((time.perf_counter() - t0) * 1e6 / args.steps)

    # --- the other launch shape of the same step, for reference
    other = (run_three if one_launch_23 else run_12) if args.four_calls else run_four
    us_per_step_other = None
    if not args.no_other_form:
        for i in range(5):
            other(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            other(i)
        torch.cuda.synchronize()
        us_per_step_other = (time.perf_counter() - t0) * 1e6 / args.steps

    # --- the same step recorded once per (query set, summary copy) pair in a HIP graph and replayed: the launch
    # gaps of the host-issued step are replaced by the graph's own dispatch.  Checked against the eager bits.
    us_per_step_graph = us_per_step_graph_many = graph_steps = None
    if not args.no_graph:
        import math as _m
        ncomb = len(qsets) * len(summ_copies) // _m.gcd(len(qsets), len(summ_copies))
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            run(0)                                      # warm-up on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graphs = []
        for i in range(ncomb):
            gph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gph):
                run(i)
            graphs.append(gph)
        run(1)
        torch.cuda.synchronize()
        eager_bits = layer.out.view(torch.int16).clone()
        layer.out.fill_(5.0)
        graphs[1 % ncomb].replay()
        torch.cuda.synchronize()
        assert torch.equal(layer.out.view(torch.int16), eager_bits), "graph replay differs from the eager step"
        for i in range(args.warmup):
            graphs[i % ncomb].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            graphs[i % ncomb].replay()
        torch.cuda.synchronize()
        us_per_step_graph = (time.perf_counter() - t0) * 1e6 / args.steps
        assert layer.status() == 0, "device fault during the graph replays"
        del graphs
        # one graph holding `ncomb` consecutive steps (as the layers of a model share one graph): the replay cost
        # is paid once per `ncomb` steps
        many = torch.cuda.CUDAGraph()
        with torch.cuda.graph(many):
            for i in range(ncomb):
                run(i)
        nrep = max(1, args.steps // ncomb)
        for _ in range(2):
            many.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(nrep):
            many.replay()
        torch.cuda.synchronize()
        us_per_step_graph_many = (time.perf_counter() - t0) * 1e6 / (nrep * ncomb)
        graph_steps = ncomb
        assert layer.status() == 0, "device fault during the graph replays"
        del many

    # --- spread of the step time: the same K steps with a stream event between consecutive steps
    # (no host synchronisation inside; the event records cost a little, so `value` stays the
    # figure of the plain run above)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    evs[0].record()
    for i in range(args.steps):
        run(i)
        evs[i + 1].record()
    torch.cuda.synchronize()
    per_step = sorted(evs[i].elapsed_time(evs[i + 1]) * 1e3 for i in range(args.steps))
    pct = lambda f: round(per_step[min(int(f * len(per_step)), len(per_step) - 1)], 2)
    step_spread = dict(p10=pct(0.10), median=pct(0.50), p90=pct(0.90), note="stream events between steps")

    # --- the same K steps again with every kernel bracketed by HIP events on the
    # launch stream (start/stop timestamps of the kernel itself); the bracketing
    # slows the step down, so it is kept out of `value`
    kernels = {}
    us_per_step_events = None
    if not args.no_kernel_events:
        sp.profile_enable(args.steps)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            run(i)
        torch.cuda.synchronize()
        us_per_step_events = (time.perf_counter() - t0) * 1e6 / args.steps
        for name in ("score", "select_hist", "select", "resolve", "decode"):
            n, mean, mn = sp.profile_read(name)
            if n:
                label = "select+resolve" if (name == "select" and not args.four_calls) else name
                kernels[label] = dict(launches=n, mean_us=round(mean, 3), min_us=round(mn, 3))
        sp.profile_enable(0)
        assert layer.status() == 0, "device fault during the event-bracketed pass"

    # --- when the timed step attends the sink / recent pages beside stages 2+3: the plain three-launch step with
    # the same event bracketing, to say what that side work costs the launch of stages 2+3 and what stage 4 takes
    # over all pages
    forced_split = (not args.four_calls) and sp.forced_split_supported
    plain_kernels = {}
    if forced_split and not args.no_kernel_events:
        sp.profile_enable(args.steps)
        for i in range(args.steps):
            layer.step3(qsets[i % len(qsets)], summ_copies[i % len(summ_copies)])
        torch.cuda.synchronize()
        for name, label in (("select", "select+resolve"), ("decode", "decode")):
            n, mean, mn = sp.profile_read(name)
            if n:
                plain_kernels[label] = dict(launches=n, mean_us=round(mean, 3), min_us=round(mn, 3))
        sp.profile_read("score")
        sp.profile_enable(0)
        run(0)                                                         # leave the timed step's results in the buffers
        torch.cuda.synchronize()

    # --- yardstick: a plain streaming read of 128 MiB per launch from the same pool (cold: the
    # launches walk through 2 GiB), timed with the same kernel events
    stream_gbps = None
    if not args.no_kernel_events:
        sp.profile_enable(32)
        pool_u8 = layer.kv_pool.view(torch.uint8).reshape(-1)
        chunk = 128 << 20
        nchunks = pool_u8.numel() // chunk
        for i in range(32):
            sp.probe_stream_read(pool_u8[(i % nchunks) * chunk:], chunk, layer.ws)
        torch.cuda.synchronize()
        n, mean, mn = sp.profile_read("probe")
        sp.profile_enable(0)
        if n:
            stream_gbps = round(chunk / mean / 1e3, 1)

    # --- byte accounting (Eq. 1 / Eq. 2 of the paper's envelope for this workload)
    # attended tokens = set bits of the page masks (whole pages unless partitions are smaller than a page)
    mask_bits = layer.valid_mask.to(torch.int32) & 0xFFFF
    in_list = torch.arange(mask_bits.shape[1], device=dev)[None, :] < layer.npages[:, None]
    attended_tokens = int(sum(((mask_bits >> t) & 1)[in_list].sum().item() for t in range(16)))
    kv_bytes = attended_tokens * 2 * w.head_dim * 2                    # 512 B per attended token
    page_bytes = int(layer.npages.sum().item()) * 8192                 # what page-granular gathering reads
    score_bytes = int(layer.summaries.numel())                         # summary bytes of the (padded) rows
    dec_us = kernels.get("decode", {}).get("mean_us") or None
    sc_us = kernels.get("score", {}).get("mean_us") or None
    # bytes stage 4's launch itself moves: with the forced split, the sink / recent pages (whole pages: one-page
    # partitions) were attended by the launch of stages 2+3
    dec_bytes, side_bytes, side_us = kv_bytes, 0, 0.0
    if forced_split:
        for b in range(w.batch):
            pages = w.pages(b)
            lo, hi = min(w.sink_pages, pages), max(pages - w.recent_pages, 0)
            forced_tokens = w.seq_lens[b] if lo >= hi else 16 * lo + (w.seq_lens[b] - 16 * hi)
            side_bytes += forced_tokens * w.num_kv_heads * 2 * w.head_dim * 2
        dec_bytes = kv_bytes - side_bytes
        if plain_kernels.get("select+resolve") and kernels.get("select+resolve"):
            side_us = max(0.0, kernels["select+resolve"]["mean_us"] - plain_kernels["select+resolve"]["mean_us"])
    roofline = None
    attended = None
    if dec_us:
        # the metric's figure: all attended K/V bytes of the step over the time spent attending them (stage 4's
        # launch plus what the side work adds to the launch of stages 2+3)
        attended = dict(bytes=kv_bytes, us=round(dec_us + side_us, 3), gbps=round(kv_bytes / (dec_us + side_us) / 1e3, 1),
                        pct_peak=round(100 * kv_bytes / (dec_us + side_us) / 1e3 / PEAK_HBM_GBPS, 2),
                        side_bytes=side_bytes, side_us=round(side_us, 3))
        ach = dec_bytes / dec_us / 1e3                                 # GB/s
        kernel = "spin_decode_tokens_kernel<8>" if w.partition_tokens < 16 else \
            f"spin_decode_kernel<{args.decode_waves or 8}, {args.decode_depth or 2}>"
        traffic, traffic_note = read_traffic(os.path.join(ROOT, "profiles", f"{args.workload}_stage_kernels_pmc.txt"),
                                             kernel)
        roofline = dict(bound="hbm", kernel=kernel, achieved=round(ach, 1), peak=PEAK_HBM_GBPS,
                        unit="GB/s", frac=round(ach / PEAK_HBM_GBPS, 4), traffic=traffic, traffic_note=traffic_note,
                        algorithmic_bytes=dec_bytes, whole_page_bytes=page_bytes - side_bytes, mean_us=dec_us)
        if plain_kernels.get("decode"):
            pd = plain_kernels["decode"]["mean_us"]
            roofline["all_pages_in_stage_4"] = dict(mean_us=pd, algorithmic_bytes=kv_bytes,
                                                    achieved=round(kv_bytes / pd / 1e3, 1),
                                                    frac=round(kv_bytes / pd / 1e3 / PEAK_HBM_GBPS, 4))

    # --- CPU oracle on a bounded sample of the same workload, same run
    cpu = None
    parity = None
    if not args.no_cpu:
        run(0)                                                         # query set 0, summary copy 0
        torch.cuda.synchronize()
        q_bits = qsets[0].view(torch.int16).cpu().numpy().view(np.uint16)
        picked, prepared, results, cpu_us, cpu_all = cpu_oracle_leg(layer, natural, q_bits, args.cpu_rows,
                                                                     args.cpu_reps, pool)
        if pool is not None:
            pool.close()
        from oracle import attend as oattend, bf16 as obf16
        out = obf16.decode(layer.out.view(torch.int16).cpu().numpy().view(np.uint16))
        page_ids = layer.page_ids.cpu().numpy()
        npages = layer.npages.cpu().numpy()
        worst, same_sel = 0.0, 0
        vmask = layer.valid_mask.cpu().numpy().view(np.uint16)
        for (r, b, h, q, summ, page_map, pages, chan), res in zip(prepared, results):
            gp = page_ids[r, :npages[r]].tolist()
            gm = [int(m) for m in vmask[r, :npages[r]]]
            same_sel += int(gp == res["page_ids"] and gm == [int(m) for m in res["masks"]])
            pg = obf16.decode(pages[np.asarray(gp, dtype=np.int64)])
            ks, vs = oattend.gather_tokens(pg[:, 0], pg[:, 1], gm)   # the GPU's own page list and masks
            ref, _ = oattend.attend(q, ks, vs, layer.scale)
            g = w.group
            err = np.abs(out[b, h * g:(h + 1) * g] - ref) - (2e-2 + 1e-2 * np.abs(ref))
            worst = max(worst, float(err.max()))
        parity = dict(rows=len(picked), rows_same_selection_as_fp64=same_sel, worst_excess_over_tolerance=worst,
                      ok=bool(worst <= 0.0))
        cpu = dict(value=round(cpu_us, 1), unit="us/layer", cores=1, kind="oracle",
                   sample=f"{len(picked)} of {w.rows} rows of the same step, {args.cpu_reps} repetitions, "
                          f"scaled by {w.rows / len(picked):.0f}; host has {os.cpu_count()} logical CPUs",
                   all_cores=cpu_all, cpu_model=cpu_model(),
                   note="all_cores: the same rows dealt to worker processes (one single-threaded oracle each), "
                        "wall clock of the slowest, same scaling")

    line = {
        "metric": METRIC if args.workload == "cfg1" else f"sparse decode µs/layer + attended-KV HBM GB/s (% peak), {w.name}",
        "value": round(us_per_step, 2), "unit": "us/layer", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(us_per_step / 1e3, 5),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "context": w.seq_lens[0], "q_heads": w.num_q_heads,
                   "kv_heads": w.num_kv_heads, "head_dim": w.head_dim, "page_tokens": w.page_tokens,
                   "partition_tokens": w.partition_tokens, "score": ["minmax", "sketch", "repmax"][w.score_kind],
                   "topk_partitions": w.topk, "decode_splits": sp.decode_splits, "decode_waves": args.decode_waves or 8, "query_sets": len(qsets),
                   "summary_copies": len(summ_copies)},
        "attended_kv_gbps": attended["gbps"] if attended else None,
        "attended_kv_pct_peak": attended["pct_peak"] if attended else None,
        "attended_kv": attended,
        "step_launches": "four stage calls" if args.four_calls else (
            "stages 1-3 in one call (stage 1 counts stage 2's histogram, stage 2's launch resolves), attention (3 launches)" if fused_12
            else ("score, select+resolve with the sink / recent pages attended on the side, attention over the "
                  "other pages (3 launches)" if forced_split else "score, select+resolve, attention (3 launches)")),
        "kernels_plain_three_launch_step": plain_kernels or None,
        ("us_per_layer_fused_calls" if args.four_calls else "us_per_layer_four_calls"): round(us_per_step_other, 2) if us_per_step_other else None,
        "us_per_layer_repeats": [round(x, 2) for x in more],
        "us_per_layer_graph_replay": round(us_per_step_graph, 2) if us_per_step_graph else None,
        "us_per_layer_graph_replay_many": dict(value=round(us_per_step_graph_many, 2), steps_per_graph=graph_steps)
        if us_per_step_graph_many else None,
        "us_per_layer_with_kernel_events": round(us_per_step_events, 2) if us_per_step_events else None,
        "us_per_layer_spread": step_spread,
        "kernel_us_sum": round(sum(k["mean_us"] for k in kernels.values()), 2) if kernels else None,
        "kernels": kernels,
        "score_gbps": round(score_bytes / sc_us / 1e3, 1) if sc_us else None,
        "stream_read_128MiB_gbps": stream_gbps,
        "ideal_us_at_peak": round((kv_bytes + score_bytes) / PEAK_HBM_GBPS / 1e3, 2),
        "roofline": roofline, "cpu_baseline": cpu, "parity": parity,
        "paper_context": "end-to-end on A100/B200 (not this metric): 1.66-5.66x throughput, 7-9x lower TTFT "
                         "vs vLLM; up to 58% lower TPOT vs original sparse implementations",
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
