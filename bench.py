#!/usr/bin/env python3
"""Benchmark of the sparse-decode hot path on one MI355X.

One "step" = one pass of the whole path (score -> select -> resolve -> attend)
for one layer over one batch of synthetic input, resident in HBM.  Prints ONE
JSON line; see the design doc for the byte accounting behind `roofline`.
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
    ap.add_argument("--workload", default="cfg1", choices=["cfg1", "cfg2", "cfg3", "cfg4"],
                    help="cfg1: the headline all-resident layer (the metric's workload); cfg2: token partitions scored "
                         "on a key sketch; cfg3: 128-token blocks with representative keys; cfg4: hierarchical HBM "
                         "budget, 64 decode steps")
    ap.add_argument("--copy-mode", default="both", choices=["memcpy", "gather", "both"])
    ap.add_argument("--budget-frac", type=float, default=0.25)
    ap.add_argument("--four-calls", action="store_true",
                    help="time the four separate stage calls as the step (default: stages 2+3 share one launch)")
    ap.add_argument("--decode-splits", type=int, default=0, help="split-K factor of the attention kernel (0: library default)")
    ap.add_argument("--decode-waves", type=int, default=0, help="wavefronts per attention workgroup (0: library default)")
    ap.add_argument("--decode-depth", type=int, default=0, help="page buffers per attention wavefront (0: library default)")
    ap.add_argument("--score-waves", type=int, default=0, help="wavefronts per stage-1 workgroup (0: library default)")
    ap.add_argument("--score-tiles", type=int, default=0, help="summary tiles per stage-1 workgroup (0: library default)")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="do not bracket kernels with HIP events during the timed region")
    return ap.parse_args()


def read_traffic(path):
    """HBM bytes per launch of the decode kernel from the committed counter summary, or None."""
    try:
        txt = open(path).read()
    except OSError:
        return None
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", txt, re.M)
    return float(m.group(1)) if m else None


def cpu_oracle_leg(layer, natural, q_bits, rows, reps):
    """Times the fp64 oracle (as it stands) on `rows` rows of the same workload
    and checks the GPU's output for those rows against it."""
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
    t0 = time.perf_counter()
    results = None
    for _ in range(reps):
        results = [ostep.decode_row(q, summ, w.score_kind, w.seq_lens[b], w.page_tokens,
                                    w.partition_tokens, w.topk, w.topk_includes_forced, w.sink_pages,
                                    w.recent_pages, page_map, r, pages, layer.scale, channels=chan)
                   for (r, b, h, q, summ, page_map, pages, chan) in prepared]
    dt = (time.perf_counter() - t0) / reps
    if limiter is not None:
        limiter.restore_original_limits() if hasattr(limiter, "restore_original_limits") else None
    us_per_layer = dt * 1e6 * (w.rows / len(picked))
    return picked, prepared, results, us_per_layer


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
    for exact, policy in ((False, 0), (True, 0), (False, 1)):
        for mode in modes:
            if (exact or policy) and mode != modes[-1]:
                continue
            layer = hier.HierLayer(w, budget_frac=args.budget_frac, n_ts=64, evict_exact=exact, copy_mode=mode,
                                   lru_policy=policy, decode_splits=args.decode_splits,
                                   decode_waves=args.decode_waves, decode_depth=args.decode_depth)
            q = layer.q0
            lat, persist, prev = [], [], None
            layer.spin.profile_enable(steps)          # kernels bracketed by HIP events on the launch stream
            trace = [[] for _ in range(w.rows)] if (mode == modes[-1] and not exact and not policy and not args.no_cpu) else None
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
            key = f"{mode}{'_evict_exact' if exact else ''}{'_set_assoc8' if policy else ''}"
            results[key] = dict(hit_rate=round(overall, 4), hit_rate_after_step0=round(warm, 4),
                                misses_per_step=round(layer.stats["misses_after_first"] / (steps - 1), 1),
                                selected_per_step=round(layer.stats["selected"] / steps, 1),
                                step_us_median=round(lat_w[len(lat_w) // 2], 1), step_us_p90=round(lat_w[int(0.9 * len(lat_w))], 1),
                                first_step_us=round(lat[0], 1), topk_persistence=round(float(np.mean(persist)), 4),
                                kernel_us=kern, pool_gib=round(layer.pool_slots * 8192 / 2**30, 2),
                                host_kv_gib=round(layer.host_kv.numel() * 2 / 2**30, 2))
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


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (every stage is independent per (request, KV head) "
              "row and no collective is involved); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

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
    w = {"cfg1": synth.config1, "cfg2": synth.config2, "cfg3": synth.config3}[args.workload]()
    layer, natural = runner.build_device_layer(w, device=dev, keep_natural=not args.no_cpu,
                                               decode_splits=args.decode_splits, decode_waves=args.decode_waves,
                                               decode_depth=args.decode_depth, score_waves=args.score_waves,
                                               score_tiles_per_wg=args.score_tiles)
    # stages 2+3 share a launch only for rows the one-launch kernel takes (at most 16384 partitions)
    one_launch_23 = max(w.partitions(b) for b in range(w.batch)) <= 16384
    if not one_launch_23:
        args.four_calls = True
    sp = layer.spin

    # distinct query sets (seeds base+1000+i) and distinct summary copies
    qsets = [layer.q0] + [synth.make_queries_on_device(w, w.seed + 1000 + i, dev) for i in range(1, args.query_sets)]
    summ_copies = [layer.summaries] + [layer.summaries.clone() for _ in range(1, args.layers)]
    torch.cuda.synchronize()

    def run_four(i):
        layer.step(qsets[i % len(qsets)], summ_copies[i % len(summ_copies)])

    def run_three(i):
        layer.step3(qsets[i % len(qsets)], summ_copies[i % len(summ_copies)])

    # the step as timed: score, select+resolve in one launch, attention (three
    # launches, same results bit for bit); the four separate calls are timed beside it
    run = run_four if args.four_calls else run_three

    for i in range(args.warmup):
        run(i)
    torch.cuda.synchronize()
    assert layer.status() == 0, "device fault during warm-up"

    # --- timed region: exactly K steps of the four-call sequence
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        run(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    us_per_step = dt * 1e6 / args.steps
    assert layer.status() == 0, "device fault during the timed region"

    # --- the other launch shape of the same step, for reference
    other = run_three if args.four_calls else run_four
    us_per_step_other = None
    if one_launch_23:
        for i in range(5):
            other(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            other(i)
        torch.cuda.synchronize()
        us_per_step_other = (time.perf_counter() - t0) * 1e6 / args.steps

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
    roofline = None
    if dec_us:
        ach = kv_bytes / dec_us / 1e3                                  # GB/s
        traffic = read_traffic(os.path.join(ROOT, "profiles", f"{args.workload}_stage_kernels_pmc.txt"))
        roofline = dict(bound="hbm", kernel="spin_decode_tokens_kernel" if w.partition_tokens < 16 else "spin_decode_kernel", achieved=round(ach, 1), peak=PEAK_HBM_GBPS,
                        unit="GB/s", frac=round(ach / PEAK_HBM_GBPS, 4), traffic=traffic,
                        algorithmic_bytes=kv_bytes, whole_page_bytes=page_bytes, mean_us=dec_us)

    # --- CPU oracle on a bounded sample of the same workload, same run
    cpu = None
    parity = None
    if not args.no_cpu:
        run(0)                                                         # query set 0, summary copy 0
        torch.cuda.synchronize()
        q_bits = qsets[0].view(torch.int16).cpu().numpy().view(np.uint16)
        picked, prepared, results, cpu_us = cpu_oracle_leg(layer, natural, q_bits, args.cpu_rows, args.cpu_reps)
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
                          f"scaled by {w.rows / len(picked):.0f}; host has {os.cpu_count()} logical CPUs")

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
        "attended_kv_gbps": roofline["achieved"] if roofline else None,
        "attended_kv_pct_peak": round(100 * roofline["frac"], 2) if roofline else None,
        "step_launches": "four stage calls" if args.four_calls else "score, select+resolve, attention (3 launches)",
        ("us_per_layer_three_launches" if args.four_calls else "us_per_layer_four_calls"): round(us_per_step_other, 2) if us_per_step_other else None,
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
