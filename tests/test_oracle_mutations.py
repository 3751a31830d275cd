"""Do the pins pin?  Each case plants one plausible mistake in the oracle's source (a wrong reduction, a
flipped comparison, a dropped term, an off-by-one, a transposed operand), in a child process, and runs the
oracle's pin tests there: they must fail.  A pin file that stays green under a planted mistake would mean
the oracle could carry that mistake unnoticed.  CPU only; the product code is not involved."""
import json
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))

# (oracle module, source text, replacement, pin files that must notice)
MISTAKES = [
    # stage 1
    ("score", "s[p] = per_head.max()", "s[p] = per_head.min()", ["test_oracle_score.py"]),
    ("score", "np.maximum(q * mins[p][None, :], q * maxs[p][None, :])",
     "np.minimum(q * mins[p][None, :], q * maxs[p][None, :])", ["test_oracle_score.py"]),
    ("score", "np.maximum(q * mins[p][None, :], q * maxs[p][None, :])",
     "(q * maxs[p][None, :])", ["test_oracle_score.py"]),
    ("score", "return (sketch @ qc.T).max(axis=1)", "return (sketch @ qc.T).sum(axis=1)", ["test_oracle_score.py"]),
    ("score", "qc = q[:, np.asarray(channels, dtype=np.int64)]", "qc = q[:, :len(channels)]", ["test_oracle_score.py"]),
    ("score", "return dots.max(axis=(1, 2))", "return dots.max(axis=2).mean(axis=1)", ["test_oracle_score.py"]),
    # Index
    ("index", "        t1 = min(t0 + partition_tokens, seq_len)\n        mins[p]",
     "        t1 = t0 + partition_tokens\n        mins[p]", ["test_oracle_score.py"]),
    ("index", "maxs[p] = K[t0:t1].max(axis=0)", "maxs[p] = K[t0:t1].mean(axis=0)", ["test_oracle_score.py"]),
    ("index", "mean = K[t0:t1].sum(axis=0) / float(t1 - t0)", "mean = K[t0:t1].sum(axis=0) / float(sub)",
     ["test_oracle_score.py"]),
    ("index", "out[p, r] = out[p, 0]", "out[p, r] = 0.0", ["test_oracle_score.py"]),
    ("varpart", "blk.sum(axis=0) / float(tokens[p])", "blk.sum(axis=0) / float(page_tokens)", ["test_oracle_varpart.py"]),
    # stage 2
    ("select", "return (-s, i)", "return (-s, -i)", ["test_oracle_select.py"]),
    ("select", "return (-s, i)", "return (s, i)", ["test_oracle_select.py"]),
    ("select", "kprime = topk - len(forced) if topk_includes_forced else topk", "kprime = topk",
     ["test_oracle_select.py"]),
    ("select", "cands = [p for p in range(P) if p not in fset]", "cands = [p for p in range(P)]",
     ["test_oracle_select.py"]),
    # stage 3 and the replacement policy
    ("resolve", "return (1 << n) - 1", "return (1 << page_tokens) - 1", ["test_oracle_resolve.py"]),
    ("resolve", "masks[pg] = masks.get(pg, 0) | (1 << (t % page_tokens))", "masks[pg] = 1 << (t % page_tokens)",
     ["test_oracle_resolve.py"]),
    ("lru", "evict = t <= x", "evict = t < x", ["test_oracle_lru.py"]),
    ("lru", "cache.ts[s] = max(cache.ts[s] - 1, 0)", "cache.ts[s] = cache.ts[s]", ["test_oracle_lru.py"]),
    ("lru", "ts_star = min(step, n - 1)", "ts_star = step % n", ["test_oracle_lru.py"]),
    ("lru", "net = max(0, demand - free)", "net = demand", ["test_oracle_lru.py"]),
    ("lru", "        for t in range(n):\n            if cum + hist[t] >= net:",
     "        for t in reversed(range(n)):\n            if cum + hist[t] >= net:", ["test_oracle_lru.py"]),
    ("lru", "for p, s in zip(misses, free_slots):", "for p, s in zip(misses, reversed(free_slots)):",
     ["test_oracle_lru.py"]),
    ("lru", "    for s in range(keep, S):\n        p = cache.page[s]", "    for s in range(keep + 1, S):\n        p = cache.page[s]",
     ["test_oracle_lru.py"]),
    ("lru", "far = max(victims, key=lambda r: (resident[r], r))", "far = min(victims, key=lambda r: (resident[r], r))",
     ["test_oracle_lru.py"]),
    ("lru", "if best is None or cache.ts[base + w] < best:", "if best is None or cache.ts[base + w] > best:",
     ["test_oracle_lru_setassoc.py"]),
    ("lru", "            if any(cache.page[base + w] not in selected for w in range(ways)):\n                break",
     "            if True:\n                break", ["test_oracle_lru_setassoc.py"]),
    ("lru", "st = mix32(row, p) % sets", "st = p % sets", ["test_oracle_lru_setassoc.py"]),
    # variable-length partitions, pinned partitions
    ("varpart", "n = min(max(tokens[p] - page_tokens * k, 0), page_tokens)", "n = page_tokens", ["test_oracle_varpart.py"]),
    ("varpart", "if all(x in fp for x in partition_page_list(first_page, tokens, p, page_tokens))] if fp else []",
     "if any(x in fp for x in partition_page_list(first_page, tokens, p, page_tokens))] if fp else []",
     ["test_oracle_varpart.py"]),
    ("varpart", "mins[p], maxs[p] = blk.min(axis=0), blk.max(axis=0)", "mins[p], maxs[p] = blk.max(axis=0), blk.min(axis=0)",
     ["test_oracle_varpart.py"]),
    ("select", "out[p] = math.inf", "out[p] = -math.inf", ["test_oracle_select.py"]),
    # byte model
    ("envelope", "return 2 * B * L * H * d * e * beta * N", "return B * L * H * d * e * beta * N", ["test_oracle_envelope.py"]),
    ("envelope", "rho * topk_bytes / bw_pcie", "rho * score_bytes / bw_pcie", ["test_oracle_envelope.py"]),
    # stage 4
    ("attend", "logits = scale * (q @ K_S.T)", "logits = q @ K_S.T", ["test_oracle_attend.py"]),
    ("attend", "out = (w @ V_S) / l", "out = (w @ K_S) / l", ["test_oracle_attend.py"]),
    ("attend", "out = (w @ V_S) / l", "out = (w @ V_S)", ["test_oracle_attend.py"]),
    ("attend", "l = sum(p[1] * np.exp(p[0] - m) for p in parts)", "l = sum(p[1] for p in parts)",
     ["test_oracle_attend.py"]),
    # storage rounding
    ("bf16", "q = int(np.rint(np.ldexp(m, 8)))   # in [128, 256]", "q = int(np.floor(np.ldexp(m, 8)))",
     ["test_oracle_bf16.py"]),
]


def _run(files, spec):
    env = dict(os.environ)
    if spec:
        env["SPIN_ORACLE_MUTATION"] = spec
    else:
        env.pop("SPIN_ORACLE_MUTATION", None)
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"] +
                          [os.path.join(HERE, f) for f in files], env=env, capture_output=True, text=True, timeout=600)


CASES = [m for m in MISTAKES if m[1] is not None]
_results = {}


def _result(case):
    """The child runs of all cases, started together on first use (a few at a time)."""
    if not _results:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=max(1, min(6, (os.cpu_count() or 2) - 1))) as pool:
            futures = {i: pool.submit(_run, files, json.dumps([module, old, new]))
                       for i, (module, old, new, files) in enumerate(CASES)}
            for i, f in futures.items():
                _results[i] = f.result()
    return _results[case]


@pytest.mark.parametrize("case", range(len(CASES)))
def test_a_planted_mistake_fails_the_pins(case):
    module, old, new, files = CASES[case]
    r = _result(case)
    # 1 = tests failed (what is wanted); anything else (0 = the pins did not notice, 2+ = the mistake did not apply)
    assert r.returncode == 1, f"oracle/{module}.py with {old!r} -> {new!r}: exit {r.returncode}\n{r.stdout[-1500:]}\n{r.stderr[-500:]}"
    assert "planted mistake does not apply" not in r.stdout + r.stderr


def test_pins_are_green_without_a_planted_mistake():
    files = sorted({f for _, old, _, fs in MISTAKES if old is not None for f in fs})
    r = _run(files, None)
    assert r.returncode == 0, r.stdout[-2000:]
