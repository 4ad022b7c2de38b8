#!/usr/bin/env python3
"""Benchmark of the knowledge-base retrieval hot path on one MI355X.

A step is one kb_query over one batch of synthetic queries (query norms, sampling pass, threshold,
scan with fused scale / tag filter / threshold filter, bucket, final top-k) with the knowledge base and
the queries already resident in HBM.  The default workload is the filtered knowledge base the metric is
quoted on: N = 2^20 keys, d = 1024, bf16, 256 masked queries, k = 32.

Prints ONE JSON line.  `roofline` describes the scan kernel: achieved = algorithmic bytes per launch /
average launch duration (HIP events recorded around the scan launch on its own stream, inside the timed
region).  `cpu_baseline` is the fp64 oracle timed on the host cores on a bounded sample of the same
batch; the same sample is used to check the GPU result, and no throughput is printed if that check fails.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "fp8": 5000.0}     # MI355X dense matrix peaks
DRAW_TEMPERATURE = 0.05
# Vector-ALU roof for the weighted random selection: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-instructions per second.
VALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
# Lane-instructions per (query, entry) pair of the key computation: a quarter of a 10-round Philox4x32 call (20), the
# uniform variate (3), two logarithms with their scalings and negations (6), score scaling (3), key (2), test (2).
DRAW_OPS_PER_PAIR = 36
# HBM bytes per launch of the main-pass scan kernel, from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE (KiB per dispatch),
# each scaled by what the same counter reads for a copy of known size.  A record applies to one workload, the default
# kernel choice and the kernel sources it was taken on: `sources` is scan_sources_digest() at that time, and the
# figure is reported as null once any of those files has changed.
SCAN_TRAFFIC = {
    "filtered": {"fetch_kib": 1087874, "fetch_scale": 2.0, "write_kib": 9422, "write_scale": 1.0, "sources": "547dc9f240a12fd4"},
}
SCAN_SOURCES = ["kb_scan_wide.hpp", "kb_scan.hpp", "kb_scan_sp.hpp", "kb_epilogue.hpp", "kb_internal.hpp", "kb_configs.hpp"]


def scan_sources_digest() -> str:
    import hashlib

    h = hashlib.sha256()
    for name in SCAN_SOURCES:
        with open(os.path.join(ROOT, "paper_2602_14293_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


SCAN_TIMING_STRIDE = 4


def scan_timing_stride(steps: int) -> int:
    return SCAN_TIMING_STRIDE if steps >= 4 * SCAN_TIMING_STRIDE else 1


def scan_traffic_bytes(workload: str, tuned: bool):
    rec = SCAN_TRAFFIC.get(workload)
    if rec is None or tuned or rec["sources"] != scan_sources_digest():
        return None
    return rec["fetch_kib"] * 1024 * rec["fetch_scale"] + rec["write_kib"] * 1024 * rec["write_scale"]


def make_workload(name: str, seed: int, device):
    from paper_2602_14293_amd import workloads as W

    if name == "filtered":
        return W.filtered(seed=seed, device=device), "filtered KB: N=1048576 d=1024 bf16, Q=256 masked queries, k=32"
    if name == "filtered-q128":
        return (W.filtered(seed=seed, Q=128, k=16, device=device),
                "growing-KB query shape: N=1048576 d=1024 bf16, Q=128 masked queries, k=16")
    if name == "clustered":
        return W.clustered(seed=seed, device=device), "clustered KB: N=65536 d=768 bf16, Q=64, k=16"
    if name == "tiny":
        return W.tiny(seed=seed, device=device), "tiny KB: N=4096 d=256 fp32, Q=8, k=8"
    if name == "compressed":
        return (W.compressed(seed=seed, device=device),
                "compressed KB: N=4194304 d=768 fp8-e4m3 + row scale, Q=1024 bf16 queries, k=64")
    if name == "compressed-q8":
        return (W.compressed(seed=seed, device=device, fp8_queries=True),
                "compressed KB: N=4194304 d=768 fp8-e4m3 + row scale, Q=1024 fp8-e4m3 queries, k=64")
    raise SystemExit(f"unknown workload {name}")


def _median(xs):
    xs = sorted(xs)
    return xs[len(xs) // 2]


def run_quantize(args, torch, kbmod, W, dev):
    """kb_quantize_rows on 2^20 x 1024 bf16 rows (what building a compressed knowledge base of that size costs) and
    on a 1024 x 768 bf16 query batch.  Algorithmic traffic: the rows read once, one byte per element and one scale
    per row written."""
    gen = torch.Generator(device=dev)
    gen.manual_seed(args.seed)
    out = []
    for n, d in ((1 << 20, 1024), (1024, 768)):
        x = torch.randn(n, d, generator=gen, device=dev).to(torch.bfloat16)
        for _ in range(args.warmup):
            kbmod.quantize_rows(x)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        for e0, e1 in evs:
            e0.record()
            kbmod.quantize_rows(x)
            e1.record()
        torch.cuda.synchronize()
        ms = _median([e0.elapsed_time(e1) for e0, e1 in evs])
        nbytes = n * d * 3 + n * 4
        out.append({"rows": n, "d": d, "ms": ms, "GBps": nbytes / (ms * 1e-3) / 1e9, "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS})
        del x
    print(json.dumps({"metric": "kb_quantize_rows, bf16 rows to e4m3 codes + row scale", "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
                      "warmup": args.warmup, "dtype": "bf16 -> fp8_e4m3", "data": "synthetic", "shapes": out,
                      "roofline": {"bound": "hbm", "kernel": "quantize_rows_kernel", "achieved": out[0]["GBps"], "peak": HBM_PEAK_GBPS,
                                   "unit": "GB/s", "frac": out[0]["frac_of_hbm_peak"], "traffic": None}}))


def run_two_stage(args, torch, kbmod, W, dev):
    """Two-stage retrieval on a grouped knowledge base (2^20 rows in 1024 clusters, d = 1024 bf16): per batch size and
    nprobe, the latency of centroid ranking + kb_query_probe against the exhaustive kb_query, and the recall@k of the
    two-stage result against the exhaustive one; the first batch is also checked against the CPU oracle."""
    C, k = 1024, 32
    w, cent, off = W.grouped(seed=args.seed, C=C, mean_size=1024, d=1024, spread=0.03, Q=32, k=k, dtype=torch.bfloat16, device=dev)
    N = w.N
    kb = kbmod.KnowledgeBase(w.d, kbmod.KB_BF16, N)
    kb.keys[:N].copy_(w.keys)
    kb.append_in_place(N)
    kb.normalize()
    ckb = kbmod.KnowledgeBase(w.d, kbmod.KB_BF16, C)
    ckb.append(cent.contiguous())
    ckb.normalize()

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        for e0, e1 in evs:
            e0.record()
            out = fn()
            e1.record()
        torch.cuda.synchronize()
        return _median([e0.elapsed_time(e1) for e0, e1 in evs]), out

    def recall(found, exact):
        f, e = found.cpu().numpy(), exact.cpu().numpy()
        return float(sum(len(set(a[a >= 0]) & set(b[b >= 0])) / max(len(set(b[b >= 0])), 1) for a, b in zip(f, e)) / len(f))

    rows = []
    for Q in (1, 8, 32):
        q = w.queries[:Q].contiguous()
        t_full, (ei, es) = timed(lambda: kb.query(q, k))
        for nprobe in (1, 4, 16):
            def two():
                probe, _ = ckb.query(q, nprobe)
                return kb.query_probe(q, k, off, probe)
            t_two, (gi, gs) = timed(two)
            rows.append({"Q": Q, "nprobe": nprobe, "two_stage_ms": t_two, "exhaustive_ms": t_full, "speedup": t_full / t_two,
                         "recall_at_k": recall(gi, ei), "rows_scored_per_query": nprobe * N // C})
    result = {"metric": "two-stage retrieval latency and recall@32, N=1M d=1024 bf16, 1024 clusters", "unit": "ms", "n_gpus": 1,
              "steps": args.steps, "warmup": args.warmup, "dtype": "bf16", "data": "synthetic",
              "config": {"workload": f"grouped KB: N={N} d=1024 bf16 in 1024 clusters (spread 0.03 per coordinate), k=32", "seed": args.seed},
              "cases": rows}
    if not args.no_cpu_baseline:
        from oracle import compare, kb_oracle

        nq, nprobe = 8, 4
        q = w.queries[:nq].contiguous()
        probe, _ = ckb.query(q, nprobe)
        gi, gs = kb.query_probe(q, k, off, probe)
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        o_idx, o_sc, o_probe, full = kb_oracle.two_stage(W.key_bits(w.keys), kb_oracle.BF16, W.key_bits(cent), kb_oracle.BF16, off.cpu().numpy(),
                                                         W.key_bits(q), kb_oracle.BF16, nprobe, k)
        c1 = time.perf_counter()
        same = [r for r in range(nq) if set(probe[r].cpu().tolist()) == set(o_probe[r].tolist())]
        rep = compare.check(gi.cpu().numpy()[same], gs.cpu().numpy()[same], full[same], k, 2e-3, label="two-stage bench parity")
        exact_idx, _ = kb_oracle.query(W.key_bits(w.keys), kb_oracle.BF16, W.key_bits(q), kb_oracle.BF16, k)
        result["cpu_baseline"] = {"value": nq / (c1 - c0), "unit": "queries/s", "cores": kb_oracle.num_threads(), "kind": "oracle",
                                  "sample": f"{nq} queries, nprobe {nprobe}: centroid ranking + fp64 scores of all {N} keys restricted to the probed clusters, {c1 - c0:.1f} s"}
        result["parity"] = {"queries_checked": rep.queries, "same_probe_set": len(same), "max_score_err": rep.max_score_err,
                            "recall_at_k_vs_oracle_exact": kb_oracle.recall_at_k(gi.cpu().numpy(), exact_idx)}
    print(json.dumps(result))


def run_maintain(args, torch, kbmod, W, dev):
    """Maintenance of the filtered knowledge base (2^20 x 1024 bf16, tagged): revise 8192 gains, remove a random 10 %
    of the entries, query with the removed entries in place, compact into a second store, query the compacted store."""
    w, desc = make_workload("filtered", args.seed, dev)
    N, d, Q, k = w.N, w.d, w.Q, w.k
    gen = torch.Generator(device=dev)
    gen.manual_seed(args.seed + 5)

    def timed(fn, reps):
        for _ in range(2):
            fn()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for e0, e1 in evs:
            e0.record()
            fn()
            e1.record()
        torch.cuda.synchronize()
        return _median([e0.elapsed_time(e1) for e0, e1 in evs])

    src = kbmod.KnowledgeBase(d, kbmod.KB_BF16, N, tagged=True)
    src.keys.copy_(w.keys)
    src.tags.copy_(w.tags)
    src.append_in_place(N)
    src.normalize()
    out_i = torch.empty((Q, k), dtype=torch.int32, device=dev)
    out_s = torch.empty((Q, k), dtype=torch.float32, device=dev)
    q_before = timed(lambda: src.query(w.queries, k, w.qmask, out_i, out_s), args.steps)
    gain = torch.empty(N, dtype=torch.float32, device=dev).uniform_(0.25, 4.0, generator=gen)
    upd_i = torch.randperm(N, generator=gen, device=dev)[:8192].to(torch.int32)
    upd_v = torch.empty(8192, dtype=torch.float32, device=dev).uniform_(0.0, 8.0, generator=gen)
    t_update = timed(lambda: kbmod.update_gain(gain, upd_i, upd_v, 0.5), args.steps)
    rm = torch.randperm(N, generator=gen, device=dev)[:N // 10].to(torch.int32)
    t_remove = timed(lambda: src.remove(rm), args.steps)
    q_removed = timed(lambda: src.query(w.queries, k, w.qmask, out_i, out_s), args.steps)
    live = N - N // 10
    dsts = []

    def compact_once():
        dst = kbmod.KnowledgeBase(d, kbmod.KB_BF16, live, tagged=True)
        dsts.append(dst)
        while len(dsts) > 1:
            dsts.pop(0).close()
        got, _, _ = src.compact_into(dst, gain=gain)
        assert got == live

    t_compact = timed(compact_once, 5)       # includes the allocation of the destination and the one synchronisation
    dst = dsts[-1]
    q_compacted = timed(lambda: dst.query(w.queries, k, w.qmask, out_i, out_s), args.steps)
    nbytes = live * (2 * d * 2 + 2 * (4 + 8 + 4)) + N * (4 + 4 + 4)
    print(json.dumps({"metric": "knowledge-base maintenance, N=1M d=1024 bf16", "unit": "ms", "n_gpus": 1, "steps": args.steps,
                      "dtype": "bf16", "data": "synthetic", "config": {"workload": desc + "; 8192 gains revised, 10 % removed, compacted"},
                      "update_gain_ms": t_update, "remove_ms": t_remove, "compact_ms": t_compact,
                      "query_ms": {"before": q_before, "with_removed_entries": q_removed, "compacted": q_compacted},
                      "roofline": {"bound": "hbm", "kernel": "kb_compact (count + offset scan + gather, with the host synchronisation)",
                                   "achieved": nbytes / (t_compact * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                   "frac": nbytes / (t_compact * 1e-3) / 1e9 / HBM_PEAK_GBPS, "traffic": None, "algorithmic_bytes": nbytes}}))


def run_growing(args, torch, kbmod, W, dev):
    """The growing knowledge base: 2^20 rows, then 64 rounds of (append 16384 rows, normalize, 128 masked
    queries, k = 16).  A step is one round; append + normalize and the query are timed separately."""
    N0, n_new, rounds, d, Q, k = 1 << 20, 16384, 64, 1024, 128, 16
    keys0, tags0, centers = W.growing_base(seed=args.seed, device=dev)
    kb = kbmod.KnowledgeBase(d, kbmod.KB_BF16, N0 + rounds * n_new, tagged=True)
    kb.keys[:N0].copy_(keys0)
    kb.tags[:N0].copy_(tags0)
    del keys0, tags0
    kb.append_in_place(N0)
    kb.normalize()
    for t in args.tune:
        name, val = t.split("=")
        kb.set_tuning(name, int(val))
    out_i = torch.empty((Q, k), dtype=torch.int32, device=dev)
    out_s = torch.empty((Q, k), dtype=torch.float32, device=dev)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    t_append, t_query = [], []
    for r in range(rounds):
        rows, tags, queries, qmask = W.growing_round(args.seed, r, n_new, d, Q, centers, device=dev)
        if r == 0:      # untimed warm-up of the query path on the initial knowledge base
            for _ in range(args.warmup):
                kb.query(queries, k, qmask, out_i, out_s)
            kb.set_tuning("profile_stride", scan_timing_stride(rounds))
            kb.profile_begin(rounds)
        torch.cuda.synchronize()
        ev[0].record()
        kb.append(rows, tags=tags)
        kb.normalize()
        ev[1].record()
        kb.query(queries, k, qmask, out_i, out_s)
        ev[2].record()
        torch.cuda.synchronize()
        t_append.append(ev[0].elapsed_time(ev[1]))
        t_query.append(ev[1].elapsed_time(ev[2]))
    scan_ms_total, scan_calls = kb.profile_end()
    n_first, n_last = N0 + n_new, N0 + rounds * n_new
    row_bytes = d * 2
    q_first, q_last = _median(t_query[:8]), _median(t_query[-8:])
    # algorithmic bytes of a round's scan: the rows as of that round (+ norm and tag) and the query block
    alg = [(N0 + (r + 1) * n_new) * (row_bytes + 12) + Q * row_bytes for r in range(rounds)]
    call_frac = [alg[r] / (t_query[r] * 1e-3) / 1e9 / HBM_PEAK_GBPS for r in range(rounds)]
    timed_rounds = list(range(scan_timing_stride(rounds) // 2, rounds, scan_timing_stride(rounds)))      # the rounds whose scan kernel carried an event pair
    scan_achieved = sum(alg[r] for r in timed_rounds) / (scan_ms_total * 1e-3) / 1e9 if scan_calls == len(timed_rounds) else None
    result = {
        "metric": "KB top-k queries/sec + key-scan HBM GB/s (% of peak), N=1M d=1024 bf16",
        "value": Q * rounds / (sum(t_query) * 1e-3), "unit": "queries/s", "n_gpus": 1, "steps": rounds, "warmup": args.warmup,
        "ms_per_step": (sum(t_query) + sum(t_append)) / rounds, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "growing KB: 1048576 -> 2097152 rows in 64 rounds of +16384, d=1024 bf16, Q=128 masked queries, k=16",
                   "seed": args.seed},
        "append_normalize_ms": {"median": _median(t_append), "min": min(t_append), "max": max(t_append),
                                "GBps_median": n_new * row_bytes / (_median(t_append) * 1e-3) / 1e9},
        "query_ms": {"first_8_rounds_median": q_first, "last_8_rounds_median": q_last, "min": min(t_query), "max": max(t_query),
                     "per_round": [round(t, 4) for t in t_query]},
        "key_scan_GBps": {"first_8_rounds": n_first * row_bytes / (q_first * 1e-3) / 1e9,
                          "last_8_rounds": n_last * row_bytes / (q_last * 1e-3) / 1e9},
        "call_frac_of_hbm_peak": {"min": min(call_frac), "median": _median(call_frac), "max": max(call_frac)},
        "queries_per_s": {"first_8_rounds": Q / (q_first * 1e-3), "last_8_rounds": Q / (q_last * 1e-3)},
        "counters_last_round": kb.counters(),
        "roofline": {"bound": "hbm", "kernel": "scan kernel, main pass (all rounds)", "achieved": scan_achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": None if scan_achieved is None else scan_achieved / HBM_PEAK_GBPS, "traffic": None,
                     "kernel_ms": scan_ms_total / max(scan_calls, 1), "algorithmic_bytes": sum(alg[r] for r in timed_rounds) / len(timed_rounds),
                     "launches_timed": scan_calls, "timing_stride": scan_timing_stride(rounds)},
    }
    if not args.no_cpu_baseline:
        n = kb.size
        w = W.Workload("growing", kb.keys[:n], queries, k, tags=kb.tags[:n], qmask=qmask)
        result["cpu_baseline"], result["parity"] = parity_and_baseline(args, torch, kbmod, W, w, kbmod.KB_BF16, k, out_i.cpu().numpy(),
                                                                       out_s.cpu().numpy(), None, min(args.oracle_queries, 64))
        result["cpu_baseline"]["sample"] += " (the last round)"
    kb.close()
    return result


def run_q_sweep(args, torch, kbmod, W, dev):
    """Query-batch sweep on the N = 2^20, d = 1024 bf16 knowledge base (masked, k = 32): where the path goes from
    streaming-bound to matrix-core-bound."""
    w = W.filtered(seed=args.seed, Q=512, device=dev)
    kb = kbmod.KnowledgeBase(w.d, kbmod.KB_BF16, w.N, tagged=True)
    kb.keys.copy_(w.keys)
    kb.tags.copy_(w.tags)
    kb.append_in_place(w.N)
    kb.normalize()
    key_bytes = w.N * w.d * 2
    rows = []
    for Q in (1, 8, 32, 64, 128, 256, 512):
        queries, qmask = w.queries[:Q].contiguous(), w.qmask[:Q].contiguous()
        out_i = torch.empty((Q, w.k), dtype=torch.int32, device=dev)
        out_s = torch.empty((Q, w.k), dtype=torch.float32, device=dev)
        for _ in range(args.warmup):
            kb.query(queries, w.k, qmask, out_i, out_s)
        torch.cuda.synchronize()
        kb.profile_begin(args.steps)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            kb.query(queries, w.k, qmask, out_i, out_s)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        scan_ms, n = kb.profile_end()
        scan_ms /= max(n, 1)
        rows.append({"Q": Q, "ms_per_query_batch": ms, "queries_per_s": Q / (ms * 1e-3), "scan_kernel_ms": scan_ms,
                     "scan_key_GBps": key_bytes / (scan_ms * 1e-3) / 1e9, "scan_TFLOPs": 2.0 * Q * w.N * w.d / (scan_ms * 1e-3) / 1e12})
    print(json.dumps({"metric": "query-batch sweep, N=1048576 d=1024 bf16 masked k=32", "steps": args.steps, "warmup": args.warmup,
                      "n_gpus": 1, "data": "synthetic", "sweep": rows}))


TIGHT_TAU = 1e-5            # the error the kernels reach on the same stored bits; fp8 queries: 1e-4; keys of a draw: 2e-5
ALL_WORKLOADS = ["tiny", "clustered", "filtered", "compressed", "compressed-q8", "filtered-q128", "growing"]


def parity_and_baseline(args, torch, kbmod, W, w, code, k, gi, gs, gain, nq):
    """The oracle, as it stands, on the first nq queries of the batch against all keys: timed (cpu_baseline), and
    the GPU result judged by the acceptance rule at the dtype tolerance and at the tight one.  Raises on a mismatch."""
    from oracle import compare, kb_oracle

    N, Q = w.N, w.Q
    masked = w.qmask is not None
    key_bits = W.key_bits(w.keys)
    q_bits = W.key_bits(w.queries[:nq])
    tags = W.word_bits(w.tags) if masked else None
    qm = W.word_bits(w.qmask[:nq]) if masked else None
    okind = {kbmod.KB_F32: kb_oracle.F32, kbmod.KB_BF16: kb_oracle.BF16, kbmod.KB_FP8_E4M3: kb_oracle.FP8_E4M3}[code]
    qkind = {torch.float32: kb_oracle.F32, torch.bfloat16: kb_oracle.BF16, torch.float8_e4m3fn: kb_oracle.FP8_E4M3}[w.queries.dtype]
    c0 = time.perf_counter()
    oi, osc, full = kb_oracle.query(key_bits, okind, q_bits, qkind, k,
                                    row_scale=None if w.scale is None else w.scale.cpu().numpy(), tags=tags, qmask=qm,
                                    return_scores=True)
    if gain is not None:       # keys of the same draw from the fp64 scores; selection is part of the timed work
        full = kb_oracle.selection_keys(full, gain.cpu().numpy(), DRAW_TEMPERATURE, args.seed, 0)
        for r in range(nq):
            kb_oracle.select(full[r], k, tags=tags, qmask=None if qm is None else qm[r])
    c1 = time.perf_counter()
    tau = 2e-4 if gain is not None else {kbmod.KB_F32: 1e-5, kbmod.KB_BF16: 2e-3, kbmod.KB_FP8_E4M3: 2e-2}[code]
    tight_tau = 2e-5 if gain is not None else 1e-4 if w.queries.dtype == torch.float8_e4m3fn else TIGHT_TAU
    rep, tight = compare.check(gi[:nq], gs[:nq], full, k, tau, tags=tags, qmask=qm, label="bench parity", tight_tau=tight_tau)
    baseline = {"value": nq / (c1 - c0), "unit": "queries/s", "cores": kb_oracle.num_threads(), "kind": "oracle",
                "sample": f"first {nq} of the {Q} queries against all {N} keys (fp64 brute force + full sort), {c1 - c0:.1f} s"}
    parity = {"queries_checked": rep.queries, "tau": tau, "strict": rep.strict, "near_tie": rep.near_tie,
              "tight_tau": tight_tau, "tight_strict": tight.strict, "tight_near_tie": tight.near_tie,
              "max_score_err": rep.max_score_err}
    return baseline, parity


def run_query_workload(args, torch, kbmod, W, dev, name):
    w, desc = make_workload(name, args.seed, dev)
    code = {torch.float32: kbmod.KB_F32, torch.bfloat16: kbmod.KB_BF16, torch.float8_e4m3fn: kbmod.KB_FP8_E4M3}[w.keys.dtype]
    kb = kbmod.KnowledgeBase(w.d, code, w.N, tagged=w.tags is not None)
    kb.keys.copy_(w.keys)
    if w.scale is not None:
        kb.scale.copy_(w.scale)
    if w.tags is not None:
        kb.tags.copy_(w.tags)
    kb.append_in_place(w.N)
    kb.normalize()
    for t in args.tune:
        tname, val = t.split("=")
        kb.set_tuning(tname, int(val))
    queries = w.queries.contiguous()
    qmask = w.qmask
    Q, k, N, d = w.Q, w.k, w.N, w.d
    out_i = torch.empty((Q, k), dtype=torch.int32, device=dev)
    out_s = torch.empty((Q, k), dtype=torch.float32, device=dev)
    gain = None
    if args.draw:
        gen = torch.Generator(device=dev)
        gen.manual_seed(args.seed + 17)
        gain = torch.empty(N, dtype=torch.float32, device=dev).uniform_(0.25, 4.0, generator=gen)

        def draw_step(queries, k, qmask, out_i, out_s):
            return kb.query_sampled(queries, k, gain, DRAW_TEMPERATURE, args.seed, qmask, 0, out_i, out_s)

        kb.query = draw_step      # every call below times the draw
        desc += f"; weighted random selection, temperature {DRAW_TEMPERATURE}"

    for _ in range(args.warmup):
        kb.query(queries, k, qmask, out_i, out_s)
    torch.cuda.synchronize()
    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    if args.graph:
        graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
        with torch.cuda.graph(graph, stream=side):
            kb.query(queries, k, qmask, out_i, out_s)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        # one eager, timed launch afterwards gives the scan kernel's duration for the roofline entry
        kb.profile_begin(1)
        kb.query(queries, k, qmask, out_i, out_s)
        torch.cuda.synchronize()
        scan_ms_total, scan_calls = kb.profile_end()
    else:
        # The scan kernel of every SCAN_TIMING_STRIDE-th timed step carries an event pair (all of them in a short
        # run): a timed launch costs the stream about 12 us of idle time around it, which belongs to the
        # measurement, not to the call.
        stride = scan_timing_stride(args.steps)
        kb.set_tuning("profile_stride", stride)
        kb.profile_begin((args.steps + stride - 1) // stride)      # (launch stride / 2 of every run of `stride` launches is the timed one)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            kb.query(queries, k, qmask, out_i, out_s)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        scan_ms_total, scan_calls = kb.profile_end()
        kb.set_tuning("profile_stride", 1)
    counters = kb.counters()
    # a second, untimed-for-the-headline pass with one event pair per call: spread of the per-call latency
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(min(args.steps, 50))]
    for e0, e1 in evs:
        e0.record()
        kb.query(queries, k, qmask, out_i, out_s)
        e1.record()
    torch.cuda.synchronize()
    per_call = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    flushed = None
    if args.flushed:
        # the same call after 1 GiB of unrelated writes has gone through the caches (keys and queries come from HBM)
        junk = torch.empty(1 << 28, dtype=torch.float32, device=dev)
        cold = []
        for _ in range(min(args.steps, 10)):
            junk.fill_(1.0)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            kb.query(queries, k, qmask, out_i, out_s)
            e1.record()
            torch.cuda.synchronize()
            cold.append(e0.elapsed_time(e1))
        del junk
        cold.sort()
        flushed = {"median": cold[len(cold) // 2], "min": cold[0], "max": cold[-1], "calls": len(cold)}

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    qps = Q / (ms_per_step * 1e-3)
    key_bytes = N * d * w.keys.element_size()
    # algorithmic bytes of one scan launch: every key row once (+ its fp32 norm, + its 64-bit tag when a
    # mask is given) and the query block once
    scan_bytes = N * (d * w.keys.element_size() + 4 + (8 if qmask is not None else 0)) + Q * d * queries.element_size()
    scan_ms = scan_ms_total / max(scan_calls, 1)
    achieved = scan_bytes / (scan_ms * 1e-3) / 1e9
    flops = 2.0 * Q * N * d
    small_path = counters["sample_keys"] == 0 and counters["candidates"] == 0 and N <= 16384
    result = {
        "metric": "KB top-k queries/sec + key-scan HBM GB/s (% of peak), N=1M d=1024 bf16",
        "value": qps,
        "unit": "queries/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_call_events": {"median": per_call[len(per_call) // 2], "min": per_call[0], "max": per_call[-1], "calls": len(per_call)},
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {kbmod.KB_F32: "f32", kbmod.KB_BF16: "bf16", kbmod.KB_FP8_E4M3: "fp8_e4m3"}[code],
        "data": "synthetic",
        "config": {"workload": desc, "seed": args.seed, "checksum": W.checksum(w.keys[:4096], w.queries)},
        "key_scan_GBps": key_bytes / (ms_per_step * 1e-3) / 1e9,
        "key_scan_frac_of_hbm_peak": key_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "call_frac_of_hbm_peak": scan_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "mfma_TFLOPs": flops / (ms_per_step * 1e-3) / 1e12,
        "counters": counters,
        "launch": "hip graph replay" if args.graph else "eager",
        "roofline": {"bound": "hbm", "kernel": "scoring kernel of the small-knowledge-base path" if small_path else "scan kernel, main pass",
                     "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": scan_traffic_bytes(name, bool(args.tune) or args.draw),
                     "kernel_ms": scan_ms, "algorithmic_bytes": scan_bytes, "launches_timed": scan_calls,
                     "timing_stride": 1 if args.graph else scan_timing_stride(args.steps)},
    }
    if flushed is not None:
        result["ms_per_call_flushed"] = flushed

    # Above the ridge (large Q) the matrix cores, not HBM, bound the scan: report against the dense MFMA peak of the
    # type the contraction runs in (fp8 keys with bf16 queries are widened to bf16; fp8 with fp8 queries run in fp8).
    mfma_peak = None if code == kbmod.KB_F32 else MFMA_PEAK_TFLOPS["fp8" if queries.dtype == torch.float8_e4m3fn else "bf16"]
    if mfma_peak is not None and flops / (mfma_peak * 1e12) > scan_bytes / (HBM_PEAK_GBPS * 1e9):
        result["roofline"] = {"bound": "mfma", "kernel": "scan kernel, main pass", "achieved": flops / (scan_ms * 1e-3) / 1e12,
                              "peak": mfma_peak, "unit": "TFLOP/s", "frac": flops / (scan_ms * 1e-3) / 1e12 / mfma_peak,
                              "traffic": None, "kernel_ms": scan_ms, "algorithmic_flops": flops, "launches_timed": scan_calls}

    if args.draw:
        ops = float(DRAW_OPS_PER_PAIR) * Q * N
        result["roofline"] = {"bound": "alu", "kernel": "scan kernel, main pass, keys of the weighted random selection",
                              "achieved": ops / (scan_ms * 1e-3) / 1e12, "peak": VALU_PEAK_TOPS, "unit": "Tops/s",
                              "frac": ops / (scan_ms * 1e-3) / 1e12 / VALU_PEAK_TOPS, "traffic": None, "kernel_ms": scan_ms,
                              "algorithmic_ops": ops, "launches_timed": scan_calls}

    if not args.no_cpu_baseline:
        # a bounded sample: the whole batch up to 256 queries of 2^20 keys, 64 queries of the 2^22-key store
        nq = min(args.oracle_queries, Q, max(8, int(256 * (1 << 20) / max(N, 1))))
        result["cpu_baseline"], result["parity"] = parity_and_baseline(args, torch, kbmod, W, w, code, k, out_i.cpu().numpy(),
                                                                       out_s.cpu().numpy(), gain, nq)
    kb.close()
    return result


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="filtered",
                    help="tiny | clustered | filtered (default, the workload the metric is quoted on) | compressed | compressed-q8 | "
                         "filtered-q128 | growing | all (one JSON line per workload, in that order)")
    ap.add_argument("--seed", type=int, default=2000)
    ap.add_argument("--oracle-queries", type=int, default=256, help="queries of the batch given to the CPU oracle")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 1 GiB device-to-device elementwise copy (a dispatch of known traffic that "
                         "calibrates rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--tune", action="append", default=[], help="name=value performance knob (repeatable)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one kb_query in a HIP graph and time replays (for the launch-latency-bound workloads; "
                         "the scan kernel is then not timed on its own)")
    ap.add_argument("--flushed", action="store_true",
                    help="also time calls that follow 1 GiB of unrelated writes (caches flushed: the small workloads from HBM)")
    ap.add_argument("--draw", action="store_true",
                    help="time the weighted random selection (kb_query_sampled: gains uniform in [0.25, 4], temperature "
                         "0.05) instead of the plain top-k")
    ap.add_argument("--two-stage", action="store_true", help="time centroid ranking + kb_query_probe against the exhaustive query and report recall@k instead")
    ap.add_argument("--maintain", action="store_true", help="time kb_update_gain / kb_remove / kb_compact and queries around them instead")
    ap.add_argument("--quantize", action="store_true", help="time kb_quantize_rows instead")
    ap.add_argument("--q-sweep", action="store_true", help="time query batches of 1..512 on the N=2^20 bf16 knowledge base instead")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py measures one GPU: the retrieval path is built and measured on a single MI355X "
                         "(--gpus must be 1).")

    import torch

    from paper_2602_14293_amd import kb as kbmod
    from paper_2602_14293_amd import workloads as W

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    kbmod.lib()     # raises if libkb.so has not been built: there is no fallback path
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.q_sweep:
        return run_q_sweep(args, torch, kbmod, W, dev)
    if args.quantize:
        return run_quantize(args, torch, kbmod, W, dev)
    if args.maintain:
        return run_maintain(args, torch, kbmod, W, dev)
    if args.two_stage:
        return run_two_stage(args, torch, kbmod, W, dev)
    for name in (ALL_WORKLOADS if args.workload == "all" else [args.workload]):
        if args.workload == "all":
            args.flushed = name in ("tiny", "clustered")        # the two that fit in the caches
        result = run_growing(args, torch, kbmod, W, dev) if name == "growing" else run_query_workload(args, torch, kbmod, W, dev, name)
        print(json.dumps(result), flush=True)
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
