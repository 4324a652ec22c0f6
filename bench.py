#!/usr/bin/env python3
"""Benchmark of span-restricted decode attention on one MI355X.

A "step" is one span_decode_attn call (all of: locate work, q.K scores, online softmax, p.V, merge)
over one batch of synthetic input that is already resident in HBM.  The headline workload is the
arithmetic-evaluation-shaped one (config 3: batch 64, 32 heads x 128, 512 cached tokens, ~30 % of them
in the span, fp16).  Steps rotate over several independent (K, V, span) copies so that the bytes touched
between two uses of a buffer exceed the on-package cache: the figure is HBM bandwidth, not cache bandwidth.

Prints ONE JSON line:
  value    = span bytes (K and V rows inside the intervals) * steps / wall time of the timed region  [GB/s];
             the timed region of exactly `steps` calls (synchronize on both sides, nothing else inside) is run
             `rounds` times and the median round is reported
  roofline = same bytes / average call duration from HIP events on the launch stream, against 8 TB/s
  workloads, coverage_sweep, instances, few_query, unstructured_masks = the other configurations, each with its
             dense control, timed in the same run (compact rows)
  cpu_baseline = the fp64 CPU oracle on the same workload, timed on the host cores

Other modes: --microbench (the paper's kernel micro-benchmark), --phase-trace (where the time of one call goes,
needs the `trace` build), --pmc-summary (turns rocprofv3 counter CSVs into the HBM-traffic figure).
"""
import argparse
import dataclasses
import json
import os
import statistics
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0           # MI355X HBM3E, published peak
LLC_BYTES = 256 * 1024 * 1024    # on-package last-level cache to defeat by rotation
EVENT_LEAD_IN = 8                # untimed calls in front of the start event of an event-timed round
PAPER_CONTEXT = {"gain": "up to 28% more tokens/s end to end (27.7% at 1536-1792 output tokens)",
                 "hardware": "1x NVIDIA A100 80GB, LLaMA-7B, batch 48", "source": "paper abstract and Sec. 4.1"}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--rounds", type=int, default=7,
                    help="the timed region of exactly --steps calls is repeated this many times; the median round "
                         "is reported (all rounds are listed)")
    ap.add_argument("--config", type=int, default=3, help="workload id 1..5 (headline: 3)")
    ap.add_argument("--copies", type=int, default=0, help="independent KV copies to rotate over (0 = auto)")
    ap.add_argument("--coverage", type=float, default=None, help="config 5 only: uniform span coverage")
    ap.add_argument("--num-splits", type=int, default=0)
    ap.add_argument("--q-len", type=int, default=1,
                    help="with --only span or --phase-trace: time / trace the few-query call with this many new tokens "
                         "per sequence instead of the decode step (diagnostic; the bytes counted stay the span's K / V)")
    ap.add_argument("--uniform-grid", action="store_true",
                    help="do not pass per-sequence token counts (every sequence gets the same number of slices)")
    ap.add_argument("--no-host-lists", action="store_true",
                    help="do not hand the host copies of the span lists to the call (the kernel then walks the device "
                         "lists itself)")
    ap.add_argument("--only", choices=["all", "span", "dense"], default="all",
                    help="'span' / 'dense' run just that timed loop of the headline config (for profiling one kernel)")
    ap.add_argument("--no-others", action="store_true", help="skip the rows for the other configurations")
    ap.add_argument("--microbench", action="store_true",
                    help="instead of the headline run: the paper's kernel micro-benchmark (Sec. 5.2), speedup of "
                         "50 %-sparse masks over dense for sparsity block sizes 32..256 and 1024..8096 cached tokens")
    ap.add_argument("--phase-trace", action="store_true",
                    help="instead of the headline run: per-workgroup phase times of one call of --config "
                         "(needs --variant trace)")
    ap.add_argument("--variant", default="", help="load libspanattn_<variant>.so, a measurement build of the library")
    ap.add_argument("--pmc-summary", nargs="+", metavar="DIR",
                    help="no GPU work: read rocprofv3 --pmc output directories (FETCH_SIZE / WRITE_SIZE runs made with "
                         "--calibrate-copy) and print HBM bytes per decode call")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch a plain 1 GiB-in / 1 GiB-out elementwise kernel (reference for HBM traffic counters)")
    return ap.parse_args()


def validated_tokens(sp):
    import paper_2404_09336_amd as span
    code, _, _, tok = span.span_validate(sp.offsets, sp.starts, sp.ends, sp.ctx_lens)
    assert code == 0, code
    return tok


class Workload:
    """`copies` independent instances of one config: tensors on the GPU plus prepared calls.  `kv` hands in the
    (q, K, V) tensors of an earlier workload of the same shape and seeds (the spans are drawn anew)."""

    def __init__(self, cfg, copies, device, coverage=None, num_splits=0, exact=True, kv=None, spans=None,
                 host_lists=True, q_len=1):
        import numpy as np
        import torch
        import paper_2404_09336_amd as span
        from workloads import draw_qkv, draw_spans
        self.cfg = cfg
        self.span_calls, self.dense_calls, self.kv = [], [], []
        self.span_bytes, self.dense_bytes, self.coverages = [], [], []
        self.host = []
        row_pair = 2 * cfg.head_dim * cfg.elt_bytes * cfg.heads     # K and V bytes per position, all heads
        for c in range(copies):
            sp = spans[c] if spans else draw_spans(cfg, seed=cfg.seed(c), coverage=coverage)
            tok = validated_tokens(sp)
            q, K, V = kv[c] if kv else draw_qkv(cfg, sp.ctx_lens, seed=cfg.seed(c), device=device)
            self.kv.append((q, K, V))
            dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(device)
            off, st, en, ctx = dev(sp.offsets), dev(sp.starts), dev(sp.ends), dev(sp.ctx_lens)
            self.span_calls.append(span.prepare_span_decode_attn(q, K, V, off, st, en, ctx, np.float32(cfg.scale),
                                                                 max_tokens=int(tok.max()), num_splits=num_splits,
                                                                 tokens_per_seq=tok if exact else None,
                                                                 host_spans=(sp.offsets, sp.starts, sp.ends)
                                                                 if exact and host_lists else None))
            self.dense_calls.append(span.prepare_dense_decode_attn(
                q, K, V, ctx, np.float32(cfg.scale), max_tokens=int(sp.ctx_lens.max()),
                tokens_per_seq=sp.ctx_lens.astype(np.int64) if exact else None))
            self.span_bytes.append(int(tok.sum()) * row_pair)
            self.dense_bytes.append(int(sp.ctx_lens.astype(np.int64).sum()) * row_pair)
            self.coverages.append(sp.coverage())
            if c == 0:
                self.host.append((sp, q, K, V))
        self.one_query_calls, self.q_len = self.span_calls, q_len
        if q_len > 1:          # diagnostic runs of the few-query call: it takes the place of the span call
            self.span_calls = few_query_calls(self, q_len, device)
        self.plan = span.span_plan_query(self.span_calls[0].desc)
        self.coverage = sum(self.coverages) / len(self.coverages)


def auto_copies(cfg, touched=None):
    """Enough copies that the span bytes touched in one rotation are >= 2x the last-level cache."""
    import numpy as np
    from workloads import draw_spans
    if touched is None:
        sp = draw_spans(cfg)
        touched = int(sp.tokens_per_seq().sum()) * 2 * cfg.head_dim * cfg.elt_bytes * cfg.heads
    alloc = 2 * cfg.batch * cfg.heads * cfg.max_len * cfg.head_dim * cfg.elt_bytes
    n = int(np.ceil(2 * LLC_BYTES / max(touched, 1)))
    n = max(2, n)                                   # always alternate buffers, even when one call exceeds the cache
    n = max(1, min(n, 16, max(1, (48 << 30) // alloc)))
    return n


def timed_loop(calls, nbytes, steps, warmup, rounds=1):
    """Warm up, then time exactly `steps` calls, `rounds` times over, two ways: by the wall clock, bracketed by
    synchronize() on both sides with nothing but the calls in between; and, in a round of its own, by HIP events
    recorded on the launch stream (the events would add their own cost to the wall-clock region).  The event round
    is led in by a few untimed calls, so that the first timed call is already queued when the GPU reaches the start
    event: the events then bracket exactly `steps` launches running back to back (the kernel's average launch
    duration plus the gap between two launches), with no host launch latency inside.  Every round starts at the
    same rotated copy, so all rounds move the same bytes.  Returns the median round of each kind and the
    per-round times."""
    import torch
    n = len(calls)
    for i in range(warmup):
        calls[i % n]()
    total_bytes = sum(nbytes[i % n] for i in range(steps))
    walls, evs = [], []
    for _ in range(max(1, rounds)):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            calls[i % n]()
        torch.cuda.synchronize()
        walls.append(time.perf_counter() - t0)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for i in range(EVENT_LEAD_IN):          # untimed: the GPU is busy while the timed calls are being enqueued
            calls[(i - EVENT_LEAD_IN) % n]()
        ev0.record()
        for i in range(steps):
            calls[i % n]()
        ev1.record()
        torch.cuda.synchronize()
        evs.append(ev0.elapsed_time(ev1) * 1e-3)
    wall, ev_s = statistics.median(walls), statistics.median(evs)
    return {"wall_s": wall, "event_s": ev_s, "bytes_per_call": total_bytes / steps,
            "us_per_call_wall": wall / steps * 1e6, "us_per_call_event": ev_s / steps * 1e6,
            "gbps_wall": total_bytes / wall / 1e9, "gbps_event": total_bytes / ev_s / 1e9,
            "rounds_us_per_call_wall": [round(w / steps * 1e6, 3) for w in walls],
            "rounds_us_per_call_event": [round(e / steps * 1e6, 3) for e in evs]}


def prewarm(calls, seconds=0.3):
    """Untimed: keeps the GPU busy long enough for its clocks to settle before anything is measured."""
    import torch
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for i in range(64):
            calls[i % len(calls)]()
        torch.cuda.synchronize()


def compact_row(wl, steps, dense_steps=None, rounds=3):
    """One line of the side tables: span and dense control timed with HIP events (median of `rounds`)."""
    s = timed_loop(wl.span_calls, wl.span_bytes, steps, max(5, steps // 10), rounds)
    d = timed_loop(wl.dense_calls, wl.dense_bytes, dense_steps or max(10, steps // 4), 5, rounds)
    return {"name": wl.cfg.name, "coverage": round(wl.coverage, 4),
            "span_mb": round(s["bytes_per_call"] / 1e6, 1), "span_us": round(s["us_per_call_event"], 2),
            "span_gbps": round(s["gbps_event"], 1), "span_pct_peak": round(100 * s["gbps_event"] / HBM_PEAK_GBPS, 2),
            "dense_us": round(d["us_per_call_event"], 2), "dense_gbps": round(d["gbps_event"], 1),
            "speedup_vs_dense": round(d["us_per_call_event"] / s["us_per_call_event"], 3),
            "slices_per_pair": wl.plan["max_splits"], "workgroups": wl.plan["workgroups"]}


def few_query_calls(wl, q_len, device):
    """Prepared few-query calls on the workload's tensors: the new tokens are the last q_len cache rows."""
    import numpy as np
    import torch
    import paper_2404_09336_amd as span
    from workloads import draw_queries
    calls = []
    for c, one in enumerate(wl.one_query_calls):
        _, K, V, off, st, en, ctx, _ = one._keepalive
        q = draw_queries(wl.cfg, q_len, seed=wl.cfg.seed(c), device=device)
        q_pos = (ctx - q_len).to(torch.int32)
        calls.append(span.prepare_span_decode_attn_multi(q, K, V, off, st, en, q_pos, np.float32(wl.cfg.scale),
                                                         max_tokens=one.desc.max_tokens,
                                                         tokens_per_seq=getattr(one.desc, "_tokens_keepalive", None)))
    return calls


def few_query_table(wl, device, steps, single_us):
    """The few-query entry point on the same workload: q_len new tokens per sequence share one pass over the span
    (each under its causal limit).  Reports the time per call and per token next to the one-token call."""
    import numpy as np
    import torch
    import paper_2404_09336_amd as span
    from workloads import draw_queries
    cfg, table = wl.cfg, {}
    for q_len in (2, 4, 8, 16, 32):
        calls = few_query_calls(wl, q_len, device)
        r = timed_loop(calls, wl.span_bytes, steps, max(5, steps // 10), 3)
        us = r["us_per_call_event"]
        table[f"q_len_{q_len}"] = {"us_per_call": round(us, 2), "us_per_token": round(us / q_len, 2),
                                   "tokens_per_s": round(cfg.batch * q_len / us * 1e6, 0),
                                   "speedup_per_token_vs_one_query": round(single_us * q_len / us, 3),
                                   "passes_over_span": -(-q_len // span.span_plan_query(calls[0].desc)["queries_per_pass"])}
    return table


def other_workloads(device, args):
    """Configs 2, 4, 5 with their dense controls; config 5 with one interval per sequence against the dense call;
    config 5 at uniform coverages (speedup against sparsity); the other (type, head_dim) instances at the
    headline shape; per-token random masks as interval lists."""
    import torch
    from workloads import CONFIGS, full_cover_spans, draw_spans
    out = {"workloads": {}, "coverage_sweep": {}, "instances": {}}
    for cid in (2, 4):
        wl = Workload(CONFIGS[cid], auto_copies(CONFIGS[cid]), device)
        out["workloads"][f"config{cid}"] = compact_row(wl, 600)
        del wl
        torch.cuda.empty_cache()
    cfg5 = CONFIGS[5]
    wl5 = Workload(cfg5, 2, device)
    out["workloads"]["config5"] = compact_row(wl5, 80, 24)
    dense_us = out["workloads"]["config5"]["dense_us"]
    ctxs = [draw_spans(cfg5, seed=cfg5.seed(c)).ctx_lens for c in range(2)]
    full = Workload(cfg5, 2, device, kv=wl5.kv, spans=[full_cover_spans(c) for c in ctxs])
    f = timed_loop(full.span_calls, full.span_bytes, 24, 4, 3)
    out["workloads"]["config5_one_interval_control"] = {
        "span_path_us": round(f["us_per_call_event"], 2), "dense_call_us": dense_us,
        "span_path_overhead_pct": round(100.0 * (f["us_per_call_event"] / dense_us - 1.0), 2),
        "note": "one interval [0, len) per sequence through span_decode_attn against dense_decode_attn (the paper's "
                "keep-everything check of its kernel: within 7 %, Sec. 4.1)"}
    del full
    for cov in (0.05, 0.10, 0.25, 0.50):
        w = Workload(cfg5, 2, device, coverage=cov, kv=wl5.kv)
        s = timed_loop(w.span_calls, w.span_bytes, 60 if cov < 0.2 else 30, 5, 3)
        out["coverage_sweep"][f"{int(round(cov * 100))}pct"] = {
            "span_mb": round(s["bytes_per_call"] / 1e6, 1), "span_us": round(s["us_per_call_event"], 2),
            "span_gbps": round(s["gbps_event"], 1), "speedup_vs_dense": round(dense_us / s["us_per_call_event"], 2)}
        del w
    del wl5
    torch.cuda.empty_cache()
    base = CONFIGS[3]
    for dtype, D in (("f32", 128), ("f32", 64), ("f16", 64), ("bf16", 128), ("bf16", 64)):
        cfg = dataclasses.replace(base, dtype=dtype, head_dim=D, name=f"config3-shape-{dtype}-d{D}")
        wl = Workload(cfg, auto_copies(cfg), device)
        row = compact_row(wl, 400)
        out["instances"][f"{dtype}_d{D}"] = {k: row[k] for k in ("span_mb", "span_us", "span_gbps", "span_pct_peak",
                                                                 "dense_us", "dense_gbps", "speedup_vs_dense")}
        del wl
        torch.cuda.empty_cache()
    return out


def secondary_bytes(wl):
    """Bytes a span call moves besides the K / V rows of the span (first rotated copy), itemised so that they
    cannot hide inside the headline figure: q, out, span metadata, and the slices' partial states (written once,
    read once by the merging workgroup) when a (batch, head) pair is cut into several slices."""
    cfg, plan = wl.cfg, wl.plan
    sp = wl.host[0][0]
    pairs = cfg.batch * cfg.heads
    partial = 2 * plan["workgroups"] * plan["queries_per_pass"] * (cfg.head_dim + 2) * 4 if plan["max_splits"] > 1 else 0
    return {"q": wl.q_len * pairs * cfg.head_dim * cfg.elt_bytes, "out": wl.q_len * pairs * cfg.head_dim * 4,
            "span_metadata": 8 * int(sp.starts.size) + 4 * (cfg.batch + 1),
            "partial_states_write_plus_read": partial}


def cpu_baseline(wl, budget_s=10.0):
    """The oracle as it stands on the host cores, on whole batches of the same workload; plus the smallest workload
    (config 1) on one thread."""
    import numpy as np
    import oracle
    from workloads import CONFIGS, draw_qkv, draw_spans, to_host_raw
    sp, q, K, V = wl.host[0]
    hq, hK, hV = to_host_raw(q), to_host_raw(K), to_host_raw(V)
    reps, t0 = 0, time.perf_counter()
    while True:
        oracle.span_attn(hq, hK, hV, sp.offsets, sp.starts, sp.ends, np.float32(wl.cfg.scale), dtype=wl.cfg.dtype)
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or reps >= 1000:
            break
    res = {"value": wl.span_bytes[0] * reps / dt / 1e9, "unit": "GB/s", "cores": oracle.num_threads(),
           "kind": "oracle", "ms_per_call": dt / reps * 1e3,
           "sample": f"{reps} whole batch(es) of config {wl.cfg.cfg_id} ({wl.cfg.name}), fp64 two-pass softmax over "
                     f"span rows, OpenMP over heads"}
    try:
        from threadpoolctl import threadpool_limits
        cfg1 = CONFIGS[1]
        sp1 = draw_spans(cfg1)
        q1, K1, V1 = draw_qkv(cfg1, sp1.ctx_lens)
        a = (to_host_raw(q1), to_host_raw(K1), to_host_raw(V1), sp1.offsets, sp1.starts, sp1.ends, np.float32(cfg1.scale))
        with threadpool_limits(limits=1, user_api="openmp"):
            oracle.span_attn(*a, dtype=cfg1.dtype)
            n, t0 = 200, time.perf_counter()
            for _ in range(n):
                oracle.span_attn(*a, dtype=cfg1.dtype)
            res["config1_one_thread_ms_per_call"] = round((time.perf_counter() - t0) / n * 1e3, 4)
    except Exception as e:  # the headline baseline above does not depend on this extra
        res["config1_one_thread_ms_per_call"] = f"unavailable: {type(e).__name__}"
    return res


PAPER_MICROBENCH = {"speedup_vs_hf_geomean": {"32": 0.97, "64": 1.2, "128": 1.6, "256": 1.6, "all": 1.29},
                    "hardware": "1x NVIDIA A100 80GB, batch 64, vs Hugging Face self-attention",
                    "source": "paper Sec. 5.2"}


def microbench(device, steps, warmup):
    """The kernel micro-benchmark of Sec. 5.2: one new token, batch 64, 1024..8096 cached tokens, random masks that
    keep 50 % of the context in runs of `sparsity block size` tokens.  The masks travel the paper's way: blocked
    (block index, bit mask) encoding with 256-token blocks, converted by the library into interval lists.  The
    speedup is over this library's own dense control (the paper's baseline, Hugging Face attention, is absent).
    Besides the paper's run lengths 32..256, unstructured masks with runs of 1..16 tokens are timed."""
    import numpy as np
    import torch
    import paper_2404_09336_amd as span
    from workloads import DecodeConfig, draw_qkv, full_cover_spans, microbench_spans, random_mask_spans
    rows, fine_rows, logsum, overhead = [], [], {}, {}
    for L in (1024, 2048, 4096, 8096):
        cfg = DecodeConfig(100, f"microbench-{L}", 64, 32, 128, L, L, "f16", 2e-3)
        ctx = np.full(cfg.batch, L, np.int32)
        q, K, V = draw_qkv(cfg, ctx, seed=L, device=device)
        dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(device)
        row_pair = 2 * cfg.head_dim * cfg.elt_bytes * cfg.heads
        dense = span.prepare_dense_decode_attn(q, K, V, dev(ctx), np.float32(cfg.scale), max_tokens=L,
                                               tokens_per_seq=ctx.astype(np.int64))
        n = max(20, steps // max(1, L // 512))
        d = timed_loop([dense], [L * cfg.batch * row_pair], n, max(5, warmup // 8))
        # the span path with nothing masked against the dense path (the paper runs its sparse kernel on a
        # keep-everything mask against the dense implementation and finds it within 7 %, Sec. 4.1 "Results")
        full = full_cover_spans(ctx)
        fc = span.prepare_span_decode_attn(q, K, V, dev(full.offsets), dev(full.starts), dev(full.ends), dev(ctx),
                                           np.float32(cfg.scale), max_tokens=L, tokens_per_seq=ctx.astype(np.int64))
        f = timed_loop([fc], [L * cfg.batch * row_pair], n, max(5, warmup // 8))
        overhead[str(L)] = round(100.0 * (f["us_per_call_event"] / d["us_per_call_event"] - 1.0), 2)

        def time_mask(sp):
            boff, bidx, bm = span.span_intervals_to_blocks(256, sp.offsets, sp.starts, sp.ends)   # the paper's format
            off, st, en = span.span_blocks_to_intervals(256, boff, bidx, bm)                       # what the kernel takes
            code, _, _, tok = span.span_validate(off, st, en, ctx)
            assert code == 0
            call = span.prepare_span_decode_attn(q, K, V, dev(off), dev(st), dev(en), dev(ctx), np.float32(cfg.scale),
                                                 max_tokens=int(tok.max()), tokens_per_seq=tok)
            s = timed_loop([call], [int(tok.sum()) * row_pair], n, max(5, warmup // 8))
            return s, tok, len(st)

        for sbs in (32, 64, 128, 256):
            s, tok, n_int = time_mask(microbench_spans(cfg.batch, L, sbs, seed=1000 * L + sbs))
            sp_up = d["us_per_call_event"] / s["us_per_call_event"]
            rows.append({"cached_tokens": L, "sparsity_block": sbs, "kept": round(float(tok.sum()) / (L * cfg.batch), 3),
                         "intervals_per_seq": round(n_int / cfg.batch, 1), "span_us": round(s["us_per_call_event"], 2),
                         "dense_us": round(d["us_per_call_event"], 2), "speedup_vs_dense": round(sp_up, 3),
                         "span_gbps": round(s["gbps_event"], 1)})
            logsum.setdefault(str(sbs), []).append(np.log(sp_up))
        for run in (1, 2, 4, 8, 16):
            s, tok, n_int = time_mask(random_mask_spans(cfg.batch, L, run, seed=77 * L + run))
            fine_rows.append({"cached_tokens": L, "run_length": run, "kept": round(float(tok.sum()) / (L * cfg.batch), 3),
                              "intervals_per_seq": round(n_int / cfg.batch, 1),
                              "span_us": round(s["us_per_call_event"], 2), "dense_us": round(d["us_per_call_event"], 2),
                              "speedup_vs_dense": round(d["us_per_call_event"] / s["us_per_call_event"], 3),
                              "span_gbps": round(s["gbps_event"], 1)})
        del q, K, V, dense, fc
        torch.cuda.empty_cache()
    geo = {k: round(float(np.exp(np.mean(v))), 3) for k, v in logsum.items()}
    geo["all"] = round(float(np.exp(np.mean([x for v in logsum.values() for x in v]))), 3)
    return {"metric": "speedup of 50%-sparse span attention over dense decode (kernel micro-benchmark)",
            "unit": "x", "value": geo["all"], "geomean_by_sparsity_block": geo, "rows": rows,
            "unstructured_rows": fine_rows,
            "span_path_overhead_pct_at_sparsity_0": overhead, "n_gpus": 1,
            "dtype": "f32", "data": "synthetic",
            "config": {"storage_dtype": "f16", "workload": "batch 64, 32 heads x 128, 1 query token, 1024/2048/4096/8096 cached tokens, "
                                   "50 % kept in runs of 32/64/128/256 (paper) and 1/2/4/8/16 (unstructured), masks via "
                                   "256-token blocked encoding"},
            "paper_context": PAPER_MICROBENCH}


STAMP_NAMES = ["entry", "metadata_read", "positions_tabulated", "first_rows_consumed", "all_rows_consumed",
               "waves_merged", "out_stored_one_slice", "state_published_acked", "ticket_returned",
               "slices_merged_out_stored", "interval_range_read"]
STAMP_ORDER = [0, 10, 1, 2, 3, 4, 5, 6, 7, 8, 9]


def phase_trace(args, device):
    """Per-workgroup times of the phases of ONE call in a stream of back-to-back calls (diagnostic `trace` build:
    thread 0 of every workgroup stamps a 100 MHz clock at each phase boundary)."""
    import ctypes
    import numpy as np
    import torch
    import paper_2404_09336_amd as span
    from workloads import CONFIGS
    lib = span.load_library()
    if not hasattr(lib, "span_debug_set_trace"):
        print("bench.py: --phase-trace needs the trace build: python -m paper_2404_09336_amd.build trace, then "
              "--variant trace", file=sys.stderr)
        sys.exit(4)
    lib.span_debug_set_trace.argtypes = [ctypes.c_void_p, ctypes.c_size_t]
    lib.span_debug_set_trace.restype = None
    cfg = CONFIGS[args.config]
    wl = Workload(cfg, args.copies or auto_copies(cfg), device, coverage=args.coverage, num_splits=args.num_splits,
                  exact=not args.uniform_grid, host_lists=not args.no_host_lists, q_len=args.q_len)
    calls = wl.span_calls if args.only != "dense" else wl.dense_calls
    wgs = max(span.span_plan_query(c.desc)["workgroups"] for c in calls)
    buf = torch.zeros((wgs, 16), dtype=torch.int64, device=device)
    prewarm(calls)
    lib.span_debug_set_trace(ctypes.c_void_p(buf.data_ptr()), wgs)   # workgroups beyond `wgs` would not stamp
    samples = []
    for rep in range(8):                                # eight traced calls, each the last of a burst of 50
        for i in range(47):
            calls[i % len(calls)]()
        buf.zero_()
        for i in range(47, 50):                         # the zeroing must not sit right in front of the traced call
            calls[i % len(calls)]()
        torch.cuda.synchronize()
        last = calls[49 % len(calls)]                   # every workgroup of the last call has overwritten its row
        samples.append(buf.cpu().numpy()[:span.span_plan_query(last.desc)["workgroups"]].copy())
    lib.span_debug_set_trace(None, 0)
    rows = {}
    spans_us = []
    for t in samples:
        t = t.astype(np.float64)
        start = t[:, 0].min()
        spans_us.append((t.max() - start) / 100.0)
        for k in STAMP_ORDER:
            col = t[:, k]
            col = col[col >= start]                     # a stamp the last call did not write is zero or older
            if col.size == 0:
                continue
            rel = (col - start) / 100.0                 # microseconds since the first workgroup entered
            rows.setdefault(STAMP_NAMES[k], []).append([float(np.percentile(rel, p)) for p in (0, 50, 95, 100)] + [int(col.size)])
    table = {}
    for name, v in rows.items():
        a = np.array(v)
        table[name] = {"min_us": round(float(np.median(a[:, 0])), 2), "p50_us": round(float(np.median(a[:, 1])), 2),
                       "p95_us": round(float(np.median(a[:, 2])), 2), "max_us": round(float(np.median(a[:, 3])), 2),
                       "workgroups": int(np.median(a[:, 4]))}
    r = timed_loop(calls, wl.span_bytes if args.only != "dense" else wl.dense_bytes, 500, 50, 3)
    idx = 49 % len(calls)
    print(json.dumps({"mode": "phase-trace", "config": cfg.cfg_id, "kernel": args.only if args.only != "all" else "span",
                      "traced_copy": idx, "plan": span.span_plan_query(calls[idx].desc),
                      "kv_bytes_of_traced_call": (wl.span_bytes if args.only != "dense" else wl.dense_bytes)[idx],
                      "first_entry_to_last_stamp_us": round(float(np.median(spans_us)), 2),
                      "us_per_call_hip_events_with_stamps": round(r["us_per_call_event"], 2),
                      "phases_us_since_first_entry": table}), flush=True)


def pmc_summary(dirs):
    """rocprofv3 --pmc CSVs -> mean counter value per decode call and per 1 GiB calibration kernel."""
    import csv
    import glob
    out = {}
    for d in dirs:
        for path in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
            agg = {}
            for r in csv.DictReader(open(path)):
                n = r["Kernel_Name"]
                if "decode_kernel" in n:
                    key = "decode_kernel"
                elif "neg" in n.lower() and int(r["Grid_Size"]) >= (1 << 24):
                    key = "copy_1GiB"
                else:
                    continue
                agg.setdefault((r["Counter_Name"], key), []).append(float(r["Counter_Value"]))
            for (counter, key), v in agg.items():
                out.setdefault(counter, {})[key] = {"mean": statistics.mean(v), "dispatches": len(v)}
    res = {"counters": out}
    try:
        # both counters count KiB; the calibration kernel reads 1 GiB and writes 1 GiB
        fs = (1 << 20) / out["FETCH_SIZE"]["copy_1GiB"]["mean"]
        ws = (1 << 20) / out["WRITE_SIZE"]["copy_1GiB"]["mean"]
        fetch = out["FETCH_SIZE"]["decode_kernel"]["mean"] * 1024 * fs
        write = out["WRITE_SIZE"]["decode_kernel"]["mean"] * 1024 * ws
        res.update({"fetch_scale": round(fs, 4), "write_scale": round(ws, 4), "fetch_bytes": int(fetch),
                    "write_bytes": int(write), "hbm_bytes_per_call": int(fetch + write)})
    except KeyError:
        pass
    print(json.dumps(res), flush=True)


def read_traffic(cfg_id):
    """(HBM bytes per call measured offline with rocprofv3 --pmc, the commit they were measured at), see profiles/;
    (None, None) if not recorded."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(path):
        return None, None
    try:
        doc = json.load(open(path))
        return doc.get(f"config{cfg_id}", {}).get("hbm_bytes_per_call"), doc.get("measured_at_commit")
    except (ValueError, OSError):
        return None, None


def source_revision():
    try:
        return subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], capture_output=True, text=True,
                              timeout=5).stdout.strip() or None
    except (OSError, subprocess.SubprocessError):
        return None


def main():
    args = parse_args()
    if args.pmc_summary:
        pmc_summary(args.pmc_summary)
        return
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (one MI355X); --gpus must be 1. The path shards over batch "
              "or heads with no collective, but no multi-GPU run exists here.", file=sys.stderr)
        sys.exit(2)
    if args.variant:
        os.environ["SPAN_ATTN_VARIANT"] = args.variant
    import torch
    import paper_2404_09336_amd as span
    from workloads import CONFIGS
    span.load_library()                      # fail loudly if the HIP library is not built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    device = torch.device("cuda:0")
    torch.cuda.set_device(device)

    if args.microbench:
        print(json.dumps(microbench(device, args.steps, args.warmup)), flush=True)
        return
    if args.phase_trace:
        phase_trace(args, device)
        return

    cfg = CONFIGS[args.config]
    copies = args.copies or auto_copies(cfg)
    if args.q_len > 1 and args.only != "span":
        print("bench.py: --q-len needs --only span (or --phase-trace)", file=sys.stderr)
        sys.exit(2)
    wl = Workload(cfg, copies, device, coverage=args.coverage, num_splits=args.num_splits,
                  exact=not args.uniform_grid, host_lists=not args.no_host_lists, q_len=args.q_len)

    if args.calibrate_copy:
        # a plain elementwise kernel that reads 1 GiB and writes 1 GiB (torch's same-dtype copy_ is a DMA
        # memcpy, not a kernel, so it would not show up in per-kernel counters)
        src = torch.ones(1 << 28, dtype=torch.float32, device=device)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            torch.neg(src, out=dst)
        torch.cuda.synchronize()
        del src, dst

    res_span = res_dense = res_hot = None
    prewarm(wl.span_calls if args.only != "dense" else wl.dense_calls)
    if args.only in ("all", "span"):
        res_span = timed_loop(wl.span_calls, wl.span_bytes, args.steps, args.warmup, args.rounds)
    if args.only in ("all", "dense"):
        dsteps = max(10, args.steps // 4) if args.only == "all" else args.steps
        res_dense = timed_loop(wl.dense_calls, wl.dense_bytes, dsteps, max(5, args.warmup // 4),
                               3 if args.only == "all" else args.rounds)
    if args.only == "all":
        res_hot = timed_loop(wl.span_calls[:1], wl.span_bytes[:1], max(10, args.steps // 4), max(5, args.warmup // 4), 3)

    main_res = res_span or res_dense
    out = {
        "metric": "span-KV HBM GB/s" if res_span else "dense-KV HBM GB/s (control)",
        "value": round(main_res["gbps_wall"], 2), "unit": "GB/s",
        "pct_of_hbm_peak": round(100.0 * main_res["gbps_wall"] / HBM_PEAK_GBPS, 2),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "rounds": args.rounds,
        "ms_per_step": round(main_res["us_per_call_wall"] * 1e-3, 6),
        "ms_per_step_of_each_round": [round(u * 1e-3, 6) for u in main_res["rounds_us_per_call_wall"]],
        "calls_per_s": round(1e6 / main_res["us_per_call_wall"], 1),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config {cfg.cfg_id} ({cfg.name}): batch {cfg.batch}, {cfg.heads} heads x "
                               f"{cfg.head_dim}, KV length {cfg.min_len}-{cfg.max_len}, {args.q_len} query token"
                               + ("s (few-query call)" if args.q_len > 1 else ""),
                   "storage_dtype": cfg.dtype, "arithmetic": "fp32 multiply-accumulate, fp32 softmax, fp32 output",
                   "span_coverage": round(wl.coverage, 4),
                   "span_bytes_per_call": int(main_res["bytes_per_call"]),
                   "secondary_bytes_per_call": secondary_bytes(wl),
                   "kv_copies_rotated": copies, "plan": wl.plan, "library_variant": args.variant or "product",
                   "source_revision": source_revision()},
        "roofline": {"bound": "hbm", "achieved": round(main_res["gbps_event"], 2), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(main_res["gbps_event"] / HBM_PEAK_GBPS, 4),
                     "traffic": read_traffic(cfg.cfg_id)[0] if res_span and args.q_len == 1 else None,
                     "traffic_measured_at_commit": read_traffic(cfg.cfg_id)[1] if res_span and args.q_len == 1 else None,
                     "us_per_call_hip_events": round(main_res["us_per_call_event"], 3)},
        "paper_context": PAPER_CONTEXT,
    }
    if res_span and res_dense:
        out["speedup_vs_dense"] = round(res_dense["us_per_call_wall"] / res_span["us_per_call_wall"], 3)
        out["dense_control"] = {"us_per_call": round(res_dense["us_per_call_wall"], 3),
                                "gbps": round(res_dense["gbps_wall"], 2),
                                "pct_of_hbm_peak": round(100.0 * res_dense["gbps_wall"] / HBM_PEAK_GBPS, 2),
                                "bytes_per_call": int(res_dense["bytes_per_call"])}
    if res_hot:
        out["hot_cache_gbps_not_counted"] = round(res_hot["gbps_wall"], 2)

    if args.only == "all" and not args.no_others and args.config == 3 and not args.variant:
        out["few_query"] = few_query_table(wl, device, 300, res_span["us_per_call_event"])
        out.update(other_workloads(device, args))

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
