#!/usr/bin/env python3
"""Benchmark of span-restricted decode attention on one MI355X.

A "step" is one span_decode_attn call (all of: locate work, q.K scores, online softmax, p.V, merge)
over one batch of synthetic input that is already resident in HBM.  The headline workload is the
arithmetic-evaluation-shaped one (config 3: batch 64, 32 heads x 128, 512 cached tokens, ~30 % of them
in the span, fp16).  Steps rotate over several independent (K, V, span) copies so that the bytes touched
between two uses of a buffer exceed the on-package cache: the figure is HBM bandwidth, not cache bandwidth.

Prints ONE JSON line:
  value    = span bytes (K and V rows inside the intervals) * steps / wall time of the timed region  [GB/s]
  roofline = same bytes / average call duration from HIP events on the launch stream, against 8 TB/s
  cpu_baseline = the fp64 CPU oracle on the same workload, timed on the host cores
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0           # MI355X HBM3E, published peak
LLC_BYTES = 256 * 1024 * 1024    # on-package last-level cache to defeat by rotation
PAPER_CONTEXT = {"gain": "up to 28% more tokens/s end to end (27.7% at 1536-1792 output tokens)",
                 "hardware": "1x NVIDIA A100 80GB, LLaMA-7B, batch 48", "source": "paper abstract and Sec. 4.1"}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4000)
    ap.add_argument("--warmup", type=int, default=400)
    ap.add_argument("--config", type=int, default=3, help="workload id 1..5 (headline: 3)")
    ap.add_argument("--copies", type=int, default=0, help="independent KV copies to rotate over (0 = auto)")
    ap.add_argument("--coverage", type=float, default=None, help="config 5 only: uniform span coverage")
    ap.add_argument("--num-splits", type=int, default=0)
    ap.add_argument("--uniform-grid", action="store_true",
                    help="do not pass per-sequence token counts (every sequence gets the same number of slices)")
    ap.add_argument("--only", choices=["all", "span", "dense"], default="all",
                    help="'span' / 'dense' run just that timed loop (for profiling one kernel)")
    ap.add_argument("--others", action="store_true", help="also time configs 2, 4, 5 (reported under 'workloads')")
    ap.add_argument("--microbench", action="store_true",
                    help="instead of the headline run: the paper's kernel micro-benchmark (Sec. 5.2), speedup of "
                         "50 %-sparse masks over dense for sparsity block sizes 32..256 and 1024..8096 cached tokens")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch a plain 1 GiB-in / 1 GiB-out elementwise kernel (reference for HBM traffic counters)")
    return ap.parse_args()


class Workload:
    """`copies` independent instances of one config: tensors on the GPU plus prepared calls."""

    def __init__(self, cfg_id, copies, device, coverage=None, num_splits=0, exact=True):
        import numpy as np
        import torch
        import paper_2404_09336_amd as span
        from workloads import CONFIGS, draw_qkv, draw_spans
        self.cfg = cfg = CONFIGS[cfg_id]
        self.span_calls, self.dense_calls = [], []
        self.span_bytes, self.dense_bytes, self.coverages = [], [], []
        self.host = []
        row_pair = 2 * cfg.head_dim * cfg.elt_bytes * cfg.heads     # K and V bytes per position, all heads
        for c in range(copies):
            sp = draw_spans(cfg, seed=cfg.seed(c), coverage=coverage)
            code, _, _, tok = span.span_validate(sp.offsets, sp.starts, sp.ends, sp.ctx_lens)
            assert code == 0, code
            q, K, V = draw_qkv(cfg, sp.ctx_lens, seed=cfg.seed(c), device=device)
            dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(device)
            off, st, en, ctx = dev(sp.offsets), dev(sp.starts), dev(sp.ends), dev(sp.ctx_lens)
            self.span_calls.append(span.prepare_span_decode_attn(q, K, V, off, st, en, ctx, np.float32(cfg.scale),
                                                                 max_tokens=int(tok.max()), num_splits=num_splits,
                                                                 tokens_per_seq=tok if exact else None))
            self.dense_calls.append(span.prepare_dense_decode_attn(
                q, K, V, ctx, np.float32(cfg.scale), max_tokens=int(sp.ctx_lens.max()),
                tokens_per_seq=sp.ctx_lens.astype(np.int64) if exact else None))
            self.span_bytes.append(int(tok.sum()) * row_pair)
            self.dense_bytes.append(int(sp.ctx_lens.astype(np.int64).sum()) * row_pair)
            self.coverages.append(sp.coverage())
            if c == 0:
                self.host.append((sp, q, K, V))
        self.plan = span.span_plan_query(self.span_calls[0].desc)
        self.partition = (self.plan["max_splits"], self.plan["slice_tokens"], self.plan["workgroups"])


def few_query_table(wl, device, steps, single_us):
    """The few-query entry point on the same workload: q_len new tokens per sequence share one pass over the span
    (each under its causal limit).  Reports the time per call and per token next to the one-token call."""
    import numpy as np
    import torch
    import paper_2404_09336_amd as span
    from workloads import draw_queries
    cfg, table = wl.cfg, {}
    for q_len in (2, 4, 8):
        calls = []
        for c, one in enumerate(wl.span_calls):
            _, K, V, off, st, en, ctx, _ = one._keepalive
            q = draw_queries(cfg, q_len, seed=cfg.seed(c), device=device)
            q_pos = (ctx - q_len).to(torch.int32)            # the new tokens are the last q_len cache rows
            calls.append(span.prepare_span_decode_attn_multi(q, K, V, off, st, en, q_pos, np.float32(cfg.scale),
                                                             max_tokens=one.desc.max_tokens,
                                                             tokens_per_seq=getattr(one.desc, "_tokens_keepalive", None)))
        r = timed_loop(calls, wl.span_bytes, steps, max(5, steps // 10))
        us = r["us_per_call_event"]
        table[f"q_len_{q_len}"] = {"us_per_call": round(us, 2), "us_per_token": round(us / q_len, 2),
                                   "tokens_per_s": round(cfg.batch * q_len / us * 1e6, 0),
                                   "speedup_per_token_vs_one_query": round(single_us * q_len / us, 3),
                                   "passes_over_span": -(-q_len // 4)}
    return table


def auto_copies(cfg_id):
    """Enough copies that the span bytes touched in one rotation are >= 2x the last-level cache."""
    import numpy as np
    import paper_2404_09336_amd as span  # noqa: F401
    from workloads import CONFIGS, draw_spans
    cfg = CONFIGS[cfg_id]
    sp = draw_spans(cfg)
    touched = int(sp.tokens_per_seq().sum()) * 2 * cfg.head_dim * cfg.elt_bytes * cfg.heads
    alloc = 2 * cfg.batch * cfg.heads * cfg.max_len * cfg.head_dim * cfg.elt_bytes
    n = int(np.ceil(2 * LLC_BYTES / max(touched, 1)))
    n = max(2, n)                                   # always alternate buffers, even when one call exceeds the cache
    n = max(1, min(n, 16, max(1, (48 << 30) // alloc)))
    return n


def timed_loop(calls, nbytes, steps, warmup):
    """Warm up, then time exactly `steps` calls: wall clock bracketed by synchronize, plus HIP events
    recorded on the launch stream.  Returns dict with per-call times and byte rates."""
    import torch
    n = len(calls)
    for i in range(warmup):
        calls[i % n]()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    total_bytes = sum(nbytes[i % n] for i in range(steps))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for i in range(steps):
        calls[i % n]()
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ev_s = ev0.elapsed_time(ev1) * 1e-3
    return {"wall_s": wall, "event_s": ev_s, "bytes_per_call": total_bytes / steps,
            "us_per_call_wall": wall / steps * 1e6, "us_per_call_event": ev_s / steps * 1e6,
            "gbps_wall": total_bytes / wall / 1e9, "gbps_event": total_bytes / ev_s / 1e9}


def secondary_bytes(wl):
    """Bytes a span call moves besides the K / V rows of the span (first rotated copy), itemised so that they
    cannot hide inside the headline figure: q, out, span metadata, and the slices' partial states (written once,
    read once by the merging workgroup) when a (batch, head) pair is cut into several slices."""
    cfg, plan = wl.cfg, wl.plan
    sp = wl.host[0][0]
    pairs = cfg.batch * cfg.heads
    partial = 2 * plan["workgroups"] * (cfg.head_dim + 2) * 4 if plan["max_splits"] > 1 else 0
    return {"q": pairs * cfg.head_dim * cfg.elt_bytes, "out": pairs * cfg.head_dim * 4,
            "span_metadata": 8 * int(sp.starts.size) + 4 * (cfg.batch + 1),
            "partial_states_write_plus_read": partial}


def cpu_baseline(wl, budget_s=12.0):
    """The oracle as it stands on the host cores, on whole batches of the same workload."""
    import numpy as np
    import oracle
    from workloads import to_host_raw
    sp, q, K, V = wl.host[0]
    hq, hK, hV = to_host_raw(q), to_host_raw(K), to_host_raw(V)
    reps, t0 = 0, time.perf_counter()
    while True:
        oracle.span_attn(hq, hK, hV, sp.offsets, sp.starts, sp.ends, np.float32(wl.cfg.scale), dtype=wl.cfg.dtype)
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or reps >= 1000:
            break
    return {"value": wl.span_bytes[0] * reps / dt / 1e9, "unit": "GB/s", "cores": oracle.num_threads(),
            "kind": "oracle", "ms_per_call": dt / reps * 1e3,
            "sample": f"{reps} whole batch(es) of config {wl.cfg.cfg_id} ({wl.cfg.name}), fp64 two-pass softmax over "
                      f"span rows, OpenMP over heads"}


PAPER_MICROBENCH = {"speedup_vs_hf_geomean": {"32": 0.97, "64": 1.2, "128": 1.6, "256": 1.6, "all": 1.29},
                    "hardware": "1x NVIDIA A100 80GB, batch 64, vs Hugging Face self-attention",
                    "source": "paper Sec. 5.2"}


def microbench(device, steps, warmup):
    """The kernel micro-benchmark of Sec. 5.2: one new token, batch 64, 1024..8096 cached tokens, random masks that
    keep 50 % of the context in runs of `sparsity block size` tokens.  The masks travel the paper's way: blocked
    (block index, bit mask) encoding with 256-token blocks, converted by the library into interval lists.  The
    speedup is over this library's own dense control (the paper's baseline, Hugging Face attention, is absent)."""
    import numpy as np
    import torch
    import paper_2404_09336_amd as span
    from workloads import DecodeConfig, draw_qkv, full_cover_spans, microbench_spans
    rows, logsum, overhead = [], {}, {}
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
        for sbs in (32, 64, 128, 256):
            sp = microbench_spans(cfg.batch, L, sbs, seed=1000 * L + sbs)
            boff, bidx, bm = span.span_intervals_to_blocks(256, sp.offsets, sp.starts, sp.ends)   # the paper's format
            off, st, en = span.span_blocks_to_intervals(256, boff, bidx, bm)                       # what the kernel takes
            code, _, _, tok = span.span_validate(off, st, en, ctx)
            assert code == 0
            call = span.prepare_span_decode_attn(q, K, V, dev(off), dev(st), dev(en), dev(ctx), np.float32(cfg.scale),
                                                 max_tokens=int(tok.max()), tokens_per_seq=tok)
            s = timed_loop([call], [int(tok.sum()) * row_pair], n, max(5, warmup // 8))
            sp_up = d["us_per_call_event"] / s["us_per_call_event"]
            rows.append({"cached_tokens": L, "sparsity_block": sbs, "kept": round(float(tok.sum()) / (L * cfg.batch), 3),
                         "intervals_per_seq": round(len(st) / cfg.batch, 1), "span_us": round(s["us_per_call_event"], 2),
                         "dense_us": round(d["us_per_call_event"], 2), "speedup_vs_dense": round(sp_up, 3),
                         "span_gbps": round(s["gbps_event"], 1)})
            logsum.setdefault(str(sbs), []).append(np.log(sp_up))
        del q, K, V, dense, fc
        torch.cuda.empty_cache()
    geo = {k: round(float(np.exp(np.mean(v))), 3) for k, v in logsum.items()}
    geo["all"] = round(float(np.exp(np.mean([x for v in logsum.values() for x in v]))), 3)
    return {"metric": "speedup of 50%-sparse span attention over dense decode (kernel micro-benchmark)",
            "unit": "x", "value": geo["all"], "geomean_by_sparsity_block": geo, "rows": rows,
            "span_path_overhead_pct_at_sparsity_0": overhead, "n_gpus": 1,
            "dtype": "f32", "data": "synthetic",
            "config": {"storage_dtype": "f16", "workload": "batch 64, 32 heads x 128, 1 query token, 1024/2048/4096/8096 cached tokens, "
                                   "50 % kept in runs of 32/64/128/256, masks via 256-token blocked encoding"},
            "paper_context": PAPER_MICROBENCH}


def read_traffic(cfg_id):
    """HBM bytes per call measured offline with rocprofv3 --pmc (see profiles/); None if not recorded."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(path):
        return None
    try:
        return json.load(open(path)).get(f"config{cfg_id}", {}).get("hbm_bytes_per_call")
    except (ValueError, OSError):
        return None


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (one MI355X); --gpus must be 1. The path shards over batch "
              "or heads with no collective, but no multi-GPU run exists here.", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2404_09336_amd as span
    span.load_library()                      # fail loudly if the HIP library is not built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    device = torch.device("cuda:0")
    torch.cuda.set_device(device)

    if args.microbench:
        print(json.dumps(microbench(device, args.steps, args.warmup)), flush=True)
        return

    copies = args.copies or auto_copies(args.config)
    wl = Workload(args.config, copies, device, coverage=args.coverage, num_splits=args.num_splits,
                  exact=not args.uniform_grid)
    cfg = wl.cfg

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
    if args.only in ("all", "span"):
        res_span = timed_loop(wl.span_calls, wl.span_bytes, args.steps, args.warmup)
    if args.only in ("all", "dense"):
        dsteps = max(10, args.steps // 4) if args.only == "all" else args.steps
        res_dense = timed_loop(wl.dense_calls, wl.dense_bytes, dsteps, max(5, args.warmup // 4))
    if args.only == "all":
        res_hot = timed_loop(wl.span_calls[:1], wl.span_bytes[:1], max(10, args.steps // 4), max(5, args.warmup // 4))

    main_res = res_span or res_dense
    out = {
        "metric": "span-KV HBM GB/s" if res_span else "dense-KV HBM GB/s (control)",
        "value": round(main_res["gbps_wall"], 2), "unit": "GB/s",
        "pct_of_hbm_peak": round(100.0 * main_res["gbps_wall"] / HBM_PEAK_GBPS, 2),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(main_res["us_per_call_wall"] * 1e-3, 6),
        "calls_per_s": round(1e6 / main_res["us_per_call_wall"], 1),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config {cfg.cfg_id} ({cfg.name}): batch {cfg.batch}, {cfg.heads} heads x "
                               f"{cfg.head_dim}, KV length {cfg.min_len}-{cfg.max_len}, 1 query token",
                   "storage_dtype": cfg.dtype, "arithmetic": "fp32 multiply-accumulate, fp32 softmax, fp32 output",
                   "span_coverage": round(sum(wl.coverages) / len(wl.coverages), 4),
                   "span_bytes_per_call": int(main_res["bytes_per_call"]),
                   "secondary_bytes_per_call": secondary_bytes(wl),
                   "kv_copies_rotated": copies, "plan": wl.plan},
        "roofline": {"bound": "hbm", "achieved": round(main_res["gbps_event"], 2), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(main_res["gbps_event"] / HBM_PEAK_GBPS, 4),
                     "traffic": read_traffic(cfg.cfg_id) if res_span else None,
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

    if args.others:
        if res_span:
            out["few_query"] = few_query_table(wl, device, max(20, args.steps // 4), res_span["us_per_call_event"])
        table = {}
        for cid in (2, 4, 5):
            del wl
            torch.cuda.empty_cache()
            wl = Workload(cid, auto_copies(cid), device)
            steps = max(20, args.steps // (8 if cid == 5 else 2))
            s = timed_loop(wl.span_calls, wl.span_bytes, steps, max(5, steps // 10))
            d = timed_loop(wl.dense_calls, wl.dense_bytes, max(10, steps // 4), 5)
            table[f"config{cid}"] = {"name": wl.cfg.name, "coverage": round(sum(wl.coverages) / len(wl.coverages), 4),
                                     "span_gbps": round(s["gbps_wall"], 1),
                                     "span_pct_peak": round(100 * s["gbps_wall"] / HBM_PEAK_GBPS, 2),
                                     "span_us": round(s["us_per_call_wall"], 2),
                                     "dense_us": round(d["us_per_call_wall"], 2),
                                     "dense_gbps": round(d["gbps_wall"], 1),
                                     "speedup_vs_dense": round(d["us_per_call_wall"] / s["us_per_call_wall"], 3),
                                     "splits": wl.partition[0]}
        out["workloads"] = table
        del wl
        torch.cuda.empty_cache()
        wl = Workload(args.config, 1, device)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
