"""Parity of the HIP path (through the C ABI) against the fp64 oracle, element by element, on the same
seeded inputs.  Tolerances: max-abs 1e-5 for fp32 inputs, 2e-3 for fp16 / bf16 inputs (fp32 accumulation,
fp32 output)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_09336_amd as span
from workloads import (CONFIGS, DecodeConfig, SpanBatch, draw_qkv, draw_spans, full_cover_spans, microbench_spans,
                       to_host_raw)

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "f16": 2e-3, "bf16": 2e-3}


def _dev(a, device):
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def run_span(cfg, sp, q, K, V, device, **kw):
    """By default the call gets what a caller has after span_validate: the largest span and the per-sequence
    token counts (exact slicing).  num_splits=... or tokens_per_seq=None select the uniform grid."""
    code, bs, bi, tok = span.span_validate(sp.offsets, sp.starts, sp.ends, sp.ctx_lens)
    kw.setdefault("max_tokens", int(tok.max()) if code == 0 and len(tok) else 0)
    if code == 0:
        kw.setdefault("tokens_per_seq", tok)
    out = span.span_decode_attn(q, K, V, _dev(sp.offsets, device), _dev(sp.starts, device), _dev(sp.ends, device),
                                _dev(sp.ctx_lens, device), np.float32(cfg.scale), **kw)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


def run_dense(cfg, ctx_lens, q, K, V, device, **kw):
    kw.setdefault("tokens_per_seq", np.asarray(ctx_lens, np.int64))
    out = span.dense_decode_attn(q, K, V, _dev(np.asarray(ctx_lens, np.int32), device), np.float32(cfg.scale), **kw)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


def oracle_span(cfg, sp, q, K, V):
    return oracle.span_attn(to_host_raw(q), to_host_raw(K), to_host_raw(V), sp.offsets, sp.starts, sp.ends,
                            np.float32(cfg.scale), dtype=cfg.dtype)


def oracle_dense(cfg, ctx_lens, q, K, V):
    return oracle.dense_attn(to_host_raw(q), to_host_raw(K), to_host_raw(V), ctx_lens, np.float32(cfg.scale),
                             dtype=cfg.dtype)


def check(got, ref, tol, what):
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = float(np.abs(got - ref).max())
    print(f"[parity] {what}: max-abs err {err:.3e} (tol {tol:g})", flush=True)
    assert err <= tol, f"{what}: max-abs err {err:.3e} > {tol:g}"


def small_cfg(dtype, D, B=3, H=5, L=700, min_len=None, cid=90):
    return DecodeConfig(cid, f"small-{dtype}-{D}", B, H, D, L, L if min_len is None else min_len, dtype, TOL[dtype])


# ------------------------------------------------------------------ the five workloads, full size
@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_workload_span_parity(cid, gpu_device):
    cfg = CONFIGS[cid]
    sp = draw_spans(cfg)
    assert span.span_validate(sp.offsets, sp.starts, sp.ends, sp.ctx_lens)[0] == 0
    q, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device)
    got = run_span(cfg, sp, q, K, V, gpu_device)
    check(got, oracle_span(cfg, sp, q, K, V), cfg.tol, f"config {cid} span (coverage {sp.coverage():.3f})")
    ref = oracle_span(cfg, sp, q, K, V)
    # without the per-sequence counts every sequence gets the same number of slices
    check(run_span(cfg, sp, q, K, V, gpu_device, tokens_per_seq=None), ref, cfg.tol, f"config {cid} span, uniform grid")
    # without even the bound on span tokens the grid is sized for max_len
    check(run_span(cfg, sp, q, K, V, gpu_device, tokens_per_seq=None, max_tokens=0), ref, cfg.tol,
          f"config {cid} span, uniform grid sized for max_len")


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_workload_dense_parity(cid, gpu_device):
    cfg = CONFIGS[cid]
    sp = draw_spans(cfg)
    q, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device)
    ref = oracle_dense(cfg, sp.ctx_lens, q, K, V)
    check(run_dense(cfg, sp.ctx_lens, q, K, V, gpu_device), ref, cfg.tol, f"config {cid} dense")
    # dense attention sent through the span path as one interval [0, len) (Sec. 4.1 control)
    full = full_cover_spans(sp.ctx_lens)
    check(run_span(cfg, full, q, K, V, gpu_device), ref, cfg.tol, f"config {cid} full-cover span vs dense oracle")


def test_stress_uniform_coverages(gpu_device):
    cfg = CONFIGS[5]
    base = draw_spans(cfg)
    q, K, V = draw_qkv(cfg, base.ctx_lens, device=gpu_device)
    hq, hK, hV = to_host_raw(q), to_host_raw(K), to_host_raw(V)
    for c in (0.05, 0.10, 0.25, 0.50):
        sp = draw_spans(cfg, coverage=c)          # same seed -> same ctx_lens as `base`
        assert np.array_equal(sp.ctx_lens, base.ctx_lens)
        ref = oracle.span_attn(hq, hK, hV, sp.offsets, sp.starts, sp.ends, np.float32(cfg.scale), dtype=cfg.dtype)
        check(run_span(cfg, sp, q, K, V, gpu_device), ref, cfg.tol, f"config 5 coverage {c}")


# ------------------------------------------------------------------ every (dtype, head_dim) kernel
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("D", [64, 128])
def test_all_kernel_instances(dtype, D, gpu_device):
    cfg = small_cfg(dtype, D, min_len=300)
    rng = np.random.default_rng(5 + D)
    ctx = rng.integers(cfg.min_len, cfg.max_len + 1, size=cfg.batch).astype(np.int32)
    per_seq = []
    for b in range(cfg.batch):
        cuts = np.sort(rng.choice(np.arange(0, ctx[b] + 1), size=12, replace=False))
        per_seq.append([(int(cuts[i]), int(cuts[i + 1])) for i in range(0, 12, 2)])
    sp = SpanBatch.from_lists(per_seq, ctx)
    q, K, V = draw_qkv(cfg, ctx, device=gpu_device, seed=77)
    ref = oracle_span(cfg, sp, q, K, V)
    for ns in (0, 1, 2, 5):
        check(run_span(cfg, sp, q, K, V, gpu_device, num_splits=ns), ref, cfg.tol, f"{dtype} D={D} splits={ns}")
    dref = oracle_dense(cfg, ctx, q, K, V)
    for ns in (0, 1, 3):
        check(run_dense(cfg, ctx, q, K, V, gpu_device, num_splits=ns), dref, cfg.tol, f"{dtype} D={D} dense splits={ns}")


# ------------------------------------------------------------------ split-KV partition and merge
def test_forced_split_counts_agree_with_oracle(gpu_device):
    cfg = small_cfg("f16", 128, B=2, H=3, L=3000)
    sp = SpanBatch.from_lists([[(0, 700), (1000, 1001), (1500, 2600)], [(5, 9), (2990, 3000)]], [3000, 3000])
    q, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device, seed=3)
    ref = oracle_span(cfg, sp, q, K, V)
    for ns in (1, 2, 3, 4, 7, 13, 29, 113):
        check(run_span(cfg, sp, q, K, V, gpu_device, num_splits=ns), ref, cfg.tol, f"splits={ns}")


def test_caller_workspace_is_used_and_sufficient(gpu_device):
    from paper_2404_09336_amd import binding
    cfg = small_cfg("f16", 128, B=2, H=2, L=512)
    sp = full_cover_spans([512, 300])
    q, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device, seed=4)
    d = binding.make_desc(2, 2, 128, 512, 1, 2, 0, 4)
    need = span.span_workspace_bytes(d)
    ws = torch.full((need,), 0xFF, dtype=torch.uint8, device=gpu_device)   # NaN bit patterns everywhere
    d.workspace, d.workspace_bytes = ws.data_ptr(), need
    d.stream = torch.cuda.current_stream(gpu_device).cuda_stream
    span.span_workspace_init(d)                                            # zeroes only the ticket counters
    got = run_span(cfg, sp, q, K, V, gpu_device, num_splits=4, max_tokens=0, workspace=ws)
    ref = oracle_span(cfg, sp, q, K, V)
    check(got, ref, cfg.tol, "caller workspace pre-filled with 0xFF")
    for i in range(3):   # the call leaves the counters zero: the same workspace serves the next calls
        got = run_span(cfg, sp, q, K, V, gpu_device, num_splits=4, max_tokens=0, workspace=ws)
        check(got, ref, cfg.tol, f"workspace reused, call {i + 2}")


def test_wrong_token_counts_from_the_caller(gpu_device):
    """tokens_per_seq only steers the slicing: overstating it leaves idle slices, understating it makes slices
    larger; neither changes the result (short of the slice limit) nor memory safety."""
    cfg = small_cfg("f16", 128, B=3, H=4, L=2048)
    sp = SpanBatch.from_lists([[(0, 300), (900, 1500)], [(5, 6)], [(100, 2048)]], [2048] * 3)
    q, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device, seed=21)
    ref = oracle_span(cfg, sp, q, K, V)
    true = sp.tokens_per_seq()
    for name, tok in (("exact", true), ("overstated", true * 2 + 7), ("understated", np.maximum(true // 2, 1)),
                      ("swapped", true[::-1].copy())):
        got = run_span(cfg, sp, q, K, V, gpu_device, tokens_per_seq=tok, max_tokens=0)
        check(got, ref, cfg.tol, f"tokens_per_seq {name}")
    # all zeros: one slice per sequence, so a sequence may lose what exceeds the slice limit; the others are exact
    from paper_2404_09336_amd import binding
    limit = span.span_plan_query(binding.make_desc(3, 4, 128, 2048, 1))["slice_limit"]
    got = run_span(cfg, sp, q, K, V, gpu_device, tokens_per_seq=true * 0, max_tokens=0)
    assert np.isfinite(got).all()
    fits = true <= limit
    check(got[fits], ref[fits], cfg.tol, "tokens_per_seq all zero, sequences within one slice")


# ------------------------------------------------------------------ degenerate and edge cases
def test_single_position_returns_v_row(gpu_device):
    for dtype in ("f32", "f16", "bf16"):
        cfg = small_cfg(dtype, 128, B=4, H=2, L=130)
        sp = SpanBatch.from_lists([[(0, 1)], [(129, 130)], [(64, 65)], [(17, 18)]], [130] * 4)
        q, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device, seed=5)
        got = run_span(cfg, sp, q, K, V, gpu_device)
        for b, pos in enumerate((0, 129, 64, 17)):
            assert np.array_equal(got[b], V[b, :, pos].float().cpu().numpy().astype(np.float64)), (dtype, b)


def test_empty_span_gives_zero_rows(gpu_device):
    cfg = small_cfg("f16", 128, B=3, H=2, L=64)
    sp = SpanBatch.from_lists([[(3, 9)], [], [(60, 64)]], [64, 64, 64])
    assert span.span_validate(sp.offsets, sp.starts, sp.ends, sp.ctx_lens)[:2] == (6, 1)
    q, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device, seed=6)
    for ns in (1, 2):
        got = run_span(cfg, sp, q, K, V, gpu_device, num_splits=ns, max_tokens=0)
        assert not got[1].any()
        check(got, oracle_span(cfg, sp, q, K, V), cfg.tol, f"batch with an empty span, splits={ns}")


def test_span_sizes_1_to_40_and_ragged_tails(gpu_device):
    for dtype, D in (("f16", 128), ("f32", 64), ("bf16", 64), ("f32", 128)):
        cfg = small_cfg(dtype, D, B=40, H=2, L=96)
        per_seq = [[(5, 5 + n)] if n % 2 else [(0, (n + 1) // 2), (50, 50 + n // 2)] for n in range(1, 41)]
        sp = SpanBatch.from_lists(per_seq, [96] * 40)
        q, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device, seed=7)
        check(run_span(cfg, sp, q, K, V, gpu_device), oracle_span(cfg, sp, q, K, V), cfg.tol, f"n=1..40 {dtype} D={D}")
        ctx = np.arange(1, 41, dtype=np.int32)
        check(run_dense(cfg, ctx, q, K, V, gpu_device), oracle_dense(cfg, ctx, q, K, V), cfg.tol,
              f"dense len=1..40 {dtype} D={D}")


def test_interval_order_and_split_invariance(gpu_device):
    cfg = small_cfg("f16", 128, B=1, H=4, L=1200)
    iv = [(0, 64), (100, 113), (113, 300), (512, 1000), (1190, 1200)]
    q, K, V = draw_qkv(cfg, [1200], device=gpu_device, seed=8)
    base_sp = SpanBatch.from_lists([iv], [1200])
    ref = oracle_span(cfg, base_sp, q, K, V)
    base = run_span(cfg, base_sp, q, K, V, gpu_device)
    check(base, ref, cfg.tol, "sorted list")
    rng = np.random.default_rng(9)
    for _ in range(4):
        perm = [iv[i] for i in rng.permutation(len(iv))]
        got = run_span(cfg, SpanBatch.from_lists([perm], [1200]), q, K, V, gpu_device, max_tokens=0)
        check(got, ref, cfg.tol, f"permuted list {perm}")
    pieces = [(0, 10), (10, 64), (100, 113), (113, 200), (200, 300), (512, 513), (513, 1000), (1190, 1200)]
    got = run_span(cfg, SpanBatch.from_lists([pieces], [1200]), q, K, V, gpu_device)
    check(got, ref, cfg.tol, "intervals split into touching pieces")


def test_many_intervals_per_sequence(gpu_device):
    """More than 64 intervals per sequence (several metadata chunks), including single-token intervals."""
    cfg = small_cfg("bf16", 128, B=3, H=2, L=4096)
    rng = np.random.default_rng(10)
    per_seq = []
    for k in (65, 200, 1000):
        lens = rng.integers(1, 4, size=k)
        from workloads import place_disjoint
        per_seq.append(place_disjoint(rng, lens, 0, 4096))
    sp = SpanBatch.from_lists(per_seq, [4096] * 3)
    q, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device, seed=11)
    ref = oracle_span(cfg, sp, q, K, V)
    for ns in (0, 1, 3):
        check(run_span(cfg, sp, q, K, V, gpu_device, num_splits=ns), ref, cfg.tol, f"65/200/1000 intervals splits={ns}")


def test_largest_slice_and_max_tokens_bound(gpu_device):
    """Slices far larger than one position-table window (256 rows per wave): whole long sequences per
    workgroup, span and dense, one slice and two."""
    cfg = small_cfg("f16", 128, B=2, H=2, L=9000)
    sp = SpanBatch.from_lists([[(0, 5000)], [(100, 3000), (3500, 8999)]], [9000, 9000])
    q, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device, seed=12)
    ref = oracle_span(cfg, sp, q, K, V)
    for kw in (dict(num_splits=1), dict(num_splits=2), dict()):
        check(run_span(cfg, sp, q, K, V, gpu_device, **kw), ref, cfg.tol, f"slices of thousands of rows {kw}")
    ctx = np.array([9000, 4099], np.int32)
    dref = oracle_dense(cfg, ctx, q, K, V)
    for kw in (dict(num_splits=1), dict(num_splits=2), dict()):
        check(run_dense(cfg, ctx, q, K, V, gpu_device, **kw), dref, cfg.tol, f"dense, thousands of rows per slice {kw}")
    # many short intervals in a slice that spans several windows
    rng = np.random.default_rng(12)
    from workloads import place_disjoint
    iv = place_disjoint(rng, rng.integers(1, 40, size=300), 0, 9000)
    sp2 = SpanBatch.from_lists([iv, iv[:70]], [9000, 9000])
    check(run_span(cfg, sp2, q, K, V, gpu_device, num_splits=1), oracle_span(cfg, sp2, q, K, V), cfg.tol,
          "300 intervals, one slice, several windows")


def test_rows_outside_span_never_reach_output(gpu_device):
    cfg = small_cfg("f16", 128, B=2, H=2, L=256)
    sp = SpanBatch.from_lists([[(10, 20), (100, 140)], [(0, 3), (250, 256)]], [256, 256])
    q, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device, seed=13)
    ref = oracle_span(cfg, sp, q, K, V)
    keep = torch.zeros((2, 256), dtype=torch.bool, device=gpu_device)
    for b in range(2):
        for s, e in sp.intervals(b):
            keep[b, s:e] = True
    K2, V2 = K.clone(), V.clone()
    K2.masked_fill_(~keep[:, None, :, None], float("nan"))
    V2.masked_fill_(~keep[:, None, :, None], float("inf"))
    check(run_span(cfg, sp, q, K2, V2, gpu_device), ref, cfg.tol, "NaN / Inf outside the span")


def test_microbenchmark_masks(gpu_device):
    """Masks of the paper's kernel micro-benchmark (Sec. 5.2): 50 % of the context kept in runs."""
    cfg = DecodeConfig(91, "microbench", 4, 32, 128, 2048, 2048, "f16", 2e-3)
    q, K, V = draw_qkv(cfg, [2048] * 4, device=gpu_device, seed=14)
    for sbs in (32, 64, 128, 256):
        sp = microbench_spans(4, 2048, sbs, seed=sbs)
        check(run_span(cfg, sp, q, K, V, gpu_device), oracle_span(cfg, sp, q, K, V), cfg.tol, f"sparsity block {sbs}")


def test_unstructured_masks_through_the_blocked_encoding(gpu_device):
    """Per-token random masks (the paper's kernel takes any mask, Sec. 5.2): mask -> (block index, bit mask)
    encoding of Sec. 3.3 -> interval list -> kernel, against the additive-mask brute force over all positions."""
    from oracle import blocks as ref_blocks
    from oracle import bruteforce
    cfg = DecodeConfig(92, "bitmask", 3, 2, 128, 600, 600, "f32", 1e-5)
    rng = np.random.default_rng(16)
    q, K, V = draw_qkv(cfg, [600] * 3, device=gpu_device, seed=16)
    attend = np.stack([rng.random(600) < p for p in (0.5, 0.05, 0.97)])
    boff, bidx, bmasks = [0], [], []
    for b in range(3):
        idx, masks = ref_blocks.blocks_from_positions(256, {int(p) for p in np.nonzero(attend[b])[0]})
        bidx += idx
        bmasks.append(masks)
        boff.append(len(bidx))
    off, st, en = span.span_blocks_to_intervals(256, boff, bidx, np.concatenate(bmasks))
    sp = SpanBatch(off, st, en, np.full(3, 600, np.int32))
    assert span.span_validate(sp.offsets, sp.starts, sp.ends, sp.ctx_lens)[0] == 0
    ref = bruteforce.masked_attn_from_bits(q.cpu().numpy(), K.cpu().numpy(), V.cpu().numpy(), attend,
                                           np.float32(cfg.scale))
    check(run_span(cfg, sp, q, K, V, gpu_device), ref, cfg.tol, "random bit masks via blocked encoding")


@pytest.mark.parametrize("L", [1024, 8096])
@pytest.mark.parametrize("run", [1, 2, 16])
def test_unstructured_masks_at_microbenchmark_lengths(L, run, gpu_device):
    """Per-token (run = 1) and short-run random masks at the micro-benchmark's context lengths: up to ~2000
    intervals per sequence travel through the blocked encoding into the interval kernel (64 intervals per chunk,
    256 rows per window), with and without the host copies of the lists."""
    from workloads import random_mask_spans
    cfg = DecodeConfig(97, f"unstructured-{L}-{run}", 4, 32, 128, L, L, "f16", 2e-3)
    sp0 = random_mask_spans(cfg.batch, L, run, seed=L + run)
    boff, bidx, bm = span.span_intervals_to_blocks(256, sp0.offsets, sp0.starts, sp0.ends)
    off, st, en = span.span_blocks_to_intervals(256, boff, bidx, bm)
    sp = SpanBatch(off, st, en, sp0.ctx_lens)
    assert np.array_equal(off, sp0.offsets) and np.array_equal(st, sp0.starts) and np.array_equal(en, sp0.ends)
    q, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device, seed=L + run)
    ref = oracle_span(cfg, sp, q, K, V)
    print(f"[case] L={L} run={run}: {len(st) / cfg.batch:.0f} intervals per sequence", flush=True)
    check(run_span(cfg, sp, q, K, V, gpu_device), ref, cfg.tol, f"unstructured L={L} run={run}")
    check(run_span(cfg, sp, q, K, V, gpu_device, host_spans=(off, st, en)), ref, cfg.tol,
          f"unstructured L={L} run={run}, host lists")
    check(run_span(cfg, sp, q, K, V, gpu_device, tokens_per_seq=None, num_splits=5), ref, cfg.tol,
          f"unstructured L={L} run={run}, 5 slices")


def test_non_default_stream(gpu_device):
    cfg = small_cfg("f16", 128, B=2, H=4, L=512)
    sp = SpanBatch.from_lists([[(0, 100), (400, 512)], [(7, 300)]], [512, 512])
    q, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device, seed=15)
    ref = oracle_span(cfg, sp, q, K, V)
    torch.cuda.synchronize()
    s = torch.cuda.Stream(device=gpu_device)
    with torch.cuda.stream(s):
        got = run_span(cfg, sp, q, K, V, gpu_device, num_splits=3)
    check(got, ref, cfg.tol, "side stream")


@pytest.mark.parametrize("seed", list(range(24)))
def test_random_shapes_and_lists(seed, gpu_device):
    """Random batch shapes, list structures and slicing modes; the case is printed before it runs."""
    from workloads import place_disjoint
    rng = np.random.default_rng(1000 + seed)
    dtype = ["f16", "bf16", "f32"][seed % 3]
    D = [128, 64][(seed // 3) % 2]
    B = int(rng.integers(1, 7))
    H = int(rng.choice([1, 3, 8, 32]))
    L = int(rng.choice([33, 257, 1500, 6000]))
    cfg = DecodeConfig(200 + seed, "random", B, H, D, L, L, dtype, TOL[dtype])
    ctx = rng.integers(1, L + 1, size=B).astype(np.int32)
    per_seq = []
    for b in range(B):
        n = int(ctx[b])
        k = int(rng.integers(1, min(n, 90) + 1))
        style = rng.integers(0, 3)
        hi = 1 if style == 0 else (max(1, n // k) if style == 1 else max(1, min(n // k, 7)))
        lens = rng.integers(1, hi + 1, size=k)
        per_seq.append(place_disjoint(rng, lens, 0, n))
    sp = SpanBatch.from_lists(per_seq, ctx)
    mode = seed % 4
    kw = [dict(), dict(tokens_per_seq=None), dict(num_splits=int(rng.integers(1, 9))), dict(tokens_per_seq=None, max_tokens=0)][mode]
    print(f"[case] seed {seed}: {dtype} D={D} B={B} H={H} L={L} ctx={ctx.tolist()} intervals={[len(p) for p in per_seq]} "
          f"tokens={sp.tokens_per_seq().tolist()} kw={kw}", flush=True)
    q, K, V = draw_qkv(cfg, ctx, device=gpu_device, seed=seed)
    check(run_span(cfg, sp, q, K, V, gpu_device, **kw), oracle_span(cfg, sp, q, K, V), cfg.tol, f"random case {seed} span")
    dkw = {k: v for k, v in kw.items() if k != "max_tokens"}
    check(run_dense(cfg, ctx, q, K, V, gpu_device, **dkw), oracle_dense(cfg, ctx, q, K, V), cfg.tol,
          f"random case {seed} dense")


def test_largest_supported_cache_length(gpu_device):
    """max_len = 2^22 rows with 512-byte rows (fp32, D=128): a 2 GiB slab per (batch, head), so in-slab byte
    offsets use all 31 bits; the span touches the first and the very last rows."""
    L = 1 << 22
    cfg = DecodeConfig(96, "maxlen", 1, 1, 128, L, L, "f32", 1e-5)
    g = torch.Generator(device=gpu_device).manual_seed(96)
    q = torch.randn((1, 1, 128), generator=g, device=gpu_device)
    K = torch.full((1, 1, L, 128), float("nan"), device=gpu_device)
    V = torch.full((1, 1, L, 128), float("nan"), device=gpu_device)
    iv = [(0, 40), (L // 2 - 3, L // 2 + 70), (L - 300, L)]
    for s, e in iv:
        K[0, 0, s:e] = torch.randn((e - s, 128), generator=g, device=gpu_device)
        V[0, 0, s:e] = torch.randn((e - s, 128), generator=g, device=gpu_device)
    sp = SpanBatch.from_lists([iv], [L])
    assert span.span_validate(sp.offsets, sp.starts, sp.ends, sp.ctx_lens)[0] == 0
    hq, hK, hV = q.cpu().numpy(), K.cpu().numpy(), V.cpu().numpy()
    ref = oracle.span_attn(hq, hK, hV, sp.offsets, sp.starts, sp.ends, np.float32(cfg.scale), dtype="f32")
    for kw in (dict(), dict(num_splits=3), dict(tokens_per_seq=None, max_tokens=0)):
        check(run_span(cfg, sp, q, K, V, gpu_device, **kw), ref, cfg.tol, f"max_len 2^22 {kw}")
    from paper_2404_09336_amd import binding
    lib = span.load_library()
    d = binding.make_desc(1, 1, 128, L + 1, 0)
    assert lib.span_workspace_bytes(d) == 0 and span.span_strerror(-2)        # one row more is refused
    with pytest.raises(span.SpanAttnError):
        span.span_plan_query(d)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_large_and_tiny_scores(dtype, gpu_device):
    """Scores far outside exp's comfortable range: peaky softmax (|s| in the hundreds), all scores hugely
    negative, all scores ~0 with subnormal inputs.  Only differences of scores matter (eq. (5)); nothing may
    overflow, underflow to 0/0 or turn into NaN, with one slice or several."""
    cfg = small_cfg(dtype, 128, B=3, H=4, L=900, min_len=900)
    sp = SpanBatch.from_lists([[(0, 40), (300, 700)], [(5, 6)], [(100, 900)]], [900, 900, 900])
    q, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device, seed=11)
    cases = {
        "peaky": (q * 12, K * 6),                                   # scores ~ N(0, 72 * sqrt(128)) * scale
        "all very negative": (q.abs() * 20, -K.abs() * 20),          # every product negative: scores ~ -3e3
        "tiny": (q * 1e-4, K * 1e-4 if dtype != "f16" else K * 1e-3),   # fp16: K * 1e-3 is partly subnormal
    }
    for name, (qq, KK) in cases.items():
        qq, KK = qq.to(q.dtype).contiguous(), KK.to(K.dtype).contiguous()
        ref = oracle_span(cfg, sp, qq, KK, V)
        for kw in (dict(), dict(num_splits=5, tokens_per_seq=None)):
            check(run_span(cfg, sp, qq, KK, V, gpu_device, **kw), ref, cfg.tol, f"{dtype} {name} {kw}")
