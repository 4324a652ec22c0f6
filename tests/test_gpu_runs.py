"""Run mode (the caller also hands in host copies of the span lists; the slices' position runs then travel in the
kernel arguments): same plan, same rows per wave, same arithmetic order as the device-list path, so the outputs
must be equal bit for bit; the fp64 oracle bounds them both.  All calls go through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_09336_amd as span
from workloads import (CONFIGS, DecodeConfig, SpanBatch, draw_qkv, draw_queries, draw_spans, place_disjoint,
                       to_host_raw)

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-5, "f16": 2e-3, "bf16": 2e-3}


def _dev(a, device):
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def both_paths(cfg, sp, q, K, V, device, expect_runs=None, **kw):
    """Returns (output with host lists, output without, oracle); asserts the first two are identical."""
    lists = [_dev(a, device) for a in (sp.offsets, sp.starts, sp.ends, sp.ctx_lens)]
    tok = sp.tokens_per_seq()
    kw.setdefault("max_tokens", int(tok.max()))
    with_lists = span.prepare_span_decode_attn(q, K, V, *lists, np.float32(cfg.scale),
                                               host_spans=(sp.offsets, sp.starts, sp.ends), **kw)
    plan = span.span_plan_query(with_lists.desc)
    if expect_runs is not None:
        assert plan["runs_in_arguments"] == expect_runs, plan
    a = with_lists().clone()
    b = span.span_decode_attn(q, K, V, *lists, np.float32(cfg.scale), tokens_per_seq=tok, **kw)
    torch.cuda.synchronize()
    assert torch.equal(a, b), "run mode differs from the device-list path"
    ref = oracle.span_attn(to_host_raw(q), to_host_raw(K), to_host_raw(V), sp.offsets, sp.starts, sp.ends,
                           np.float32(cfg.scale), dtype=cfg.dtype)
    got = a.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    err = float(np.abs(got - ref).max())
    print(f"[parity] run mode {cfg.name}: runs_in_arguments={plan['runs_in_arguments']} workgroups={plan['workgroups']} "
          f"max-abs err {err:.3e} (tol {cfg.tol:g})", flush=True)
    assert err <= cfg.tol
    return plan


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_workloads_with_host_lists(cid, gpu_device):
    """Configs 2 and 4 are sliced raggedly and fit the run tables.  Configs 1 and 3 need no slice table (every
    sequence is one slice), and config 5 does not fit (slices of > 1024 positions): those take the device lists,
    with the token counts taken from the host lists."""
    cfg = CONFIGS[cid]
    for copy in range(2):
        sp = draw_spans(cfg, seed=cfg.seed(copy))
        q, K, V = draw_qkv(cfg, sp.ctx_lens, seed=cfg.seed(copy), device=gpu_device)
        both_paths(cfg, sp, q, K, V, gpu_device, expect_runs=cid in (2, 4))


def ragged_batch(rng, B, L, lo, hi):
    """B sequences with different numbers of attended positions in [lo, hi], 1-6 intervals each."""
    per_seq = []
    for b in range(B):
        n_tok = int(rng.integers(lo, hi + 1)) if b else hi
        k = min(n_tok, int(rng.integers(1, 7)))
        cuts = np.sort(rng.choice(np.arange(1, n_tok), size=k - 1, replace=False)) if k > 1 else np.array([], int)
        per_seq.append(place_disjoint(rng, np.diff(np.concatenate(([0], cuts, [n_tok]))), 0, L))
    return SpanBatch.from_lists(per_seq, np.full(B, L, np.int32))


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("D", [64, 128])
def test_every_instance_and_slice_shape(dtype, D, gpu_device):
    """All (type, head_dim) instances on ragged batches whose slices are tiny (single rows), quarters (< 384 rows)
    and interleaved (>= 384 rows, up to the 1024 rows the mode takes per slice), and one batch past that limit."""
    rng = np.random.default_rng(D + len(dtype))
    # (sequences, heads, cache length, fewest and most attended positions, expected mode)
    for B, H, L, lo, hi, expect in ((3, 5, 300, 1, 130, None), (4, 32, 1500, 100, 1400, True),
                                    (8, 32, 3000, 500, 1900, None), (8, 32, 9000, 5000, 8990, None),
                                    (6, 64, 9000, 7000, 8990, False)):
        cfg = DecodeConfig(96, f"runs-{dtype}-{D}-{hi}", B, H, D, L, L, dtype, TOL[dtype])
        sp = ragged_batch(rng, B, L, lo, hi)
        q, K, V = draw_qkv(cfg, sp.ctx_lens, seed=hi + D, device=gpu_device)
        plan = both_paths(cfg, sp, q, K, V, gpu_device, expect_runs=expect)
        print(f"[plan] B={B} H={H} tokens {lo}..{hi}: {plan}", flush=True)
        del q, K, V


@pytest.mark.parametrize("seed", list(range(16)))
def test_random_lists(seed, gpu_device):
    """Random shapes and list structures, ragged lengths, unsorted and touching intervals; the case is printed."""
    rng = np.random.default_rng(7000 + seed)
    dtype = ["f16", "bf16", "f32"][seed % 3]
    D = [128, 64][(seed // 3) % 2]
    B, H = int(rng.integers(1, 9)), int(rng.choice([1, 4, 32, 40]))
    L = int(rng.choice([60, 700, 3000]))
    cfg = DecodeConfig(400 + seed, "random-runs", B, H, D, L, L, dtype, TOL[dtype])
    ctx = rng.integers(max(2, L // 3), L + 1, size=B).astype(np.int32)
    per_seq = []
    for b in range(B):
        n = int(ctx[b])
        k = int(rng.integers(1, min(n, 30) + 1))
        hi = max(1, n // k) if seed % 2 else max(1, min(n // k, 9))
        iv = place_disjoint(rng, rng.integers(1, hi + 1, size=k), 0, n)
        if seed % 4 == 3:
            rng.shuffle(iv)                                  # the kernel takes any order of disjoint intervals
        per_seq.append([tuple(int(x) for x in p) for p in iv])
    sp = SpanBatch.from_lists(per_seq, ctx)
    print(f"[case] seed {seed}: {dtype} D={D} B={B} H={H} L={L} ctx={ctx.tolist()} "
          f"intervals={[len(p) for p in per_seq]}", flush=True)
    q, K, V = draw_qkv(cfg, ctx, seed=seed, device=gpu_device)
    both_paths(cfg, sp, q, K, V, gpu_device)


def test_few_query_append_and_static_calls_take_host_lists(gpu_device):
    cfg = CONFIGS[2]
    sp = draw_spans(cfg)
    tok = sp.tokens_per_seq()
    q1, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device)
    lists = [_dev(a, gpu_device) for a in (sp.offsets, sp.starts, sp.ends)]
    host = (sp.offsets, sp.starts, sp.ends)
    kw = dict(max_tokens=int(tok.max()))
    for q_len in (2, 4, 6):
        q = draw_queries(cfg, q_len, device=gpu_device)
        q_pos = _dev((sp.ctx_lens - q_len).astype(np.int32), gpu_device)
        a = span.span_decode_attn_multi(q, K, V, *lists, q_pos, np.float32(cfg.scale), host_spans=host, **kw)
        b = span.span_decode_attn_multi(q, K, V, *lists, q_pos, np.float32(cfg.scale), tokens_per_seq=tok, **kw)
        torch.cuda.synchronize()
        assert torch.equal(a, b), f"few-query call, {q_len} tokens"
    # static scratch
    out = torch.empty_like(q1, dtype=torch.float32)
    ctx = _dev(sp.ctx_lens, gpu_device)
    a = span.span_decode_attn_static(q1, K, V, *lists, ctx, np.float32(cfg.scale), out, host_spans=host, **kw).clone()
    b = span.span_decode_attn(q1, K, V, *lists, ctx, np.float32(cfg.scale), tokens_per_seq=tok, **kw)
    torch.cuda.synchronize()
    assert torch.equal(a, b), "static-scratch call"
    # append: the new token overwrites the last cache row of every sequence
    g = torch.Generator(device=gpu_device).manual_seed(5)
    k_new = torch.randn(q1.shape, generator=g, device=gpu_device).to(K.dtype)
    v_new = torch.randn(q1.shape, generator=g, device=gpu_device).to(K.dtype)
    pos = _dev((sp.ctx_lens - 1).astype(np.int32), gpu_device)
    Ka, Va, Kb, Vb = K.clone(), V.clone(), K.clone(), V.clone()
    a = span.span_decode_attn_append(q1, k_new, v_new, Ka, Va, pos, *lists, np.float32(cfg.scale), host_spans=host, **kw)
    b = span.span_decode_attn_append(q1, k_new, v_new, Kb, Vb, pos, *lists, np.float32(cfg.scale), tokens_per_seq=tok, **kw)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(Ka.view(torch.int16), Kb.view(torch.int16))
    K2, V2 = K.clone(), V.clone()
    for i in range(cfg.batch):
        K2[i, :, int(sp.ctx_lens[i]) - 1] = k_new[i]
        V2[i, :, int(sp.ctx_lens[i]) - 1] = v_new[i]
    ref = oracle.span_attn(to_host_raw(q1), to_host_raw(K2), to_host_raw(V2), sp.offsets, sp.starts, sp.ends,
                           np.float32(cfg.scale), dtype=cfg.dtype)
    assert float(np.abs(a.cpu().numpy().astype(np.float64) - ref).max()) <= cfg.tol


def test_dense_call_ignores_host_lists(gpu_device):
    """A descriptor reused for the dense control may still carry the host lists: they mean nothing there."""
    import ctypes
    from paper_2404_09336_amd.binding import make_desc
    cfg = CONFIGS[1]
    sp = draw_spans(cfg)
    q, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device)
    ctx = _dev(sp.ctx_lens, gpu_device)
    ref = span.dense_decode_attn(q, K, V, ctx, np.float32(cfg.scale), num_splits=1)
    d = make_desc(cfg.batch, cfg.heads, cfg.head_dim, cfg.max_len, 0, int(sp.starts.size), num_splits=1,
                  stream=torch.cuda.current_stream(gpu_device).cuda_stream, host_spans=(sp.offsets, sp.starts, sp.ends))
    out = torch.zeros_like(ref)
    rc = span.load_library().dense_decode_attn(ctypes.byref(d), q.data_ptr(), K.data_ptr(), V.data_ptr(),
                                               ctx.data_ptr(), float(np.float32(cfg.scale)), out.data_ptr())
    torch.cuda.synchronize()
    assert rc == 0 and torch.equal(out, ref)
