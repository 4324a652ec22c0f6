"""Fused KV-append + attention (the step before the path in a decode loop, Sec. 2.2 "KV-cache"): parity with
the oracle run on the updated cache, and the cache itself bit-exact."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_09336_amd as span
from workloads import DecodeConfig, SpanBatch, draw_qkv, to_host_raw

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-5, "f16": 2e-3, "bf16": 2e-3}


def _dev(a, device):
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def _bits(t):
    a = to_host_raw(t)
    return a.view(np.uint32) if a.dtype == np.float32 else a


def _updated(K, k_new, pos):
    K2 = K.clone()
    for b, p in enumerate(pos):
        if 0 <= p < K.shape[2]:
            K2[b, :, p, :] = k_new[b]
    return K2


def run_case(dtype, D, per_seq, ctx, pos, device, seed, num_splits=0, max_len=None, dense=False):
    B, H = len(ctx), 3
    L = max_len or int(max(ctx))
    cfg = DecodeConfig(95, "append", B, H, D, L, L, dtype, TOL[dtype])
    q, K, V = draw_qkv(cfg, np.asarray(ctx, np.int32), device=device, seed=seed)   # rows >= ctx are NaN, incl. append_pos
    g = torch.Generator(device=device).manual_seed(seed + 1)
    k_new = torch.randn((B, H, D), generator=g, device=device).to(K.dtype)
    v_new = torch.randn((B, H, D), generator=g, device=device).to(K.dtype)
    new_ctx = np.asarray([max(c, p + 1) if 0 <= p < L else c for c, p in zip(ctx, pos)], np.int32)
    K_ref, V_ref = _updated(K, k_new, pos), _updated(V, v_new, pos)
    if dense:
        out = span.dense_decode_attn_append(q, k_new, v_new, K, V, _dev(np.asarray(pos, np.int32), device),
                                            _dev(new_ctx, device), np.float32(cfg.scale), num_splits=num_splits,
                                            tokens_per_seq=new_ctx.astype(np.int64) if num_splits == 0 else None)
        ref = oracle.dense_attn(to_host_raw(q), to_host_raw(K_ref), to_host_raw(V_ref), new_ctx, np.float32(cfg.scale),
                                dtype=dtype)
    else:
        sp = SpanBatch.from_lists(per_seq, new_ctx)
        code, _, _, tok = span.span_validate(sp.offsets, sp.starts, sp.ends, sp.ctx_lens)
        assert code == 0
        out = span.span_decode_attn_append(q, k_new, v_new, K, V, _dev(np.asarray(pos, np.int32), device),
                                           _dev(sp.offsets, device), _dev(sp.starts, device), _dev(sp.ends, device),
                                           np.float32(cfg.scale), num_splits=num_splits, max_tokens=int(tok.max()),
                                           tokens_per_seq=tok if num_splits == 0 else None)
        ref = oracle.span_attn(to_host_raw(q), to_host_raw(K_ref), to_host_raw(V_ref), sp.offsets, sp.starts, sp.ends,
                               np.float32(cfg.scale), dtype=dtype)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    err = float(np.abs(got - ref).max())
    print(f"[parity] append {dtype} D={D} splits={num_splits} dense={dense}: max-abs err {err:.3e}", flush=True)
    assert err <= TOL[dtype]
    # the caches now hold the new rows, everything else untouched (NaN rows compared as bits)
    assert np.array_equal(_bits(K), _bits(K_ref)) and np.array_equal(_bits(V), _bits(V_ref))


@pytest.mark.parametrize("dtype,D", [("f16", 128), ("bf16", 128), ("f32", 64), ("f32", 128), ("f16", 64)])
def test_append_inside_recent_interval(dtype, D, gpu_device):
    ctx = [200, 77, 300]                       # rows held before the new token
    pos = [200, 77, 300]                       # the new token goes right behind them
    per_seq = [[(0, 16), (50, 90), (180, 201)], [(70, 78)], [(0, 301)]]
    for ns in (0, 1, 3):
        run_case(dtype, D, per_seq, ctx, pos, gpu_device, seed=41, num_splits=ns, max_len=320)


def test_append_dense_and_ragged(gpu_device):
    for ns in (0, 1, 4):
        run_case("f16", 128, None, [511, 1, 130, 64], [511, 1, 130, 64], gpu_device, seed=42, num_splits=ns,
                 max_len=512, dense=True)


def test_append_only_position_and_not_in_span(gpu_device):
    # sequence 0: the span is just the new token; sequence 1: the new row is written but not attended;
    # sequence 2: append_pos out of range -> nothing is appended
    run_case("f16", 128, [[(10, 11)], [(0, 5)], [(0, 5)]], [10, 10, 10], [10, 10, -1], gpu_device, seed=43, max_len=64)
    # overwrite a row in the middle of an attended interval
    run_case("bf16", 128, [[(0, 40)], [(3, 9), (20, 30)]], [40, 30], [17, 25], gpu_device, seed=44, max_len=64)


def test_append_at_workload_scale(gpu_device):
    from workloads import CONFIGS, draw_spans
    cfg = CONFIGS[3]
    sp = draw_spans(cfg)
    ctx_before = sp.ctx_lens - 1                              # the last attended position is the new token
    q, K, V = draw_qkv(cfg, ctx_before, device=gpu_device)
    g = torch.Generator(device=gpu_device).manual_seed(5)
    k_new = torch.randn(q.shape, generator=g, device=gpu_device).to(K.dtype)
    v_new = torch.randn(q.shape, generator=g, device=gpu_device).to(K.dtype)
    pos = ctx_before.astype(np.int32)
    K_ref, V_ref = _updated(K, k_new, pos), _updated(V, v_new, pos)
    tok = sp.tokens_per_seq()
    out = span.span_decode_attn_append(q, k_new, v_new, K, V, _dev(pos, gpu_device), _dev(sp.offsets, gpu_device),
                                       _dev(sp.starts, gpu_device), _dev(sp.ends, gpu_device), np.float32(cfg.scale),
                                       max_tokens=int(tok.max()), tokens_per_seq=tok)
    torch.cuda.synchronize()
    ref = oracle.span_attn(to_host_raw(q), to_host_raw(K_ref), to_host_raw(V_ref), sp.offsets, sp.starts, sp.ends,
                           np.float32(cfg.scale), dtype=cfg.dtype)
    err = float(np.abs(out.cpu().numpy() - ref).max())
    print(f"[parity] append at config 3 scale: max-abs err {err:.3e}")
    assert err <= cfg.tol
    assert np.array_equal(_bits(K), _bits(K_ref))


def test_append_happens_even_when_nothing_is_attended(gpu_device):
    """A sequence whose span is empty (the validator would flag it) or whose ctx_len is 0 gets an all-zero output
    row, and its new K / V row is in the cache all the same."""
    B, H, D, L = 3, 3, 128, 64
    cfg = DecodeConfig(97, "append-empty", B, H, D, L, L, "f16", 2e-3)
    q, K, V = draw_qkv(cfg, np.array([20, 20, 20], np.int32), device=gpu_device, seed=45)
    g = torch.Generator(device=gpu_device).manual_seed(46)
    k_new = torch.randn((B, H, D), generator=g, device=gpu_device).half()
    v_new = torch.randn((B, H, D), generator=g, device=gpu_device).half()
    pos = [20, 20, 20]
    K_ref, V_ref = _updated(K, k_new, pos), _updated(V, v_new, pos)
    off = np.array([0, 1, 1, 2], np.int32)                        # sequence 1 has no interval
    st, en = np.array([0, 5], np.int32), np.array([21, 21], np.int32)
    for ns in (0, 3):
        Kc, Vc = K.clone(), V.clone()
        out = span.span_decode_attn_append(q, k_new, v_new, Kc, Vc, _dev(np.asarray(pos, np.int32), gpu_device),
                                           _dev(off, gpu_device), _dev(st, gpu_device), _dev(en, gpu_device),
                                           np.float32(cfg.scale), num_splits=ns)
        torch.cuda.synchronize()
        ref = oracle.span_attn(to_host_raw(q), to_host_raw(K_ref), to_host_raw(V_ref), off, st, en,
                               np.float32(cfg.scale), dtype="f16")
        got = out.cpu().numpy().astype(np.float64)
        assert np.array_equal(got[1], np.zeros_like(got[1])) and np.abs(got - ref).max() <= cfg.tol
        assert np.array_equal(_bits(Kc), _bits(K_ref)) and np.array_equal(_bits(Vc), _bits(V_ref))
        Kc, Vc = K.clone(), V.clone()
        ctx = np.array([21, 0, 21], np.int32)                     # dense form: sequence 1 claims no rows
        out = span.dense_decode_attn_append(q, k_new, v_new, Kc, Vc, _dev(np.asarray(pos, np.int32), gpu_device),
                                            _dev(ctx, gpu_device), np.float32(cfg.scale), num_splits=ns)
        torch.cuda.synchronize()
        ref = oracle.dense_attn(to_host_raw(q), to_host_raw(K_ref), to_host_raw(V_ref), ctx, np.float32(cfg.scale),
                                dtype="f16")
        got = out.cpu().numpy().astype(np.float64)
        assert np.array_equal(got[1], np.zeros_like(got[1])) and np.abs(got - ref).max() <= cfg.tol
        assert np.array_equal(_bits(Kc), _bits(K_ref)) and np.array_equal(_bits(Vc), _bits(V_ref))
