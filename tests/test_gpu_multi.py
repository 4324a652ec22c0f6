"""Parity of the few-query entry point (several new tokens of a sequence share its span, each under the
causal limit) against the fp64 oracle, through the C ABI.  Same tolerances as the single-query path."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_09336_amd as span
from workloads import CONFIGS, DecodeConfig, SpanBatch, draw_qkv, draw_queries, draw_spans, to_host_raw

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "f16": 2e-3, "bf16": 2e-3}


def _dev(a, device):
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def run_multi(cfg, sp, q, K, V, q_pos, device, **kw):
    code, _, _, tok = span.span_validate(sp.offsets, sp.starts, sp.ends, sp.ctx_lens)
    assert code == 0
    kw.setdefault("max_tokens", int(tok.max()))
    kw.setdefault("tokens_per_seq", tok)
    out = span.span_decode_attn_multi(q, K, V, _dev(sp.offsets, device), _dev(sp.starts, device),
                                      _dev(sp.ends, device), None if q_pos is None else _dev(q_pos, device),
                                      np.float32(cfg.scale), **kw)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


def oracle_multi(cfg, sp, q, K, V, q_pos):
    return oracle.span_attn_multi(to_host_raw(q), to_host_raw(K), to_host_raw(V), sp.offsets, sp.starts, sp.ends,
                                  q_pos, np.float32(cfg.scale), dtype=cfg.dtype)


def check(got, ref, tol, what):
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = float(np.abs(got - ref).max())
    print(f"[parity] {what}: max-abs err {err:.3e} (tol {tol:g})", flush=True)
    assert err <= tol, f"{what}: max-abs err {err:.3e} > {tol:g}"


def new_tokens_at_the_end(sp, q_len):
    """The q_len new tokens are the last q_len cache rows of each sequence; token 0 sits at ctx_len - q_len."""
    return (sp.ctx_lens.astype(np.int64) - q_len).astype(np.int32)


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("q_len", [2, 4, 16])
def test_workload_multi_parity(cid, q_len, gpu_device):
    """The five workloads: every span ends with the recent-token interval, so the new tokens are inside it."""
    cfg = CONFIGS[cid]
    sp = draw_spans(cfg)
    _, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device)
    q = draw_queries(cfg, q_len, device=gpu_device)
    q_pos = new_tokens_at_the_end(sp, q_len)
    ref = oracle_multi(cfg, sp, q, K, V, q_pos)
    check(run_multi(cfg, sp, q, K, V, q_pos, gpu_device), ref, cfg.tol, f"config {cid}, {q_len} query tokens")
    check(run_multi(cfg, sp, q, K, V, q_pos, gpu_device, tokens_per_seq=None), ref, cfg.tol,
          f"config {cid}, {q_len} query tokens, uniform grid")


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("q_len", [1, 2, 3, 4, 5, 8, 13, 16, 17, 40])
def test_multi_all_kernel_instances(dtype, D, q_len, gpu_device):
    """Every (type, head_dim) instance, token counts that pad a pass (3), fill it (2, 4) and need several (5, 8);
    ragged sequences, forced slicing so that the cross-workgroup merge runs per query token."""
    cfg = DecodeConfig(91, "multi", 3, 5, D, 700, 300, dtype, TOL[dtype])
    rng = np.random.default_rng(100 * D + q_len)
    ctx = rng.integers(cfg.min_len, cfg.max_len + 1, size=cfg.batch).astype(np.int32)
    per_seq = []
    for b in range(cfg.batch):
        n = int(ctx[b])
        a = int(rng.integers(1, 40))
        s1 = int(rng.integers(a + 1, n // 2))
        e1 = int(rng.integers(s1 + 1, n // 2 + 60))
        per_seq.append([(0, a), (s1, e1), (n - 37, n)])
    sp = SpanBatch.from_lists(per_seq, ctx)
    _, K, V = draw_qkv(cfg, ctx, seed=cfg.seed() + q_len, device=gpu_device)
    q = draw_queries(cfg, q_len, device=gpu_device)
    q_pos = new_tokens_at_the_end(sp, q_len)
    ref = oracle_multi(cfg, sp, q, K, V, q_pos)
    check(run_multi(cfg, sp, q, K, V, q_pos, gpu_device), ref, cfg.tol, f"{dtype} D={D} q_len={q_len}")
    for splits in (3, 7):
        check(run_multi(cfg, sp, q, K, V, q_pos, gpu_device, num_splits=splits, tokens_per_seq=None), ref, cfg.tol,
              f"{dtype} D={D} q_len={q_len} splits={splits}")
    ref_all = oracle_multi(cfg, sp, q, K, V, None)
    check(run_multi(cfg, sp, q, K, V, None, gpu_device), ref_all, cfg.tol, f"{dtype} D={D} q_len={q_len} no limit")


def test_multi_limit_cases(gpu_device):
    """Limits that fall before the span (zero rows), inside an interval, in a gap, and beyond the cache."""
    cfg = DecodeConfig(92, "multi-limits", 5, 4, 128, 600, 600, "f16", 2e-3)
    ctx = np.full(cfg.batch, 600, np.int32)
    per_seq = [[(10, 50), (300, 420)]] * cfg.batch
    sp = SpanBatch.from_lists(per_seq, ctx)
    _, K, V = draw_qkv(cfg, ctx, device=gpu_device)
    q = draw_queries(cfg, 4, device=gpu_device)
    q_pos = np.array([5, 8, 48, 100, 2**31 - 1], np.int32)   # nothing / first rows appear / interval end / gap / all (no overflow)
    ref = oracle_multi(cfg, sp, q, K, V, q_pos)
    got = run_multi(cfg, sp, q, K, V, q_pos, gpu_device)
    check(got, ref, cfg.tol, "limit cases")
    assert np.array_equal(got[0], np.zeros_like(got[0]))            # tokens at 5..8 see nothing of [10, 50)
    assert np.array_equal(got[1, :2], np.zeros_like(got[1, :2]))    # tokens at 8, 9 see nothing; 10, 11 do
    assert np.abs(got[1, 2:]).max() > 0
    for splits in (2, 5):
        check(run_multi(cfg, sp, q, K, V, q_pos, gpu_device, num_splits=splits, tokens_per_seq=None), ref, cfg.tol,
              f"limit cases, {splits} slices")


def test_one_token_through_the_multi_entry_equals_the_decode_call(gpu_device):
    cfg = CONFIGS[2]
    sp = draw_spans(cfg)
    q1, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device)
    dev = lambda a: _dev(a, gpu_device)
    tok = sp.tokens_per_seq()
    single = span.span_decode_attn(q1, K, V, dev(sp.offsets), dev(sp.starts), dev(sp.ends), dev(sp.ctx_lens),
                                   np.float32(cfg.scale), max_tokens=int(tok.max()), tokens_per_seq=tok)
    multi = span.span_decode_attn_multi(q1[:, None].contiguous(), K, V, dev(sp.offsets), dev(sp.starts),
                                        dev(sp.ends), None, np.float32(cfg.scale), max_tokens=int(tok.max()),
                                        tokens_per_seq=tok)
    torch.cuda.synchronize()
    assert torch.equal(single, multi[:, 0])
    # with a limit: one token that may not see the last 10 rows of its span
    q_pos = (sp.ctx_lens - 11).astype(np.int32)
    got = run_multi(cfg, sp, q1[:, None].contiguous(), K, V, q_pos, gpu_device)
    check(got, oracle_multi(cfg, sp, q1[:, None].contiguous(), K, V, q_pos), cfg.tol, "one token with a limit")


def test_single_query_entry_points_reject_several_tokens(gpu_device):
    cfg = CONFIGS[1]
    sp = draw_spans(cfg)
    q, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device)
    lib = span.load_library()
    from paper_2404_09336_amd.binding import make_desc
    import ctypes
    d = make_desc(cfg.batch, cfg.heads, cfg.head_dim, cfg.max_len, 0, int(sp.starts.size), q_len=2)
    out = torch.zeros((cfg.batch, cfg.heads, cfg.head_dim), device=gpu_device)
    dev = lambda a: _dev(a, gpu_device)
    off, st, en = dev(sp.offsets), dev(sp.starts), dev(sp.ends)
    rc = lib.span_decode_attn(ctypes.byref(d), q.data_ptr(), K.data_ptr(), V.data_ptr(), off.data_ptr(),
                              st.data_ptr(), en.data_ptr(), None, 0.1, out.data_ptr())
    assert rc == -2   # SPAN_ERR_SHAPE
    d.q_len = 65
    rc = lib.span_decode_attn_multi(ctypes.byref(d), q.data_ptr(), K.data_ptr(), V.data_ptr(), off.data_ptr(),
                                    st.data_ptr(), en.data_ptr(), None, 0.1, out.data_ptr())
    assert rc == -2


@pytest.mark.parametrize("seed", list(range(18)))
def test_multi_random_shapes_and_lists(seed, gpu_device):
    """Random shapes, list structures (up to 90 intervals, single positions, long runs), token counts, limits and
    slicing modes; the case is printed before it runs."""
    from workloads import place_disjoint
    rng = np.random.default_rng(3000 + seed)
    dtype = ["f16", "bf16", "f32"][seed % 3]
    D = [128, 64][(seed // 3) % 2]
    B, H = int(rng.integers(1, 6)), int(rng.choice([1, 3, 8, 32]))
    L = int(rng.choice([40, 300, 1500, 5000]))
    q_len = int(rng.integers(1, 10)) if seed % 3 else int(rng.integers(10, 36))
    cfg = DecodeConfig(300 + seed, "random-multi", B, H, D, L, L, dtype, TOL[dtype])
    ctx = rng.integers(q_len + 1, L + 1, size=B).astype(np.int32)
    per_seq = []
    for b in range(B):
        n = int(ctx[b])
        k = int(rng.integers(1, min(n, 90) + 1))
        style = rng.integers(0, 3)
        hi = 1 if style == 0 else (max(1, n // k) if style == 1 else max(1, min(n // k, 7)))
        per_seq.append(place_disjoint(rng, rng.integers(1, hi + 1, size=k), 0, n))
    sp = SpanBatch.from_lists(per_seq, ctx)
    limit_style = seed % 3          # tokens at the end of the cache / anywhere (also before the span) / no limit
    q_pos = [(ctx - q_len).astype(np.int32), rng.integers(-3, L, size=B).astype(np.int32), None][limit_style]
    kw = [dict(), dict(tokens_per_seq=None), dict(num_splits=int(rng.integers(1, 9)), tokens_per_seq=None)][(seed // 3) % 3]
    print(f"[case] seed {seed}: {dtype} D={D} B={B} H={H} L={L} q_len={q_len} ctx={ctx.tolist()} "
          f"intervals={[len(p) for p in per_seq]} q_pos={None if q_pos is None else q_pos.tolist()} kw={kw}", flush=True)
    _, K, V = draw_qkv(cfg, ctx, device=gpu_device, seed=seed)
    q = draw_queries(cfg, q_len, device=gpu_device)
    check(run_multi(cfg, sp, q, K, V, q_pos, gpu_device, **kw), oracle_multi(cfg, sp, q, K, V, q_pos), cfg.tol,
          f"random few-query case {seed}")


def _poison(K, V, b, rows, gpu_device):
    """NaN into K and alternating +Inf / -Inf into V on the given cache rows of sequence b (all heads)."""
    idx = torch.as_tensor(rows, device=gpu_device, dtype=torch.long)
    K[b, :, idx] = float("nan")
    sign = torch.where(idx % 2 == 0, 1.0, -1.0).to(V.dtype)
    V[b, :, idx] = (sign * float("inf"))[None, :, None].expand(V.shape[1], -1, V.shape[3])


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("q_len", [1, 2, 3, 4, 6, 11, 16, 21])
def test_poisoned_span_rows_past_the_limits_have_no_influence(dtype, D, q_len, gpu_device):
    """GPU twin of the oracle pin of the same name (masked positions have no influence, Sec. 2.2 mask paragraph).
    Span rows after the last query token's causal limit hold NaN (K) and +-Inf (V), as an uninitialised
    pre-allocated cache may: every output row must still equal the oracle's, which never looks at them.  Runs the
    one-token call with a limit, the 2- and 4-token kernels, padded and multi-pass token counts, unsplit and sliced."""
    cfg = DecodeConfig(93, "multi-poison", 3, 4, D, 420, 330, dtype, TOL[dtype])
    rng = np.random.default_rng(500 + q_len)
    ctx = rng.integers(cfg.min_len, cfg.max_len + 1, size=cfg.batch).astype(np.int32)
    per_seq, q_pos, hidden = [], [], []
    for b in range(cfg.batch):
        n = int(ctx[b])
        tail = int(rng.integers(40, 90))                      # the recent interval [n - tail, n)
        per_seq.append([(0, 17), (60 + 11 * b, 150 + 7 * b), (n - tail, n)])
        p0 = [n - tail + 5, 100 + 7 * b, n - q_len - 9][b]     # limit inside the tail / inside the middle interval / near the end
        q_pos.append(p0)
        last_seen = p0 + q_len - 1
        hidden.append([p for s, e in per_seq[b] for p in range(s, e) if p > last_seen])
        assert hidden[b], "every sequence needs span rows past its last limit"
    sp = SpanBatch.from_lists(per_seq, ctx)
    q_pos = np.array(q_pos, np.int32)
    _, K, V = draw_qkv(cfg, ctx, seed=cfg.seed() + q_len, device=gpu_device)
    q = draw_queries(cfg, q_len, device=gpu_device)
    clean = oracle_multi(cfg, sp, q, K, V, q_pos)
    for b in range(cfg.batch):
        _poison(K, V, b, hidden[b], gpu_device)
    ref = oracle_multi(cfg, sp, q, K, V, q_pos)
    assert np.array_equal(ref, clean) and np.isfinite(ref).all()      # the oracle does not look at those rows
    check(run_multi(cfg, sp, q, K, V, q_pos, gpu_device), ref, cfg.tol, f"poisoned {dtype} D={D} q_len={q_len}")
    check(run_multi(cfg, sp, q, K, V, q_pos, gpu_device, tokens_per_seq=None), ref, cfg.tol,
          f"poisoned {dtype} D={D} q_len={q_len}, uniform grid")
    for splits in (2, 5):
        check(run_multi(cfg, sp, q, K, V, q_pos, gpu_device, num_splits=splits, tokens_per_seq=None), ref, cfg.tol,
              f"poisoned {dtype} D={D} q_len={q_len}, {splits} slices")


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("q_len", [2, 4, 7, 16, 19])
def test_a_row_only_later_tokens_see_does_not_touch_the_earlier_ones(dtype, q_len, gpu_device):
    """The row at the last token's own position holds +Inf in V: the last token's output is not finite (in the
    oracle too), every earlier token's row must equal the oracle's finite result (no 0 * Inf)."""
    cfg = DecodeConfig(94, "multi-band", 2, 3, 128, 300, 300, dtype, TOL[dtype])
    ctx = np.full(cfg.batch, 300, np.int32)
    sp = SpanBatch.from_lists([[(3, 40), (200, 300)], [(0, 9), (120, 180), (250, 300)]], ctx)
    q_pos = np.array([260, 270], np.int32)
    _, K, V = draw_qkv(cfg, ctx, device=gpu_device)
    q = draw_queries(cfg, q_len, device=gpu_device)
    for b in range(cfg.batch):
        V[b, :, int(q_pos[b]) + q_len - 1] = float("inf")
    ref = oracle_multi(cfg, sp, q, K, V, q_pos)
    assert np.isfinite(ref[:, :q_len - 1]).all() and not np.isfinite(ref[:, q_len - 1]).any()
    for kw in (dict(), dict(num_splits=3, tokens_per_seq=None)):
        code, _, _, tok = span.span_validate(sp.offsets, sp.starts, sp.ends, sp.ctx_lens)
        kw.setdefault("tokens_per_seq", tok)
        out = span.span_decode_attn_multi(q, K, V, _dev(sp.offsets, gpu_device), _dev(sp.starts, gpu_device),
                                          _dev(sp.ends, gpu_device), _dev(q_pos, gpu_device), np.float32(cfg.scale),
                                          max_tokens=int(tok.max()), **kw)
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        check(got[:, :q_len - 1], ref[:, :q_len - 1], cfg.tol, f"band row, {dtype} q_len={q_len} {sorted(kw)}")
        assert not np.isfinite(got[:, q_len - 1]).any()


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("q_len", [3, 16])
def test_peaked_scores_with_a_long_light_tail_in_the_matrix_pass(dtype, q_len, gpu_device):
    """One span row outweighs every other by 2^15 and 2^20, but the other ~5000 rows together still carry 13 % and
    0.5 % of the sum.  The sixteen-token pass feeds the weights to the matrix cores as 16-bit values: weights that far
    below the largest must neither vanish (fp16's normal range ends 2^14 below one) nor lose the sum's accuracy.
    Scores are set exactly through one non-zero query component."""
    L = 5000
    cfg = DecodeConfig(95, f"multi-peaked-{dtype}", 2, 2, 128, L, L, dtype, TOL[dtype])
    ctx = np.full(cfg.batch, L, np.int32)
    sp = SpanBatch.from_lists([[(0, L)], [(0, 2500), (2600, L)]], ctx)
    _, K, V = draw_qkv(cfg, ctx, device=gpu_device)
    q = torch.zeros((cfg.batch, q_len, cfg.heads, cfg.head_dim), dtype=K.dtype, device=gpu_device)
    q[..., 0] = 16.0
    per_unit = 16.0 * float(np.float32(cfg.scale))            # score per unit of K[..., 0]
    K[..., 0] = (-15.0 * np.log(2.0)) / per_unit              # every row: weight 2^-15 of the heavy one
    K[1, :, :, 0] = (-20.0 * np.log(2.0)) / per_unit          # second sequence: 2^-20
    K[:, :, 7, 0] = 0.0                                       # the heavy row
    q_pos = new_tokens_at_the_end(sp, q_len)
    ref = oracle_multi(cfg, sp, q, K, V, q_pos)
    heavy = V[:, :, 7].float().cpu().numpy().astype(np.float64)
    share = np.abs(ref[:, 0] - heavy).max()
    assert share > 1e-3, "the tail must matter in the reference, or the case proves nothing"
    for kw in (dict(), dict(num_splits=5, tokens_per_seq=None)):
        got = run_multi(cfg, sp, q, K, V, q_pos, gpu_device, **kw)
        check(got, ref, 2e-5, f"peaked {dtype} q_len={q_len} {sorted(kw)}")
