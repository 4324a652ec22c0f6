"""The hand-over of the slices' partial states between workgroups (publish, acknowledge, ticket, last arrival
re-reads) must never let the merging workgroup see a stale value.  The merge order is fixed, so a sliced call is
bit-reproducible: thousands of back-to-back calls on ONE workspace must all give the first call's bits, and those
must agree with the oracle.  A stale read (a state of the previous call, or a half-written one) would show up as
a differing output row."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_09336_amd as span
from workloads import CONFIGS, DecodeConfig, SpanBatch, draw_qkv, draw_queries, draw_spans, to_host_raw

pytestmark = pytest.mark.gpu

CALLS = 4096
RING = 16            # output buffers written in turn, compared together


def _dev(a, device):
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def hammer(cfg, sp, device, what, **plan_kw):
    tok = sp.tokens_per_seq()
    q, K, V = draw_qkv(cfg, sp.ctx_lens, device=device)
    lists = [_dev(a, device) for a in (sp.offsets, sp.starts, sp.ends, sp.ctx_lens)]
    kw = dict(max_tokens=int(tok.max()))
    kw.update(plan_kw)
    first = span.prepare_span_decode_attn(q, K, V, *lists, np.float32(cfg.scale), **kw)
    plan = span.span_plan_query(first.desc)
    assert plan["max_splits"] > 1, plan
    workspace = first._keepalive[-1]
    outs = [torch.empty_like(first.out) for _ in range(RING)]
    calls = [span.prepare_span_decode_attn(q, K, V, *lists, np.float32(cfg.scale), outs[i], workspace=workspace, **kw)
             for i in range(RING)]
    want = first().clone()
    torch.cuda.synchronize()
    ref = oracle.span_attn(to_host_raw(q), to_host_raw(K), to_host_raw(V), sp.offsets, sp.starts, sp.ends,
                           np.float32(cfg.scale), dtype=cfg.dtype)
    assert float(np.abs(want.cpu().numpy().astype(np.float64) - ref).max()) <= cfg.tol
    done = 0
    while done < CALLS:
        for _ in range(8):                      # 8 x RING calls back to back, nothing else on the stream in between
            for c in calls:
                c()
            done += RING
        differing = sum(int((o != want).sum()) for o in outs)     # (the last RING outputs; earlier ones were overwritten)
        assert differing == 0, f"{what}: {differing} output elements differ from the first call after {done} calls"
        for o in outs:
            o.fill_(float("nan"))
    print(f"[handover] {what}: {done} calls, {plan['max_splits']} slices per pair at most, {plan['workgroups']} "
          f"workgroups, runs_in_arguments={plan['runs_in_arguments']}: all outputs bit-identical", flush=True)


@pytest.mark.parametrize("cid", [2, 4])
@pytest.mark.parametrize("host_lists", [False, True])
def test_sliced_workloads_are_bit_reproducible(cid, host_lists, gpu_device):
    cfg = CONFIGS[cid]
    sp = draw_spans(cfg)
    kw = dict(host_spans=(sp.offsets, sp.starts, sp.ends)) if host_lists else dict(tokens_per_seq=sp.tokens_per_seq())
    hammer(cfg, sp, gpu_device, f"config {cid}, {'run' if host_lists else 'table'} mode", **kw)


@pytest.mark.parametrize("heads", [8, 3])
def test_one_pair_in_113_slices_is_bit_reproducible(heads, gpu_device):
    """Every slice of the 113 is a single workgroup of 17 positions: tickets arrive as close together as they can.
    Consecutive workgroups go to consecutive XCDs (8 of them, each with its own L2), heads varying fastest: with 8
    heads all slices of a pair share one XCD, with 3 heads they are spread over all eight, so the states really
    cross L2s on their way to the merging workgroup."""
    cfg = DecodeConfig(98, f"handover-113-{heads}", 2, heads, 128, 2048, 2048, "f16", 2e-3)
    sp = SpanBatch.from_lists([[(0, 700), (900, 2048)], [(5, 1900)]], [2048, 2048])
    hammer(cfg, sp, gpu_device, f"113 forced slices, {heads} heads", num_splits=113)


def test_slices_spread_over_all_xcds_are_bit_reproducible(gpu_device):
    """A ragged batch with 5 heads (not a multiple of the 8 XCDs): the slices of one pair run on different XCDs."""
    cfg = DecodeConfig(99, "handover-5-heads", 6, 5, 128, 4096, 4096, "bf16", 2e-3)
    rng = np.random.default_rng(99)
    from workloads import place_disjoint
    per_seq = [place_disjoint(rng, rng.integers(50, 700, size=4), 0, 4096) for _ in range(cfg.batch)]
    sp = SpanBatch.from_lists(per_seq, np.full(cfg.batch, 4096, np.int32))
    hammer(cfg, sp, gpu_device, "6 sequences x 5 heads, table mode", tokens_per_seq=sp.tokens_per_seq())
    hammer(cfg, sp, gpu_device, "6 sequences x 5 heads, 9 slices each", num_splits=9)


def test_uniform_grid_with_empty_slices_is_bit_reproducible(gpu_device):
    """Without the token counts short sequences leave slices empty: their slots are never written and must be
    ignored, not read as the previous call's state."""
    cfg = CONFIGS[4]
    sp = draw_spans(cfg)
    hammer(cfg, sp, gpu_device, "config 4, uniform grid")


@pytest.mark.parametrize("q_len", [2, 5, 16])
def test_sliced_few_query_calls_are_bit_reproducible(q_len, gpu_device):
    """The few-query passes hand over one state per query token and slice (two tokens: vector-ALU pass; five and
    sixteen: the sixteen-token pass, five leaving eleven states of the slot unwritten)."""
    cfg = CONFIGS[2]
    sp = draw_spans(cfg)
    tok = sp.tokens_per_seq()
    _, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device)
    q = draw_queries(cfg, q_len, device=gpu_device)
    lists = [_dev(a, gpu_device) for a in (sp.offsets, sp.starts, sp.ends)]
    q_pos_host = (sp.ctx_lens - q_len).astype(np.int32)
    q_pos = _dev(q_pos_host, gpu_device)
    kw = dict(max_tokens=int(tok.max()), tokens_per_seq=tok)
    first = span.prepare_span_decode_attn_multi(q, K, V, *lists, q_pos, np.float32(cfg.scale), **kw)
    plan = span.span_plan_query(first.desc)
    assert plan["max_splits"] > 1 and plan["queries_per_pass"] == (2 if q_len == 2 else 16), plan
    workspace = first._keepalive[-1]
    outs = [torch.empty_like(first.out) for _ in range(RING)]
    calls = [span.prepare_span_decode_attn_multi(q, K, V, *lists, q_pos, np.float32(cfg.scale), outs[i],
                                                 workspace=workspace, **kw) for i in range(RING)]
    want = first().clone()
    torch.cuda.synchronize()
    ref = oracle.span_attn_multi(to_host_raw(q), to_host_raw(K), to_host_raw(V), sp.offsets, sp.starts, sp.ends,
                                 q_pos_host, np.float32(cfg.scale), dtype=cfg.dtype)
    assert float(np.abs(want.cpu().numpy().astype(np.float64) - ref).max()) <= cfg.tol
    done = 0
    while done < CALLS // 4:
        for _ in range(4):
            for c in calls:
                c()
            done += RING
        differing = sum(int((o != want).sum()) for o in outs)
        assert differing == 0, f"{q_len} tokens: {differing} output elements differ from the first call after {done} calls"
        for o in outs:
            o.fill_(float("nan"))
    print(f"[handover] few-query, {q_len} tokens: {done} calls, {plan['max_splits']} slices per pair at most, "
          f"{plan['workgroups']} workgroups: all outputs bit-identical", flush=True)
