"""The between-tokens step: the list-based oracle against its definition on position sets (CPU), the
HIP kernel against the oracle bit for bit, and a decode loop over a group of tokens recorded as one
HIP graph (append + attention + advance) against the oracle stepping the same tokens on the host."""
import numpy as np
import pytest
import torch

import oracle
from oracle.advance import advance as oracle_advance
from workloads import DecodeConfig, SpanBatch, draw_qkv, place_disjoint, to_host_raw


def _random_lists(rng, B, L):
    per_seq = []
    for _ in range(B):
        k = int(rng.integers(1, 6))
        lens = rng.integers(1, max(2, L // (2 * k)), size=k)
        per_seq.append(place_disjoint(rng, lens, 0, L))
    return per_seq


def _positions(intervals):
    s = set()
    for a, e in intervals:
        s.update(range(a, e))
    return s


def test_oracle_advance_is_the_set_definition():
    rng = np.random.default_rng(21)
    L = 40
    for trial in range(400):
        B = int(rng.integers(1, 5))
        per_seq = _random_lists(rng, B, L)
        sp = SpanBatch.from_lists(per_seq, np.full(B, L, np.int32))
        off, st, en = sp.offsets.tolist(), sp.starts.tolist(), sp.ends.tolist()
        pos = []
        for b in range(B):       # often right at an interval's end, sometimes anywhere, sometimes out of range
            ends_b = [e - 1 for _, e in per_seq[b]]
            pos.append(int(rng.choice(ends_b)) if rng.random() < 0.6 else int(rng.integers(-2, L + 1)))
        ctx = [p + 1 for p in pos]
        before = [_positions(sp.intervals(b)) for b in range(B)]
        pos2, ctx2 = list(pos), list(ctx)
        oracle_advance(off, st, en, pos2, ctx2, L)
        for b in range(B):
            after = _positions(zip(st[off[b]:off[b + 1]], en[off[b]:off[b + 1]]))
            p = pos[b]
            if p < 0 or p + 1 >= L:
                assert after == before[b] and pos2[b] == p and ctx2[b] == ctx[b]
                continue
            want = before[b] | {p + 1} if (p in before[b] and p + 1 not in before[b]) else before[b]
            assert after == want, (per_seq[b], p)
            assert pos2[b] == p + 1 and ctx2[b] == ctx[b] + 1
            # still a list of disjoint, non-empty intervals in the same order
            iv = list(zip(st[off[b]:off[b + 1]], en[off[b]:off[b + 1]]))
            assert all(a < e for a, e in iv) and sum(e - a for a, e in iv) == len(after)


def test_oracle_advance_by_several_tokens_is_the_set_definition():
    """n tokens per step: the interval the appended tokens closed grows by the next n positions, if all are free."""
    rng = np.random.default_rng(24)
    L = 60
    for trial in range(600):
        n = int(rng.integers(2, 6))
        B = int(rng.integers(1, 4))
        per_seq = _random_lists(rng, B, L)
        sp = SpanBatch.from_lists(per_seq, np.full(B, L, np.int32))
        off, st, en = sp.offsets.tolist(), sp.starts.tolist(), sp.ends.tolist()
        pos = []
        for b in range(B):       # often such that the appended tokens end an interval
            ends_b = [e - n for _, e in per_seq[b]]
            pos.append(int(rng.choice(ends_b)) if rng.random() < 0.7 else int(rng.integers(-2, L + 1)))
        before = [_positions(sp.intervals(b)) for b in range(B)]
        pos2 = list(pos)
        oracle_advance(off, st, en, pos2, None, L, count=n)
        for b in range(B):
            after = _positions(zip(st[off[b]:off[b + 1]], en[off[b]:off[b + 1]]))
            p = pos[b]
            if p < 0 or p + 2 * n > L:
                assert after == before[b] and pos2[b] == p
                continue
            nxt = set(range(p + n, p + 2 * n))
            closes = any(e == p + n for _, e in per_seq[b])
            want = before[b] | nxt if (closes and not (nxt & before[b])) else before[b]
            assert after == want, (per_seq[b], p, n)
            assert pos2[b] == p + n
            iv = list(zip(st[off[b]:off[b + 1]], en[off[b]:off[b + 1]]))
            assert all(a < e for a, e in iv) and sum(e - a for a, e in iv) == len(after)


@pytest.mark.gpu
def test_kernel_advances_by_several_tokens_like_the_oracle(gpu_device):
    import paper_2404_09336_amd as span
    rng = np.random.default_rng(25)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(gpu_device)
    for trial in range(20):
        n = int(rng.integers(2, 9))
        B, L = int(rng.integers(1, 400)), int(rng.choice([64, 500, 4096]))
        per_seq = _random_lists(rng, B, L)
        sp = SpanBatch.from_lists(per_seq, np.full(B, L, np.int32))
        pos = np.array([(per_seq[b][int(rng.integers(len(per_seq[b])))][1] - n) if rng.random() < 0.7
                        else int(rng.integers(-2, L + 1)) for b in range(B)], np.int32)
        ctx = np.maximum(pos + n, 0).astype(np.int32)
        off, st, en = sp.offsets.tolist(), sp.starts.tolist(), sp.ends.tolist()
        pos_o, ctx_o = pos.tolist(), ctx.tolist()
        d_off, d_st, d_en, d_pos, d_ctx = dev(sp.offsets), dev(sp.starts), dev(sp.ends), dev(pos), dev(ctx)
        for step in range(3):
            oracle_advance(off, st, en, pos_o, ctx_o, L, count=n)
            span.span_advance(d_off, d_st, d_en, d_pos, d_ctx, max_len=L, q_len=n)
            torch.cuda.synchronize()
            assert d_en.cpu().tolist() == en and d_pos.cpu().tolist() == pos_o, (trial, step, n)
        assert d_ctx.cpu().tolist() == ctx_o and d_st.cpu().tolist() == st


@pytest.mark.gpu
def test_kernel_matches_oracle_bit_for_bit(gpu_device):
    import paper_2404_09336_amd as span
    rng = np.random.default_rng(22)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(gpu_device)
    for trial in range(30):
        B, L = int(rng.integers(1, 700)), int(rng.choice([64, 500, 4096]))
        per_seq = _random_lists(rng, B, L)
        if trial % 3 == 0:                                      # touching neighbours: p + 1 already in the span
            per_seq[0] = [(2, 5), (5, 9)]
        sp = SpanBatch.from_lists(per_seq, np.full(B, L, np.int32))
        pos = np.array([(per_seq[b][int(rng.integers(len(per_seq[b])))][1] - 1) if rng.random() < 0.7
                        else int(rng.integers(-2, L + 1)) for b in range(B)], np.int32)
        if trial % 3 == 0:
            pos[0] = 4
        ctx = (pos + 1).astype(np.int32)
        off, st, en = sp.offsets.tolist(), sp.starts.tolist(), sp.ends.tolist()
        pos_o, ctx_o = pos.tolist(), ctx.tolist()
        d_off, d_st, d_en, d_pos, d_ctx = dev(sp.offsets), dev(sp.starts), dev(sp.ends), dev(pos), dev(ctx)
        for step in range(3):
            with_ctx = step != 1                                # ctx_lens is optional
            oracle_advance(off, st, en, pos_o, ctx_o if with_ctx else None, L)
            span.span_advance(d_off, d_st, d_en, d_pos, d_ctx if with_ctx else None, max_len=L)
            torch.cuda.synchronize()
            assert d_en.cpu().tolist() == en and d_pos.cpu().tolist() == pos_o, (trial, step)
            assert d_st.cpu().tolist() == st
        assert d_ctx.cpu().tolist() == ctx_o


@pytest.mark.gpu
def test_group_of_tokens_as_one_graph(gpu_device):
    """Six tokens of one group: the HIP graph [append + span attention, advance] is replayed once per token
    with nothing but the new q / k / v rows changing on the host side."""
    import paper_2404_09336_amd as span
    cfg = DecodeConfig(93, "loop", 6, 8, 128, 900, 900, "f16", 2e-3)
    rng = np.random.default_rng(23)
    tokens = 6
    start_len = rng.integers(300, 800, size=cfg.batch).astype(np.int32)    # tokens already in the cache
    per_seq = []
    for b in range(cfg.batch):
        n = int(start_len[b])
        per_seq.append([(0, 17), (40 + 3 * b, 120 + 5 * b), (n - 9, n + 1)])   # the last interval holds the new token
    sp = SpanBatch.from_lists(per_seq, start_len + 1)
    _, K, V = draw_qkv(cfg, start_len, device=gpu_device)                  # rows >= start_len are NaN
    gen = torch.Generator(device=gpu_device)
    gen.manual_seed(5)
    new = [torch.randn((tokens, cfg.batch, cfg.heads, cfg.head_dim), generator=gen, device=gpu_device).half()
           for _ in range(3)]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(gpu_device)
    off, st, en, pos = dev(sp.offsets), dev(sp.starts), dev(sp.ends), dev(start_len)
    q, kn, vn = (torch.empty_like(new[0][0]) for _ in range(3))
    out = torch.empty((cfg.batch, cfg.heads, cfg.head_dim), dtype=torch.float32, device=gpu_device)
    tok_final = sp.tokens_per_seq() + tokens                               # plan for the group's last token
    side = torch.cuda.Stream(device=gpu_device)
    call = span.prepare_span_decode_attn_append(q, kn, vn, K, V, pos, off, st, en, np.float32(cfg.scale), out,
                                                max_tokens=int(tok_final.max()), tokens_per_seq=tok_final,
                                                stream=side.cuda_stream)
    adv = span.prepare_span_advance(off, st, en, pos, max_len=cfg.max_len, stream=side.cuda_stream)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call()
        adv()

    hK, hV = to_host_raw(K).copy(), to_host_raw(V).copy()
    o_off, o_st, o_en, o_pos = sp.offsets.tolist(), sp.starts.tolist(), sp.ends.tolist(), start_len.tolist()
    for t in range(tokens):
        q.copy_(new[0][t]); kn.copy_(new[1][t]); vn.copy_(new[2][t])
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        # host side: append the rows, attend over the span as it stands, then advance
        hk_new, hv_new = to_host_raw(new[1][t]), to_host_raw(new[2][t])
        for b in range(cfg.batch):
            hK[b, :, o_pos[b]] = hk_new[b]
            hV[b, :, o_pos[b]] = hv_new[b]
        ref = oracle.span_attn(to_host_raw(new[0][t]), hK, hV, np.array(o_off, np.int32), np.array(o_st, np.int32),
                               np.array(o_en, np.int32), np.float32(cfg.scale), dtype="f16")
        err = float(np.abs(out.cpu().numpy().astype(np.float64) - ref).max())
        print(f"[loop] token {t}: max-abs err {err:.3e}", flush=True)
        assert np.isfinite(out.cpu().numpy()).all() and err <= cfg.tol, (t, err)
        oracle_advance(o_off, o_st, o_en, o_pos, None, cfg.max_len)
        assert en.cpu().tolist() == o_en and pos.cpu().tolist() == o_pos
    assert np.array_equal(to_host_raw(K), hK, equal_nan=False) or np.array_equal(
        to_host_raw(K).view(np.uint16), hK.view(np.uint16))
    assert np.array_equal(to_host_raw(V).view(np.uint16), hV.view(np.uint16))
