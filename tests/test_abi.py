"""Host-side checks of the C-ABI library that need no GPU: exported symbols, argument checking,
work-partition arithmetic, and the validator against the oracle's (bit-exact)."""
import ctypes
import itertools
import os
import re

import numpy as np
import pytest

import oracle
import paper_2404_09336_amd as span
from paper_2404_09336_amd import binding
from test_oracle_validate import load_golden

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "span_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(span_\w+|dense_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = span.load_library()
    names = declared_functions()
    assert {"span_decode_attn", "dense_decode_attn", "span_validate", "span_plan_query", "span_workspace_bytes",
            "span_workspace_init", "span_strerror", "span_last_hip_error", "span_blocks_to_intervals",
            "span_intervals_to_blocks", "span_build", "span_decode_attn_append", "dense_decode_attn_append",
            "span_decode_attn_multi", "span_advance", "span_decode_attn_static",
            "span_decode_attn_multi_append"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_strerror_covers_all_codes():
    seen = set()
    for code in range(-7, 7):
        s = span.span_strerror(code)
        assert s and s != "unknown code"
        seen.add(s)
    assert len(seen) == 14
    assert span.span_strerror(99) == "unknown code"


def _call_span(desc, ptrs=(1, 1, 1, 1, 1, 1, 1, 1)):
    lib = span.load_library()
    q, k, v, off, st, en, ctx, out = [ctypes.c_void_p(p) if p else None for p in ptrs]
    return lib.span_decode_attn(ctypes.byref(desc) if desc is not None else None, q, k, v, off, st, en, ctx, 0.1, out)


def test_argument_errors_are_reported_before_any_launch():
    ok = dict(batch=2, heads=4, head_dim=128, max_len=64, dtype_code=1, num_intervals=4)
    mk = lambda **kw: binding.make_desc(**{**ok, **kw})
    assert _call_span(None) == -1
    assert _call_span(mk(), ptrs=(0, 1, 1, 1, 1, 1, 1, 1)) == -1
    assert _call_span(mk(), ptrs=(1, 1, 1, 0, 1, 1, 1, 1)) == -1
    assert _call_span(mk(), ptrs=(1, 1, 1, 1, 1, 1, 1, 0)) == -1
    assert _call_span(mk(head_dim=96)) == -2
    assert _call_span(mk(batch=0)) == -2
    assert _call_span(mk(max_len=(1 << 22) + 1)) == -2
    assert _call_span(mk(dtype_code=7)) == -3
    # several slices but no workspace / a short one / a misaligned one
    need = span.span_workspace_bytes(mk(num_splits=2))
    assert need > 0
    assert _call_span(mk(num_splits=2)) == -4
    assert _call_span(mk(num_splits=2, workspace_ptr=4096, workspace_bytes=need - 1)) == -4
    assert _call_span(mk(num_splits=2, workspace_ptr=4096 + 64, workspace_bytes=need)) == -4
    lib = span.load_library()
    assert lib.dense_decode_attn(ctypes.byref(mk()), 1, 1, 1, None, 0.1, 1) == -1
    assert lib.dense_decode_attn(ctypes.byref(mk(head_dim=32)), 1, 1, 1, 1, 0.1, 1) == -2


def test_argument_errors_of_the_few_query_and_advance_calls():
    """All of these return before any launch (the pointers are fakes)."""
    lib = span.load_library()
    mk = lambda **kw: binding.make_desc(**{**dict(batch=2, heads=4, head_dim=128, max_len=64, dtype_code=1,
                                                  num_intervals=4, q_len=3), **kw})
    P = ctypes.c_void_p
    multi = lambda d, q=1, off=1, out=1: lib.span_decode_attn_multi(
        ctypes.byref(d), P(q) if q else None, P(1), P(1), P(off) if off else None, P(1), P(1), None, 0.1,
        P(out) if out else None)
    assert multi(mk(), q=0) == -1 and multi(mk(), off=0) == -1 and multi(mk(), out=0) == -1
    assert multi(mk(q_len=65)) == -2 and multi(mk(q_len=-1)) == -2 and multi(mk(head_dim=32)) == -2
    assert multi(mk(num_splits=2)) == -4                       # several slices need a workspace
    # every other entry point takes one query token only
    assert _call_span(mk()) == -2
    assert lib.dense_decode_attn(ctypes.byref(mk()), 1, 1, 1, 1, 0.1, 1) == -2
    assert lib.span_decode_attn_append(ctypes.byref(mk()), 1, 1, 1, 1, 1, 1, 1, 1, 1, 0.1, 1) == -2
    adv = lambda d, off=1, en=1, pos=1: lib.span_advance(ctypes.byref(d) if d is not None else None,
                                                         P(off) if off else None, P(1), P(en) if en else None,
                                                         P(pos) if pos else None, None)
    assert adv(None) == -1 and adv(mk(), off=0) == -1 and adv(mk(), en=0) == -1 and adv(mk(), pos=0) == -1
    assert adv(mk(batch=0)) == -2


def test_partition_arithmetic_uniform():
    for B, H, L, mt, ns in itertools.product([1, 8, 64, 300], [1, 32], [1, 100, 512, 4096, 16384, 1 << 22],
                                             [0, 1, 63, 157, 5000], [0, 1, 2, 5, 64]):
        d = binding.make_desc(B, H, 128, L, 1, 10, mt, ns)
        info = span.span_plan_query(d)
        splits, slice_tokens = info["max_splits"], info["slice_tokens"]
        max_tok = min(mt, L) if mt > 0 else L
        limit = info["slice_limit"]
        assert not info["exact"] and info["workgroups"] == B * H * splits
        assert 1 <= slice_tokens <= limit and splits <= 65535
        assert splits * slice_tokens >= max_tok              # every position has an owner
        assert (splits - 1) * slice_tokens < max_tok         # and no slice is useless
        if ns and -(-max_tok // ns) <= limit - 16 and ns <= max_tok:
            assert splits <= ns
        ws = span.span_workspace_bytes(d)
        assert ws == info["workspace_bytes"] and (ws == 0) == (splits == 1)
        if splits > 1:
            assert ws >= B * H * (splits * (128 + 2) + 1) * 4


def test_partition_arithmetic_exact():
    rng = np.random.default_rng(3)
    for trial in range(300):
        B = int(rng.integers(1, 70))
        H = int(rng.choice([1, 8, 32]))
        L = int(rng.choice([64, 512, 4096, 16384]))
        tok = rng.integers(0, L + 1, size=B)
        if trial % 5 == 0:
            tok[:] = int(rng.integers(1, L + 1))             # uniform batch
        mt = int(tok.max()) if trial % 2 else 0
        d = binding.make_desc(B, H, 128, L, 1, 10, mt, 0, tokens_per_seq=tok)
        info = span.span_plan_query(d)
        if not info["exact"]:
            continue
        T = info["slice_tokens"]
        assert 1 <= T <= info["slice_limit"]
        assert info["workgroups"] % H == 0 and B <= info["workgroups"] // H <= 768
        # enough slices of at most T positions to hold every sequence
        assert info["workgroups"] // H >= sum(max(1, -(-int(n) // T)) for n in tok) - B
        assert info["max_splits"] * T >= tok.max()
        assert (info["workspace_bytes"] == 0) == (info["max_splits"] == 1)
    # equal token counts near one chip-load stay unsplit; num_splits > 0 turns the table off
    tok = np.full(64, 156)
    assert span.span_plan_query(binding.make_desc(64, 32, 128, 512, 1, 10, 168, 0, tokens_per_seq=tok))["max_splits"] == 1
    assert not span.span_plan_query(binding.make_desc(64, 32, 128, 512, 1, 10, 168, 2, tokens_per_seq=tok))["exact"]
    assert not span.span_plan_query(binding.make_desc(1025, 1, 128, 512, 1, 10, 0, 0,
                                                      tokens_per_seq=np.ones(1025)))["exact"]


def test_partition_follows_the_query_token_count():
    """One resident round is 2048 workgroups for one query token, 1536 for two, 1024 for the four-token pass and for
    the sixteen-token pass (16-bit types with head_dim 128, from three tokens on), and a ragged batch of 30
    sequences (two slices per sequence wanted) is capped by it; the workspace grows with the tokens one pass serves
    (1, 2, 4 or 16), never with q_len itself."""
    tok = np.linspace(1500, 4096, 30).astype(np.int64)
    plans, plans32 = {}, {}
    for q_len in (0, 1, 2, 3, 4, 5, 8, 64):
        plans[q_len] = span.span_plan_query(binding.make_desc(30, 32, 128, 4096, 1, 10, 4096, 0, tokens_per_seq=tok, q_len=q_len))
        plans32[q_len] = span.span_plan_query(binding.make_desc(30, 32, 128, 4096, 0, 10, 4096, 0, tokens_per_seq=tok, q_len=q_len))
    assert plans[0] == plans[1]
    assert [plans[q]["queries_per_pass"] for q in (1, 2, 3, 4, 5, 64)] == [1, 2, 16, 16, 16, 16]
    assert [plans32[q]["queries_per_pass"] for q in (1, 2, 3, 4, 5, 64)] == [1, 2, 4, 4, 4, 4]    # fp32: vector units only
    assert 1536 < plans[1]["workgroups"] <= 1920           # 2 x 30 slices per head wanted, 64 would fit
    assert 1024 < plans[2]["workgroups"] <= 1536 and 768 < plans32[4]["workgroups"] <= 1024
    assert 960 <= plans[8]["workgroups"] <= 1024           # 30 x 32 pairs nearly fill the round by themselves
    assert plans[3] == plans[4] == plans[5] == plans[8] == plans[64]
    assert plans32[3] == plans32[4] == plans32[8] == plans32[64]
    per_slot = lambda pl: (pl["workspace_bytes"] - 3840) / pl["workgroups"]      # 3840 B of counters at this size
    assert abs(per_slot(plans[1]) - 130 * 4) < 2 and abs(per_slot(plans[2]) - 2 * 130 * 4) < 2
    assert abs(per_slot(plans32[4]) - 4 * 130 * 4) < 2 and abs(per_slot(plans[8]) - 16 * 130 * 4) < 2
    few = np.linspace(1500, 4096, 6).astype(np.int64)
    sliced = span.span_plan_query(binding.make_desc(6, 32, 128, 4096, 1, 10, 4096, 0, tokens_per_seq=few, q_len=8))
    assert 192 < sliced["workgroups"] <= 1024 and sliced["max_splits"] > 1
    counters = 6 * 32 * 4
    assert abs((sliced["workspace_bytes"] - counters) / sliced["workgroups"] - 16 * 130 * 4) < 8
    # head_dim 64 has no sixteen-token pass either
    d8 = binding.make_desc(30, 32, 64, 4096, 1, 10, 4096, 0, tokens_per_seq=tok, q_len=8)
    assert span.span_plan_query(d8)["queries_per_pass"] == 4
    for bad in (-1, 65):
        d = binding.make_desc(8, 32, 128, 4096, 1, 10, 4096, 0, q_len=bad)
        with pytest.raises(span.SpanAttnError):
            span.span_plan_query(d)


def test_level_batches_with_enough_pairs_are_not_sliced():
    """At least 512 (batch, head) pairs and the longest sequence within 35 % of the mean: one workgroup per pair."""
    rng = np.random.default_rng(8)
    tok = rng.integers(420, 560, size=16)
    level = binding.make_desc(16, 32, 128, 4096, 1, 16, int(tok.max()), 0, tokens_per_seq=tok)
    plan = span.span_plan_query(level)
    assert plan["max_splits"] == 1 and plan["workgroups"] == 512 and plan["workspace_bytes"] == 0
    ragged = tok.copy()
    ragged[0] = 1100                                             # one long sequence: slices level the work again
    plan = span.span_plan_query(binding.make_desc(16, 32, 128, 4096, 1, 16, 1100, 0, tokens_per_seq=ragged))
    assert plan["max_splits"] > 1 and 512 < plan["workgroups"] <= 1024
    few = binding.make_desc(8, 32, 128, 4096, 1, 16, int(tok.max()), 0, tokens_per_seq=tok[:8])   # 256 pairs
    assert span.span_plan_query(few)["max_splits"] > 1


def test_small_batches_aim_at_a_quarter_round_of_large_slices():
    """Few, large slices: a quarter of a resident round (512 workgroups), or two slices per sequence on average if
    that is more, never beyond one round (2048)."""
    plan = lambda B, tok: span.span_plan_query(binding.make_desc(B, 32, 128, 16384, 1, 10, int(np.max(tok)), 0,
                                                                 tokens_per_seq=np.asarray(tok, np.int64)))
    one = plan(1, [8000])
    assert one["workgroups"] == 512 and one["max_splits"] == 16 and one["slice_tokens"] == 500
    eight = plan(8, np.linspace(200, 1600, 8))
    assert 384 < eight["workgroups"] <= 512
    sixteen = plan(16, np.linspace(110, 1100, 16))
    assert 768 < sixteen["workgroups"] <= 1024
    big = plan(32, np.linspace(1000, 8000, 32))
    assert 1700 < big["workgroups"] <= 2048
    # without the counts: the same room, spread evenly
    uni = span.span_plan_query(binding.make_desc(8, 32, 128, 16384, 1, 10, 1600, 0))
    assert uni["workgroups"] == 512 and uni["max_splits"] == 2


def test_validator_matches_oracle_on_golden_cases():
    for ctx, off, st, en, exp in load_golden():
        got = span.span_validate(off, st, en, ctx)
        assert got[:3] == exp
        ref = oracle.validate(off, st, en, ctx)
        assert got[:3] == ref[:3]


def test_validator_bit_exact_exhaustive_tiny():
    pts = range(-1, 5)
    pairs = list(itertools.product(pts, pts))
    for k in range(0, 4):
        for combo in itertools.product(pairs, repeat=k):
            st = [c[0] for c in combo]
            en = [c[1] for c in combo]
            got = span.span_validate([0, k], st, en, [3])
            ref = oracle.validate([0, k], st, en, [3])
            assert got[:3] == ref[:3], (st, en)
            if got[0] == 0:
                assert np.array_equal(got[3], ref[3])


def test_validator_bit_exact_random_batches():
    rng = np.random.default_rng(7)
    from workloads import CONFIGS, draw_spans
    for trial in range(300):
        cfg = CONFIGS[int(rng.choice([1, 2, 3, 4]))]
        sp = draw_spans(cfg, seed=1000 + trial)
        off, st, en, ctx = sp.offsets.copy(), sp.starts.copy(), sp.ends.copy(), sp.ctx_lens.copy()
        kind = trial % 6
        i = int(rng.integers(0, st.shape[0]))
        b = int(rng.integers(0, ctx.shape[0]))
        if kind == 1:
            st[i] = en[i] + int(rng.integers(0, 3))
        elif kind == 2:
            en[i] = ctx.max() + int(rng.integers(1, 50))
        elif kind == 3:
            j = int(rng.integers(0, st.shape[0]))
            st[[i, j]] = st[[j, i]]
            en[[i, j]] = en[[j, i]]
        elif kind == 4:
            off[b + 1] = off[b] + int(rng.integers(-2, 1))
        elif kind == 5:
            st[i] = st[i] - int(rng.integers(1, 40))
        got = span.span_validate(off, st, en, ctx)
        ref = oracle.validate(off, st, en, ctx)
        assert got[:3] == ref[:3], (trial, kind)
        if got[0] == 0:
            assert np.array_equal(got[3], ref[3])


def test_validator_offsets_two_sequences_exhaustive():
    st, en = [0, 2, 1], [1, 3, 2]
    for off in itertools.product(range(-1, 5), repeat=3):
        assert span.span_validate(list(off), st, en, [3, 3])[:3] == oracle.validate(list(off), st, en, [3, 3])[:3]
