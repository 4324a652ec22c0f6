"""Pins for the few-query form of the fp64 oracle (several new tokens share one span, each under the
causal mask of Sec. 2.2): library attention with a boolean mask, the brute-force additive mask, the
single-query oracle on clipped spans, and closed forms.  CPU only."""
import numpy as np
import torch

import oracle
from oracle import bruteforce

TIGHT = 1e-12


def _spans(per_seq):
    off, st, en = [0], [], []
    for iv in per_seq:
        for s, e in iv:
            st.append(s)
            en.append(e)
        off.append(len(st))
    return np.array(off, np.int32), np.array(st, np.int32).reshape(-1), np.array(en, np.int32).reshape(-1)


def _rand(rng, B, Qn, H, L, D):
    q = rng.standard_normal((B, Qn, H, D)).astype(np.float32)
    K = rng.standard_normal((B, H, L, D)).astype(np.float32)
    V = rng.standard_normal((B, H, L, D)).astype(np.float32)
    return q, K, V


def _attend_bits(per_seq, q_pos, Qn, L):
    """bool [B, Qn, L]: position p visible to query j  <=>  p in span and p <= q_pos[b] + j."""
    B = len(per_seq)
    bits = np.zeros((B, Qn, L), dtype=bool)
    for b, iv in enumerate(per_seq):
        for s, e in iv:
            bits[b, :, s:e] = True
        if q_pos is not None:
            for j in range(Qn):
                bits[b, j, int(q_pos[b]) + j + 1:] = False
    return bits


PER_SEQ = [[(0, 4), (9, 12), (30, 41)], [(2, 3), (3, 20), (36, 40)], [(37, 41)]]
Q_POS = np.array([37, 36, 37], np.int32)     # sequence 1: the tail interval is only partly visible to early queries


def test_multi_equals_library_sdpa_with_mask():
    """Each (b, j) row == torch's scaled_dot_product_attention in float64 under the boolean mask
    span AND causal.  All dimensions differ, so a transposed q layout ([B,H,Qn,D]) cannot pass."""
    rng = np.random.default_rng(11)
    B, Qn, H, L, D = 3, 4, 5, 41, 24
    q, K, V = _rand(rng, B, Qn, H, L, D)
    off, st, en = _spans(PER_SEQ)
    scale = np.float32(0.21)
    got = oracle.span_attn_multi(q, K, V, off, st, en, Q_POS, scale)
    bits = _attend_bits(PER_SEQ, Q_POS, Qn, L)
    for b in range(B):
        tq = torch.from_numpy(q[b]).double().permute(1, 0, 2)          # [H, Qn, D]
        tk, tv = torch.from_numpy(K[b]).double(), torch.from_numpy(V[b]).double()
        mask = torch.from_numpy(bits[b])[None, :, :]                    # [1, Qn, L] broadcast over heads
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=float(scale))
        np.testing.assert_allclose(got[b], ref.permute(1, 0, 2).numpy(), rtol=0, atol=TIGHT)


def test_many_tokens_equal_library_sdpa_with_mask():
    """Eighteen query tokens (more than any pass of the GPU path serves at once), limits running through two
    intervals and a gap: every row against torch's float64 attention under the span-and-causal mask."""
    rng = np.random.default_rng(15)
    B, Qn, H, L, D = 2, 18, 3, 64, 12
    per_seq = [[(0, 5), (20, 33), (40, 64)], [(3, 30), (45, 58)]]
    q_pos = np.array([28, 41], np.int32)      # limits 28..45 and 41..58
    q, K, V = _rand(rng, B, Qn, H, L, D)
    off, st, en = _spans(per_seq)
    scale = np.float32(0.17)
    got = oracle.span_attn_multi(q, K, V, off, st, en, q_pos, scale)
    bits = _attend_bits(per_seq, q_pos, Qn, L)
    assert bits.any(axis=2).all()
    for b in range(B):
        tq = torch.from_numpy(q[b]).double().permute(1, 0, 2)
        tk, tv = torch.from_numpy(K[b]).double(), torch.from_numpy(V[b]).double()
        mask = torch.from_numpy(bits[b])[None, :, :]
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=float(scale))
        np.testing.assert_allclose(got[b], ref.permute(1, 0, 2).numpy(), rtol=0, atol=TIGHT)


def test_multi_equals_bruteforce_additive_mask():
    rng = np.random.default_rng(12)
    B, Qn, H, L, D = 3, 3, 2, 41, 8
    q, K, V = _rand(rng, B, Qn, H, L, D)
    off, st, en = _spans(PER_SEQ)
    got = oracle.span_attn_multi(q, K, V, off, st, en, Q_POS, 0.3)
    bits = _attend_bits(PER_SEQ, Q_POS, Qn, L)
    for j in range(Qn):
        ref = bruteforce.masked_attn_from_bits(q[:, j], K, V, bits[:, j], 0.3)
        np.testing.assert_allclose(got[:, j], ref, rtol=0, atol=TIGHT)


def test_each_query_is_a_single_query_call_on_the_clipped_span():
    """Row j == the single-query oracle given q[:, j] and the span cut off after q_pos + j."""
    rng = np.random.default_rng(13)
    B, Qn, H, L, D = 3, 4, 3, 41, 16
    q, K, V = _rand(rng, B, Qn, H, L, D)
    off, st, en = _spans(PER_SEQ)
    got = oracle.span_attn_multi(q, K, V, off, st, en, Q_POS, 0.25)
    for j in range(Qn):
        clipped = []
        for b, iv in enumerate(PER_SEQ):
            last = int(Q_POS[b]) + j
            clipped.append([(s, min(e, last + 1)) for s, e in iv if s <= last])
        o2, s2, e2 = _spans(clipped)
        ref = oracle.span_attn(np.ascontiguousarray(q[:, j]), K, V, o2, s2, e2, 0.25)
        np.testing.assert_allclose(got[:, j], ref, rtol=0, atol=1e-15)


def test_no_limit_means_every_query_sees_the_whole_span():
    rng = np.random.default_rng(14)
    B, Qn, H, L, D = 3, 2, 3, 41, 16
    q, K, V = _rand(rng, B, Qn, H, L, D)
    off, st, en = _spans(PER_SEQ)
    got = oracle.span_attn_multi(q, K, V, off, st, en, None, 0.25)
    for j in range(Qn):
        ref = oracle.span_attn(np.ascontiguousarray(q[:, j]), K, V, off, st, en, 0.25)
        np.testing.assert_array_equal(got[:, j], ref)
    far = oracle.span_attn_multi(q, K, V, off, st, en, np.full(B, L, np.int32), 0.25)
    np.testing.assert_array_equal(far, got)


def test_single_query_form_is_the_special_case():
    rng = np.random.default_rng(15)
    B, H, L, D = 3, 3, 41, 16
    q, K, V = _rand(rng, B, 1, H, L, D)
    off, st, en = _spans(PER_SEQ)
    got = oracle.span_attn_multi(q, K, V, off, st, en, None, 0.25)
    ref = oracle.span_attn(np.ascontiguousarray(q[:, 0]), K, V, off, st, en, 0.25)
    np.testing.assert_array_equal(got[:, 0], ref)


def test_closed_forms_under_the_causal_limit():
    """Zero queries: row j is the mean of the V rows visible to it.  A limit before the first span
    position leaves nothing visible: zeros.  A query that sees exactly one position returns that V row."""
    rng = np.random.default_rng(16)
    B, Qn, H, L, D = 1, 3, 2, 20, 6
    _, K, V = _rand(rng, B, Qn, H, L, D)
    q = np.zeros((B, Qn, H, D), np.float32)
    off, st, en = _spans([[(5, 8), (10, 13)]])
    got = oracle.span_attn_multi(q, K, V, off, st, en, np.array([10], np.int32), 0.4)
    vis = [[5, 6, 7, 10], [5, 6, 7, 10, 11], [5, 6, 7, 10, 11, 12]]
    for j in range(Qn):
        np.testing.assert_allclose(got[0, j], V[0][:, vis[j]].astype(np.float64).mean(axis=1), rtol=0, atol=TIGHT)
    q2 = rng.standard_normal((B, Qn, H, D)).astype(np.float32)
    got = oracle.span_attn_multi(q2, K, V, off, st, en, np.array([3], np.int32), 0.4)
    np.testing.assert_array_equal(got[0, 0], 0.0)                       # sees up to 3: nothing
    np.testing.assert_array_equal(got[0, 1], 0.0)                       # up to 4: nothing
    np.testing.assert_array_equal(got[0, 2], V[0][:, 5].astype(np.float64))   # up to 5: one position


def test_poisoned_rows_outside_the_visible_set_have_no_influence():
    """NaN in K / V rows that are outside the span, or inside it but after every query's limit, changes nothing."""
    rng = np.random.default_rng(17)
    B, Qn, H, L, D = 1, 2, 2, 24, 8
    q, K, V = _rand(rng, B, Qn, H, L, D)
    off, st, en = _spans([[(1, 5), (12, 20)]])
    q_pos = np.array([14], np.int32)                                    # queries see up to 14 and 15
    ref = oracle.span_attn_multi(q, K, V, off, st, en, q_pos, 0.3)
    K2, V2 = K.copy(), V.copy()
    hidden = [0] + list(range(5, 12)) + list(range(16, 24))
    K2[:, :, hidden] = np.nan
    V2[:, :, hidden] = np.nan
    got = oracle.span_attn_multi(q, K2, V2, off, st, en, q_pos, 0.3)
    np.testing.assert_array_equal(got, ref)
    K2[:, :, 15] = np.nan                                               # visible to query 1 only
    got = oracle.span_attn_multi(q, K2, V2, off, st, en, q_pos, 0.3)
    np.testing.assert_array_equal(got[0, 0], ref[0, 0])
    assert np.isnan(got[0, 1]).all()


def test_reduced_precision_inputs_are_widened_exactly():
    rng = np.random.default_rng(18)
    B, Qn, H, L, D = 2, 2, 2, 16, 8
    q, K, V = _rand(rng, B, Qn, H, L, D)
    off, st, en = _spans([[(0, 9)], [(4, 16)]])
    q_pos = np.array([7, 14], np.int32)
    for name, tdt in (("f16", torch.float16), ("bf16", torch.bfloat16)):
        tq, tk, tv = (torch.from_numpy(a).to(tdt) for a in (q, K, V))
        raw = [t.view(torch.int16).numpy().view(np.uint16) for t in (tq, tk, tv)]
        got = oracle.span_attn_multi(raw[0], raw[1], raw[2], off, st, en, q_pos, 0.35, dtype=name)
        ref = oracle.span_attn_multi(tq.float().numpy(), tk.float().numpy(), tv.float().numpy(), off, st, en,
                                     q_pos, 0.35)
        np.testing.assert_array_equal(got, ref)
