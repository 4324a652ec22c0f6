"""Pins for the fp64 oracle: everything here runs on the CPU and compares the oracle with
something that is not the oracle — a library routine, a closed form, brute force, or an
invariant fixed by the mathematics of Sec. 2.2 eqs. (4)-(6) and Sec. 3.3."""
import itertools
import math

import numpy as np
import pytest
import torch

import oracle
from oracle import bruteforce

TIGHT = 1e-12


def _rand(rng, B, H, L, D):
    q = rng.standard_normal((B, H, D)).astype(np.float32)
    K = rng.standard_normal((B, H, L, D)).astype(np.float32)
    V = rng.standard_normal((B, H, L, D)).astype(np.float32)
    return q, K, V


def _spans(per_seq):
    off, st, en = [0], [], []
    for iv in per_seq:
        for s, e in iv:
            st.append(s)
            en.append(e)
        off.append(len(st))
    return np.array(off, np.int32), np.array(st, np.int32).reshape(-1), np.array(en, np.int32).reshape(-1)


# ---------------------------------------------------------------- library routine
def test_dense_equals_library_sdpa():
    """Dense oracle == torch's scaled_dot_product_attention in float64 (textbook softmax(qK^T s)V)."""
    rng = np.random.default_rng(1)
    B, H, L, D = 3, 5, 37, 24          # all different, so a transposed operand cannot pass
    q, K, V = _rand(rng, B, H, L, D)
    scale = np.float32(0.173)
    ctx = np.array([37, 20, 1], np.int32)
    got = oracle.dense_attn(q, K, V, ctx, scale)
    for b in range(B):
        n = int(ctx[b])
        tq = torch.from_numpy(q[b]).double()[:, None, :]
        tk = torch.from_numpy(K[b, :, :n]).double()
        tv = torch.from_numpy(V[b, :, :n]).double()
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=float(scale))[:, 0, :].numpy()
        np.testing.assert_allclose(got[b], ref, rtol=0, atol=TIGHT)


def test_full_cover_equals_dense():
    """A span that keeps every position is dense attention (Sec. 4.1 / 4.2: the two kernels are
    equivalent at sparsity 0)."""
    rng = np.random.default_rng(2)
    B, H, L, D = 4, 3, 50, 16
    q, K, V = _rand(rng, B, H, L, D)
    ctx = np.array([50, 7, 33, 1], np.int32)
    off, st, en = _spans([[(0, int(n))] for n in ctx])
    a = oracle.span_attn(q, K, V, off, st, en, 0.25)
    d = oracle.dense_attn(q, K, V, ctx, 0.25)
    np.testing.assert_allclose(a, d, rtol=0, atol=1e-13)


def test_span_equals_library_on_gathered_rows():
    """Span oracle == library softmax attention over the gathered span rows."""
    rng = np.random.default_rng(3)
    B, H, L, D = 2, 3, 64, 12
    q, K, V = _rand(rng, B, H, L, D)
    per_seq = [[(0, 5), (9, 10), (40, 64)], [(3, 4), (4, 17)]]
    off, st, en = _spans(per_seq)
    got = oracle.span_attn(q, K, V, off, st, en, 0.3)
    for b in range(B):
        idx = np.concatenate([np.arange(s, e) for s, e in per_seq[b]])
        s = torch.from_numpy(K[b][:, idx]).double() @ torch.from_numpy(q[b]).double()[:, :, None]
        a = torch.softmax(s[:, :, 0] * float(np.float32(0.3)), dim=-1)
        ref = (a[:, None, :] @ torch.from_numpy(V[b][:, idx]).double())[:, 0, :].numpy()
        np.testing.assert_allclose(got[b], ref, rtol=0, atol=TIGHT)


# ---------------------------------------------------------------- brute force over masks
def test_bruteforce_all_masks_tiny():
    """Every non-empty subset of 8 positions, as an additive 0 / -inf mask over all positions."""
    rng = np.random.default_rng(4)
    L, D = 8, 5
    q, K, V = _rand(rng, 1, 2, L, D)
    scale = 1.0 / math.sqrt(D)
    for bits in range(1, 1 << L):
        iv, p = [], 0
        while p < L:
            if bits >> p & 1:
                s = p
                while p < L and bits >> p & 1:
                    p += 1
                iv.append((s, p))
            else:
                p += 1
        off, st, en = _spans([iv])
        got = oracle.span_attn(q, K, V, off, st, en, scale)
        ref = bruteforce.masked_attn(q, K, V, [iv], [L], scale)
        np.testing.assert_allclose(got, ref, rtol=0, atol=TIGHT)


def test_bruteforce_random_small():
    rng = np.random.default_rng(5)
    for _ in range(20):
        B, H, L, D = 2, 2, int(rng.integers(4, 33)), int(rng.integers(1, 9))
        q, K, V = _rand(rng, B, H, L, D)
        ctx = rng.integers(2, L + 1, size=B)
        per_seq = []
        for b in range(B):
            cuts = np.sort(rng.choice(np.arange(0, ctx[b] + 1), size=min(6, ctx[b] + 1) // 2 * 2, replace=False))
            per_seq.append([(int(cuts[i]), int(cuts[i + 1])) for i in range(0, len(cuts), 2)])
        off, st, en = _spans(per_seq)
        got = oracle.span_attn(q, K, V, off, st, en, 0.41)
        ref = bruteforce.masked_attn(q, K, V, per_seq, ctx, 0.41)
        np.testing.assert_allclose(got, ref, rtol=0, atol=TIGHT)


# ---------------------------------------------------------------- special cases and closed forms
def test_single_position_returns_v_row_exactly():
    rng = np.random.default_rng(6)
    q, K, V = _rand(rng, 3, 2, 19, 7)
    per_seq = [[(0, 1)], [(18, 19)], [(7, 8)]]
    off, st, en = _spans(per_seq)
    got = oracle.span_attn(q, K, V, off, st, en, 0.5)
    for b, iv in enumerate(per_seq):
        assert np.array_equal(got[b], V[b, :, iv[0][0], :].astype(np.float64))


def test_zero_query_gives_mean_of_span_rows():
    rng = np.random.default_rng(7)
    q, K, V = _rand(rng, 1, 3, 40, 6)
    q[:] = 0
    iv = [(2, 9), (20, 31)]
    off, st, en = _spans([iv])
    got = oracle.span_attn(q, K, V, off, st, en, 0.7)
    idx = np.r_[2:9, 20:31]
    np.testing.assert_allclose(got[0], V[0][:, idx].astype(np.float64).mean(axis=1), rtol=0, atol=TIGHT)


def test_equal_keys_give_mean_of_span_rows():
    rng = np.random.default_rng(8)
    q, K, V = _rand(rng, 1, 2, 30, 6)
    K[0, :, 5:25] = K[0, :, 5:6]
    off, st, en = _spans([[(5, 12), (15, 25)]])
    got = oracle.span_attn(q, K, V, off, st, en, 0.9)
    idx = np.r_[5:12, 15:25]
    np.testing.assert_allclose(got[0], V[0][:, idx].astype(np.float64).mean(axis=1), rtol=0, atol=TIGHT)


def test_equal_values_returned_whatever_the_scores():
    rng = np.random.default_rng(9)
    q, K, V = _rand(rng, 1, 2, 30, 6)
    V[0, :, :, :] = V[0, :, 3:4, :]
    off, st, en = _spans([[(1, 4), (10, 29)]])
    got = oracle.span_attn(q, K, V, off, st, en, 1.3)
    np.testing.assert_allclose(got[0], V[0, :, 3].astype(np.float64), rtol=0, atol=TIGHT)


def test_key_shift_invariance():
    """Adding u to every span key adds the constant scale*q.u to every score: softmax unchanged."""
    rng = np.random.default_rng(10)
    B, H, L, D = 1, 2, 24, 8
    # small integers: sums and products are exact in fp32, so the shifted keys are exact
    q = rng.integers(-3, 4, (B, H, D)).astype(np.float32)
    K = rng.integers(-3, 4, (B, H, L, D)).astype(np.float32)
    V = rng.standard_normal((B, H, L, D)).astype(np.float32)
    u = rng.integers(-3, 4, D).astype(np.float32)
    off, st, en = _spans([[(0, 3), (8, 20)]])
    a = oracle.span_attn(q, K, V, off, st, en, 0.125)
    b = oracle.span_attn(q, K + u, V, off, st, en, 0.125)
    np.testing.assert_allclose(a, b, rtol=0, atol=TIGHT)


def test_two_positions_logistic():
    rng = np.random.default_rng(11)
    q, K, V = _rand(rng, 1, 4, 12, 5)
    scale = np.float32(0.37)
    off, st, en = _spans([[(2, 3), (9, 10)]])
    got = oracle.span_attn(q, K, V, off, st, en, scale)
    for h in range(4):
        s0 = float(scale) * float(q[0, h].astype(np.float64) @ K[0, h, 2].astype(np.float64))
        s1 = float(scale) * float(q[0, h].astype(np.float64) @ K[0, h, 9].astype(np.float64))
        sig = 1.0 / (1.0 + math.exp(-(s0 - s1)))
        ref = sig * V[0, h, 2].astype(np.float64) + (1.0 - sig) * V[0, h, 9].astype(np.float64)
        np.testing.assert_allclose(got[0, h], ref, rtol=0, atol=TIGHT)


def test_dominant_key_selects_its_value_row():
    rng = np.random.default_rng(12)
    q, K, V = _rand(rng, 1, 1, 16, 4)
    q[0, 0] = [1, 0, 0, 0]
    K[0, 0, :, 0] = 0.0
    K[0, 0, 11, 0] = 60.0                   # score gap 60 with scale 1: weights of the rest < e^-60
    off, st, en = _spans([[(0, 16)]])
    got = oracle.span_attn(q, K, V, off, st, en, 1.0)
    np.testing.assert_allclose(got[0, 0], V[0, 0, 11].astype(np.float64), rtol=0, atol=1e-20 * 1e4)


def test_scale_is_applied_to_scores():
    """Doubling scale == doubling q (both exact in binary), and scale 0 gives the mean."""
    rng = np.random.default_rng(13)
    q, K, V = _rand(rng, 1, 2, 20, 6)
    off, st, en = _spans([[(0, 7), (9, 20)]])
    a = oracle.span_attn(q, K, V, off, st, en, 0.5)
    b = oracle.span_attn(q * 2, K, V, off, st, en, 0.25)
    np.testing.assert_allclose(a, b, rtol=0, atol=TIGHT)
    z = oracle.span_attn(q, K, V, off, st, en, 0.0)
    idx = np.r_[0:7, 9:20]
    np.testing.assert_allclose(z[0], V[0][:, idx].astype(np.float64).mean(axis=1), rtol=0, atol=TIGHT)


def test_convexity_and_weights():
    rng = np.random.default_rng(14)
    q, K, V = _rand(rng, 2, 3, 48, 10)
    per_seq = [[(0, 6), (20, 25), (40, 48)], [(5, 30)]]
    off, st, en = _spans(per_seq)
    got = oracle.span_attn(q, K, V, off, st, en, 0.4)
    for b in range(2):
        idx = np.concatenate([np.arange(s, e) for s, e in per_seq[b]])
        lo = V[b][:, idx].min(axis=1).astype(np.float64)
        hi = V[b][:, idx].max(axis=1).astype(np.float64)
        assert (got[b] >= lo - 1e-15).all() and (got[b] <= hi + 1e-15).all()
    # weights sum to one: with V == 1 everywhere the output is 1
    ones = np.ones_like(V)
    np.testing.assert_allclose(oracle.span_attn(q, K, ones, off, st, en, 0.4), 1.0, rtol=0, atol=TIGHT)


# ---------------------------------------------------------------- invariances
def test_interval_order_invariance():
    rng = np.random.default_rng(15)
    q, K, V = _rand(rng, 1, 3, 64, 8)
    iv = [(0, 4), (10, 13), (13, 20), (33, 50), (60, 64)]
    base = oracle.span_attn(q, K, V, *_spans([iv]), 0.35)
    for perm in itertools.islice(itertools.permutations(iv), 0, 120, 7):
        got = oracle.span_attn(q, K, V, *_spans([list(perm)]), 0.35)
        np.testing.assert_allclose(got, base, rtol=0, atol=1e-13)


def test_split_interval_invariance():
    rng = np.random.default_rng(16)
    q, K, V = _rand(rng, 1, 3, 64, 8)
    base = oracle.span_attn(q, K, V, *_spans([[(3, 40), (50, 64)]]), 0.35)
    for cut in (4, 17, 39):
        got = oracle.span_attn(q, K, V, *_spans([[(3, cut), (cut, 40), (50, 57), (57, 64)]]), 0.35)
        np.testing.assert_allclose(got, base, rtol=0, atol=1e-13)


def test_rows_outside_span_have_no_influence():
    """Even NaN / Inf outside the span must not reach the output (an interval kernel never reads them)."""
    rng = np.random.default_rng(17)
    q, K, V = _rand(rng, 2, 2, 40, 8)
    per_seq = [[(2, 9), (30, 35)], [(0, 1), (39, 40)]]
    off, st, en = _spans(per_seq)
    base = oracle.span_attn(q, K, V, off, st, en, 0.3)
    Kp, Vp = K.copy(), V.copy()
    for b in range(2):
        keep = np.zeros(40, bool)
        for s, e in per_seq[b]:
            keep[s:e] = True
        Kp[b][:, ~keep] = np.nan
        Vp[b][:, ~keep] = np.inf
    got = oracle.span_attn(q, Kp, Vp, off, st, en, 0.3)
    assert np.array_equal(got, base)


def test_heads_share_the_span_and_sequences_do_not():
    rng = np.random.default_rng(18)
    q, K, V = _rand(rng, 2, 3, 20, 4)
    per_seq = [[(0, 5)], [(10, 20)]]
    got = oracle.span_attn(q, K, V, *_spans(per_seq), 0.5)
    for b in range(2):
        for h in range(3):
            one = oracle.span_attn(q[b:b + 1, h:h + 1], K[b:b + 1, h:h + 1], V[b:b + 1, h:h + 1],
                                   *_spans([per_seq[b]]), 0.5)
            np.testing.assert_allclose(got[b, h], one[0, 0], rtol=0, atol=TIGHT)


# ---------------------------------------------------------------- group states + log-sum-exp merge
def test_group_states_merge_to_one_shot_result():
    rng = np.random.default_rng(19)
    q, K, V = _rand(rng, 2, 2, 96, 8)
    iv = [(0, 10), (12, 30), (31, 32), (50, 90)]
    off, st, en = _spans([iv, iv])
    full = oracle.span_attn(q, K, V, off, st, en, 0.45)
    for groups in ([[0], [1], [2], [3]], [[0, 3], [1, 2]], [[0, 1, 2, 3], []], [[], [2], [0, 1, 3]]):
        for b, h in ((0, 0), (1, 1)):
            states = [oracle.span_state(q, K, V, b, h, [iv[i] for i in g], 0.45) for g in groups]
            merged = oracle.lse_merge([s[0] for s in states], [s[1] for s in states], [s[2] for s in states])
            np.testing.assert_allclose(merged, full[b, h], rtol=0, atol=TIGHT)


def test_state_of_single_position_and_empty_group():
    rng = np.random.default_rng(20)
    q, K, V = _rand(rng, 1, 1, 8, 4)
    m, l, acc = oracle.span_state(q, K, V, 0, 0, [(5, 6)], 0.5)
    s = float(np.float32(0.5)) * float(q[0, 0].astype(np.float64) @ K[0, 0, 5].astype(np.float64))
    assert m == pytest.approx(s, abs=1e-15) and l == 1.0
    assert np.array_equal(acc, V[0, 0, 5].astype(np.float64))
    m, l, acc = oracle.span_state(q, K, V, 0, 0, [], 0.5)
    assert m == -np.inf and l == 0.0 and not acc.any()
    assert not oracle.lse_merge([-np.inf, -np.inf], [0.0, 0.0], np.zeros((2, 4))).any()


def test_empty_span_gives_zeros_and_flag():
    rng = np.random.default_rng(21)
    q, K, V = _rand(rng, 2, 2, 8, 4)
    off, st, en = _spans([[], [(1, 3)]])
    out, empty = oracle.span_attn(q, K, V, off, st, en, 0.5, return_empty=True)
    assert empty.tolist() == [True, False]
    assert not out[0].any() and out[1].any()


# ---------------------------------------------------------------- 16-bit storage types
def test_fp16_widening_all_bit_patterns():
    """Single-position spans return the stored V row exactly, so they expose the fp16 decoder:
    all 65536 patterns against numpy's float16."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    B, D = 512, 128
    V = bits.reshape(B, 1, 1, D)
    K = np.zeros_like(V)
    q = np.zeros((B, 1, D), np.uint16)
    off, st, en = _spans([[(0, 1)]] * B)
    got = oracle.span_attn(q, K, V, off, st, en, 1.0, dtype="f16").reshape(-1)
    ref = bits.view(np.float16).astype(np.float64)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    # (-0.0 comes back as +0.0: the output is a sum that starts from +0.0)


def test_bf16_widening_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    B, D = 512, 128
    V = bits.reshape(B, 1, 1, D)
    K = np.zeros_like(V)
    q = np.zeros((B, 1, D), np.uint16)
    off, st, en = _spans([[(0, 1)]] * B)
    got = oracle.span_attn(q, K, V, off, st, en, 1.0, dtype="bf16").reshape(-1)
    ref = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).double().numpy()
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_16bit_inputs_equal_fp32_inputs_of_the_same_values(dtype):
    """The oracle on raw 16-bit storage == the oracle on the same values held as fp32."""
    from workloads import to_host_raw, torch_dtype
    g = torch.Generator().manual_seed(22)
    B, H, L, D = 2, 3, 40, 16
    q = torch.randn((B, H, D), generator=g).to(torch_dtype(dtype))
    K = torch.randn((B, H, L, D), generator=g).to(torch_dtype(dtype))
    V = torch.randn((B, H, L, D), generator=g).to(torch_dtype(dtype))
    off, st, en = _spans([[(0, 9), (30, 40)], [(4, 5)]])
    a = oracle.span_attn(to_host_raw(q), to_host_raw(K), to_host_raw(V), off, st, en, 0.25, dtype=dtype)
    b = oracle.span_attn(q.float().numpy(), K.float().numpy(), V.float().numpy(), off, st, en, 0.25)
    assert np.array_equal(a, b)
