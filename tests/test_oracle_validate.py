"""The oracle's span-list validator against (a) hand-classified cases and (b) an independent
bitmap checker over an exhaustive enumeration of tiny lists."""
import itertools
import os

import numpy as np

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "validator_cases.txt")


def load_golden():
    cases = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        ctx, off, st, en, exp = [[int(x) for x in part.split()] for part in line.split("|")]
        cases.append((ctx, off, st, en, tuple(exp)))
    return cases


def bitmap_check(ctx_lens, offsets, starts, ends):
    """Independent checker: marks positions in a per-sequence bitmap and looks for positions that do
    not exist, intervals that mark nothing, double marking, and going backwards."""
    B = len(ctx_lens)
    tokens = [0] * B
    for b in range(B):
        if (b == 0 and offsets[0] != 0) or offsets[b + 1] < offsets[b] or offsets[b + 1] > len(starts):
            return 1, b, -1, tokens
        mine = list(zip(starts[offsets[b]:offsets[b + 1]], ends[offsets[b]:offsets[b + 1]]))
        if not mine:
            return 6, b, -1, tokens
        bitmap = [False] * max(ctx_lens[b], 0)
        prev_start = None
        for i, (s, e) in enumerate(mine):
            cells = list(range(s, e))
            if s < 0 or e > len(bitmap):
                return 2, b, i, tokens
            if not cells:
                return 3, b, i, tokens
            if prev_start is not None and s >= prev_start and any(bitmap[c] for c in cells):
                return 4, b, i, tokens
            if prev_start is not None and s < prev_start:
                return 5, b, i, tokens
            for c in cells:
                bitmap[c] = True
            prev_start = s
        tokens[b] = sum(bitmap)
    return 0, -1, -1, tokens


def test_golden_cases():
    for ctx, off, st, en, exp in load_golden():
        code, bs, bi, _ = oracle.validate(off, st, en, ctx)
        assert (code, bs, bi) == exp, (ctx, off, st, en)


def test_bitmap_checker_agrees_with_golden():
    for ctx, off, st, en, exp in load_golden():
        assert bitmap_check(ctx, off, st, en)[:3] == exp


def test_exhaustive_single_sequence():
    """All lists of up to 3 intervals with endpoints in [-1, len+1], len in 1..4."""
    n = 0
    for L in range(1, 5):
        pts = range(-1, L + 2)
        pairs = list(itertools.product(pts, pts))
        for k in range(0, 4):
            if k == 3 and L > 3:
                continue
            for combo in itertools.product(pairs, repeat=k):
                st = [c[0] for c in combo]
                en = [c[1] for c in combo]
                code, bs, bi, tok = oracle.validate([0, k], st, en, [L])
                ecode, ebs, ebi, etok = bitmap_check([L], [0, k], st, en)
                assert (code, bs, bi) == (ecode, ebs, ebi), (L, st, en)
                if code == 0:
                    assert tok.tolist() == etok
                n += 1
    assert n > 70000


def test_exhaustive_offsets_two_sequences():
    st, en = [0, 2, 1], [1, 3, 2]
    for off in itertools.product(range(-1, 5), repeat=3):
        code, bs, bi, _ = oracle.validate(list(off), st, en, [3, 3])
        assert (code, bs, bi) == bitmap_check([3, 3], list(off), st, en)[:3], off


def test_tokens_per_seq_on_workloads():
    from workloads import CONFIGS, draw_spans
    for cid in (1, 2, 3, 4):
        sp = draw_spans(CONFIGS[cid])
        code, bs, bi, tok = oracle.validate(sp.offsets, sp.starts, sp.ends, sp.ctx_lens)
        assert (code, bs, bi) == (0, -1, -1)
        assert tok.tolist() == sp.tokens_per_seq().tolist()
