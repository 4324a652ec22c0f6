"""Span builder (anchors + references -> interval list, Sec. 3.2) against a set-based reference."""
import numpy as np
import pytest

import paper_2404_09336_amd as span
from oracle import builder as ref


def arithmetic_trace():
    """A token layout with the reference structure of the paper's arithmetic example (Fig. 5): a task line
    closed by anchor 0, two working lines that each refer to the previous line, an anchor 1, a line that
    refers to anchors 0 and 1 and ends with anchor 2, and a last line that refers to 0, 1 and 2.
    Token counts are made up; only the structure matters."""
    lines = [(0, 14), (14, 39), (39, 52), (52, 63), (63, 70)]      # [start, end) of each line
    anchors = [(0, 14), (39, 52), (52, 63)]                        # anchor k names the line it closes
    refs = [None, [-1], [-1], [0, 1], [0, 1, 2]]                   # what each line attends to
    return lines, anchors, refs


def test_arithmetic_trace_structure():
    lines, anchors, refs = arithmetic_trace()
    # while the 4th line (index 3) is written, 5 tokens in: task line + anchor-1 line + the line itself
    got = span.span_build(anchors, refs[3], 0, lines[2][0], lines[3][0], lines[3][0] + 5)
    assert got == [(0, 14), (39, 57)]            # anchor 1's line touches the current line: one interval
    # the 3rd line refers to the previous line only
    got = span.span_build(anchors, refs[2], 0, lines[1][0], lines[2][0], lines[2][0] + 1)
    assert got == [(14, 40)]
    # the last line: all three anchors, 7 tokens in; anchors 1 and 2 and the line are contiguous
    got = span.span_build(anchors, refs[4], 0, lines[3][0], lines[4][0], 70)
    assert got == [(0, 14), (39, 70)]


def test_summarization_line_ranges():
    """Fig. 7 style: instruction always attended, line-number anchors, references are line ranges,
    plus the previous summary sentence (Sec. 4.2)."""
    instr = 20
    sent = [(instr + 30 * i, instr + 30 * (i + 1)) for i in range(31)]     # 31 article sentences
    art_end = sent[-1][1]
    # second summary sentence refers to lines 17-19; previous sentence is [art_end, art_end + 25)
    got = span.span_build(sent, [(17, 19), -1], instr, art_end, art_end + 25, art_end + 25 + 4)
    assert got == [(0, instr), (sent[17][0], sent[19][1]), (art_end, art_end + 29)]
    assert got == ref.build(sent, [(17, 19), -1], instr, art_end, art_end + 25, art_end + 29)


def test_random_against_set_reference():
    rng = np.random.default_rng(0)
    for trial in range(500):
        ctx = int(rng.integers(1, 400))
        na = int(rng.integers(0, 12))
        cuts = np.sort(rng.integers(0, ctx + 1, size=2 * na)).reshape(na, 2) if na else np.zeros((0, 2), int)
        if trial % 3 == 0 and na:                      # overlapping / nested anchor ranges too
            cuts = np.sort(rng.integers(0, ctx + 1, size=(na, 2)), axis=1)
        anchors = [(int(a), int(b)) for a, b in cuts]
        refs = []
        for _ in range(int(rng.integers(0, 6))):
            kind = rng.integers(0, 3)
            if kind == 0 or na == 0:
                refs.append(-1)
            elif kind == 1:
                refs.append(int(rng.integers(0, na)))
            else:
                f = int(rng.integers(0, na))
                refs.append((f, int(rng.integers(f, na))))
        cur = int(rng.integers(0, ctx + 1))
        prev = int(rng.integers(0, cur + 1))
        prefix = int(rng.integers(0, ctx + 1)) if trial % 2 else 0
        got = span.span_build(anchors, refs, prefix, prev, cur, ctx)
        assert got == ref.build(anchors, refs, prefix, prev, cur, ctx), (anchors, refs, prefix, prev, cur, ctx)
        if got:
            flat = np.array(got, np.int32)
            code = span.span_validate([0, len(got)], flat[:, 0], flat[:, 1], [ctx])[0]
            assert code == 0
            assert all(b[0] > a[1] for a, b in zip(got, got[1:]))          # non-touching


def test_errors():
    A = [(0, 5), (5, 9)]
    for args, code in (((A, [2], 0, 0, 9, 10), 2), ((A, [(1, 0)], 0, 0, 9, 10), 2), ((A, [-2], 0, 0, 9, 10), 2),
                       (([(0, 50)], [0], 0, 0, 9, 10), 2), (([(6, 5)], [0], 0, 0, 9, 10), 2),
                       ((A, [0], 11, 0, 9, 10), 2), ((A, [0], 0, 9, 8, 10), 2), ((A, [0], 0, 0, 11, 10), 2)):
        with pytest.raises(span.SpanAttnError) as e:
            span.span_build(*args)
        assert e.value.code == code, args
    assert span.span_build([], [], 0, 0, 0, 0) == []
    assert span.span_build(A, [], 0, 0, 10, 10) == []          # nothing referenced, nothing written yet


def test_many_intervals_grow_the_output():
    anchors = [(4 * i, 4 * i + 2) for i in range(100)]
    got = span.span_build(anchors, [(0, 99)], 0, 400, 400, 401)
    assert got == ref.build(anchors, [(0, 99)], 0, 400, 400, 401) and len(got) == 101


@pytest.mark.gpu
def test_decode_loop_over_lines(gpu_device):
    """The span path inside a toy decode loop: for every new token of two 'lines', rebuild the span from the
    anchor table and the line's references, attend with the HIP kernel, compare with the fp64 oracle."""
    import torch
    import oracle
    from workloads import DecodeConfig, draw_qkv, to_host_raw
    lines, anchors, refs = arithmetic_trace()
    B, H, D, L = 2, 4, 128, 80
    cfg = DecodeConfig(93, "loop", B, H, D, L, L, "f16", 2e-3)
    q, K, V = draw_qkv(cfg, [L, L], device=gpu_device, seed=31, poison=False)
    hq, hK, hV = to_host_raw(q), to_host_raw(K), to_host_raw(V)
    worst = 0.0
    for line in (3, 4):
        for t in range(lines[line][0] + 1, lines[line][1] + 1, 3):          # ctx_len as the line grows
            per_seq = [span.span_build(anchors, refs[line], 0, lines[line - 1][0], lines[line][0], t),
                       [(0, t)]]                                             # sequence 1 is emitting references: dense
            off = np.array([0, len(per_seq[0]), len(per_seq[0]) + 1], np.int32)
            st = np.array([s for iv in per_seq for s, _ in iv], np.int32)
            en = np.array([e for iv in per_seq for _, e in iv], np.int32)
            ctx = np.array([t, t], np.int32)
            code, _, _, tok = span.span_validate(off, st, en, ctx)
            assert code == 0
            dev = lambda a: torch.from_numpy(a).to(gpu_device)
            out = span.span_decode_attn(q, K, V, dev(off), dev(st), dev(en), dev(ctx), np.float32(cfg.scale),
                                        max_tokens=int(tok.max()), tokens_per_seq=tok)
            torch.cuda.synchronize()
            want = oracle.span_attn(hq, hK, hV, off, st, en, np.float32(cfg.scale), dtype="f16")
            worst = max(worst, float(np.abs(out.cpu().numpy() - want).max()))
    print(f"[parity] decode loop over lines: worst max-abs err {worst:.3e}")
    assert worst <= cfg.tol
