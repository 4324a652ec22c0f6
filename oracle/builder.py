"""Set-based reference for building a span from anchors and references (TEST INFRASTRUCTURE).

Sec. 3.2: the context is partitioned into groups of contiguous tokens, each named by an anchor that
follows it; before a line is generated the model emits references (anchor ids; `[-1]` = the previous
line, Fig. 5; `(a-b)` = a range of line-number anchors, Fig. 7); the tokens of the line then attend only
to the referenced groups, plus what is always kept (the instruction, Sec. 4.2; and the line being written
itself, which a causal decoder always sees).  Everything here is a plain Python set of positions.
"""
from .blocks import maximal_runs


def span_positions(anchors, refs, prefix_end, prev_line_start, cur_line_start, ctx_len):
    pos = set(range(0, prefix_end)) | set(range(cur_line_start, ctx_len))
    for r in refs:
        first, last = (r, r) if isinstance(r, int) else r
        if first == -1:
            pos |= set(range(prev_line_start, cur_line_start))
        else:
            for k in range(first, last + 1):
                pos |= set(range(anchors[k][0], anchors[k][1]))
    return pos


def build(anchors, refs, prefix_end, prev_line_start, cur_line_start, ctx_len):
    return maximal_runs(span_positions(anchors, refs, prefix_end, prev_line_start, cur_line_start, ctx_len))
