"""The step between two decode steps of one group of tokens, on plain Python lists.

TEST INFRASTRUCTURE.  Anchors and references are generated once per group of tokens (Sec. 3.2,
"Overhead"), so within a group the span only gains the tokens just decoded.  Stated on position sets:
with n tokens per step and p the position the first of the last step's tokens was appended at,

    S' = S + {p + n, ..., p + 2n - 1}   if an interval of S ends at p + n and none of those positions is in S,
    S' = S                              otherwise,

and the append position (and the context length) move on by n.  `advance` does that on the interval
arrays, in place, the way a caller would: the interval that ends at p + n grows by n positions.  n = 1 is
the one-token decode step.
"""


def advance(offsets, starts, ends, append_pos, ctx_lens, max_len, count=1):
    """offsets/starts/ends/append_pos/ctx_lens: Python lists of ints (ctx_lens may be None); updated in place."""
    n = count
    for b in range(len(append_pos)):
        p = append_pos[b]
        if p < 0 or p + 2 * n > max_len:
            continue
        mine = range(offsets[b], offsets[b + 1])
        nxt = set(range(p + n, p + 2 * n))
        holds_next = any(starts[i] <= q < ends[i] for i in mine for q in nxt)
        if not holds_next:
            for i in mine:
                if starts[i] < ends[i] and ends[i] == p + n:
                    ends[i] = p + 2 * n
        append_pos[b] = p + n
        if ctx_lens is not None:
            ctx_lens[b] += n
