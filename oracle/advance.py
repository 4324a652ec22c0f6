"""The step between two decode steps of one group of tokens, on plain Python lists.

TEST INFRASTRUCTURE.  Anchors and references are generated once per group of tokens (Sec. 3.2,
"Overhead"), so within a group the span only gains the token just decoded.  Stated on position sets:
with p the position the last token was appended at,

    S' = S + {p + 1}   if p is in S and p + 1 is not,     S' = S otherwise,

and the append position (and the context length) move on by one.  `advance` does that on the interval
arrays, in place, the way a caller would: the interval that ends at p + 1 grows by one position.
"""


def advance(offsets, starts, ends, append_pos, ctx_lens, max_len):
    """offsets/starts/ends/append_pos/ctx_lens: Python lists of ints (ctx_lens may be None); updated in place."""
    for b in range(len(append_pos)):
        p = append_pos[b]
        if p < 0 or p + 1 >= max_len:
            continue
        mine = range(offsets[b], offsets[b + 1])
        holds_next = any(starts[i] <= p + 1 < ends[i] for i in mine)
        if not holds_next:
            for i in mine:
                if starts[i] < ends[i] and ends[i] == p + 1:
                    ends[i] = p + 2
        append_pos[b] = p + 1
        if ctx_lens is not None:
            ctx_lens[b] += 1
