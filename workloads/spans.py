"""Seeded span lists shaped like the paper's two tasks.

A span is, per sequence, a sorted list of pairwise-disjoint half-open KV-position
intervals [start, end): an always-kept instruction prefix, the ranges named by
the references, and the most recent tokens (Sec. 3.2 "Token generation",
Fig. 5 and Fig. 7, Sec. 4.2 on the always-attended instruction and previous
sentence).  Intervals are shared by all heads of a sequence (Sec. 3.3: metadata
is kept per request).
"""
from dataclasses import dataclass
import numpy as np

from .configs import DecodeConfig


@dataclass
class SpanBatch:
    offsets: np.ndarray   # int32 [batch+1]; intervals of sequence b are offsets[b]..offsets[b+1]-1
    starts: np.ndarray    # int32 [offsets[-1]], inclusive
    ends: np.ndarray      # int32 [offsets[-1]], exclusive
    ctx_lens: np.ndarray  # int32 [batch], number of valid KV rows per sequence

    @property
    def batch(self) -> int:
        return int(self.ctx_lens.shape[0])

    def intervals(self, b: int):
        lo, hi = int(self.offsets[b]), int(self.offsets[b + 1])
        return [(int(s), int(e)) for s, e in zip(self.starts[lo:hi], self.ends[lo:hi])]

    def tokens_per_seq(self) -> np.ndarray:
        out = np.zeros(self.batch, dtype=np.int64)
        for b in range(self.batch):
            out[b] = sum(e - s for s, e in self.intervals(b))
        return out

    def coverage(self) -> float:
        return float(self.tokens_per_seq().sum()) / float(self.ctx_lens.astype(np.int64).sum())

    @staticmethod
    def from_lists(per_seq, ctx_lens) -> "SpanBatch":
        offsets = [0]
        starts, ends = [], []
        for iv in per_seq:
            for s, e in iv:
                starts.append(s)
                ends.append(e)
            offsets.append(len(starts))
        return SpanBatch(np.asarray(offsets, dtype=np.int32),
                         np.asarray(starts, dtype=np.int32).reshape(-1),
                         np.asarray(ends, dtype=np.int32).reshape(-1),
                         np.asarray(ctx_lens, dtype=np.int32).reshape(-1))


def place_disjoint(rng: np.random.Generator, lengths, lo: int, hi: int):
    """Place intervals of the given lengths, in order, without overlap in [lo, hi).

    The free room is split by k sorted uniform gaps, so the result is sorted,
    disjoint and possibly adjacent.  Returns a list of (start, end).
    """
    lengths = [int(x) for x in lengths]
    free = (hi - lo) - sum(lengths)
    if free < 0:
        raise ValueError("intervals do not fit")
    gaps = np.sort(rng.integers(0, free + 1, size=len(lengths)))
    out, used = [], 0
    for g, n in zip(gaps, lengths):
        s = lo + int(g) + used
        out.append((s, s + n))
        used += n
    return out


def _draw_lengths_fit(rng, k, lo_len, hi_len, room):
    while True:
        lens = rng.integers(lo_len, hi_len + 1, size=k)
        if int(lens.sum()) <= room:
            return lens


def draw_spans(cfg: DecodeConfig, seed=None, coverage=None) -> SpanBatch:
    """Span lists and context lengths for one of the five workloads.

    `coverage` (a fraction) only applies to the stress workload: every sequence
    then uses that target instead of drawing one from {5, 10, 25, 50} %.
    """
    rng = np.random.default_rng(cfg.seed() if seed is None else seed)
    B = cfg.batch
    ctx = rng.integers(cfg.min_len, cfg.max_len + 1, size=B).astype(np.int32)
    per_seq = []
    for b in range(B):
        L = int(ctx[b])
        if cfg.cfg_id == 1:
            lens = rng.integers(8, 33, size=3)
            iv = place_disjoint(rng, lens, 0, L - 16) + [(L - 16, L)]
        elif cfg.cfg_id == 2:
            k = int(rng.integers(4, 13))
            lens = _draw_lengths_fit(rng, k, 16, 128, L - 32 - 64)
            iv = [(0, 64)] + place_disjoint(rng, lens, 64, L - 32) + [(L - 32, L)]
        elif cfg.cfg_id == 3:
            lens = rng.integers(4, 17, size=2)
            iv = [(0, 128)] + place_disjoint(rng, lens, 128, L - 8) + [(L - 8, L)]
        elif cfg.cfg_id == 4:
            generated = int(rng.integers(1, 193))
            art_lo, art_hi = 48, L - generated
            k = int(rng.integers(1, 4))
            lens = _draw_lengths_fit(rng, k, 50, 400, art_hi - art_lo)
            recent = min(128, generated)
            iv = [(0, 48)] + place_disjoint(rng, lens, art_lo, art_hi) + [(L - recent, L)]
        elif cfg.cfg_id == 5:
            k = int(rng.integers(16, 65))
            c = float(rng.choice([0.05, 0.10, 0.25, 0.50])) if coverage is None else float(coverage)
            total = max(k, int(round(c * L)))
            cuts = np.sort(rng.choice(np.arange(1, total), size=k - 1, replace=False))
            lens = np.diff(np.concatenate(([0], cuts, [total])))
            iv = place_disjoint(rng, lens, 0, L)
        else:
            raise ValueError(f"unknown config {cfg.cfg_id}")
        per_seq.append(iv)
    return SpanBatch.from_lists(per_seq, ctx)


def full_cover_spans(ctx_lens) -> SpanBatch:
    """One interval [0, len) per sequence: the dense-attention-through-the-span-path control (Sec. 4.1)."""
    ctx_lens = np.asarray(ctx_lens, dtype=np.int32)
    return SpanBatch.from_lists([[(0, int(L))] for L in ctx_lens], ctx_lens)


def microbench_spans(batch: int, length: int, sparsity_block: int, seed: int, keep: float = 0.5) -> SpanBatch:
    """Masks of the kernel micro-benchmark (Sec. 5.2): the context is cut into
    runs of `sparsity_block` tokens and a random `keep` fraction of the runs is
    attended.  Neighbouring kept runs are joined into one interval."""
    rng = np.random.default_rng(seed)
    nblk = length // sparsity_block
    nkeep = max(1, int(round(keep * nblk)))
    per_seq = []
    for _ in range(batch):
        kept = np.sort(rng.choice(nblk, size=nkeep, replace=False))
        iv = []
        for blk in kept:
            s, e = int(blk) * sparsity_block, (int(blk) + 1) * sparsity_block
            if iv and iv[-1][1] == s:
                iv[-1] = (iv[-1][0], e)
            else:
                iv.append((s, e))
        per_seq.append(iv)
    return SpanBatch.from_lists(per_seq, np.full(batch, length, dtype=np.int32))


def random_mask_spans(batch: int, length: int, run: int, seed: int, keep: float = 0.5) -> SpanBatch:
    """Unstructured masks (the paper's kernel takes any mask, Sec. 5.2): the context is cut into runs of `run`
    tokens, each kept with probability `keep` independently (run = 1: every token decides for itself); the
    newest token always attends itself.  Returned as the interval list of the kept positions."""
    rng = np.random.default_rng(seed)
    per_seq = []
    for _ in range(batch):
        kept = np.repeat(rng.random(-(-length // run)) < keep, run)[:length]
        kept[-1] = True
        edges = np.flatnonzero(np.diff(np.concatenate(([0], kept.view(np.int8), [0]))))
        per_seq.append(list(zip(edges[0::2].tolist(), edges[1::2].tolist())))
    return SpanBatch.from_lists(per_seq, np.full(batch, length, dtype=np.int32))
