"""Set-based reference for the blocked span encoding (TEST INFRASTRUCTURE).

Sec. 3.3 "Attention span encoding" / Fig. 3: the context is cut into blocks of a fixed size; a request
lists the blocks that hold span positions, each with its block index and a per-token binary mask;
untouched blocks are left out.  Here everything goes through a plain Python set of positions, so the
answers are obvious: an encoding and an interval list are equivalent iff their position sets are equal,
and the canonical interval list of a set is its maximal runs in ascending order.
"""
import numpy as np


def positions_from_blocks(block_size, block_idx, block_masks):
    """block_masks: one row of block_size // 32 uint32 words per block (bit t%32 of word t//32 = token t)."""
    pos = set()
    for j, blk in enumerate(block_idx):
        for t in range(block_size):
            if (int(block_masks[j][t // 32]) >> (t % 32)) & 1:
                pos.add(int(blk) * block_size + t)
    return pos


def positions_from_intervals(intervals):
    pos = set()
    for s, e in intervals:
        pos.update(range(int(s), int(e)))
    return pos


def maximal_runs(positions):
    """Canonical interval list of a position set: sorted, disjoint, non-touching."""
    out = []
    for p in sorted(positions):
        if out and out[-1][1] == p:
            out[-1][1] = p + 1
        else:
            out.append([p, p + 1])
    return [(s, e) for s, e in out]


def blocks_from_positions(block_size, positions):
    """Ascending touched blocks: (block_idx list, masks uint32 [n, block_size // 32])."""
    idx = sorted({p // block_size for p in positions})
    masks = np.zeros((len(idx), block_size // 32), dtype=np.uint32)
    row = {blk: j for j, blk in enumerate(idx)}
    for p in positions:
        t = p % block_size
        masks[row[p // block_size], t // 32] |= np.uint32(1 << (t % 32))
    return idx, masks
