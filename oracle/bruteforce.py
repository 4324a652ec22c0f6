"""Brute-force masked softmax attention in numpy float64 (small inputs only).

TEST INFRASTRUCTURE.  Second formulation of the oracle, written from the mask
definition instead of the span: build the additive mask M over *all* ctx_len positions
(0 where the position is attended, -inf elsewhere), take the softmax of M + S over the
whole row, and multiply by all of V (Sec. 2.2, eqs. (4)-(6) and the paragraph on the
attention mask).  Every row of K and V is read, so rows outside the span must be finite.
"""
import numpy as np


def mask_from_intervals(intervals, ctx_len: int) -> np.ndarray:
    """Additive mask row: 0.0 on the union of the intervals, -inf elsewhere."""
    M = np.full(ctx_len, -np.inf, dtype=np.float64)
    for s, e in intervals:
        M[max(0, s):max(0, min(e, ctx_len))] = 0.0
    return M


def masked_attn_row(q, K, V, mask_row, scale) -> np.ndarray:
    """q [D], K/V [ctx_len, D] as float64, mask_row [ctx_len] of 0 / -inf -> out [D]."""
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    S = (K @ q) * np.float64(np.float32(scale))          # eq. (4), one row
    Z = mask_row + S                                     # M (+) S
    if not np.isfinite(Z).any():
        return np.zeros(V.shape[1], dtype=np.float64)
    Z = Z - Z[np.isfinite(Z)].max()
    A = np.exp(Z)                                        # exp(-inf) = 0 on forbidden positions
    A = A / A.sum()                                      # eq. (5)
    return A @ V                                         # eq. (6)


def masked_attn(q, K, V, per_seq_intervals, ctx_lens, scale) -> np.ndarray:
    """q [B,H,D], K/V [B,H,Lmax,D] float arrays -> out [B,H,D] float64."""
    B, H, _, D = K.shape
    out = np.zeros((B, H, D), dtype=np.float64)
    for b in range(B):
        n = int(ctx_lens[b])
        M = mask_from_intervals(per_seq_intervals[b], n)
        for h in range(H):
            out[b, h] = masked_attn_row(q[b, h], K[b, h, :n], V[b, h, :n], M, scale)
    return out


def masked_attn_from_bits(q, K, V, attend, scale) -> np.ndarray:
    """attend: bool [B, L] (True = position attended).  q [B,H,D], K/V [B,H,L,D] -> out [B,H,D] float64."""
    B, H, L, D = K.shape
    out = np.zeros((B, H, D), dtype=np.float64)
    for b in range(B):
        M = np.where(np.asarray(attend[b], dtype=bool), 0.0, -np.inf)
        for h in range(H):
            out[b, h] = masked_attn_row(q[b, h], K[b, h], V[b, h], M, scale)
    return out
