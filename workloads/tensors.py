"""Seeded q / K / V tensors in the pre-allocated KV-cache layout.

q: [batch, heads, head_dim]; K, V: [batch, heads, max_len, head_dim], contiguous
(a per-request cache pre-allocated to its maximum length, Sec. 2.3 and Sec. 4 "Hardware and software").
Values are N(0,1) drawn in fp32 and rounded once to the workload's type; rows at
positions >= ctx_lens[b] are never valid and are filled with NaN so that any
read of them shows up in the result.
"""
import numpy as np
import torch

from .configs import DecodeConfig

_TORCH_DTYPES = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def torch_dtype(name: str) -> torch.dtype:
    return _TORCH_DTYPES[name]


def draw_qkv(cfg: DecodeConfig, ctx_lens, seed=None, device="cpu", poison=True):
    """Returns (q, K, V) on `device`.  Drawn one sequence at a time to bound the fp32 temporaries."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(int(cfg.seed() if seed is None else seed))
    dt = torch_dtype(cfg.dtype)
    B, H, D, L = cfg.batch, cfg.heads, cfg.head_dim, cfg.max_len
    q = torch.randn((B, H, D), generator=gen, device=dev, dtype=torch.float32).to(dt)
    K = torch.empty((B, H, L, D), device=dev, dtype=dt)
    V = torch.empty((B, H, L, D), device=dev, dtype=dt)
    for b in range(B):
        K[b].copy_(torch.randn((H, L, D), generator=gen, device=dev, dtype=torch.float32))
        V[b].copy_(torch.randn((H, L, D), generator=gen, device=dev, dtype=torch.float32))
        n = int(ctx_lens[b])
        if poison and n < L:
            K[b, :, n:, :] = float("nan")
            V[b, :, n:, :] = float("nan")
    return q, K, V


def draw_queries(cfg: DecodeConfig, q_len: int, seed=None, device="cpu"):
    """Query rows of `q_len` consecutive new tokens per sequence: [batch, q_len, heads, head_dim]."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(int(cfg.seed() if seed is None else seed) + 7919 * int(q_len))
    q = torch.randn((cfg.batch, int(q_len), cfg.heads, cfg.head_dim), generator=gen, device=dev, dtype=torch.float32)
    return q.to(torch_dtype(cfg.dtype))


def to_host_raw(t: torch.Tensor) -> np.ndarray:
    """Host copy with the exact bits: float32 stays float32; fp16 / bf16 become uint16 bit patterns."""
    t = t.detach().contiguous().cpu()
    if t.dtype == torch.float32:
        return t.numpy()
    if t.dtype in (torch.float16, torch.bfloat16):
        return t.view(torch.int16).numpy().view(np.uint16)
    raise TypeError(f"unsupported dtype {t.dtype}")
