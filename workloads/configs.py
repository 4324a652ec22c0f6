"""The five decode-attention workloads, as shapes only.

Shapes follow the paper's set-up: LLaMA-7B heads (32 x 128, Sec. 2.3 and 4),
batch sizes 8-64 (Sec. 2.3, 4.1, 5.2), contexts 512-2048 tokens (Sec. 4.1),
stretched to 16384 for the stress case.  Config ids are 1-based.
"""
from dataclasses import dataclass
import math


@dataclass(frozen=True)
class DecodeConfig:
    cfg_id: int
    name: str
    batch: int
    heads: int
    head_dim: int
    max_len: int          # allocated KV length (rows per (batch, head) slab)
    min_len: int          # ctx_lens are drawn uniformly in [min_len, max_len]
    dtype: str            # "f32" | "f16" | "bf16"  (type of q, K, V)
    tol: float            # max-abs error allowed against the fp64 oracle

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)

    @property
    def elt_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def seed(self, iteration: int = 0) -> int:
        return 20240409 + 1000 * self.cfg_id + iteration


CONFIGS = {
    1: DecodeConfig(1, "tiny-f32", 1, 4, 64, 256, 256, "f32", 1e-5),
    2: DecodeConfig(2, "7b-mha-f16", 8, 32, 128, 2048, 2048, "f16", 2e-3),
    3: DecodeConfig(3, "arith-f16", 64, 32, 128, 512, 512, "f16", 2e-3),
    4: DecodeConfig(4, "summ-f16", 16, 32, 128, 4096, 2048, "f16", 2e-3),
    5: DecodeConfig(5, "stress-bf16", 32, 32, 128, 16384, 4096, "bf16", 2e-3),
}


def get_config(cfg_id: int) -> DecodeConfig:
    return CONFIGS[int(cfg_id)]
