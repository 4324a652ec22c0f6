"""Seeded synthetic inputs for span-sparse decode attention.

This package only *draws inputs*: span lists (numpy, host) and q/K/V tensors
(torch, on the device asked for).  It holds none of the method's arithmetic
(no dot products, no softmax, no validation rules), so both the HIP path and
the CPU oracle can be fed from it without sharing any code of their own.
"""
from .configs import CONFIGS, DecodeConfig, get_config
from .spans import (SpanBatch, draw_spans, place_disjoint, full_cover_spans, microbench_spans,
                    random_mask_spans)
from .tensors import draw_qkv, draw_queries, to_host_raw, torch_dtype

__all__ = [
    "CONFIGS", "DecodeConfig", "get_config",
    "SpanBatch", "draw_spans", "place_disjoint", "full_cover_spans", "microbench_spans", "random_mask_spans",
    "draw_qkv", "draw_queries", "to_host_raw", "torch_dtype",
]
