"""Span-restricted decode attention for MI355X (gfx950): thin Python binding over the C-ABI
library `libspanattn.so` (hand-written HIP kernels).  Argument marshalling only; there is no
CPU or PyTorch fallback — if the library is not built, calls raise."""
from .binding import (PreparedCall, SpanAttnError, dense_decode_attn, lib_path, load_library,  # noqa: F401
                      prepare_dense_decode_attn, prepare_span_decode_attn, span_blocks_to_intervals, span_build,
                      span_intervals_to_blocks, span_decode_attn, span_plan_query, span_strerror, span_validate, span_workspace_bytes, span_workspace_init)
