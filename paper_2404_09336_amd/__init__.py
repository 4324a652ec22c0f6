"""Span-restricted decode attention for MI355X (gfx950): thin Python binding over the C-ABI
library `libspanattn.so` (hand-written HIP kernels).  Argument marshalling only; there is no
CPU or PyTorch fallback — if the library is not built, calls raise."""
from .binding import (  # noqa: F401
    PreparedCall, SpanAttnError, lib_path, load_library,
    span_decode_attn, dense_decode_attn, span_decode_attn_append, dense_decode_attn_append,
    span_decode_attn_multi, prepare_span_decode_attn_multi, span_decode_attn_multi_append,
    prepare_span_decode_attn_multi_append, span_decode_attn_static, prepare_span_decode_attn_static,
    span_advance, prepare_span_advance,
    prepare_span_decode_attn, prepare_dense_decode_attn, prepare_span_decode_attn_append,
    prepare_dense_decode_attn_append,
    span_validate, span_build, span_blocks_to_intervals, span_intervals_to_blocks,
    span_plan_query, span_workspace_bytes, span_workspace_init, span_strerror,
)
