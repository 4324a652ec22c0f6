"""Span-restricted decode attention for MI355X (gfx950): thin Python binding over the C-ABI
library `libspanattn.so` (hand-written HIP kernels).  Argument marshalling only; there is no
CPU or PyTorch fallback — if the library is not built, calls raise."""
from .binding import (SpanAttnError, dense_decode_attn, lib_path, load_library, span_decode_attn,  # noqa: F401
                      span_plan_splits, span_strerror, span_validate, span_workspace_bytes)
