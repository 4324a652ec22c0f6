"""ctypes binding with the same names as the C entry points of include/span_attn.h.

Tensors are torch tensors that already live on the GPU; this module only checks their type and
contiguity, fills the descriptor, and passes raw device pointers and the current HIP stream.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libspanattn.so")
_lib = None

SPAN_F32, SPAN_F16, SPAN_BF16 = 0, 1, 2


class SpanAttnError(RuntimeError):
    def __init__(self, code, where):
        self.code = int(code)
        super().__init__(f"{where} failed with code {code}: {span_strerror(code)}")


class _Desc(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("max_len", ctypes.c_int32), ("dtype", ctypes.c_int32), ("num_intervals", ctypes.c_int32),
                ("max_tokens", ctypes.c_int32), ("num_splits", ctypes.c_int32),
                ("tokens_per_seq", ctypes.c_void_p), ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
                ("stream", ctypes.c_void_p), ("q_len", ctypes.c_int32),
                ("host_span_offsets", ctypes.c_void_p), ("host_span_starts", ctypes.c_void_p),
                ("host_span_ends", ctypes.c_void_p)]


class PlanInfo(ctypes.Structure):
    _fields_ = [("exact", ctypes.c_int32), ("slice_tokens", ctypes.c_int32), ("max_splits", ctypes.c_int32),
                ("slice_limit", ctypes.c_int32), ("workgroups", ctypes.c_int64), ("workspace_bytes", ctypes.c_int64),
                ("runs_in_arguments", ctypes.c_int32), ("queries_per_pass", ctypes.c_int32)]

    def as_dict(self):
        return {"exact": bool(self.exact), "slice_tokens": self.slice_tokens, "max_splits": self.max_splits,
                "slice_limit": self.slice_limit, "workgroups": self.workgroups, "workspace_bytes": self.workspace_bytes,
                "runs_in_arguments": bool(self.runs_in_arguments), "queries_per_pass": int(self.queries_per_pass)}


def lib_path() -> str:
    """The product library, or the measurement variant of it that SPAN_ATTN_VARIANT names (see build.py)."""
    variant = os.environ.get("SPAN_ATTN_VARIANT", "")
    return os.path.join(_HERE, f"libspanattn_{variant}.so") if variant else _LIB_PATH


def load_library():
    """Loads libspanattn.so; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build it with "
                               "`python -m paper_2404_09336_amd.build` (needs hipcc)")
        lib = ctypes.CDLL(path)
        P, I32, F = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float
        DP = ctypes.POINTER(_Desc)
        lib.span_decode_attn.argtypes = [DP, P, P, P, P, P, P, P, F, P]
        lib.span_decode_attn.restype = ctypes.c_int
        lib.span_decode_attn_static.argtypes = [DP, P, P, P, P, P, P, P, F, P]
        lib.span_decode_attn_static.restype = ctypes.c_int
        lib.span_decode_attn_multi.argtypes = [DP, P, P, P, P, P, P, P, F, P]
        lib.span_decode_attn_multi.restype = ctypes.c_int
        lib.dense_decode_attn.argtypes = [DP, P, P, P, P, F, P]
        lib.dense_decode_attn.restype = ctypes.c_int
        lib.span_decode_attn_append.argtypes = [DP, P, P, P, P, P, P, P, P, P, F, P]
        lib.span_decode_attn_append.restype = ctypes.c_int
        lib.dense_decode_attn_append.argtypes = [DP, P, P, P, P, P, P, P, F, P]
        lib.dense_decode_attn_append.restype = ctypes.c_int
        lib.span_decode_attn_multi_append.argtypes = [DP, P, P, P, P, P, P, P, P, P, F, P]
        lib.span_decode_attn_multi_append.restype = ctypes.c_int
        lib.span_advance.argtypes = [DP, P, P, P, P, P]
        lib.span_advance.restype = ctypes.c_int
        lib.span_validate.argtypes = [I32, I32, P, P, P, P, P, P, P]
        lib.span_validate.restype = ctypes.c_int
        lib.span_plan_query.argtypes = [DP, ctypes.POINTER(PlanInfo)]
        lib.span_plan_query.restype = ctypes.c_int
        lib.span_workspace_bytes.argtypes = [DP]
        lib.span_workspace_bytes.restype = ctypes.c_size_t
        lib.span_workspace_init.argtypes = [DP]
        lib.span_workspace_init.restype = ctypes.c_int
        lib.span_blocks_to_intervals.argtypes = [I32, I32, P, P, P, I32, P, P, P, P]
        lib.span_blocks_to_intervals.restype = ctypes.c_int
        lib.span_intervals_to_blocks.argtypes = [I32, I32, P, P, P, I32, P, P, P, P]
        lib.span_intervals_to_blocks.restype = ctypes.c_int
        lib.span_build.argtypes = [I32, P, P, I32, P, P, I32, I32, I32, I32, I32, P, P, P]
        lib.span_build.restype = ctypes.c_int
        lib.span_strerror.argtypes = [ctypes.c_int]
        lib.span_strerror.restype = ctypes.c_char_p
        lib.span_last_hip_error.restype = ctypes.c_int
        _lib = lib
    return _lib


def span_strerror(code: int) -> str:
    return load_library().span_strerror(int(code)).decode()


def _dtype_code(t):
    import torch
    try:
        return {torch.float32: SPAN_F32, torch.float16: SPAN_F16, torch.bfloat16: SPAN_BF16}[t.dtype]
    except KeyError:
        raise TypeError(f"unsupported dtype {t.dtype}") from None


def make_desc(batch, heads, head_dim, max_len, dtype_code, num_intervals=0, max_tokens=0, num_splits=0,
              workspace_ptr=0, workspace_bytes=0, stream=0, tokens_per_seq=None, q_len=0, host_spans=None) -> _Desc:
    """tokens_per_seq: host int64 numpy array [batch] or None.  host_spans: (offsets, starts, ends) host int32
    arrays, copies of the device span lists, or None.  The descriptor keeps references to the host arrays."""
    d = _Desc(batch, heads, head_dim, max_len, dtype_code, num_intervals, max_tokens, num_splits, None,
              workspace_ptr or None, workspace_bytes, stream or None, int(q_len), None, None, None)
    if host_spans is not None:
        off, st, en = (np.ascontiguousarray(a, dtype=np.int32).reshape(-1) for a in host_spans)
        if off.shape[0] != batch + 1 or st.shape[0] != num_intervals or en.shape[0] != num_intervals:
            raise ValueError("host_spans must be (offsets[batch+1], starts[num_intervals], ends[num_intervals])")
        if st.shape[0] == 0:                       # keep the pointers non-NULL for an empty list
            st, en = np.zeros(1, np.int32), np.zeros(1, np.int32)
        d._host_spans_keepalive = (off, st, en)
        d.host_span_offsets, d.host_span_starts, d.host_span_ends = off.ctypes.data, st.ctypes.data, en.ctypes.data
    if tokens_per_seq is not None:
        tok = np.ascontiguousarray(tokens_per_seq, dtype=np.int64).reshape(-1)
        if tok.shape[0] != batch:
            raise ValueError("tokens_per_seq must have one entry per sequence")
        d._tokens_keepalive = tok
        d.tokens_per_seq = tok.ctypes.data
    return d


def span_plan_query(desc: _Desc) -> dict:
    info = PlanInfo()
    rc = load_library().span_plan_query(ctypes.byref(desc), ctypes.byref(info))
    if rc != 0:
        raise SpanAttnError(rc, "span_plan_query")
    return info.as_dict()


def span_workspace_bytes(desc: _Desc) -> int:
    return int(load_library().span_workspace_bytes(ctypes.byref(desc)))


def span_workspace_init(desc: _Desc) -> None:
    """Zeroes the ticket counters at the head of desc.workspace (enqueued on desc.stream)."""
    rc = load_library().span_workspace_init(ctypes.byref(desc))
    if rc != 0:
        raise SpanAttnError(rc, "span_workspace_init")


def prepare_span_advance(span_offsets, span_starts, span_ends, append_pos, ctx_lens=None, *, max_len, stream=None,
                         q_len=0):
    """Device int32 tensors; span_ends, append_pos and ctx_lens (optional) are updated in place on the GPU.
    q_len: tokens appended per step (0 or 1 for the one-token calls)."""
    import torch
    lib = load_library()
    batch, n_int = int(append_pos.numel()), int(span_starts.numel())
    if stream is None:
        stream = torch.cuda.current_stream(append_pos.device).cuda_stream
    desc = make_desc(batch, 1, 64, int(max_len), SPAN_F32, n_int, stream=stream, q_len=q_len)
    args = (ctypes.byref(desc), _i32_dev(span_offsets, batch + 1, "span_offsets"), _i32_dev(span_starts, n_int, "span_starts"),
            _i32_dev(span_ends, n_int, "span_ends"), _i32_dev(append_pos, batch, "append_pos"),
            _i32_dev(ctx_lens, batch, "ctx_lens") if ctx_lens is not None else None)
    keep = (span_offsets, span_starts, span_ends, append_pos, ctx_lens)
    return PreparedCall("span_advance", lib.span_advance, desc, args, None, keep)


def span_advance(span_offsets, span_starts, span_ends, append_pos, ctx_lens=None, *, max_len, stream=None, q_len=0):
    prepare_span_advance(span_offsets, span_starts, span_ends, append_pos, ctx_lens, max_len=max_len, stream=stream,
                         q_len=q_len)()


def span_validate(span_offsets, span_starts, span_ends, ctx_lens):
    """Host arrays in, (code, first_bad_seq, first_bad_interval, tokens_per_seq[int64]) out."""
    off = np.ascontiguousarray(span_offsets, dtype=np.int32)
    st = np.ascontiguousarray(span_starts, dtype=np.int32).reshape(-1)
    en = np.ascontiguousarray(span_ends, dtype=np.int32).reshape(-1)
    ctx = np.ascontiguousarray(ctx_lens, dtype=np.int32).reshape(-1)
    if off.shape != (ctx.shape[0] + 1,) or st.shape != en.shape:
        raise ValueError("span_offsets must have batch+1 entries and starts / ends equal lengths")
    bs, bi = np.full(1, -7, np.int32), np.full(1, -7, np.int32)
    tok = np.zeros(ctx.shape[0], dtype=np.int64)
    vp = lambda a: ctypes.c_void_p(a.ctypes.data)
    rc = load_library().span_validate(ctx.shape[0], st.shape[0], vp(off), vp(st), vp(en), vp(ctx), vp(bs), vp(bi),
                                      vp(tok))
    if rc < 0:
        raise SpanAttnError(rc, "span_validate")
    return int(rc), int(bs[0]), int(bi[0]), tok


def span_blocks_to_intervals(block_size, block_offsets, block_idx, block_masks):
    """Host arrays of the blocked encoding in -> (span_offsets, span_starts, span_ends) int32 arrays out.
    block_masks: uint32 [num_blocks, block_size // 32].  Raises SpanAttnError on a malformed encoding."""
    lib = load_library()
    boff = np.ascontiguousarray(block_offsets, dtype=np.int32)
    bidx = np.ascontiguousarray(block_idx, dtype=np.int32).reshape(-1)
    bm = np.ascontiguousarray(block_masks, dtype=np.uint32).reshape(-1)
    batch = boff.shape[0] - 1
    if bm.shape[0] != bidx.shape[0] * (block_size // 32 if block_size > 0 else 0) and block_size > 0 and block_size % 32 == 0:
        raise ValueError("block_masks must hold block_size/32 words per block")
    vp = lambda a: ctypes.c_void_p(a.ctypes.data)
    off = np.zeros(batch + 1, np.int32)
    needed = np.zeros(1, np.int32)
    cap = max(16, 2 * bidx.shape[0])
    while True:
        st, en = np.zeros(cap, np.int32), np.zeros(cap, np.int32)
        rc = lib.span_blocks_to_intervals(batch, int(block_size), vp(boff), vp(bidx), vp(bm), cap, vp(off), vp(st),
                                          vp(en), vp(needed))
        if rc == -6:
            cap = int(needed[0])
            continue
        if rc != 0:
            raise SpanAttnError(rc, "span_blocks_to_intervals")
        n = int(needed[0])
        return off, st[:n].copy(), en[:n].copy()


def span_intervals_to_blocks(block_size, span_offsets, span_starts, span_ends):
    """Interval lists in -> (block_offsets, block_idx, block_masks[num_blocks, block_size//32]) out."""
    lib = load_library()
    off = np.ascontiguousarray(span_offsets, dtype=np.int32)
    st = np.ascontiguousarray(span_starts, dtype=np.int32).reshape(-1)
    en = np.ascontiguousarray(span_ends, dtype=np.int32).reshape(-1)
    batch = off.shape[0] - 1
    vp = lambda a: ctypes.c_void_p(a.ctypes.data)
    boff = np.zeros(batch + 1, np.int32)
    needed = np.zeros(1, np.int32)
    words = max(1, block_size // 32)
    cap = max(16, 2 * st.shape[0])
    while True:
        bidx, bm = np.zeros(cap, np.int32), np.zeros(cap * words, np.uint32)
        rc = lib.span_intervals_to_blocks(batch, int(block_size), vp(off), vp(st), vp(en), cap, vp(boff), vp(bidx),
                                          vp(bm), vp(needed))
        if rc == -6:
            cap = int(needed[0])
            continue
        if rc != 0:
            raise SpanAttnError(rc, "span_intervals_to_blocks")
        n = int(needed[0])
        return boff, bidx[:n].copy(), bm[:n * words].reshape(n, words).copy()


def span_build(anchors, refs, prefix_end, prev_line_start, cur_line_start, ctx_len):
    """One sequence: anchors = [(start, end), ...] by anchor id; refs = ids, (first, last) id ranges, or -1 for
    the previous line.  Returns the list of (start, end) intervals, sorted, disjoint and non-touching."""
    lib = load_library()
    a_st = np.ascontiguousarray([a[0] for a in anchors], dtype=np.int32)
    a_en = np.ascontiguousarray([a[1] for a in anchors], dtype=np.int32)
    firsts, lasts = [], []
    for r in refs:
        f, l = (r, r) if np.isscalar(r) else r
        firsts.append(f)
        lasts.append(l)
    r_f = np.ascontiguousarray(firsts, dtype=np.int32)
    r_l = np.ascontiguousarray(lasts, dtype=np.int32)
    vp = lambda x: ctypes.c_void_p(x.ctypes.data) if x.size else None
    needed = np.zeros(1, np.int32)
    cap = 16
    while True:
        st, en = np.zeros(cap, np.int32), np.zeros(cap, np.int32)
        rc = lib.span_build(len(anchors), vp(a_st), vp(a_en), len(refs), vp(r_f), vp(r_l), int(prefix_end),
                            int(prev_line_start), int(cur_line_start), int(ctx_len), cap, vp(st), vp(en), vp(needed))
        if rc == -6:
            cap = int(needed[0])
            continue
        if rc != 0:
            raise SpanAttnError(rc, "span_build")
        n = int(needed[0])
        return list(zip(st[:n].tolist(), en[:n].tolist()))


def _check_qkv(q, k_cache, v_cache, multi=False):
    if not (q.is_cuda and k_cache.is_cuda and v_cache.is_cuda):
        raise ValueError("q, k_cache and v_cache must be GPU tensors")
    if not (q.is_contiguous() and k_cache.is_contiguous() and v_cache.is_contiguous()):
        raise ValueError("q, k_cache and v_cache must be contiguous")
    B, H, L, D = k_cache.shape
    if multi:
        if q.dim() != 4 or (q.shape[0], q.shape[2], q.shape[3]) != (B, H, D) or v_cache.shape != k_cache.shape:
            raise ValueError("expected q [B,Q,H,D] and k_cache / v_cache [B,H,L,D]")
    elif tuple(q.shape) != (B, H, D) or v_cache.shape != k_cache.shape:
        raise ValueError("expected q [B,H,D] and k_cache / v_cache [B,H,L,D]")
    if not (q.dtype == k_cache.dtype == v_cache.dtype):
        raise ValueError("q, k_cache, v_cache must share one dtype")
    return B, H, L, D


def _i32_dev(t, n, name):
    import torch
    if t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous() or t.numel() < n:
        raise ValueError(f"{name} must be a contiguous int32 GPU tensor with at least {n} entries")
    return t.data_ptr()


def _prepare(q, k_cache, v_cache, out, num_intervals, max_tokens, num_splits, workspace, stream, tokens_per_seq,
             multi=False, host_spans=None):
    import torch
    B, H, L, D = _check_qkv(q, k_cache, v_cache, multi)
    if out is None:
        out = torch.empty(tuple(q.shape), dtype=torch.float32, device=q.device)
    elif out.dtype != torch.float32 or not out.is_cuda or not out.is_contiguous() or out.shape != q.shape:
        raise ValueError("out must be a contiguous fp32 GPU tensor shaped like q")
    if stream is None:
        stream = torch.cuda.current_stream(q.device).cuda_stream
    desc = make_desc(B, H, D, L, _dtype_code(q), num_intervals, int(max_tokens), int(num_splits), 0, 0, stream,
                     tokens_per_seq, q_len=q.shape[1] if multi else 0, host_spans=host_spans)
    need = span_workspace_bytes(desc)
    if need:
        fresh = workspace is None
        if fresh:
            workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
        desc.workspace = workspace.data_ptr()
        desc.workspace_bytes = workspace.numel() * workspace.element_size()
        if fresh:
            span_workspace_init(desc)   # a workspace handed in by the caller must already be initialised
    return desc, out, workspace


def prepare_span_decode_attn_multi(q, k_cache, v_cache, span_offsets, span_starts, span_ends, q_pos, scale,
                                   out=None, *, max_tokens=0, num_splits=0, workspace=None, stream=None,
                                   tokens_per_seq=None, host_spans=None) -> "PreparedCall":
    """Few-query variant: q [B,Q,H,D], q_pos int32 GPU tensor [B] or None, out fp32 [B,Q,H,D]."""
    lib = load_library()
    n_int = int(span_starts.numel())
    desc, out, workspace = _prepare(q, k_cache, v_cache, out, n_int, max_tokens, num_splits, workspace, stream,
                                    tokens_per_seq, multi=True, host_spans=host_spans)
    off_p = _i32_dev(span_offsets, desc.batch + 1, "span_offsets")
    st_p = _i32_dev(span_starts, n_int, "span_starts")
    en_p = _i32_dev(span_ends, n_int, "span_ends")
    pos_p = _i32_dev(q_pos, desc.batch, "q_pos") if q_pos is not None else None
    args = (ctypes.byref(desc), q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(), off_p, st_p, en_p, pos_p,
            float(scale), out.data_ptr())
    keep = (q, k_cache, v_cache, span_offsets, span_starts, span_ends, q_pos, workspace)
    return PreparedCall("span_decode_attn_multi", lib.span_decode_attn_multi, desc, args, out, keep)


def span_decode_attn_multi(q, k_cache, v_cache, span_offsets, span_starts, span_ends, q_pos, scale, out=None,
                           **kw):
    return prepare_span_decode_attn_multi(q, k_cache, v_cache, span_offsets, span_starts, span_ends, q_pos, scale,
                                          out, **kw)()


class PreparedCall:
    """One fully marshalled call: holds the descriptor, raw pointers and the tensors they point into, so
    that invoking it costs a single ctypes call (used by tight loops such as the benchmark)."""

    def __init__(self, name, fn, desc, args, out, keepalive):
        self.name, self._fn, self.desc, self._args, self.out, self._keepalive = name, fn, desc, args, out, keepalive

    def __call__(self):
        rc = self._fn(*self._args)
        if rc != 0:
            raise SpanAttnError(rc, self.name)
        return self.out


def prepare_span_decode_attn(q, k_cache, v_cache, span_offsets, span_starts, span_ends, ctx_lens, scale, out=None, *,
                             max_tokens=0, num_splits=0, workspace=None, stream=None,
                             tokens_per_seq=None, host_spans=None) -> PreparedCall:
    """host_spans: optional (offsets, starts, ends) host copies of the device span lists (see span_attn.h)."""
    lib = load_library()
    n_int = int(span_starts.numel())
    desc, out, workspace = _prepare(q, k_cache, v_cache, out, n_int, max_tokens, num_splits, workspace, stream,
                                    tokens_per_seq, host_spans=host_spans)
    off_p = _i32_dev(span_offsets, desc.batch + 1, "span_offsets")
    st_p = _i32_dev(span_starts, n_int, "span_starts")
    en_p = _i32_dev(span_ends, n_int, "span_ends")
    ctx_p = _i32_dev(ctx_lens, desc.batch, "ctx_lens") if ctx_lens is not None else None
    args = (ctypes.byref(desc), q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(), off_p, st_p, en_p, ctx_p,
            float(scale), out.data_ptr())
    keep = (q, k_cache, v_cache, span_offsets, span_starts, span_ends, ctx_lens, workspace)
    return PreparedCall("span_decode_attn", lib.span_decode_attn, desc, args, out, keep)


STATIC_SCRATCH_BYTES = 4 << 20


def prepare_span_decode_attn_static(q, k_cache, v_cache, span_offsets, span_starts, span_ends, ctx_lens, scale, out, *,
                                    max_tokens=0, num_splits=0, stream=None, tokens_per_seq=None,
                                    host_spans=None) -> PreparedCall:
    """span_decode_attn on the library's own scratch array: no workspace is created or passed, `out` is the
    caller's.  Invoking the prepared call allocates nothing."""
    import torch
    lib = load_library()
    B, H, L, D = _check_qkv(q, k_cache, v_cache)
    if out is None or out.dtype != torch.float32 or not out.is_cuda or not out.is_contiguous() or out.shape != q.shape:
        raise ValueError("out must be a contiguous fp32 GPU tensor shaped like q")
    if stream is None:
        stream = torch.cuda.current_stream(q.device).cuda_stream
    n_int = int(span_starts.numel())
    desc = make_desc(B, H, D, L, _dtype_code(q), n_int, int(max_tokens), int(num_splits), 0, 0, stream, tokens_per_seq,
                     host_spans=host_spans)
    ctx_p = _i32_dev(ctx_lens, B, "ctx_lens") if ctx_lens is not None else None
    args = (ctypes.byref(desc), q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(),
            _i32_dev(span_offsets, B + 1, "span_offsets"), _i32_dev(span_starts, n_int, "span_starts"),
            _i32_dev(span_ends, n_int, "span_ends"), ctx_p, float(scale), out.data_ptr())
    keep = (q, k_cache, v_cache, span_offsets, span_starts, span_ends, ctx_lens, out)
    return PreparedCall("span_decode_attn_static", lib.span_decode_attn_static, desc, args, out, keep)


def span_decode_attn_static(q, k_cache, v_cache, span_offsets, span_starts, span_ends, ctx_lens, scale, out, **kw):
    return prepare_span_decode_attn_static(q, k_cache, v_cache, span_offsets, span_starts, span_ends, ctx_lens, scale,
                                           out, **kw)()


def prepare_dense_decode_attn(q, k_cache, v_cache, ctx_lens, scale, out=None, *, max_tokens=0, num_splits=0,
                              workspace=None, stream=None, tokens_per_seq=None) -> PreparedCall:
    lib = load_library()
    desc, out, workspace = _prepare(q, k_cache, v_cache, out, 0, max_tokens, num_splits, workspace, stream,
                                    tokens_per_seq)
    ctx_p = _i32_dev(ctx_lens, desc.batch, "ctx_lens")
    args = (ctypes.byref(desc), q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(), ctx_p, float(scale),
            out.data_ptr())
    return PreparedCall("dense_decode_attn", lib.dense_decode_attn, desc, args, out,
                        (q, k_cache, v_cache, ctx_lens, workspace))


def _check_new_rows(q, k_new, v_new):
    for t, name in ((k_new, "k_new"), (v_new, "v_new")):
        if not t.is_cuda or not t.is_contiguous() or t.dtype != q.dtype or tuple(t.shape) != tuple(q.shape):
            raise ValueError(f"{name} must be a contiguous GPU tensor shaped and typed like q")


def prepare_span_decode_attn_append(q, k_new, v_new, k_cache, v_cache, append_pos, span_offsets, span_starts,
                                    span_ends, scale, out=None, *, max_tokens=0, num_splits=0, workspace=None,
                                    stream=None, tokens_per_seq=None, host_spans=None) -> PreparedCall:
    lib = load_library()
    n_int = int(span_starts.numel())
    desc, out, workspace = _prepare(q, k_cache, v_cache, out, n_int, max_tokens, num_splits, workspace, stream,
                                    tokens_per_seq, host_spans=host_spans)
    _check_new_rows(q, k_new, v_new)
    args = (ctypes.byref(desc), q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), k_cache.data_ptr(),
            v_cache.data_ptr(), _i32_dev(append_pos, desc.batch, "append_pos"),
            _i32_dev(span_offsets, desc.batch + 1, "span_offsets"), _i32_dev(span_starts, n_int, "span_starts"),
            _i32_dev(span_ends, n_int, "span_ends"), float(scale), out.data_ptr())
    keep = (q, k_new, v_new, k_cache, v_cache, append_pos, span_offsets, span_starts, span_ends, workspace)
    return PreparedCall("span_decode_attn_append", lib.span_decode_attn_append, desc, args, out, keep)


def prepare_dense_decode_attn_append(q, k_new, v_new, k_cache, v_cache, append_pos, ctx_lens, scale, out=None, *,
                                     max_tokens=0, num_splits=0, workspace=None, stream=None,
                                     tokens_per_seq=None) -> PreparedCall:
    lib = load_library()
    desc, out, workspace = _prepare(q, k_cache, v_cache, out, 0, max_tokens, num_splits, workspace, stream,
                                    tokens_per_seq)
    _check_new_rows(q, k_new, v_new)
    args = (ctypes.byref(desc), q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), k_cache.data_ptr(),
            v_cache.data_ptr(), _i32_dev(append_pos, desc.batch, "append_pos"),
            _i32_dev(ctx_lens, desc.batch, "ctx_lens"), float(scale), out.data_ptr())
    keep = (q, k_new, v_new, k_cache, v_cache, append_pos, ctx_lens, workspace)
    return PreparedCall("dense_decode_attn_append", lib.dense_decode_attn_append, desc, args, out, keep)


def prepare_span_decode_attn_multi_append(q, k_new, v_new, k_cache, v_cache, append_pos, span_offsets, span_starts,
                                          span_ends, scale, out=None, *, max_tokens=0, num_splits=0, workspace=None,
                                          stream=None, tokens_per_seq=None, host_spans=None) -> PreparedCall:
    """Few-query append: q, k_new, v_new [B,Q,H,D]; token j of sequence b goes to cache row append_pos[b] + j."""
    lib = load_library()
    n_int = int(span_starts.numel())
    desc, out, workspace = _prepare(q, k_cache, v_cache, out, n_int, max_tokens, num_splits, workspace, stream,
                                    tokens_per_seq, multi=True, host_spans=host_spans)
    _check_new_rows(q, k_new, v_new)
    args = (ctypes.byref(desc), q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), k_cache.data_ptr(),
            v_cache.data_ptr(), _i32_dev(append_pos, desc.batch, "append_pos"),
            _i32_dev(span_offsets, desc.batch + 1, "span_offsets"), _i32_dev(span_starts, n_int, "span_starts"),
            _i32_dev(span_ends, n_int, "span_ends"), float(scale), out.data_ptr())
    keep = (q, k_new, v_new, k_cache, v_cache, append_pos, span_offsets, span_starts, span_ends, workspace)
    return PreparedCall("span_decode_attn_multi_append", lib.span_decode_attn_multi_append, desc, args, out, keep)


def span_decode_attn_multi_append(q, k_new, v_new, k_cache, v_cache, append_pos, span_offsets, span_starts, span_ends,
                                  scale, out=None, **kw):
    return prepare_span_decode_attn_multi_append(q, k_new, v_new, k_cache, v_cache, append_pos, span_offsets,
                                                 span_starts, span_ends, scale, out, **kw)()


def span_decode_attn_append(q, k_new, v_new, k_cache, v_cache, append_pos, span_offsets, span_starts, span_ends,
                            scale, out=None, **kw):
    """Writes the new token's K / V rows into the caches at append_pos[b] and attends over the updated cache."""
    return prepare_span_decode_attn_append(q, k_new, v_new, k_cache, v_cache, append_pos, span_offsets, span_starts,
                                           span_ends, scale, out, **kw)()


def dense_decode_attn_append(q, k_new, v_new, k_cache, v_cache, append_pos, ctx_lens, scale, out=None, **kw):
    return prepare_dense_decode_attn_append(q, k_new, v_new, k_cache, v_cache, append_pos, ctx_lens, scale, out,
                                            **kw)()


def span_decode_attn(q, k_cache, v_cache, span_offsets, span_starts, span_ends, ctx_lens, scale, out=None, *,
                     max_tokens=0, num_splits=0, workspace=None, stream=None, tokens_per_seq=None, host_spans=None):
    """out[b,h,:] = softmax over the span's positions of scale*q.K, times V.  Returns `out` (fp32)."""
    return prepare_span_decode_attn(q, k_cache, v_cache, span_offsets, span_starts, span_ends, ctx_lens, scale, out,
                                    max_tokens=max_tokens, num_splits=num_splits, workspace=workspace,
                                    stream=stream, tokens_per_seq=tokens_per_seq, host_spans=host_spans)()


def dense_decode_attn(q, k_cache, v_cache, ctx_lens, scale, out=None, *, max_tokens=0, num_splits=0,
                      workspace=None, stream=None, tokens_per_seq=None):
    """Dense control: every position below ctx_lens[b] is attended."""
    return prepare_dense_decode_attn(q, k_cache, v_cache, ctx_lens, scale, out, max_tokens=max_tokens,
                                     num_splits=num_splits, workspace=workspace, stream=stream,
                                     tokens_per_seq=tokens_per_seq)()
