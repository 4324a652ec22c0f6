"""fp64 CPU oracle for span-restricted decode attention.

TEST INFRASTRUCTURE.  Only tests, the smoke check and the benchmark's CPU-baseline leg
may import this package; the HIP library and its Python binding never do, and this
package never imports them.

Two independent formulations live here:
  * `span_oracle.c` (plain C, double precision, compiled with gcc): sums over the span's
    positions only; also the few-query form (causal limit over the span), the dense
    control, group states + log-sum-exp merge, and the span-list validator.
  * `bruteforce.py` (numpy float64): additive 0 / -inf mask over *all* positions and a
    full-length softmax, as the mask is defined in Sec. 2.2; small inputs only.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "span_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

DTYPE_CODES = {"f32": 0, "f16": 1, "bf16": 2}

VALIDATION_NAMES = {0: "OK", 1: "OFFSETS", 2: "RANGE", 3: "EMPTY_INTERVAL", 4: "OVERLAP", 5: "UNSORTED",
                    6: "EMPTY_SPAN"}


def build(force: bool = True) -> str:
    """Compile span_oracle.c with gcc (-O2, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.run(["gcc", "-O2", "-fopenmp", "-std=c11", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"],
                       check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        lib = ctypes.CDLL(_LIB)
        vp, ip, dp = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
        ci, cf = ctypes.c_int, ctypes.c_float
        lib.oracle_span_attn.argtypes = [ci, ci, ci, ci, ci, vp, vp, vp, ip, ip, ip, cf, dp, ip]
        lib.oracle_span_attn_multi.argtypes = [ci, ci, ci, ci, ci, ci, vp, vp, vp, ip, ip, ip, ip, cf, dp]
        lib.oracle_dense_attn.argtypes = [ci, ci, ci, ci, ci, vp, vp, vp, ip, cf, dp]
        lib.oracle_span_state.argtypes = [ci, ci, ci, ci, vp, vp, vp, ci, ci, ip, ip, ci, cf, dp, dp, dp]
        lib.oracle_lse_merge.argtypes = [ci, ci, dp, dp, dp, dp]
        lib.oracle_validate.argtypes = [ci, ci, ip, ip, ip, ip, ip, ip, ip]
        lib.oracle_num_threads.restype = ci
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _raw(a: np.ndarray, dtype: str) -> np.ndarray:
    want = np.float32 if dtype == "f32" else np.uint16
    a = np.ascontiguousarray(a)
    if dtype == "f16" and a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != want:
        raise TypeError(f"dtype {dtype} needs a {want} array (raw bits for 16-bit types), got {a.dtype}")
    return a


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def span_attn(q, K, V, offsets, starts, ends, scale, dtype="f32", return_empty=False):
    """q [B,H,D], K/V [B,H,Lmax,D] (float32, or uint16 bit patterns for f16 / bf16) -> float64 [B,H,D]."""
    q, K, V = _raw(q, dtype), _raw(K, dtype), _raw(V, dtype)
    B, H, Lmax, D = K.shape
    assert q.shape == (B, H, D) and V.shape == K.shape
    offsets, starts, ends = _i32(offsets), _i32(starts), _i32(ends)
    assert offsets.shape == (B + 1,)
    out = np.zeros((B, H, D), dtype=np.float64)
    empty = np.zeros(B, dtype=np.int32)
    rc = _load().oracle_span_attn(B, H, D, Lmax, DTYPE_CODES[dtype], _ptr(q), _ptr(K), _ptr(V), _ptr(offsets),
                                  _ptr(starts), _ptr(ends), np.float32(scale), _ptr(out), _ptr(empty))
    assert rc == 0
    return (out, empty.astype(bool)) if return_empty else out


def span_attn_multi(q, K, V, offsets, starts, ends, q_pos, scale, dtype="f32"):
    """Few-query form.  q [B,Qn,H,D], K/V [B,H,Lmax,D], q_pos int32 [B] or None -> float64 [B,Qn,H,D];
    query j of sequence b attends the span positions <= q_pos[b] + j (all of the span when q_pos is None)."""
    q, K, V = _raw(q, dtype), _raw(K, dtype), _raw(V, dtype)
    B, H, Lmax, D = K.shape
    Qn = q.shape[1]
    assert q.shape == (B, Qn, H, D) and V.shape == K.shape
    offsets, starts, ends = _i32(offsets), _i32(starts), _i32(ends)
    assert offsets.shape == (B + 1,)
    if q_pos is not None:
        q_pos = _i32(q_pos)
        assert q_pos.shape == (B,)
    out = np.zeros((B, Qn, H, D), dtype=np.float64)
    rc = _load().oracle_span_attn_multi(B, H, D, Lmax, DTYPE_CODES[dtype], Qn, _ptr(q), _ptr(K), _ptr(V),
                                        _ptr(offsets), _ptr(starts), _ptr(ends),
                                        _ptr(q_pos) if q_pos is not None else None, np.float32(scale), _ptr(out))
    assert rc == 0
    return out


def dense_attn(q, K, V, ctx_lens, scale, dtype="f32"):
    q, K, V = _raw(q, dtype), _raw(K, dtype), _raw(V, dtype)
    B, H, Lmax, D = K.shape
    ctx_lens = _i32(ctx_lens)
    assert ctx_lens.shape == (B,)
    out = np.zeros((B, H, D), dtype=np.float64)
    rc = _load().oracle_dense_attn(B, H, D, Lmax, DTYPE_CODES[dtype], _ptr(q), _ptr(K), _ptr(V), _ptr(ctx_lens),
                                   np.float32(scale), _ptr(out))
    assert rc == 0
    return out


def span_state(q, K, V, b, h, intervals, scale, dtype="f32"):
    """Un-normalised softmax state (m, l, acc[D]) of head (b,h) over the union of `intervals`."""
    q, K, V = _raw(q, dtype), _raw(K, dtype), _raw(V, dtype)
    B, H, Lmax, D = K.shape
    st = _i32([s for s, _ in intervals])
    en = _i32([e for _, e in intervals])
    m, l = ctypes.c_double(), ctypes.c_double()
    acc = np.zeros(D, dtype=np.float64)
    rc = _load().oracle_span_state(H, D, Lmax, DTYPE_CODES[dtype], _ptr(q), _ptr(K), _ptr(V), int(b), int(h),
                                   _ptr(st), _ptr(en), len(intervals), np.float32(scale),
                                   ctypes.cast(ctypes.byref(m), ctypes.c_void_p),
                                   ctypes.cast(ctypes.byref(l), ctypes.c_void_p), _ptr(acc))
    assert rc == 0
    return m.value, l.value, acc


def lse_merge(ms, ls, accs):
    ms = np.ascontiguousarray(ms, dtype=np.float64)
    ls = np.ascontiguousarray(ls, dtype=np.float64)
    accs = np.ascontiguousarray(accs, dtype=np.float64)
    G, D = accs.shape
    out = np.zeros(D, dtype=np.float64)
    rc = _load().oracle_lse_merge(G, D, _ptr(ms), _ptr(ls), _ptr(accs), _ptr(out))
    assert rc == 0
    return out


def validate(offsets, starts, ends, ctx_lens):
    """Returns (code, bad_seq, bad_interval, tokens_per_seq[int64])."""
    offsets, starts, ends, ctx_lens = _i32(offsets), _i32(starts), _i32(ends), _i32(ctx_lens)
    B = ctx_lens.shape[0]
    assert offsets.shape == (B + 1,) and starts.shape == ends.shape
    bs, bi = np.zeros(1, np.int32), np.zeros(1, np.int32)
    tok = np.zeros(B, dtype=np.int64)
    code = _load().oracle_validate(B, int(starts.shape[0]), _ptr(offsets), _ptr(starts), _ptr(ends), _ptr(ctx_lens), _ptr(bs), _ptr(bi),
                                   _ptr(tok))
    return int(code), int(bs[0]), int(bi[0]), tok
