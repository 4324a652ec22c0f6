"""span_decode_attn_static (the entry point that allocates nothing: the slices' partial states live in an array
the library owns on the device) against span_decode_attn with a caller workspace, through the C ABI.

Both run the same plan and the same kernels and the cross-slice merge has a fixed order, so the outputs must be
equal bit for bit; the oracle bounds them both.  Two calls in a row share the library's array, the second on a
smaller input; the array is then dirtied by a differently shaped call in between."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2404_09336_amd as span
from paper_2404_09336_amd.binding import make_desc
from workloads import CONFIGS, DecodeConfig, SpanBatch, draw_qkv, draw_spans, to_host_raw

pytestmark = pytest.mark.gpu


def _dev(a, device):
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


class Case:
    def __init__(self, cfg, sp, device, seed=None, **plan_kw):
        self.cfg, self.sp = cfg, sp
        code, _, _, tok = span.span_validate(sp.offsets, sp.starts, sp.ends, sp.ctx_lens)
        assert code == 0
        self.q, self.K, self.V = draw_qkv(cfg, sp.ctx_lens, seed=seed, device=device)
        self.dev = [_dev(a, device) for a in (sp.offsets, sp.starts, sp.ends, sp.ctx_lens)]
        self.kw = dict(max_tokens=int(tok.max()), tokens_per_seq=tok)
        self.kw.update(plan_kw)
        self.out = torch.full((cfg.batch, cfg.heads, cfg.head_dim), float("nan"), dtype=torch.float32, device=device)
        self.static = span.prepare_span_decode_attn_static(self.q, self.K, self.V, *self.dev, np.float32(cfg.scale),
                                                           self.out, **self.kw)

    def reference(self):
        """The existing entry point on a workspace of its own."""
        return span.span_decode_attn(self.q, self.K, self.V, *self.dev, np.float32(self.cfg.scale), **self.kw)

    def oracle(self):
        sp = self.sp
        return oracle.span_attn(to_host_raw(self.q), to_host_raw(self.K), to_host_raw(self.V), sp.offsets, sp.starts,
                                sp.ends, np.float32(self.cfg.scale), dtype=self.cfg.dtype)

    def check(self, what):
        self.out.fill_(float("nan"))
        got = self.static()
        ref = self.reference()
        torch.cuda.synchronize()
        assert torch.equal(got, ref), f"{what}: static-scratch call differs from the workspace call"
        err = float(np.abs(got.cpu().numpy().astype(np.float64) - self.oracle()).max())
        print(f"[parity] {what}: max-abs err vs oracle {err:.3e} (tol {self.cfg.tol:g})", flush=True)
        assert err <= self.cfg.tol


def small_case(device, splits):
    cfg = DecodeConfig(95, "static-small", 3, 5, 64, 500, 200, "f32", 1e-5)
    rng = np.random.default_rng(95)
    ctx = rng.integers(cfg.min_len, cfg.max_len + 1, size=cfg.batch).astype(np.int32)
    per_seq = [[(0, 9), (40 + 3 * b, 150 + 5 * b), (int(ctx[b]) - 21, int(ctx[b]))] for b in range(cfg.batch)]
    return Case(cfg, SpanBatch.from_lists(per_seq, ctx), device, num_splits=splits, tokens_per_seq=None)


def test_two_calls_in_a_row_the_second_smaller(gpu_device):
    big = Case(CONFIGS[2], draw_spans(CONFIGS[2]), gpu_device)            # sliced by the table, ~1 MB of states
    assert span.span_plan_query(big.static.desc)["max_splits"] > 1
    small = small_case(gpu_device, splits=4)                               # 15 pairs, a few slices each
    assert span.span_plan_query(small.static.desc)["max_splits"] > 1
    big.check("config 2 on the library's scratch")
    small.check("smaller input right after it")
    big.check("config 2 again")
    # a third shape whose states overwrite the counters' neighbourhood differently, then the small one again
    other = Case(CONFIGS[4], draw_spans(CONFIGS[4]), gpu_device)
    other.check("config 4 on the library's scratch")
    small.check("smaller input after config 4")
    small_case(gpu_device, splits=7).check("same small input, 7 slices")


def test_unsplit_call_needs_no_scratch_and_matches(gpu_device):
    case = Case(CONFIGS[3], draw_spans(CONFIGS[3]), gpu_device)
    assert span.span_workspace_bytes(case.static.desc) == 0
    case.check("config 3 (one slice per pair)")


def test_calls_beyond_the_limit_are_rejected_before_any_launch(gpu_device):
    cfg = CONFIGS[3]
    case = Case(cfg, draw_spans(cfg), gpu_device, num_splits=16, tokens_per_seq=None)   # 2048 pairs x 16 states
    need = span.span_workspace_bytes(case.static.desc)
    assert need > span.binding.STATIC_SCRATCH_BYTES
    case.out.fill_(7.0)
    with pytest.raises(span.SpanAttnError) as e:
        case.static()
    assert e.value.code == -7
    torch.cuda.synchronize()
    assert bool((case.out == 7.0).all())                                   # nothing ran
    assert "scratch" in span.span_strerror(-7)
