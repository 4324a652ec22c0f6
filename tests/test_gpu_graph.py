"""The calls can be recorded into a HIP graph (no allocation, no memset, no synchronisation inside) and
replayed: every replay must equal the eager result, with other work running between the replays."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_09336_amd as span
from paper_2404_09336_amd import binding
from workloads import CONFIGS, draw_qkv, draw_spans, to_host_raw

pytestmark = pytest.mark.gpu


def test_graph_replay_matches_eager_and_oracle(gpu_device):
    cfg = CONFIGS[2]                                   # several slices per (batch, head): workspace + tickets in play
    sp = draw_spans(cfg)
    tok = sp.tokens_per_seq()
    q, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(gpu_device)
    off, st, en, ctx = dev(sp.offsets), dev(sp.starts), dev(sp.ends), dev(sp.ctx_lens)

    side = torch.cuda.Stream(device=gpu_device)
    # the workspace is allocated and zeroed before capture here; the next test records the init call itself
    d = binding.make_desc(cfg.batch, cfg.heads, cfg.head_dim, cfg.max_len, 1, int(st.numel()), int(tok.max()), 0,
                          tokens_per_seq=tok)
    ws = torch.zeros(span.span_workspace_bytes(d), dtype=torch.uint8, device=gpu_device)
    out_span = torch.empty((cfg.batch, cfg.heads, cfg.head_dim), dtype=torch.float32, device=gpu_device)
    out_dense = torch.empty_like(out_span)
    ws_d = torch.zeros(span.span_workspace_bytes(binding.make_desc(
        cfg.batch, cfg.heads, cfg.head_dim, cfg.max_len, 1, 0, cfg.max_len, 0,
        tokens_per_seq=sp.ctx_lens.astype(np.int64))), dtype=torch.uint8, device=gpu_device)
    torch.cuda.synchronize()
    call_s = span.prepare_span_decode_attn(q, K, V, off, st, en, ctx, np.float32(cfg.scale), out_span,
                                           max_tokens=int(tok.max()), tokens_per_seq=tok, workspace=ws,
                                           stream=side.cuda_stream)
    call_d = span.prepare_dense_decode_attn(q, K, V, ctx, np.float32(cfg.scale), out_dense, max_tokens=cfg.max_len,
                                            tokens_per_seq=sp.ctx_lens.astype(np.int64), workspace=ws_d,
                                            stream=side.cuda_stream)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call_s()
        call_d()
        call_s()                                       # same workspace again inside one graph: counters must be back to zero

    hK, hV = to_host_raw(K), to_host_raw(V)
    for replay in range(4):
        # eager work between replays: new query values in place, plus unrelated kernels
        q.copy_(torch.randn(q.shape, device=gpu_device).to(q.dtype))
        junk = torch.randn(1 << 20, device=gpu_device).sum()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got_s, got_d = out_span.cpu().numpy().astype(np.float64), out_dense.cpu().numpy().astype(np.float64)
        eager = span.span_decode_attn(q, K, V, off, st, en, ctx, np.float32(cfg.scale), max_tokens=int(tok.max()),
                                      tokens_per_seq=tok)
        torch.cuda.synchronize()
        hq = to_host_raw(q)
        ref_s = oracle.span_attn(hq, hK, hV, sp.offsets, sp.starts, sp.ends, np.float32(cfg.scale), dtype=cfg.dtype)
        ref_d = oracle.dense_attn(hq, hK, hV, sp.ctx_lens, np.float32(cfg.scale), dtype=cfg.dtype)
        assert np.abs(got_s - ref_s).max() <= cfg.tol and np.abs(got_d - ref_d).max() <= cfg.tol, replay
        assert np.abs(got_s - eager.cpu().numpy()).max() <= 1e-6
        assert torch.isfinite(junk)


def test_workspace_init_inside_a_graph(gpu_device):
    """span_workspace_init is a kernel launch, so it can be recorded too: a graph that first re-initialises a
    workspace full of junk and then runs a sliced call gives the eager result on every replay."""
    cfg = CONFIGS[2]
    sp = draw_spans(cfg)
    tok = sp.tokens_per_seq()
    q, K, V = draw_qkv(cfg, sp.ctx_lens, device=gpu_device)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(gpu_device)
    off, st, en, ctx = dev(sp.offsets), dev(sp.starts), dev(sp.ends), dev(sp.ctx_lens)
    side = torch.cuda.Stream(device=gpu_device)
    d = binding.make_desc(cfg.batch, cfg.heads, cfg.head_dim, cfg.max_len, 1, int(st.numel()), int(tok.max()), 0,
                          tokens_per_seq=tok)
    ws = torch.full((span.span_workspace_bytes(d),), 0xAB, dtype=torch.uint8, device=gpu_device)
    out = torch.empty((cfg.batch, cfg.heads, cfg.head_dim), dtype=torch.float32, device=gpu_device)
    call = span.prepare_span_decode_attn(q, K, V, off, st, en, ctx, np.float32(cfg.scale), out,
                                         max_tokens=int(tok.max()), tokens_per_seq=tok, workspace=ws,
                                         stream=side.cuda_stream)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        span.span_workspace_init(call.desc)
        call()
    eager = span.span_decode_attn(q, K, V, off, st, en, ctx, np.float32(cfg.scale), max_tokens=int(tok.max()),
                                  tokens_per_seq=tok)
    torch.cuda.synchronize()
    for replay in range(3):
        ws.fill_(0xCD)                     # junk again between the replays (eager work on the default stream)
        out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), replay
