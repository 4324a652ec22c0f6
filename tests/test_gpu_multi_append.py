"""Few-query append (several new tokens of a sequence are appended to the cache and attend in one call): parity with
the oracle's few-query form run on the updated cache, the cache itself bit-exact, and a decode loop over a group
recorded as one HIP graph (append + attention, advance by the step's token count)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_09336_amd as span
from oracle.advance import advance as oracle_advance
from workloads import CONFIGS, DecodeConfig, SpanBatch, draw_qkv, draw_queries, draw_spans, to_host_raw

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-5, "f16": 2e-3, "bf16": 2e-3}


def _dev(a, device):
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def _bits(t):
    a = to_host_raw(t)
    return a.view(np.uint32) if a.dtype == np.float32 else a


def new_rows(cfg, q_len, device, seed):
    g = torch.Generator(device=device).manual_seed(seed)
    shape = (cfg.batch, q_len, cfg.heads, cfg.head_dim)
    mk = lambda: torch.randn(shape, generator=g, device=device).to(draw_queries(cfg, 1, device=device).dtype)
    return mk(), mk()


def updated(K, k_new, pos):
    """K with row pos[b] + j := k_new[b, j] for every token j whose row exists."""
    K2 = K.clone()
    for b, p in enumerate(pos):
        for j in range(k_new.shape[1]):
            if 0 <= p + j < K.shape[2]:
                K2[b, :, p + j, :] = k_new[b, j]
    return K2


def run_case(cfg, sp, pos, q_len, device, seed=0, what="", **kw):
    """sp describes the span AFTER the append (it is expected to hold the new positions, but need not)."""
    pos = np.asarray(pos, np.int32)
    old_len = np.clip(pos, 0, cfg.max_len).astype(np.int32)            # rows from the first new one on are NaN before the call
    _, K, V = draw_qkv(cfg, old_len, device=device, seed=cfg.seed() + seed)
    q = draw_queries(cfg, q_len, device=device, seed=cfg.seed() + seed)
    k_new, v_new = new_rows(cfg, q_len, device, seed + 1)
    K_ref, V_ref = updated(K, k_new, pos), updated(V, v_new, pos)
    code, _, _, tok = span.span_validate(sp.offsets, sp.starts, sp.ends, sp.ctx_lens)
    assert code == 0, code
    kw.setdefault("max_tokens", int(tok.max()))
    if "num_splits" not in kw:
        kw.setdefault("tokens_per_seq", tok)
    out = span.span_decode_attn_multi_append(q, k_new, v_new, K, V, _dev(pos, device), _dev(sp.offsets, device),
                                             _dev(sp.starts, device), _dev(sp.ends, device), np.float32(cfg.scale), **kw)
    torch.cuda.synchronize()
    ref = oracle.span_attn_multi(to_host_raw(q), to_host_raw(K_ref), to_host_raw(V_ref), sp.offsets, sp.starts,
                                 sp.ends, pos, np.float32(cfg.scale), dtype=cfg.dtype)
    got = out.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all(), what
    err = float(np.abs(got - ref).max())
    print(f"[parity] few-query append {what}: max-abs err {err:.3e} (tol {cfg.tol:g})", flush=True)
    assert err <= cfg.tol, what
    assert np.array_equal(_bits(K), _bits(K_ref)) and np.array_equal(_bits(V), _bits(V_ref)), f"{what}: cache bits"


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("q_len", [1, 2, 3, 4, 5, 8, 16, 23])
def test_every_instance_and_token_count(dtype, D, q_len, gpu_device):
    """The new tokens close the span's last interval; ragged sequences; unsplit and sliced."""
    cfg = DecodeConfig(99, "multi-append", 3, 5, D, 700, 700, dtype, TOL[dtype])
    rng = np.random.default_rng(10 * D + q_len)
    pos = rng.integers(300, 700 - q_len, size=cfg.batch).astype(np.int32)
    per_seq = [[(0, 11), (40 + 3 * b, 150 + 7 * b), (int(pos[b]) - 20, int(pos[b]) + q_len)] for b in range(cfg.batch)]
    sp = SpanBatch.from_lists(per_seq, pos + q_len)
    run_case(cfg, sp, pos, q_len, gpu_device, what=f"{dtype} D={D} q_len={q_len}")
    for splits in (2, 7):
        run_case(cfg, sp, pos, q_len, gpu_device, seed=splits, what=f"{dtype} D={D} q_len={q_len} splits={splits}",
                 num_splits=splits)


@pytest.mark.parametrize("cid", [2, 3, 4])
@pytest.mark.parametrize("q_len", [2, 4, 16])
def test_workload_scale(cid, q_len, gpu_device):
    """The workloads' spans end with the recent-token interval: the new tokens are its last q_len positions."""
    cfg = CONFIGS[cid]
    sp = draw_spans(cfg)
    pos = (sp.ctx_lens - q_len).astype(np.int32)
    run_case(cfg, sp, pos, q_len, gpu_device, what=f"config {cid}, {q_len} tokens")
    run_case(cfg, sp, pos, q_len, gpu_device, what=f"config {cid}, {q_len} tokens, host lists",
             host_spans=(sp.offsets, sp.starts, sp.ends))


def test_new_tokens_outside_the_span_or_the_cache(gpu_device):
    """Tokens whose positions the span does not hold are appended but not attended; rows outside [0, max_len) are
    not written; a sequence whose tokens see nothing gets zero rows."""
    cfg = DecodeConfig(100, "multi-append-edges", 4, 3, 128, 300, 300, "f16", 2e-3)
    q_len = 4
    pos = np.array([200, 100, 298, 5], np.int32)
    per_seq = [[(0, 50), (190, 200)],              # new tokens 200..203 are after the span: seen rows end at 199
               [(0, 30), (100, 102)],              # only the first two new tokens are in the span
               [(10, 60), (290, 300)],             # tokens 298, 299 fit the cache, 300 and 301 do not
               [(40, 80)]]                         # tokens at 5..8 see nothing of [40, 80)
    sp = SpanBatch.from_lists(per_seq, np.array([204, 104, 300, 80], np.int32))
    run_case(cfg, sp, pos, q_len, gpu_device, what="edge cases")
    run_case(cfg, sp, pos, q_len, gpu_device, what="edge cases, 3 slices", num_splits=3)


def test_group_of_steps_as_one_graph(gpu_device):
    """Five steps of three tokens each: the HIP graph [few-query append + attention, advance by 3] is replayed once per
    step with nothing but the new q / k / v rows changing on the host side; the oracle steps the same tokens."""
    cfg = DecodeConfig(101, "multi-loop", 5, 8, 128, 900, 900, "f16", 2e-3)
    rng = np.random.default_rng(26)
    steps, n = 5, 3
    start_len = rng.integers(300, 800, size=cfg.batch).astype(np.int32)
    per_seq = [[(0, 17), (40 + 3 * b, 120 + 5 * b), (int(start_len[b]) - 9, int(start_len[b]) + n)]
               for b in range(cfg.batch)]                      # the last interval already holds the first step's tokens
    sp = SpanBatch.from_lists(per_seq, start_len + n)
    _, K, V = draw_qkv(cfg, start_len, device=gpu_device)
    gen = torch.Generator(device=gpu_device).manual_seed(6)
    new = [torch.randn((steps, cfg.batch, n, cfg.heads, cfg.head_dim), generator=gen, device=gpu_device).half()
           for _ in range(3)]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(gpu_device)
    off, st, en, pos = dev(sp.offsets), dev(sp.starts), dev(sp.ends), dev(start_len)
    q, kn, vn = (torch.empty_like(new[0][0]) for _ in range(3))
    out = torch.empty((cfg.batch, n, cfg.heads, cfg.head_dim), dtype=torch.float32, device=gpu_device)
    tok_final = sp.tokens_per_seq() + n * (steps - 1)
    side = torch.cuda.Stream(device=gpu_device)
    call = span.prepare_span_decode_attn_multi_append(q, kn, vn, K, V, pos, off, st, en, np.float32(cfg.scale), out,
                                                      max_tokens=int(tok_final.max()), tokens_per_seq=tok_final,
                                                      stream=side.cuda_stream)
    adv = span.prepare_span_advance(off, st, en, pos, max_len=cfg.max_len, stream=side.cuda_stream, q_len=n)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call()
        adv()
    hK, hV = to_host_raw(K).copy(), to_host_raw(V).copy()
    o_off, o_st, o_en, o_pos = sp.offsets.tolist(), sp.starts.tolist(), sp.ends.tolist(), start_len.tolist()
    for t in range(steps):
        q.copy_(new[0][t]); kn.copy_(new[1][t]); vn.copy_(new[2][t])
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        hk_new, hv_new = to_host_raw(new[1][t]), to_host_raw(new[2][t])
        for b in range(cfg.batch):
            for j in range(n):
                hK[b, :, o_pos[b] + j] = hk_new[b, j]
                hV[b, :, o_pos[b] + j] = hv_new[b, j]
        ref = oracle.span_attn_multi(to_host_raw(new[0][t]), hK, hV, np.array(o_off, np.int32), np.array(o_st, np.int32),
                                     np.array(o_en, np.int32), np.array(o_pos, np.int32), np.float32(cfg.scale), dtype="f16")
        got = out.cpu().numpy().astype(np.float64)
        err = float(np.abs(got - ref).max())
        print(f"[loop] step {t}: max-abs err {err:.3e}", flush=True)
        assert np.isfinite(got).all() and err <= cfg.tol, (t, err)
        oracle_advance(o_off, o_st, o_en, o_pos, None, cfg.max_len, count=n)
        assert en.cpu().tolist() == o_en and pos.cpu().tolist() == o_pos
    assert np.array_equal(to_host_raw(K).view(np.uint16), hK.view(np.uint16))
    assert np.array_equal(to_host_raw(V).view(np.uint16), hV.view(np.uint16))
