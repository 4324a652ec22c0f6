"""The synthetic span generators produce what the workload descriptions say."""
import numpy as np
import pytest

from workloads import CONFIGS, draw_spans, full_cover_spans, microbench_spans, place_disjoint


def _check_sorted_disjoint(sp):
    for b in range(sp.batch):
        iv = sp.intervals(b)
        assert iv, "every sequence has a span"
        assert iv[0][0] >= 0 and iv[-1][1] <= sp.ctx_lens[b]
        for (s, e) in iv:
            assert s < e
        for (s0, e0), (s1, e1) in zip(iv, iv[1:]):
            assert s1 >= e0


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_shapes_and_structure(cid):
    cfg = CONFIGS[cid]
    sp = draw_spans(cfg)
    assert sp.batch == cfg.batch and sp.offsets.dtype == np.int32 and sp.offsets[0] == 0
    assert (sp.ctx_lens >= cfg.min_len).all() and (sp.ctx_lens <= cfg.max_len).all()
    _check_sorted_disjoint(sp)
    again = draw_spans(cfg)
    assert np.array_equal(again.starts, sp.starts) and np.array_equal(again.ends, sp.ends)
    other = draw_spans(cfg, seed=cfg.seed(1))
    assert not (np.array_equal(other.starts, sp.starts) and np.array_equal(other.ctx_lens, sp.ctx_lens))


def test_config_specifics():
    sp = draw_spans(CONFIGS[1])
    assert len(sp.intervals(0)) == 4 and sp.intervals(0)[-1] == (240, 256)
    sp = draw_spans(CONFIGS[2])
    for b in range(sp.batch):
        iv = sp.intervals(b)
        assert iv[0] == (0, 64) and iv[-1] == (2016, 2048) and 6 <= len(iv) <= 14
        assert all(16 <= e - s <= 128 for s, e in iv[1:-1])
    sp = draw_spans(CONFIGS[3])
    for b in range(sp.batch):
        iv = sp.intervals(b)
        assert iv[0] == (0, 128) and iv[-1] == (504, 512) and len(iv) == 4
        assert all(4 <= e - s <= 16 for s, e in iv[1:-1])
    assert 0.25 < sp.coverage() < 0.35
    sp = draw_spans(CONFIGS[4])
    for b in range(sp.batch):
        iv = sp.intervals(b)
        assert iv[0] == (0, 48) and iv[-1][1] == sp.ctx_lens[b] and 1 <= iv[-1][1] - iv[-1][0] <= 128
        assert all(50 <= e - s <= 400 for s, e in iv[1:-1]) and 3 <= len(iv) <= 5
    sp = draw_spans(CONFIGS[5])
    for b in range(sp.batch):
        assert 16 <= len(sp.intervals(b)) <= 64
    cov = sp.tokens_per_seq() / sp.ctx_lens
    assert all(min(abs(c - t) for t in (0.05, 0.10, 0.25, 0.50)) < 0.01 for c in cov)
    sp = draw_spans(CONFIGS[5], coverage=0.25)
    assert abs(sp.coverage() - 0.25) < 0.005


def test_place_disjoint_fills_exactly_when_no_room_is_left():
    rng = np.random.default_rng(0)
    assert place_disjoint(rng, [3, 4, 5], 10, 22) == [(10, 13), (13, 17), (17, 22)]
    with pytest.raises(ValueError):
        place_disjoint(rng, [3, 4, 6], 10, 22)


def test_full_cover_and_microbench():
    sp = full_cover_spans([5, 9])
    assert sp.intervals(0) == [(0, 5)] and sp.intervals(1) == [(0, 9)]
    for sbs in (32, 64, 128, 256):
        sp = microbench_spans(4, 2048, sbs, seed=3)
        _check_sorted_disjoint(sp)
        assert (sp.tokens_per_seq() == 1024).all()
        for b in range(4):
            assert all(s % sbs == 0 and e % sbs == 0 for s, e in sp.intervals(b))


def test_draw_qkv_poison_and_determinism():
    import torch
    from workloads import DecodeConfig, draw_qkv, to_host_raw
    cfg = DecodeConfig(9, "t", 2, 2, 64, 32, 8, "f16", 2e-3)
    ctx = np.array([32, 10], np.int32)
    q, K, V = draw_qkv(cfg, ctx)
    assert q.shape == (2, 2, 64) and K.shape == (2, 2, 32, 64) and K.dtype == torch.float16
    assert torch.isnan(K[1, :, 10:]).all() and torch.isfinite(K[1, :, :10]).all() and torch.isfinite(V[0]).all()
    q2, K2, _ = draw_qkv(cfg, ctx)
    assert torch.equal(q, q2) and np.array_equal(to_host_raw(K), to_host_raw(K2))
    assert to_host_raw(K).dtype == np.uint16
