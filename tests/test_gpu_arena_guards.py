"""Nothing is written outside the arena: caller-owned arenas with patterned guard zones on both
sides stay intact over decode steps, automatic evictions, multi-row calls and the fused producer."""
import numpy as np
import pytest
import torch

from paper_2605_29873_amd import inputs as X
from tests.harness import to_device

pytestmark = pytest.mark.gpu

GUARD = 1 << 20          # bytes on each side
PATTERN = 0xA5


def _guarded_ctx(mkv, wl, **kw):
    cfg = mkv.make_config(
        n_layers=wl.n_layers, batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
        head_dim=wl.head_dim, dtype=mkv.MKV_BF16 if wl.dtype == "bf16" else mkv.MKV_F32,
        max_prefill=wl.prefill_max, decode_budget=wl.decode_budget, evict_trigger=wl.evict_trigger,
        recent_window=wl.recent_window, alpha=wl.alpha,
        stream=torch.cuda.current_stream().cuda_stream, **kw)
    need = mkv.mkv_required_bytes(cfg)
    assert need > 0
    buf = torch.full((need + 2 * GUARD + 256,), PATTERN, dtype=torch.uint8, device="cuda")
    base = (buf.data_ptr() + GUARD + 255) // 256 * 256
    cfg.arena, cfg.arena_bytes = base, need
    lo = base - buf.data_ptr()
    return mkv.mkv_create(cfg), buf, lo, lo + need


def _guards_intact(buf, lo, hi):
    torch.cuda.synchronize()
    return bool((buf[:lo] == PATTERN).all()) and bool((buf[hi:] == PATTERN).all())


@pytest.mark.parametrize("G,Hkv,D,dtype,q_len,mode", [
    (4, 2, 128, "bf16", 0, 0),      # matrix-core kernels, single query
    (7, 2, 128, "bf16", 0, 1),      # per-KV-head scores
    (4, 2, 128, "bf16", 8, 0),      # two row blocks per pass
    (12, 1, 128, "bf16", 3, 0),     # several passes
    (2, 2, 64, "f32", 0, 0),        # vector-ALU kernels
    (4, 2, 64, "bf16", 0, 0),
])
def test_guard_zones_stay_intact(mkv, G, Hkv, D, dtype, q_len, mode):
    wl = X.Workload("guards", batch=3, n_layers=2, n_q_heads=G * Hkv, n_kv_heads=Hkv, head_dim=D, dtype=dtype,
                    prefill_min=5, prefill_max=300, decode_budget=40, evict_trigger=52, recent_window=4,
                    alpha=0.9, steps=0, hh_prob=0.05)
    ctx, buf, lo, hi = _guarded_ctx(mkv, wl, max_q_len=q_len, score_mode=mode, split_keys=64)
    try:
        assert _guards_intact(buf, lo, hi)         # creation clears only its own bytes
        for layer in range(wl.n_layers):
            for s in range(wl.batch):
                k, v = X.prefill_kv(wl, layer, s)
                if k.shape[0]:
                    dk, dv = to_device(k, dtype), to_device(v, dtype)
                    mkv.mkv_prefill_append(ctx, layer, s, dk.data_ptr(), dv.data_ptr(), k.shape[0])
        nq = max(1, q_len)
        tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        out = torch.empty((wl.batch, nq, wl.n_q_heads, D), dtype=tdt, device="cuda")
        t = 0
        while t < 140:                              # several evictions per sequence and layer
            for layer in range(wl.n_layers):
                per = [X.step_batch(wl, layer, t + i) for i in range(nq)]
                q, k, v = (np.stack([p[r] for p in per], axis=1) for r in range(3))
                dq, dk, dv = (to_device(a, dtype) for a in (q, k, v))
                if q_len:
                    mkv.mkv_decode_step_multi(ctx, layer, q_len, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), out.data_ptr())
                else:
                    mkv.mkv_decode_step(ctx, layer, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), out.data_ptr())
            t += nq
        assert torch.isfinite(out.float()).all()
        for layer in range(wl.n_layers):
            for s in range(wl.batch):
                assert mkv.mkv_get_lens(ctx, layer, s)[1] <= wl.evict_trigger
        assert _guards_intact(buf, lo, hi)
    finally:
        mkv.mkv_destroy(ctx)


def test_guard_zones_with_the_fused_producer(mkv):
    wl = X.Workload("guards-proj", batch=4, n_layers=1, n_q_heads=8, n_kv_heads=2, head_dim=128, dtype="bf16",
                    prefill_min=0, prefill_max=64, decode_budget=30, evict_trigger=30, recent_window=2,
                    alpha=0.8, steps=0, hh_prob=0.05)
    hidden = 512
    ctx, buf, lo, hi = _guarded_ctx(mkv, wl)
    try:
        wk, wv = X.projection_weights(wl, 0, hidden)
        dwk, dwv = to_device(wk, "bf16"), to_device(wv, "bf16")
        out = torch.empty((wl.batch, wl.n_q_heads, 128), dtype=torch.bfloat16, device="cuda")
        for t in range(70):                         # paper cadence: one token out per step from step 30 on
            x = to_device(X.step_hidden(wl, 0, t, hidden), "bf16")
            pos = torch.full((wl.batch,), t, dtype=torch.int32, device="cuda")
            mkv.mkv_project_append(ctx, 0, x.data_ptr(), dwk.data_ptr(), dwv.data_ptr(), hidden, pos.data_ptr(), 10000.0)
            q = to_device(X.step_batch(wl, 0, t)[0], "bf16")
            mkv.mkv_decode_step(ctx, 0, q.data_ptr(), None, None, out.data_ptr())
        assert mkv.mkv_get_lens(ctx, 0, 0)[1] == 30
        assert _guards_intact(buf, lo, hi)
    finally:
        mkv.mkv_destroy(ctx)


@pytest.mark.parametrize("G,Hkv,mode", [(4, 2, 0), (7, 2, 1)])
def test_guard_zones_with_deferred_compaction(mkv, G, Hkv, mode):
    # the paper's cadence on the matrix-core kernels, default capacity: slot bitmaps, hole counts
    # and pending selections live in the layer blocks of the arena; two layers, three sequences of
    # which one pauses, readers (which compact) in between
    wl = X.Workload("guards-deferred", batch=3, n_layers=2, n_q_heads=G * Hkv, n_kv_heads=Hkv, head_dim=128,
                    dtype="bf16", prefill_min=5, prefill_max=300, decode_budget=40, evict_trigger=40,
                    recent_window=4, alpha=0.9, steps=0, hh_prob=0.05)
    ctx, buf, lo, hi = _guarded_ctx(mkv, wl, score_mode=mode)
    try:
        assert _guards_intact(buf, lo, hi)
        for layer in range(wl.n_layers):
            for s in range(wl.batch):
                k, v = X.prefill_kv(wl, layer, s)
                if k.shape[0]:
                    dk, dv = to_device(k, "bf16"), to_device(v, "bf16")
                    mkv.mkv_prefill_append(ctx, layer, s, dk.data_ptr(), dv.data_ptr(), k.shape[0])
        out = torch.empty((wl.batch, wl.n_q_heads, 128), dtype=torch.bfloat16, device="cuda")
        marked = 0
        for t in range(160):
            mask = np.array([1, t % 4 != 1, 1], dtype=np.uint8)
            for layer in range(wl.n_layers):
                q, k, v = (to_device(a, "bf16") for a in X.step_batch(wl, layer, t))
                mkv.mkv_decode_step(ctx, layer, q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), mask)
            _, _, live, _ = mkv.mkv_read_slots(ctx, 1, 2, 256)
            marked = max(marked, int((~live).sum()))
            if t % 45 == 44:
                mkv.mkv_read_scores(ctx, 0, 0)
                mkv.mkv_read_kv(ctx, 1, 2, 0, 1, 128, mkv.MKV_BF16)
        assert marked >= 5 and torch.isfinite(out.float()).all()
        for layer in range(wl.n_layers):
            assert mkv.mkv_get_lens(ctx, layer, 0)[1] == 40
        assert _guards_intact(buf, lo, hi)
    finally:
        mkv.mkv_destroy(ctx)
