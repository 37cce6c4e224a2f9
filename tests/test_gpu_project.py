"""GPU tests of the fused producer (k/v projection + rotary encoding written straight into the
decode pool) against the oracle's project_kv, and of decoding with rows produced that way."""
import numpy as np
import pytest
import torch

from oracle import momentkv_oracle as O
from paper_2605_29873_amd import inputs as X
from tests.harness import Lockstep, make_ctx, to_device, from_device, storage_to_values, OUT_TOL

pytestmark = pytest.mark.gpu
THETA = 500000.0      # the rotary base of the Llama-3.1 family


def _wl(Hkv, D, G=2, B=3, **kw):
    base = dict(batch=B, n_layers=1, n_q_heads=G * Hkv, n_kv_heads=Hkv, head_dim=D, dtype="bf16",
                prefill_min=20, prefill_max=60, decode_budget=12, evict_trigger=15, recent_window=2,
                alpha=0.8, steps=0, hh_prob=0.05)
    base.update(kw)
    return X.Workload("proj", **base)


@pytest.mark.parametrize("Hkv,D,hidden,B", [
    (2, 128, 512, 3),
    (8, 128, 4096, 16),     # the Llama-3.1-8B projection at batch 16
    (4, 128, 3584, 8),      # Qwen2.5-7B
    (2, 64, 256, 70),       # two passes over the batch, the second one ragged
])
def test_projected_rows_are_within_one_rounding_step_of_the_oracle(mkv, Hkv, D, hidden, B):
    wl = _wl(Hkv, D, B=B)
    ctx = make_ctx(mkv, wl, manual_evict=True)
    rng = np.random.default_rng(5)
    try:
        wk, wv = X.projection_weights(wl, 0, hidden)
        dwk, dwv = to_device(wk, "bf16"), to_device(wv, "bf16")
        mask = np.ones(B, dtype=np.uint8)
        mask[1] = 0                                   # an inactive sequence gets no row
        q = torch.zeros((B, wl.n_q_heads, D), dtype=torch.bfloat16, device="cuda")
        out = torch.zeros_like(q)
        worst, differing, total = 0.0, 0, 0
        for t in range(3):
            x = X.step_hidden(wl, 0, t, hidden)
            pos = rng.integers(0, 131072, size=B).astype(np.int32)
            dx, dpos = to_device(x, "bf16"), torch.from_numpy(pos).cuda()
            mkv.mkv_project_append(ctx, 0, dx.data_ptr(), dwk.data_ptr(), dwv.data_ptr(), hidden,
                                   dpos.data_ptr(), THETA, mask)
            mkv.mkv_decode_step(ctx, 0, q.data_ptr(), None, None, out.data_ptr(), mask)
            torch.cuda.synchronize()
            for b in range(B):
                if not mask[b]:
                    assert mkv.mkv_get_lens(ctx, 0, b)[1] == 0
                    continue
                k_ref, v_ref = O.project_kv(x[b], wk, wv, int(pos[b]), THETA, Hkv)
                for g in range(Hkv):
                    gk, gv = mkv.mkv_read_kv(ctx, 0, b, 0, g, D, mkv.MKV_BF16)
                    assert gk.shape[0] == t + 1
                    for got, ref in ((storage_to_values(gk[t], "bf16"), k_ref[g]),
                                     (storage_to_values(gv[t], "bf16"), v_ref[g])):
                        exact = X.round_bf16(ref.astype(np.float32))
                        # one bf16 step (generous), with a floor for values near zero: the fp32 sum of
                        # `hidden` products of size ~0.05 carries an absolute error of up to ~1e-6
                        step = np.maximum(np.abs(ref) * 2.0 ** -7, 5e-6)
                        assert np.all(np.abs(got - ref) <= step), "a projected value is off by more than a rounding step"
                        differing += int(np.sum(got != exact))
                        total += got.size
                        worst = max(worst, float(np.max(np.abs(got - ref) / step)))
        # fp32 accumulation against fp64: only values next to a rounding boundary may differ
        assert differing <= max(3, total // 200), f"{differing} of {total} values rounded differently"
        print(f"projection {Hkv}x{D} hidden {hidden}: {differing}/{total} values round differently, worst {worst:.2f} steps")
    finally:
        mkv.mkv_destroy(ctx)


def _exact_inputs(rng, wl, hidden, t):
    """x and weights whose products add up exactly in fp32 (small integers times powers of two), so
    that both sides produce bit-identical rows and the lock-step tolerances stay those of the path."""
    x = rng.integers(-3, 4, size=(wl.batch, hidden)).astype(np.float32) * np.float32(0.25)
    return x


@pytest.mark.parametrize("G,Hkv,D,variant", [(4, 2, 128, 0), (4, 2, 128, 15), (2, 2, 64, 0)])
def test_decoding_with_rows_from_the_producer_in_lock_step(mkv, G, Hkv, D, variant):
    hidden = 512
    wl = _wl(Hkv, D, G=G, B=2)
    ls = Lockstep(mkv, wl, split_keys=64, attn_variant=variant)
    rng = np.random.default_rng(9)
    try:
        ls.prefill()
        n = Hkv * D
        wk = rng.integers(-2, 3, size=(n, hidden)).astype(np.float32) * np.float32(2.0 ** -5)
        wv = rng.integers(-2, 3, size=(n, hidden)).astype(np.float32) * np.float32(2.0 ** -5)
        dwk, dwv = to_device(wk, "bf16"), to_device(wv, "bf16")
        base = np.array([X.prefill_len(wl, s) + 90000 * s for s in range(wl.batch)], dtype=np.int32)
        rtol, atol = OUT_TOL["bf16"]
        for t in range(45):
            x = _exact_inputs(rng, wl, hidden, t)
            q, _, _ = X.step_batch(wl, 0, t)
            pos = base + t
            dx, dq, dpos = to_device(x, "bf16"), to_device(q, "bf16"), torch.from_numpy(pos).cuda()
            mkv.mkv_project_append(ls.ctx, 0, dx.data_ptr(), dwk.data_ptr(), dwv.data_ptr(), hidden,
                                   dpos.data_ptr(), THETA, ls.mask)
            mkv.mkv_decode_step(ls.ctx, 0, dq.data_ptr(), None, None, ls.out.data_ptr(), ls.mask)
            torch.cuda.synchronize()
            got = from_device(ls.out)
            for s in ls.seqs:
                k, v = O.project_kv(x[s], wk, wv, int(pos[s]), THETA, Hkv)
                k, v = X.round_bf16(k.astype(np.float32)), X.round_bf16(v.astype(np.float32))
                ref, _ = ls.oracles[s].decode_step(q[s], k, v, auto_evict=False)
                assert np.all(np.abs(got[s] - ref) <= atol + rtol * np.abs(ref)), f"step {t} seq {s}: output off"
                ls.check_scores(s)
            ls.capacity_check(t)          # evictions on identical scores; rows compared bit for bit
        assert ls.evictions >= 2 * 5
    finally:
        ls.close()


def test_state_and_argument_errors(mkv):
    wl = _wl(2, 128, B=2)
    ctx = make_ctx(mkv, wl, manual_evict=True)
    f32 = make_ctx(mkv, X.scaled(wl, dtype="f32"), manual_evict=True)
    z = torch.zeros(2 * 4 * 128 * 4, dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(2 * 128 * 512, dtype=torch.bfloat16, device="cuda")
    pos = torch.zeros(2, dtype=torch.int32, device="cuda")
    args = (z.data_ptr(), w.data_ptr(), w.data_ptr(), 512, pos.data_ptr(), THETA)
    try:
        with pytest.raises(mkv.MkvError) as e:       # no projected row yet
            mkv.mkv_decode_step(ctx, 0, z.data_ptr(), None, None, z.data_ptr())
        assert e.value.code == mkv.MKV_ERR_STATE
        with pytest.raises(mkv.MkvError) as e:       # only one of the two
            mkv.mkv_decode_step(ctx, 0, z.data_ptr(), z.data_ptr(), None, z.data_ptr())
        assert e.value.code == mkv.MKV_ERR_ARG
        mkv.mkv_project_append(ctx, 0, *args)
        for call in (lambda: mkv.mkv_project_append(ctx, 0, *args),                                   # twice
                     lambda: mkv.mkv_decode_step(ctx, 0, z.data_ptr(), z.data_ptr(), z.data_ptr(), z.data_ptr()),
                     lambda: mkv.mkv_evict(ctx, 0, -1)):
            with pytest.raises(mkv.MkvError) as e:
                call()
            assert e.value.code == mkv.MKV_ERR_STATE
        mkv.mkv_decode_step(ctx, 0, z.data_ptr(), None, None, z.data_ptr())
        assert mkv.mkv_get_lens(ctx, 0, 0)[1] == 1
        for bad in ((z.data_ptr(), w.data_ptr(), w.data_ptr(), 500, pos.data_ptr(), THETA),
                    (z.data_ptr(), w.data_ptr(), w.data_ptr(), 512, pos.data_ptr(), 1.0),
                    (0, w.data_ptr(), w.data_ptr(), 512, pos.data_ptr(), THETA)):
            with pytest.raises(mkv.MkvError) as e:
                mkv.mkv_project_append(ctx, 0, *bad)
            assert e.value.code == mkv.MKV_ERR_ARG
        with pytest.raises(mkv.MkvError) as e:
            mkv.mkv_project_append(f32, 0, *args)
        assert e.value.code == mkv.MKV_ERR_ARG
    finally:
        mkv.mkv_destroy(ctx)
        mkv.mkv_destroy(f32)
