"""GPU parity of the per-KV-head scoring variant (one score vector and one retained set per KV
head, the mean of Eq. 4 taken over the head's own query group) against the oracle's
`score_mode="per_kv_head"`, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import momentkv_oracle as O
from paper_2605_29873_amd import inputs as X
from tests.harness import (make_ctx, to_device, from_device, storage_to_values, OUT_TOL, SCORE_RTOL,
                           SCORE_ATOL)

pytestmark = pytest.mark.gpu


class PerHeadLockstep:
    """Sequence by sequence, vector by vector; evictions on the oracle's float32 scores."""

    def __init__(self, mkv, wl, split_keys=0, max_q_len=0, attn_variant=0):
        self.mkv, self.wl = mkv, wl
        self.ctx = make_ctx(mkv, wl, manual_evict=True, split_keys=split_keys, max_q_len=max_q_len,
                            attn_variant=attn_variant, score_mode=mkv.MKV_SCORE_PER_KV_HEAD)
        self.st = [O.MomentKVState(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.decode_budget, wl.alpha,
                                   wl.evict_trigger, wl.recent_window, score_mode="per_kv_head",
                                   decision_dtype=np.float32) for _ in range(wl.batch)]
        self.dt = mkv.MKV_BF16 if wl.dtype == "bf16" else mkv.MKV_F32
        self.tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
        self.multi = max_q_len > 0
        self.evictions = 0
        self.distinct_sets = 0
        for s in range(wl.batch):
            k, v = X.prefill_kv(wl, 0, s)
            if k.shape[0]:
                dk, dv = to_device(k, wl.dtype), to_device(v, wl.dtype)
                mkv.mkv_prefill_append(self.ctx, 0, s, dk.data_ptr(), dv.data_ptr(), k.shape[0])
            self.st[s].prefill_append(k, v)

    def close(self):
        self.mkv.mkv_destroy(self.ctx)

    def check_scores(self, s, exact=False):
        st = self.st[s]
        for g in range(self.wl.n_kv_heads):
            self.mkv.mkv_set_score_view(self.ctx, g)
            gs, gp = self.mkv.mkv_read_scores(self.ctx, 0, s)
            assert np.array_equal(gp, st.pos[g].astype(np.int32)), f"seq {s} head {g}: positions differ"
            if exact:
                assert np.array_equal(gs, st.I[g].astype(np.float32)), f"seq {s} head {g}: compacted scores differ"
            else:
                err = np.abs(gs.astype(np.float64) - st.I[g])
                assert np.all(err <= SCORE_RTOL * np.abs(st.I[g]) + SCORE_ATOL), f"seq {s} head {g}: scores off"
        self.mkv.mkv_set_score_view(self.ctx, 0)

    def check_rows(self, s):
        for g in range(self.wl.n_kv_heads):
            k, v = self.mkv.mkv_read_kv(self.ctx, 0, s, 0, g, self.wl.head_dim, self.dt)
            assert np.array_equal(storage_to_values(k, self.wl.dtype).astype(np.float64), self.st[s].Kd[g][:, 0])
            assert np.array_equal(storage_to_values(v, self.wl.dtype).astype(np.float64), self.st[s].Vd[g][:, 0])

    def feed(self, t, q_len):
        wl = self.wl
        per = [X.step_batch(wl, 0, t + i) for i in range(q_len)]
        q, k, v = (np.stack([p[r] for p in per], axis=1) for r in range(3))
        dq, dk, dv = (to_device(a, wl.dtype) for a in (q, k, v))
        out = torch.zeros((wl.batch, q_len, wl.n_q_heads, wl.head_dim), dtype=self.tdt, device="cuda")
        if q_len == 1 and (t % 2 == 0 or not self.multi):
            self.mkv.mkv_decode_step(self.ctx, 0, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), out.data_ptr())
        else:
            self.mkv.mkv_decode_step_multi(self.ctx, 0, q_len, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), out.data_ptr())
        torch.cuda.synchronize()
        got = from_device(out)
        rtol, atol = OUT_TOL[wl.dtype]
        for s in range(wl.batch):
            st = self.st[s]
            for i in range(q_len):
                ref, abar = st.decode_step(q[s, i], k[s, i], v[s, i], auto_evict=False)
                assert np.all(np.abs(got[s, i] - ref) <= atol + rtol * np.abs(ref)), f"step {t}+{i} seq {s}: output off"
            for g in range(wl.n_kv_heads):
                self.mkv.mkv_set_score_view(self.ctx, g)
                ga, _ = self.mkv.mkv_read_probs(self.ctx, 0, s, wl.n_q_heads, wl.capacity + q_len)
                assert np.all(np.abs(ga - abar[g]) <= SCORE_RTOL * abar[g] + SCORE_ATOL), f"step {t} seq {s} head {g}: abar off"
            self.check_scores(s)
            if st.n_decode > wl.evict_trigger:
                for g in range(wl.n_kv_heads):
                    self.mkv.mkv_set_score_view(self.ctx, g)
                    self.mkv.mkv_write_scores(self.ctx, 0, s, st.I[g].astype(np.float32))
                self.mkv.mkv_evict(self.ctx, 0, s)
                st.evict()
                self.evictions += 1
                self.check_scores(s, exact=True)
                self.check_rows(s)
                sets = {tuple(p.tolist()) for p in st.pos}
                self.distinct_sets = max(self.distinct_sets, len(sets))


def _wl(G, Hkv, D=128, dtype="bf16", **kw):
    base = dict(batch=2, n_layers=1, n_q_heads=G * Hkv, n_kv_heads=Hkv, head_dim=D, dtype=dtype,
                prefill_min=40, prefill_max=200, decode_budget=24, evict_trigger=30, recent_window=3,
                alpha=0.7, steps=0, hh_prob=0.05)
    base.update(kw)
    return X.Workload("perhead", **base)


@pytest.mark.parametrize("G,Hkv,D,dtype,variant", [
    (4, 4, 128, "bf16", 0),     # matrix-core kernels
    (7, 2, 128, "bf16", 0),
    (4, 2, 128, "bf16", 15),    # vector-ALU kernels on the same layer
    (2, 4, 64, "f32", 0),
    (1, 3, 64, "bf16", 0),      # no grouping: every query head scores its own KV head
])
def test_every_kv_head_keeps_its_own_tokens(mkv, G, Hkv, D, dtype, variant):
    wl = _wl(G, Hkv, D, dtype)
    ls = PerHeadLockstep(mkv, wl, split_keys=64, attn_variant=variant)
    try:
        for t in range(75):
            ls.feed(t, 1)
        assert ls.evictions >= 2 * 6
        assert ls.distinct_sets > 1, "the KV heads never disagreed: the case does not tell the modes apart"
    finally:
        ls.close()


@pytest.mark.parametrize("G,Hkv,Q", [(4, 2, 4), (4, 2, 8), (7, 2, 4)])   # 16 rows; 32 and 28 rows in two row blocks
def test_multi_query_calls(mkv, G, Hkv, Q):
    wl = _wl(G, Hkv)
    ls = PerHeadLockstep(mkv, wl, max_q_len=Q)
    try:
        t = 0
        for n in [Q, 1, 3, Q, 2, Q, Q, 1, 1, Q, 3, Q, Q, Q, 2, Q, Q, Q]:
            ls.feed(t, n)
            t += n
        assert ls.evictions >= 8 and ls.distinct_sets > 1
    finally:
        ls.close()


def test_paper_cadence_uses_the_selection_of_the_finishing_kernel(mkv):
    """Automatic one-token eviction per head (trigger = budget) against a second context that
    calls mkv_evict: bit-identical retained sets, scores and rows for every KV head."""
    wl = _wl(4, 2, decode_budget=21, evict_trigger=21, recent_window=2)
    mk = lambda manual: make_ctx(mkv, wl, manual_evict=manual, score_mode=mkv.MKV_SCORE_PER_KV_HEAD)
    auto, manual = mk(False), mk(True)
    try:
        for s in range(wl.batch):
            k, v = X.prefill_kv(wl, 0, s)
            dk, dv = to_device(k, wl.dtype), to_device(v, wl.dtype)
            for ctx in (auto, manual):
                mkv.mkv_prefill_append(ctx, 0, s, dk.data_ptr(), dv.data_ptr(), k.shape[0])
        out = torch.zeros((wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.bfloat16, device="cuda")
        distinct = 0
        for t in range(50):
            q, k, v = X.step_batch(wl, 0, t)
            dq, dk, dv = (to_device(a, wl.dtype) for a in (q, k, v))
            for ctx in (auto, manual):
                mkv.mkv_decode_step(ctx, 0, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), out.data_ptr())
            torch.cuda.synchronize()
            for s in range(wl.batch):
                if mkv.mkv_get_lens(manual, 0, s)[1] > wl.decode_budget:
                    mkv.mkv_evict(manual, 0, s)
                sets = set()
                for g in range(wl.n_kv_heads):
                    for ctx in (auto, manual):
                        mkv.mkv_set_score_view(ctx, g)
                    sa, pa = mkv.mkv_read_scores(auto, 0, s)
                    sm, pm = mkv.mkv_read_scores(manual, 0, s)
                    assert np.array_equal(pa, pm) and np.array_equal(sa.view(np.uint32), sm.view(np.uint32))
                    ka, va = mkv.mkv_read_kv(auto, 0, s, 0, g, wl.head_dim, mkv.MKV_BF16)
                    km, vm = mkv.mkv_read_kv(manual, 0, s, 0, g, wl.head_dim, mkv.MKV_BF16)
                    assert np.array_equal(ka, km) and np.array_equal(va, vm)
                    sets.add(tuple(pa.tolist()))
                distinct = max(distinct, len(sets))
        assert distinct > 1
    finally:
        mkv.mkv_destroy(auto)
        mkv.mkv_destroy(manual)


def test_score_view_bounds(mkv):
    wl = _wl(4, 2)
    ctx = make_ctx(mkv, wl, manual_evict=True, score_mode=mkv.MKV_SCORE_PER_KV_HEAD)
    plain = make_ctx(mkv, wl, manual_evict=True)
    try:
        mkv.mkv_set_score_view(ctx, 1)
        for bad in (-1, 2):
            with pytest.raises(mkv.MkvError):
                mkv.mkv_set_score_view(ctx, bad)
        mkv.mkv_set_score_view(plain, 0)
        with pytest.raises(mkv.MkvError):
            mkv.mkv_set_score_view(plain, 1)
    finally:
        mkv.mkv_destroy(ctx)
        mkv.mkv_destroy(plain)
