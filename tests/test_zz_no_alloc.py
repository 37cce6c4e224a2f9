"""mkv_decode_step_static -- the decode step whose scratch is a static array inside the library's
code object, for callers that cannot allocate -- against mkv_decode_step on a twin context: same
inputs, results bit for bit (the kernels are the same), and against the CPU oracle at the usual
tolerances.  Calls alternate between a larger and a smaller workload, so that every call finds
the array filled by a call of another shape."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import momentkv_oracle as O
from paper_2605_29873_amd import inputs as X
from tests.harness import make_ctx, oracle_state, to_device, from_device, OUT_TOL, SCORE_RTOL, SCORE_ATOL

pytestmark = pytest.mark.gpu


class Pair:
    """One workload on two contexts: `plain` steps through mkv_decode_step, `static` through
    mkv_decode_step_static; an oracle follows sequence 0."""

    def __init__(self, mkv, wl):
        self.mkv, self.wl = mkv, wl
        self.plain = make_ctx(mkv, wl, manual_evict=False)
        self.static = make_ctx(mkv, wl, manual_evict=False)
        self.st = oracle_state(wl)
        for s in range(wl.batch):
            k, v = X.prefill_kv(wl, 0, s)
            dk, dv = to_device(k, wl.dtype), to_device(v, wl.dtype)
            for c in (self.plain, self.static):
                mkv.mkv_prefill_append(c, 0, s, dk.data_ptr(), dv.data_ptr(), k.shape[0])
            if s == 0:
                self.st.prefill_append(k, v)
        tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
        self.out_p = torch.zeros((wl.batch, wl.n_q_heads, wl.head_dim), dtype=tdt, device="cuda")
        self.out_s = torch.zeros_like(self.out_p)
        self.t = 0
        self.evictions = 0

    def step(self):
        mkv, wl, t = self.mkv, self.wl, self.t
        q, k, v = X.step_batch(wl, 0, t)
        dq, dk, dv = (to_device(a, wl.dtype) for a in (q, k, v))
        mkv.mkv_decode_step(self.plain, 0, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), self.out_p.data_ptr())
        mkv.mkv_decode_step_static(self.static, 0, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), self.out_s.data_ptr())
        torch.cuda.synchronize()
        assert torch.equal(self.out_p, self.out_s), f"{wl.name} step {t}: Att differs between the two entry points"
        ref, abar = self.st.decode_step(q[0], k[0], v[0], auto_evict=False)
        rtol, atol = OUT_TOL[wl.dtype]
        err = np.abs(from_device(self.out_s)[0] - ref)
        assert np.all(err <= atol + rtol * np.abs(ref)), f"{wl.name} step {t}: Att off the oracle by {err.max():.3e}"
        ga, _ = mkv.mkv_read_probs(self.static, 0, 0, wl.n_q_heads, wl.capacity)   # read from the static array
        assert np.all(np.abs(ga - abar) <= SCORE_RTOL * abar + SCORE_ATOL), f"{wl.name} step {t}: abar off the oracle"
        fired = self.st.n_decode > wl.evict_trigger
        for s in range(wl.batch):
            sp, pp = mkv.mkv_read_scores(self.plain, 0, s)
            ss, ps = mkv.mkv_read_scores(self.static, 0, s)
            assert np.array_equal(pp, ps), f"{wl.name} step {t} seq {s}: retained sets differ"
            assert np.array_equal(sp.view(np.uint32), ss.view(np.uint32)), f"{wl.name} step {t} seq {s}: scores differ"
        if fired:
            # the oracle removes what the device removed (checked to be a legal selection on its
            # own scores up to a near-tie by the free-run tests; here the two entry points are the subject)
            self.evictions += 1
            _, ps = mkv.mkv_read_scores(self.static, 0, 0)
            self.st.remove(0, np.nonzero(~np.isin(self.st.pos[0], ps))[0])
        ss, ps = mkv.mkv_read_scores(self.static, 0, 0)
        assert np.array_equal(ps, self.st.pos[0].astype(np.int32))
        e = np.abs(ss.astype(np.float64) - self.st.I[0])
        assert np.all(e <= SCORE_RTOL * np.abs(self.st.I[0]) + SCORE_ATOL), f"{wl.name} step {t}: scores off the oracle"
        if fired or t % 16 == 0:
            dt = mkv.MKV_BF16 if wl.dtype == "bf16" else mkv.MKV_F32
            for g in range(wl.n_kv_heads):
                kp, vp = mkv.mkv_read_kv(self.plain, 0, 0, 0, g, wl.head_dim, dt)
                ks, vs = mkv.mkv_read_kv(self.static, 0, 0, 0, g, wl.head_dim, dt)
                assert np.array_equal(kp, ks) and np.array_equal(vp, vs)
        self.t += 1

    def close(self):
        self.mkv.mkv_destroy(self.plain)
        self.mkv.mkv_destroy(self.static)


def test_static_scratch_step_equals_the_arena_step_on_alternating_shapes(mkv):
    big = X.scaled(X.workloads()["cfg2"], batch=3, prefill_min=300, prefill_max=900, decode_budget=96,
                   evict_trigger=96 + 15, recent_window=8, burst_period=64, burst_keys=8, burst_len=6)
    small = X.scaled(X.workloads()["cfg1"], batch=1, prefill_min=40, prefill_max=40, decode_budget=12,
                     evict_trigger=12, recent_window=2)        # fp32 x 64 heads, the paper's cadence
    a, b = Pair(mkv, big), Pair(mkv, small)
    try:
        a.step()                      # two calls in a row, the second on the smaller input
        b.step()
        for i in range(150):
            a.step()
            b.step()
            if i % 3 == 0:
                b.step()              # the shapes also follow themselves
        assert a.evictions >= 2 and b.evictions >= 100
    finally:
        a.close()
        b.close()


def test_static_scratch_refuses_a_step_that_does_not_fit(mkv):
    lib = mkv.load()
    wl = X.Workload("wide", batch=48, n_layers=1, n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16",
                    prefill_min=16, prefill_max=16, decode_budget=8000, evict_trigger=8063, recent_window=0,
                    alpha=0.9, steps=0)
    ctx = make_ctx(mkv, wl, manual_evict=False)
    try:
        kv = torch.zeros((16, 8, 128), dtype=torch.bfloat16, device="cuda")
        for s in range(wl.batch):
            mkv.mkv_prefill_append(ctx, 0, s, kv.data_ptr(), kv.data_ptr(), 16)
        q = torch.zeros((wl.batch, 32, 128), dtype=torch.bfloat16, device="cuda")
        kn = torch.zeros((wl.batch, 8, 128), dtype=torch.bfloat16, device="cuda")
        out = torch.zeros_like(q)
        # logits alone: 48 x 32 x 8064 x 4 bytes = 49.5 MB > 32 MiB
        rc = lib.mkv_decode_step_static(ctx, 0, q.data_ptr(), kn.data_ptr(), kn.data_ptr(), out.data_ptr(), None)
        assert rc == mkv.MKV_ERR_CAPACITY
        msg = mkv.mkv_last_error(ctx)
        assert "static" in msg and str(32 << 20) in msg
        assert mkv.mkv_get_lens(ctx, 0, 0) == (16, 0, 0)          # nothing was appended
        mkv.mkv_decode_step(ctx, 0, q.data_ptr(), kn.data_ptr(), kn.data_ptr(), out.data_ptr())
        assert mkv.mkv_get_lens(ctx, 0, 0) == (16, 1, 1)
    finally:
        mkv.mkv_destroy(ctx)
