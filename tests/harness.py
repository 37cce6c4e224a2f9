"""Lock-step driver: the HIP library and the CPU oracle fed identical bits, compared per step.

Test infrastructure (imports the oracle).  Tolerances are the build's stated bars:
attention output rtol 2e-2 / atol 2e-3 with bf16 K/V (1e-4 / 1e-5 with fp32), scores rel 1e-4
(absolute floor 1e-9), retained sets / positions / moved rows bit-exact once both sides select on
the same float32 scores.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import momentkv_oracle as O
from paper_2605_29873_amd import inputs as X

OUT_TOL = {"bf16": (2e-2, 2e-3), "f32": (1e-4, 1e-5)}
SCORE_RTOL, SCORE_ATOL = 1e-4, 1e-9


def to_device(x: np.ndarray, dtype: str) -> torch.Tensor:
    """Storage-exact float32 values -> device tensor in the storage dtype."""
    if dtype == "bf16":
        bits = X.bf16_bits(x)
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


def from_device(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy()


def make_ctx(mkv, wl: X.Workload, *, manual_evict: bool, layers: int | None = None,
             split_keys: int = 0, max_prefill: int | None = None, stream: int | None = None,
             max_q_len: int = 0, attn_variant: int = 0, score_mode: int = 0):
    cfg = mkv.make_config(
        n_layers=wl.n_layers if layers is None else layers, batch=wl.batch,
        n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim,
        dtype=mkv.MKV_BF16 if wl.dtype == "bf16" else mkv.MKV_F32,
        max_prefill=wl.prefill_max if max_prefill is None else max_prefill,
        decode_budget=wl.decode_budget,
        evict_trigger=mkv.MKV_NEVER_EVICT if manual_evict else wl.evict_trigger,
        decode_capacity=wl.capacity + max(0, max_q_len - 1), recent_window=wl.recent_window,
        alpha=wl.alpha, softmax_scale=0.0, score_mode=score_mode,
        split_keys=split_keys, max_q_len=max_q_len, attn_variant=attn_variant,
        stream=stream if stream is not None else torch.cuda.current_stream().cuda_stream)
    return mkv.mkv_create(cfg)


def oracle_state(wl: X.Workload) -> O.MomentKVState:
    return O.MomentKVState(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.decode_budget, wl.alpha,
                           wl.evict_trigger, wl.recent_window, decision_dtype=np.float32)


def storage_to_values(a: np.ndarray, dtype: str) -> np.ndarray:
    return X.bf16_from_bits(a).reshape(a.shape) if dtype == "bf16" else a


class Lockstep:
    """One layer of a workload on both sides.  The GPU context never auto-evicts: at every
    eviction the oracle's float32-rounded scores are injected so that both sides select on
    identical scores, and the decision must then match bit for bit."""

    def __init__(self, mkv, wl: X.Workload, layer: int = 0, split_keys: int = 0, seqs=None,
                 active=None, n_layers: int | None = None, device_fill_unfollowed: bool = False,
                 max_q_len: int = 0, attn_variant: int = 0):
        """seqs: the sequences the oracle follows (default: all); active: the sequences the GPU
        steps (default: seqs).  Sequences that are active but not followed load the GPU at the
        real batch size; they evict through the library's own trigger check."""
        self.mkv, self.wl, self.layer = mkv, wl, layer
        self.seqs = list(range(wl.batch)) if seqs is None else list(seqs)
        self.active = list(self.seqs) if active is None else list(active)
        assert set(self.seqs) <= set(self.active)
        self.device_fill = device_fill_unfollowed   # unfollowed sequences: values drawn on the device
        self.ctx = make_ctx(mkv, wl, manual_evict=True, layers=layer + 1 if n_layers is None else n_layers,
                            split_keys=split_keys, max_q_len=max_q_len, attn_variant=attn_variant)
        self.oracles = {s: oracle_state(wl) for s in self.seqs}
        self.out = torch.zeros((wl.batch, wl.n_q_heads, wl.head_dim),
                               dtype=torch.bfloat16 if wl.dtype == "bf16" else torch.float32,
                               device="cuda")
        self.mask = np.zeros(wl.batch, dtype=np.uint8)
        self.mask[self.active] = 1
        self.max_out_err = 0.0
        self.max_score_rel = 0.0
        self.evictions = 0

    def close(self):
        if self.ctx:
            self.mkv.mkv_destroy(self.ctx)
            self.ctx = None

    def _device_kv(self, n):
        """N(0,1) rows drawn on the device in the storage dtype (for sequences nobody follows)."""
        wl = self.wl
        dt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
        shape = (n, wl.n_kv_heads, wl.head_dim)
        return (torch.randn(shape, device="cuda", dtype=torch.float32).to(dt),
                torch.randn(shape, device="cuda", dtype=torch.float32).to(dt))

    def prefill(self):
        for s in self.active:
            if self.device_fill and s not in self.oracles:
                m = X.prefill_len(self.wl, s)
                dk, dv = self._device_kv(m)
                self.mkv.mkv_prefill_append(self.ctx, self.layer, s, dk.data_ptr(), dv.data_ptr(), m)
                torch.cuda.synchronize()
                continue
            k, v = X.prefill_kv(self.wl, self.layer, s)
            half = k.shape[0] // 2                      # two appends: exercises the row offset
            for lo, hi in ((0, half), (half, k.shape[0])):
                if hi > lo:
                    dk, dv = to_device(k[lo:hi], self.wl.dtype), to_device(v[lo:hi], self.wl.dtype)
                    self.mkv.mkv_prefill_append(self.ctx, self.layer, s, dk.data_ptr(), dv.data_ptr(), hi - lo)
            torch.cuda.synchronize()
            if s in self.oracles:
                self.oracles[s].prefill_append(k, v)

    def load_snapshot(self, n_d: int, t_now: int):
        for s in self.active:
            if self.device_fill and s not in self.oracles:
                dk, dv = self._device_kv(n_d)
                rng = np.random.default_rng(s)
                pos = np.sort(rng.choice(t_now, n_d, replace=False)).astype(np.int32)
                sc = (rng.random(n_d, dtype=np.float32) * 1e-3).astype(np.float32)
                self.mkv.mkv_load_decode(self.ctx, self.layer, s, dk.data_ptr(), dv.data_ptr(), sc, pos, t_now)
                continue
            k, v, sc, pos = X.decode_snapshot(self.wl, self.layer, s, n_d, t_now)
            dk, dv = to_device(k, self.wl.dtype), to_device(v, self.wl.dtype)
            self.mkv.mkv_load_decode(self.ctx, self.layer, s, dk.data_ptr(), dv.data_ptr(), sc, pos, t_now)
            if s in self.oracles:
                self.oracles[s].load_decode(k, v, sc, pos, t_now)

    def check_scores(self, s):
        gs, gp = self.mkv.mkv_read_scores(self.ctx, self.layer, s)
        st = self.oracles[s]
        assert np.array_equal(gp, st.pos[0].astype(np.int32)), f"seq {s}: positions differ"
        ref = st.I[0]
        err = np.abs(gs.astype(np.float64) - ref)
        tol = SCORE_RTOL * np.abs(ref) + SCORE_ATOL
        self.max_score_rel = max(self.max_score_rel, float(np.max(err / (np.abs(ref) + 1e-30))))
        assert np.all(err <= tol), (f"seq {s}: score mismatch, worst rel "
                                    f"{np.max(err / (np.abs(ref) + 1e-30)):.3e}")

    def step(self, t: int, check_scores: bool = True, check_abar: bool = False):
        wl = self.wl
        q, k, v = X.step_batch(wl, self.layer, t)
        dq, dk, dv = (to_device(a, wl.dtype) for a in (q, k, v))
        self.mkv.mkv_decode_step(self.ctx, self.layer, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(),
                                 self.out.data_ptr(), self.mask)
        torch.cuda.synchronize()
        got = from_device(self.out)
        rtol, atol = OUT_TOL[wl.dtype]
        for s in self.seqs:
            st = self.oracles[s]
            ref, abar = st.decode_step(q[s], k[s], v[s], auto_evict=False)
            err = np.abs(got[s] - ref)
            self.max_out_err = max(self.max_out_err, float(err.max()))
            assert np.all(err <= atol + rtol * np.abs(ref)), \
                f"step {t} seq {s}: attention output off by {err.max():.3e}"
            if check_abar:
                ga, _ = self.mkv.mkv_read_probs(self.ctx, self.layer, s, wl.n_q_heads, wl.capacity)
                assert ga.shape == abar.shape
                assert np.all(np.abs(ga - abar) <= SCORE_RTOL * abar + SCORE_ATOL), \
                    f"step {t} seq {s}: abar mismatch"
            if check_scores:
                self.check_scores(s)
        self.capacity_check(t)

    def step_multi(self, t0: int, q_len: int, check_scores: bool = True, check_abar: bool = False):
        """q_len steps in one library call; the oracle takes them one by one (Algorithm 1 per
        token) with its capacity check held back to the end of the chunk."""
        wl = self.wl
        per_step = [X.step_batch(wl, self.layer, t0 + i) for i in range(q_len)]
        q, k, v = (np.stack([p[r] for p in per_step], axis=1) for r in range(3))   # [B, q_len, heads, D]
        dq, dk, dv = (to_device(a, wl.dtype) for a in (q, k, v))
        out = torch.zeros((wl.batch, q_len, wl.n_q_heads, wl.head_dim), dtype=self.out.dtype, device="cuda")
        self.mkv.mkv_decode_step_multi(self.ctx, self.layer, q_len, dq.data_ptr(), dk.data_ptr(),
                                       dv.data_ptr(), out.data_ptr(), self.mask)
        torch.cuda.synchronize()
        got = from_device(out)
        rtol, atol = OUT_TOL[wl.dtype]
        for s in self.seqs:
            st = self.oracles[s]
            for i in range(q_len):
                ref, abar = st.decode_step(q[s, i], k[s, i], v[s, i], auto_evict=False)
                err = np.abs(got[s, i] - ref)
                self.max_out_err = max(self.max_out_err, float(err.max()))
                assert np.all(err <= atol + rtol * np.abs(ref)), \
                    f"step {t0}+{i} seq {s}: attention output off by {err.max():.3e}"
            if check_abar:     # of the last row
                ga, _ = self.mkv.mkv_read_probs(self.ctx, self.layer, s, wl.n_q_heads, wl.capacity + q_len)
                assert ga.shape == abar.shape
                assert np.all(np.abs(ga - abar) <= SCORE_RTOL * abar + SCORE_ATOL), \
                    f"step {t0}+{q_len - 1} seq {s}: abar mismatch"
            if check_scores:
                self.check_scores(s)
        self.capacity_check(t0 + q_len - 1)

    def capacity_check(self, t: int):
        """Eq. 7 with the trigger: both sides evict on the oracle's float32 scores."""
        wl = self.wl
        for s in self.active:
            if s not in self.oracles:
                _, n_d, _ = self.mkv.mkv_get_lens(self.ctx, self.layer, s)
                if n_d > wl.evict_trigger:
                    self.mkv.mkv_evict(self.ctx, self.layer, s)
        for s in self.seqs:
            st = self.oracles[s]
            if st.n_decode > wl.evict_trigger:
                self.check_scores(s)
                inject = st.I[0].astype(np.float32)
                self.mkv.mkv_write_scores(self.ctx, self.layer, s, inject)
                before = self.snapshot_rows(s)
                self.mkv.mkv_evict(self.ctx, self.layer, s)
                st.evict()
                self.evictions += 1
                gs, gp = self.mkv.mkv_read_scores(self.ctx, self.layer, s)
                assert np.array_equal(gp, st.pos[0].astype(np.int32)), \
                    f"step {t} seq {s}: retained set differs from the oracle's"
                assert np.array_equal(gs, st.I[0].astype(np.float32)), \
                    f"step {t} seq {s}: compacted scores differ"
                self.check_rows(s, before)

    def snapshot_rows(self, s):
        """Decode rows of every KV head before an eviction, keyed by original position."""
        wl = self.wl
        _, pos = self.mkv.mkv_read_scores(self.ctx, self.layer, s)
        dt = self.mkv.MKV_BF16 if wl.dtype == "bf16" else self.mkv.MKV_F32
        rows = [self.mkv.mkv_read_kv(self.ctx, self.layer, s, 0, g, wl.head_dim, dt)
                for g in range(wl.n_kv_heads)]
        return pos, rows

    def check_rows(self, s, before):
        """Every retained row is bit-identical to the row its token had before compaction."""
        wl = self.wl
        old_pos, old_rows = before
        _, new_pos = self.mkv.mkv_read_scores(self.ctx, self.layer, s)
        idx = np.searchsorted(old_pos, new_pos)
        assert np.array_equal(old_pos[idx], new_pos)
        dt = self.mkv.MKV_BF16 if wl.dtype == "bf16" else self.mkv.MKV_F32
        st = self.oracles[s]
        for g in range(wl.n_kv_heads):
            k, v = self.mkv.mkv_read_kv(self.ctx, self.layer, s, 0, g, wl.head_dim, dt)
            assert np.array_equal(k, old_rows[g][0][idx]), f"seq {s} head {g}: K rows moved wrongly"
            assert np.array_equal(v, old_rows[g][1][idx]), f"seq {s} head {g}: V rows moved wrongly"
            assert np.array_equal(storage_to_values(k, wl.dtype).astype(np.float64), st.Kd[0][:, g])
            assert np.array_equal(storage_to_values(v, wl.dtype).astype(np.float64), st.Vd[0][:, g])

    def check_prefill_untouched(self, s):
        wl = self.wl
        dt = self.mkv.MKV_BF16 if wl.dtype == "bf16" else self.mkv.MKV_F32
        k0, v0 = X.prefill_kv(wl, self.layer, s)
        for g in range(wl.n_kv_heads):
            k, v = self.mkv.mkv_read_kv(self.ctx, self.layer, s, 1, g, wl.head_dim, dt)
            assert np.array_equal(storage_to_values(k, wl.dtype), k0[:, g])
            assert np.array_equal(storage_to_values(v, wl.dtype), v0[:, g])
