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


class Progress:
    """A line on the real stdout every `every` seconds from inside a long test (pytest's capture is
    suspended for it), so that a run that follows a workload for minutes is seen to be alive."""

    def __init__(self, capsys, label: str, every: float = 20.0):
        import time
        self.capsys, self.label, self.every = capsys, label, every
        self.clock = time.monotonic
        self.t0 = self.last = self.clock()

    def tick(self, what: str):
        now = self.clock()
        if now - self.last >= self.every:
            self.last = now
            with self.capsys.disabled():
                print(f"  [{self.label}] {what}, {now - self.t0:.0f} s", flush=True)


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
             max_q_len: int = 0, attn_variant: int = 0, score_mode: int = 0,
             decode_capacity: int | None = None):
    cfg = mkv.make_config(
        n_layers=wl.n_layers if layers is None else layers, batch=wl.batch,
        n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim,
        dtype=mkv.MKV_BF16 if wl.dtype == "bf16" else mkv.MKV_F32,
        max_prefill=wl.prefill_max if max_prefill is None else max_prefill,
        decode_budget=wl.decode_budget,
        evict_trigger=mkv.MKV_NEVER_EVICT if manual_evict else wl.evict_trigger,
        decode_capacity=(wl.capacity + max(0, max_q_len - 1)) if decode_capacity is None else decode_capacity,
        recent_window=wl.recent_window,
        alpha=wl.alpha, softmax_scale=0.0, score_mode=score_mode,
        split_keys=split_keys, max_q_len=max_q_len, attn_variant=attn_variant,
        stream=stream if stream is not None else torch.cuda.current_stream().cuda_stream)
    return mkv.mkv_create(cfg)


def oracle_state(wl: X.Workload, score_mode: str = "layer_mean") -> O.MomentKVState:
    return O.MomentKVState(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.decode_budget, wl.alpha,
                           wl.evict_trigger, wl.recent_window, score_mode=score_mode,
                           decision_dtype=np.float32)


def oracle_from_gpu(mkv, ctx, wl: X.Workload, layer: int, s: int, per_head: bool = False) -> O.MomentKVState:
    """An oracle state that starts from what the device holds for (layer, s) right now: both pools
    (every KV head), the score vector(s), the positions and the step counter, read back through
    the ABI.  Used for windows that begin in the middle of a device run; from there on the oracle
    computes everything itself."""
    st = oracle_state(wl, "per_kv_head" if per_head else "layer_mean")
    dt = mkv.MKV_BF16 if wl.dtype == "bf16" else mkv.MKV_F32
    pre = [mkv.mkv_read_kv(ctx, layer, s, 1, g, wl.head_dim, dt) for g in range(wl.n_kv_heads)]
    dec = [mkv.mkv_read_kv(ctx, layer, s, 0, g, wl.head_dim, dt) for g in range(wl.n_kv_heads)]
    val = lambda a: storage_to_values(a, wl.dtype).astype(np.float64)
    st.Kp = np.stack([val(k) for k, _ in pre], axis=1)
    st.Vp = np.stack([val(v) for _, v in pre], axis=1)
    if per_head:
        for g in range(wl.n_kv_heads):
            mkv.mkv_set_score_view(ctx, g)
            sc, pos = mkv.mkv_read_scores(ctx, layer, s)
            st.Kd[g], st.Vd[g] = val(dec[g][0])[:, None, :], val(dec[g][1])[:, None, :]
            st.I[g], st.pos[g] = sc.astype(np.float64), pos.astype(np.int64)
        mkv.mkv_set_score_view(ctx, 0)
    else:
        sc, pos = mkv.mkv_read_scores(ctx, layer, s)
        st.Kd[0] = np.stack([val(k) for k, _ in dec], axis=1)
        st.Vd[0] = np.stack([val(v) for _, v in dec], axis=1)
        st.I[0], st.pos[0] = sc.astype(np.float64), pos.astype(np.int64)
    st.t = mkv.mkv_get_lens(ctx, layer, s)[2]
    st.frozen = True
    return st


class RoundingProbe:
    """How much of the device-vs-oracle gap of an attention output is float32 rounding: at sampled
    steps the oracle's attention is taken again with float32 accumulation (same steps, other
    dtype) over the very pool the step saw, and rounded to the storage dtype like the device's
    output.  Keeps the step with the largest device gap."""

    def __init__(self, wl: X.Workload):
        self.wl = wl
        self.worst = None

    def look(self, st: O.MomentKVState, q, got, ref, t, s):
        gap = np.abs(got - ref)
        i = np.unravel_index(np.argmax(gap), gap.shape)
        if self.worst is not None and gap[i] <= self.worst["device_gap"]:
            return
        K = np.concatenate([st.Kp, st.Kd[0]])
        V = np.concatenate([st.Vp, st.Vd[0]])
        A32 = O.attention_weights(q, K, st.scale, accumulate=np.float32)
        o32 = O.attention_output(A32, V, accumulate=np.float32)
        stored = X.to_storage_values(o32, self.wl.dtype)
        self.worst = {"step": t, "seq": s, "element": tuple(int(x) for x in i), "device_gap": float(gap[i]),
                      "f32_oracle_gap": float(abs(o32[i] - ref[i])),
                      "f32_oracle_rounded_to_storage_gap": float(abs(stored[i] - ref[i]))}

    def report(self, label: str) -> str:
        w = self.worst
        if w is None:
            return f"{label}: no probe taken"
        return (f"{label}: worst probed output element at step {w['step']} seq {w['seq']} {w['element']}: "
                f"device off by {w['device_gap']:.3e}; the float32-accumulating oracle is off by "
                f"{w['f32_oracle_gap']:.3e}, and by {w['f32_oracle_rounded_to_storage_gap']:.3e} once its output "
                f"is rounded to {self.wl.dtype} like the device's")


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
        self.probe = RoundingProbe(wl)
        self.probe_every = 0               # > 0: take the rounding probe every that many steps

    def close(self):
        if self.ctx:
            self.mkv.mkv_destroy(self.ctx)
            self.ctx = None

    def follow_from_gpu(self, s: int):
        """Starts following an active sequence from the device's own state (a mid-run window)."""
        assert s in self.active and s not in self.oracles
        self.oracles[s] = oracle_from_gpu(self.mkv, self.ctx, self.wl, self.layer, s)
        self.seqs.append(s)

    def unfollow(self, s: int):
        del self.oracles[s]
        self.seqs.remove(s)

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
            if self.probe_every and t % self.probe_every == 0:
                self.probe.look(st, q[s], got[s], ref, t, s)
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


class FreeRun:
    """The library's own capacity check -- an auto-evicting context, the path a caller runs --
    under the oracle's eyes, with no score injection.

    A second, never-evicting context (the "twin") takes the same steps on the same inputs, so that
    after each step it holds the float32 scores the auto context had *before* its eviction.  The
    oracle's selection (Eq. 8) run on those exact bits must name the tokens the auto context
    dropped: retained positions, scores and rows bit for bit.  The oracle's own run (float64 state)
    is compared every step at the score tolerance; where its selection differs from the one made
    on the device's bits, the tokens in question must be a near-tie at the cut -- counted, never
    skipped -- and the oracle then removes the device's set (Eq. 9) so that the two runs remain
    comparable to the end.  The twin evicts through mkv_evict (selection kernel + row mover), the
    auto context through whatever mkv_decode_step launches (at the paper's cadence: the arg-min
    taken by the finishing kernel and the one-row shift)."""

    def __init__(self, mkv, wl: X.Workload, seqs=None, active=None, per_head: bool = False,
                 attn_variant: int = 0, split_keys: int = 0, device_fill_unfollowed: bool = False,
                 layer: int = 0, auto_capacity: int | None = None):
        self.mkv, self.wl, self.layer, self.per_head = mkv, wl, layer, per_head
        self.seqs = list(range(wl.batch)) if seqs is None else list(seqs)
        self.active = list(self.seqs) if active is None else list(active)
        assert set(self.seqs) <= set(self.active)
        self.device_fill = device_fill_unfollowed
        mode = mkv.MKV_SCORE_PER_KV_HEAD if per_head else mkv.MKV_SCORE_LAYER_MEAN
        kw = dict(layers=layer + 1, split_keys=split_keys, attn_variant=attn_variant, score_mode=mode)
        self.auto = make_ctx(mkv, wl, manual_evict=False, decode_capacity=auto_capacity, **kw)
        self.twin = make_ctx(mkv, wl, manual_evict=True, **kw)
        self.n_vec = wl.n_kv_heads if per_head else 1
        self.oracles = {s: oracle_state(wl, "per_kv_head" if per_head else "layer_mean") for s in self.seqs}
        tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
        self.out_a = torch.zeros((wl.batch, wl.n_q_heads, wl.head_dim), dtype=tdt, device="cuda")
        self.out_t = torch.zeros_like(self.out_a)
        self.mask = np.zeros(wl.batch, dtype=np.uint8)
        self.mask[self.active] = 1
        self.dt = mkv.MKV_BF16 if wl.dtype == "bf16" else mkv.MKV_F32
        self.max_out_err = self.max_score_rel = 0.0
        self.evictions = self.near_ties = 0
        self.evicted_slots = []            # slot of every one-token eviction of a followed sequence

    def close(self):
        for c in (self.auto, self.twin):
            if c:
                self.mkv.mkv_destroy(c)
        self.auto = self.twin = None

    def prefill(self):
        wl = self.wl
        for s in self.active:
            if self.device_fill and s not in self.oracles:
                m = X.prefill_len(wl, s)
                dt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
                dk = torch.randn((m, wl.n_kv_heads, wl.head_dim), device="cuda").to(dt)
                dv = torch.randn((m, wl.n_kv_heads, wl.head_dim), device="cuda").to(dt)
            else:
                k, v = X.prefill_kv(wl, self.layer, s)
                dk, dv = to_device(k, wl.dtype), to_device(v, wl.dtype)
                if s in self.oracles:
                    self.oracles[s].prefill_append(k, v)
            if dk.shape[0]:
                for c in (self.auto, self.twin):
                    self.mkv.mkv_prefill_append(c, self.layer, s, dk.data_ptr(), dv.data_ptr(), dk.shape[0])
            torch.cuda.synchronize()

    def load_snapshot(self, n_d: int, t_now: int, scores=None):
        """Both contexts (and the oracles) start from the same synthetic mid-run decode pool;
        `scores`: float32[n_d] to use instead of the generator's (planted minima and ties)."""
        assert not self.per_head
        wl = self.wl
        for s in self.active:
            k, v, sc, pos = X.decode_snapshot(wl, self.layer, s, n_d, t_now)
            if scores is not None:
                sc = np.asarray(scores[s] if isinstance(scores, dict) else scores, dtype=np.float32)
            dk, dv = to_device(k, wl.dtype), to_device(v, wl.dtype)
            for c in (self.auto, self.twin):
                self.mkv.mkv_load_decode(c, self.layer, s, dk.data_ptr(), dv.data_ptr(), sc, pos, t_now)
            if s in self.oracles:
                self.oracles[s].load_decode(k, v, sc, pos, t_now)

    def follow_from_gpu(self, s: int):
        """Starts following an active sequence from the device's own state (a mid-run window)."""
        assert s in self.active and s not in self.oracles
        self.oracles[s] = oracle_from_gpu(self.mkv, self.auto, self.wl, self.layer, s, self.per_head)
        self.seqs.append(s)

    def unfollow(self, s: int):
        del self.oracles[s]
        self.seqs.remove(s)

    def _scores(self, ctx, s, v):
        if self.per_head:
            self.mkv.mkv_set_score_view(ctx, v)
        return self.mkv.mkv_read_scores(ctx, self.layer, s)

    def _rows(self, ctx, s):
        return [self.mkv.mkv_read_kv(ctx, self.layer, s, 0, g, self.wl.head_dim, self.dt)
                for g in range(self.wl.n_kv_heads)]

    def step(self, t: int, check_rows: bool = False):
        wl, mkv, L = self.wl, self.mkv, self.layer
        q, k, v = X.step_batch(wl, L, t)
        dq, dk, dv = (to_device(a, wl.dtype) for a in (q, k, v))
        mkv.mkv_decode_step(self.auto, L, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), self.out_a.data_ptr(), self.mask)
        mkv.mkv_decode_step(self.twin, L, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), self.out_t.data_ptr(), self.mask)
        torch.cuda.synchronize()
        # same kernels on bit-identical pools: any difference means the two contexts have split
        assert torch.equal(self.out_a, self.out_t), f"step {t}: auto and twin contexts disagree on Att"
        got = from_device(self.out_a)
        rtol, atol = OUT_TOL[wl.dtype]
        for s in self.active:
            if s in self.oracles:
                continue
            if mkv.mkv_get_lens(self.twin, L, s)[1] > wl.evict_trigger:
                mkv.mkv_evict(self.twin, L, s)
        for s in self.seqs:
            st = self.oracles[s]
            ref, _ = st.decode_step(q[s], k[s], v[s], auto_evict=False)
            err = np.abs(got[s] - ref)
            self.max_out_err = max(self.max_out_err, float(err.max()))
            assert np.all(err <= atol + rtol * np.abs(ref)), f"step {t} seq {s}: attention output off by {err.max():.3e}"
            fire = st.n_decode > wl.evict_trigger
            rows_before = self._rows(self.twin, s) if (fire and check_rows) else None
            expect = []
            for vec in range(self.n_vec):
                S_g, P_g = self._scores(self.twin, s, vec)          # what the auto context selected on
                assert np.array_equal(P_g, st.pos[vec].astype(np.int32)), f"step {t} seq {s} vec {vec}: positions differ"
                ref_I = st.I[vec]
                e = np.abs(S_g.astype(np.float64) - ref_I)
                self.max_score_rel = max(self.max_score_rel, float(np.max(e / (np.abs(ref_I) + 1e-30))))
                assert np.all(e <= SCORE_RTOL * np.abs(ref_I) + SCORE_ATOL), \
                    f"step {t} seq {s} vec {vec}: score mismatch, worst rel {np.max(e / (np.abs(ref_I) + 1e-30)):.3e}"
                if not fire:
                    expect.append((S_g, P_g, None))
                    continue
                ov = O.overflow(S_g.size, wl.decode_budget)
                E_g = O.select_evict(S_g, P_g, ov, wl.recent_window)               # Eq. 8 on the device's bits
                E_o = O.select_evict(ref_I.astype(np.float32), st.pos[vec], ov, wl.recent_window)
                if not np.array_equal(E_g, E_o):
                    diff = np.setxor1d(E_g, E_o)
                    cut = np.sort(S_g[:S_g.size - wl.recent_window])[ov - 1]
                    slack = 2 * (SCORE_RTOL * abs(float(cut)) + SCORE_ATOL)
                    assert np.all(np.abs(S_g[diff] - cut) <= slack) and \
                        np.all(np.abs(ref_I[diff] - float(cut)) <= 2 * slack), \
                        f"step {t} seq {s} vec {vec}: selections differ beyond a near-tie at the cut"
                    self.near_ties += 1
                st.remove(vec, E_g)
                if ov == 1:
                    self.evicted_slots.append(int(E_g[0]))
                keep = O.survivors(S_g.size, E_g)
                expect.append((S_g[keep], P_g[keep], keep))
            if fire:
                self.evictions += 1
                mkv.mkv_evict(self.twin, L, s)
            for vec in range(self.n_vec):
                S_e, P_e, keep = expect[vec]
                for name, ctx in (("auto", self.auto), ("twin", self.twin)):
                    S_c, P_c = self._scores(ctx, s, vec)
                    assert np.array_equal(P_c, P_e), f"step {t} seq {s} vec {vec}: {name} context retained another set"
                    assert np.array_equal(S_c.view(np.uint32), S_e.view(np.uint32)), \
                        f"step {t} seq {s} vec {vec}: {name} context's scores differ"
            if self.per_head:
                mkv.mkv_set_score_view(self.auto, 0)
                mkv.mkv_set_score_view(self.twin, 0)
            if check_rows:
                rows_a = self._rows(self.auto, s)
                rows_t = self._rows(self.twin, s)
                for g in range(wl.n_kv_heads):
                    vec = g if self.per_head else 0
                    Kd = st.Kd[vec][:, 0 if self.per_head else g]
                    Vd = st.Vd[vec][:, 0 if self.per_head else g]
                    for name, rows in (("auto", rows_a), ("twin", rows_t)):
                        assert np.array_equal(storage_to_values(rows[g][0], wl.dtype).astype(np.float64), Kd), \
                            f"step {t} seq {s} head {g}: {name} K rows differ from the oracle's pool"
                        assert np.array_equal(storage_to_values(rows[g][1], wl.dtype).astype(np.float64), Vd), \
                            f"step {t} seq {s} head {g}: {name} V rows differ from the oracle's pool"
                    if rows_before is not None:
                        keep = expect[vec][2]
                        assert np.array_equal(rows_a[g][0], rows_before[g][0][keep])
                        assert np.array_equal(rows_a[g][1], rows_before[g][1][keep])


class DeferredRun:
    """A context that evicts by itself at the paper's cadence with deferred compaction (the
    token a step evicts only has its slot marked; rows are compacted every few dozen steps),
    followed by the oracle without score injection.

    mkv_read_slots shows the pool slot by slot without compacting it: after a step the selected
    slot is still marked live and keeps its score, so the float32 scores the device selected on are
    all there.  The oracle's selection (Eq. 8) on those bits must name exactly the pending slot;
    the oracle's own float64 run is compared at the score tolerance every step, near-ties between
    the two selections are counted and the oracle then removes the device's token.  Every
    `read_every` steps the ordinary readers are used as well (they compact first): positions,
    scores and rows must be the oracle's pool."""

    def __init__(self, mkv, wl: X.Workload, seqs=None, active=None, per_head: bool = False,
                 decode_capacity: int = 0, split_keys: int = 0, static_scratch: bool = False):
        self.mkv, self.wl, self.per_head = mkv, wl, per_head
        self.seqs = list(range(wl.batch)) if seqs is None else list(seqs)
        self.active = list(self.seqs) if active is None else list(active)
        mode = mkv.MKV_SCORE_PER_KV_HEAD if per_head else mkv.MKV_SCORE_LAYER_MEAN
        self.ctx = make_ctx(mkv, wl, manual_evict=False, split_keys=split_keys, score_mode=mode,
                            decode_capacity=decode_capacity)
        self.n_vec = wl.n_kv_heads if per_head else 1
        self.oracles = {s: oracle_state(wl, "per_kv_head" if per_head else "layer_mean") for s in self.seqs}
        tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
        self.out = torch.zeros((wl.batch, wl.n_q_heads, wl.head_dim), dtype=tdt, device="cuda")
        self.mask = np.zeros(wl.batch, dtype=np.uint8)
        self.mask[self.active] = 1
        self.dt = mkv.MKV_BF16 if wl.dtype == "bf16" else mkv.MKV_F32
        self.step_fn = mkv.mkv_decode_step_static if static_scratch else mkv.mkv_decode_step
        self.max_out_err = self.max_score_rel = 0.0
        self.evictions = self.near_ties = 0
        self.max_holes = 0
        self.evicted_slots = []
        self.cap_seen = 0

    def close(self):
        if self.ctx:
            self.mkv.mkv_destroy(self.ctx)
            self.ctx = None

    def prefill(self):
        wl = self.wl
        for s in self.active:
            k, v = X.prefill_kv(wl, 0, s)
            if k.shape[0]:
                dk, dv = to_device(k, wl.dtype), to_device(v, wl.dtype)
                self.mkv.mkv_prefill_append(self.ctx, 0, s, dk.data_ptr(), dv.data_ptr(), k.shape[0])
            if s in self.oracles:
                self.oracles[s].prefill_append(k, v)
        torch.cuda.synchronize()

    def load_snapshot(self, n_d: int, t_now: int):
        assert not self.per_head
        for s in self.active:
            k, v, sc, pos = X.decode_snapshot(self.wl, 0, s, n_d, t_now)
            dk, dv = to_device(k, self.wl.dtype), to_device(v, self.wl.dtype)
            self.mkv.mkv_load_decode(self.ctx, 0, s, dk.data_ptr(), dv.data_ptr(), sc, pos, t_now)
            if s in self.oracles:
                self.oracles[s].load_decode(k, v, sc, pos, t_now)

    def step(self, t: int, read: bool = False, check_abar: bool = False, active=None):
        """active: the sequences that take this step (default: all of self.active); the others
        pause -- nothing of theirs may change, marked slots and pending selection included."""
        wl, mkv = self.wl, self.mkv
        q, k, v = X.step_batch(wl, 0, t)
        dq, dk, dv = (to_device(a, wl.dtype) for a in (q, k, v))
        mask = self.mask
        if active is not None:
            mask = np.zeros(wl.batch, dtype=np.uint8)
            mask[list(active)] = 1
        self.step_fn(self.ctx, 0, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), self.out.data_ptr(), mask)
        torch.cuda.synchronize()
        got = from_device(self.out)
        rtol, atol = OUT_TOL[wl.dtype]
        cap = 16384
        for s in self.seqs:
            if not mask[s]:
                continue
            st = self.oracles[s]
            ref, abar = st.decode_step(q[s], k[s], v[s], auto_evict=False)
            err = np.abs(got[s] - ref)
            self.max_out_err = max(self.max_out_err, float(err.max()))
            assert np.all(err <= atol + rtol * np.abs(ref)), f"step {t} seq {s}: attention output off by {err.max():.3e}"
            fire = st.n_decode > wl.evict_trigger
            assert st.n_decode <= wl.decode_budget + 1, "the cadence keeps the pool at budget + 1 before an eviction"
            expect = []
            for vec in range(self.n_vec):
                if self.per_head:
                    mkv.mkv_set_score_view(self.ctx, vec)
                S, P, live, pend = mkv.mkv_read_slots(self.ctx, 0, s, cap)
                self.max_holes = max(self.max_holes, int((~live).sum()))
                self.cap_seen = max(self.cap_seen, S.size)
                idx = np.nonzero(live)[0]
                assert np.array_equal(P[idx], st.pos[vec].astype(np.int32)), f"step {t} seq {s} vec {vec}: live positions differ"
                ref_I = st.I[vec]
                e = np.abs(S[idx].astype(np.float64) - ref_I)
                self.max_score_rel = max(self.max_score_rel, float(np.max(e / (np.abs(ref_I) + 1e-30))))
                assert np.all(e <= SCORE_RTOL * np.abs(ref_I) + SCORE_ATOL), \
                    f"step {t} seq {s} vec {vec}: score mismatch, worst rel {np.max(e / (np.abs(ref_I) + 1e-30)):.3e}"
                if check_abar:
                    ga, _ = mkv.mkv_read_probs(self.ctx, 0, s, wl.n_q_heads, cap)
                    a_ref = abar[vec] if self.per_head else abar
                    assert ga.shape == a_ref.shape
                    assert np.all(np.abs(ga - a_ref) <= SCORE_RTOL * a_ref + SCORE_ATOL), f"step {t} seq {s}: abar mismatch"
                if not fire:
                    assert pend == -1, f"step {t} seq {s} vec {vec}: a selection is pending though the pool is within budget"
                    expect.append((S[idx], P[idx]))
                    continue
                E_g = O.select_evict(S[idx], P[idx], 1, wl.recent_window)          # Eq. 8 on the device's bits
                assert pend == idx[E_g[0]], \
                    f"step {t} seq {s} vec {vec}: device selected slot {pend}, the oracle's rule on the same scores slot {idx[E_g[0]]}"
                E_o = O.select_evict(ref_I.astype(np.float32), st.pos[vec], 1, wl.recent_window)
                if not np.array_equal(E_g, E_o):
                    both = np.array([E_g[0], E_o[0]])
                    cut = float(S[idx][E_g[0]])
                    slack = 2 * (SCORE_RTOL * abs(cut) + SCORE_ATOL)
                    assert np.all(np.abs(S[idx][both] - cut) <= slack) and np.all(np.abs(ref_I[both] - cut) <= 2 * slack), \
                        f"step {t} seq {s} vec {vec}: selections differ beyond a near-tie"
                    self.near_ties += 1
                st.remove(vec, E_g)
                self.evicted_slots.append(int(pend))
                keep = O.survivors(idx.size, E_g)
                expect.append((S[idx][keep], P[idx][keep]))
            if fire:
                self.evictions += 1
            if read:
                for vec in range(self.n_vec):
                    if self.per_head:
                        mkv.mkv_set_score_view(self.ctx, vec)
                    gs, gp = mkv.mkv_read_scores(self.ctx, 0, s)      # compacts first
                    assert np.array_equal(gp, expect[vec][1]), f"step {t} seq {s} vec {vec}: compacted positions differ"
                    assert np.array_equal(gs.view(np.uint32), expect[vec][0].view(np.uint32)), \
                        f"step {t} seq {s} vec {vec}: compacted scores differ"
                    S2, P2, live2, pend2 = mkv.mkv_read_slots(self.ctx, 0, s, cap)
                    assert live2.all() and pend2 == -1 and np.array_equal(P2, gp)
                assert mkv.mkv_get_lens(self.ctx, 0, s)[1] == st.n_decode
                for g in range(wl.n_kv_heads):
                    kk, vv = mkv.mkv_read_kv(self.ctx, 0, s, 0, g, wl.head_dim, self.dt)
                    vec = g if self.per_head else 0
                    col = 0 if self.per_head else g
                    assert np.array_equal(storage_to_values(kk, wl.dtype).astype(np.float64), st.Kd[vec][:, col]), \
                        f"step {t} seq {s} head {g}: K rows differ from the oracle's pool"
                    assert np.array_equal(storage_to_values(vv, wl.dtype).astype(np.float64), st.Vd[vec][:, col]), \
                        f"step {t} seq {s} head {g}: V rows differ from the oracle's pool"
            if self.per_head:
                mkv.mkv_set_score_view(self.ctx, 0)
