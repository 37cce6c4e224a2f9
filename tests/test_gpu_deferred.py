"""GPU parity of deferred compaction: at the paper's cadence (trigger = budget) on the matrix-core
kernels a step's eviction only marks the token's slot; the attention kernel masks marked slots,
the finishing kernel skips them, and the rows are compacted when the spare slots are used up or a
reader looks.  The results must be those of immediate compaction, i.e. the oracle's: the selection
is checked on the device's own float32 score bits (read slot by slot, without compacting), the
compacted pool against the oracle's pool bit for bit."""
import numpy as np
import pytest
import torch

from oracle import momentkv_oracle as O
from paper_2605_29873_amd import inputs as X
from tests.harness import DeferredRun, FreeRun, Progress, make_ctx, to_device

pytestmark = pytest.mark.gpu

WL = X.workloads()


def _wl(G, Hkv, budget, W, alpha=0.8, M=(60, 260), batch=3, **kw):
    base = dict(batch=batch, n_layers=1, n_q_heads=G * Hkv, n_kv_heads=Hkv, head_dim=128, dtype="bf16",
                prefill_min=M[0], prefill_max=M[1], decode_budget=budget, evict_trigger=budget,
                recent_window=W, alpha=alpha, steps=0, hh_prob=0.02, dip_period=32, dip_len=4)
    base.update(kw)
    return X.Workload("deferred", **base)


@pytest.mark.parametrize("G,Hkv,budget,W,per_head,capacity,read_every", [
    (4, 2, 300, 24, False, 0, 1000),      # default room (37 slots): compactions come from the room running out
    (4, 2, 300, 0, False, 0, 7),          # the paper's W = 0; a reader every 7 steps
    (7, 2, 600, 32, False, 0, 29),        # Qwen grouping, three slot blocks, 64 spare slots
    (4, 2, 300, 24, True, 0, 13),         # one score vector, bitmap and retained set per KV head
    (12, 4, 130, 10, False, 0, 11),       # 48 heads: the general finishing kernel
    (4, 2, 64, 8, False, 64 + 1 + 3, 1000),   # three spare slots only: a compaction every third step
    (2, 1, 40, 5, False, 40 + 1 + 100, 1000), # more spare slots than live tokens
    (7, 2, 1750, 32, False, 0, 211),      # a pool beyond the 1728 keys that this kernel's logit window holds at 7 rows
])
def test_deferred_compaction_free_run_under_the_oracle(mkv, G, Hkv, budget, W, per_head, capacity, read_every):
    wl = _wl(G, Hkv, budget, W)
    dr = DeferredRun(mkv, wl, seqs=[0, 2], active=[0, 2], per_head=per_head, decode_capacity=capacity)
    try:
        dr.prefill()
        steps = budget + 150
        for t in range(steps):
            dr.step(t, read=(t % read_every == read_every - 1 or t == steps - 1), check_abar=(t % 5 == 0))
        assert dr.evictions == 2 * 150
        assert dr.max_holes >= (2 if capacity else 5), "holes never accumulated: the case does not exercise the deferral"
    finally:
        dr.close()
    print(f"deferred G={G} B_d={budget} W={W} per_head={per_head}: {dr.evictions} evictions, {dr.near_ties} near-ties, "
          f"up to {dr.max_holes} holes in {dr.cap_seen} slots, evicted slots {min(dr.evicted_slots)}..{max(dr.evicted_slots)}, "
          f"max |out err| {dr.max_out_err:.2e}, max score rel {dr.max_score_rel:.2e}")


def test_deferred_compaction_with_the_static_scratch_entry_point(mkv):
    wl = _wl(4, 2, 100, 8)
    dr = DeferredRun(mkv, wl, static_scratch=True)
    try:
        dr.prefill()
        for t in range(200):
            dr.step(t, read=(t % 41 == 40 or t == 199))
        assert dr.evictions == 3 * 100 and dr.max_holes >= 6
    finally:
        dr.close()


def test_pool_loaded_above_the_budget_goes_through_the_general_selection(mkv):
    # mkv_load_decode may leave more than budget + 1 tokens after the next append: the step then
    # evicts several at once (general selection on a pool without holes), after which the cadence
    # and the deferral resume
    wl = _wl(4, 2, 100, 8, batch=2)
    dr = DeferredRun(mkv, wl)
    try:
        dr.prefill()
        for t in range(130):                                   # reach the cadence, leave holes behind
            dr.step(t)
        assert dr.max_holes >= 6
        for s in range(wl.batch):
            k, v, sc, pos = X.decode_snapshot(wl, 0, s, 104, 1000)
            dk, dv = to_device(k, wl.dtype), to_device(v, wl.dtype)
            mkv.mkv_load_decode(dr.ctx, 0, s, dk.data_ptr(), dv.data_ptr(), sc, pos, 1000)
            st = dr.oracles[s]
            st.load_decode(k, v, sc, pos, 1000)
        # one step by hand: 105 live tokens -> 5 leave together
        q, k, v = X.step_batch(wl, 0, 1000)
        dq, dk, dv = (to_device(a, wl.dtype) for a in (q, k, v))
        twin = make_ctx(mkv, wl, manual_evict=True, decode_capacity=120)      # for the pre-eviction score bits
        for s in range(wl.batch):
            kp, vp = X.prefill_kv(wl, 0, s)
            a, b = to_device(kp, wl.dtype), to_device(vp, wl.dtype)
            mkv.mkv_prefill_append(twin, 0, s, a.data_ptr(), b.data_ptr(), kp.shape[0])
            ks, vs, sc, pos = X.decode_snapshot(wl, 0, s, 104, 1000)
            a, b = to_device(ks, wl.dtype), to_device(vs, wl.dtype)
            mkv.mkv_load_decode(twin, 0, s, a.data_ptr(), b.data_ptr(), sc, pos, 1000)
        out = torch.zeros_like(dr.out)
        mkv.mkv_decode_step(dr.ctx, 0, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), dr.out.data_ptr())
        mkv.mkv_decode_step(twin, 0, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), out.data_ptr())
        torch.cuda.synchronize()
        assert torch.allclose(out.float(), dr.out.float(), rtol=0, atol=4e-3)
        for s in range(wl.batch):
            st = dr.oracles[s]
            st.decode_step(q[s], k[s], v[s], auto_evict=False)
            S, P = mkv.mkv_read_scores(twin, 0, s)
            E = O.select_evict(S, P, 5, wl.recent_window)
            st.remove(0, E)
            gs, gp = mkv.mkv_read_scores(dr.ctx, 0, s)
            keep = O.survivors(105, E)
            assert np.array_equal(gp, P[keep]) and np.array_equal(gs.view(np.uint32), S[keep].view(np.uint32))
        mkv.mkv_destroy(twin)
        for t in range(1001, 1060):                            # and on with the cadence
            dr.step(t, read=(t == 1059))
    finally:
        dr.close()


def test_explicit_minimal_capacity_keeps_compaction_immediate(mkv):
    # decode_capacity = budget + 1 leaves no spare slot: every eviction shifts the rows at once
    # (the one-row shift after the finishing kernel's selection), and no slot is ever marked
    wl = _wl(4, 2, 50, 4, batch=1)
    fr = FreeRun(mkv, wl, auto_capacity=51)
    try:
        fr.prefill()
        for t in range(90):
            fr.step(t, check_rows=(t % 9 == 0))
            S, P, live, pend = mkv.mkv_read_slots(fr.auto, 0, 0, 64)
            assert live.all() and pend == -1 and S.size == min(t + 1, 50)
        assert fr.evictions == 40
    finally:
        fr.close()


def test_sequences_that_pause_keep_their_marked_slots_and_pending_selection(mkv):
    # sequence 1 takes every third step only, sequence 2 stops for 40 steps in the middle: a paused
    # sequence's bitmap, hole count and pending selection must wait for it unchanged
    wl = _wl(4, 2, 48, 6, batch=3)
    dr = DeferredRun(mkv, wl)
    try:
        dr.prefill()
        for t in range(260):
            act = [0] + ([1] if t % 3 == 0 else []) + ([2] if not 100 <= t < 140 else [])
            dr.step(t, read=(t % 37 == 36), active=act, check_abar=(t % 7 == 0))
        dr.step(260, read=True)
        assert dr.evictions == (261 - 48) + (87 + 1 - 48) + (221 - 48) and dr.max_holes >= 5
    finally:
        dr.close()


def test_manual_calls_on_a_context_with_marked_slots(mkv):
    # mkv_evict (nothing to evict: it only compacts), mkv_write_scores (compacts, then overwrites the
    # scores both sides go on with) and a change of the score view in between the steps
    wl = _wl(4, 2, 40, 4, batch=2)
    dr = DeferredRun(mkv, wl)
    rng = np.random.default_rng(11)
    try:
        dr.prefill()
        for t in range(150):
            dr.step(t, read=(t % 50 == 49))
            if t in (60, 61, 97):
                mkv.mkv_evict(dr.ctx, 0, -1)
                for s in range(wl.batch):
                    S, P, live, pend = mkv.mkv_read_slots(dr.ctx, 0, s, 256)
                    assert live.all() and pend == -1 and S.size == 40
            if t in (75, 120):
                for s in range(wl.batch):
                    inject = (rng.random(40, dtype=np.float32) * 0.01).astype(np.float32)
                    mkv.mkv_write_scores(dr.ctx, 0, s, inject)
                    dr.oracles[s].I[0] = inject.astype(np.float64)
        assert dr.evictions == 2 * 110
    finally:
        dr.close()


def test_rows_from_the_producer_on_a_context_with_deferred_compaction(mkv):
    """mkv_project_append writes the next token's row into the first free slot at the end of the
    pool; with deferred compaction that slot may first have to be made (a compaction when the spare
    slots are used up).  Same producer, same steps on a context that compacts at once: the retained
    tokens must agree and the scores be equal up to the rounding of a different summation order."""
    wl = _wl(4, 2, 40, 4, batch=2, M=(30, 50))
    hidden, theta = 512, 500000.0
    lazy = make_ctx(mkv, wl, manual_evict=False, decode_capacity=0)
    eager = make_ctx(mkv, wl, manual_evict=False, decode_capacity=41)
    try:
        for s in range(wl.batch):
            k, v = X.prefill_kv(wl, 0, s)
            dk, dv = to_device(k, "bf16"), to_device(v, "bf16")
            for c in (lazy, eager):
                mkv.mkv_prefill_append(c, 0, s, dk.data_ptr(), dv.data_ptr(), k.shape[0])
        wk, wv = X.projection_weights(wl, 0, hidden)
        dwk, dwv = to_device(wk, "bf16"), to_device(wv, "bf16")
        out_l = torch.zeros((wl.batch, wl.n_q_heads, 128), dtype=torch.bfloat16, device="cuda")
        out_e = torch.zeros_like(out_l)
        seen_holes = 0
        for t in range(120):
            x = X.step_hidden(wl, 0, t, hidden)
            q, _, _ = X.step_batch(wl, 0, t)
            dx, dq = to_device(x, "bf16"), to_device(q, "bf16")
            dpos = torch.full((wl.batch,), 1000 + t, dtype=torch.int32, device="cuda")
            for c, o in ((lazy, out_l), (eager, out_e)):
                mkv.mkv_project_append(c, 0, dx.data_ptr(), dwk.data_ptr(), dwv.data_ptr(), hidden, dpos.data_ptr(), theta)
                mkv.mkv_decode_step(c, 0, dq.data_ptr(), None, None, o.data_ptr())
            torch.cuda.synchronize()
            assert torch.allclose(out_l.float(), out_e.float(), rtol=2e-2, atol=2e-3)
            S, P, live, pend = mkv.mkv_read_slots(lazy, 0, 0, 256)
            seen_holes = max(seen_holes, int((~live).sum()))
            if t % 23 == 22 or t == 119:
                for s in range(wl.batch):
                    sl, pl = mkv.mkv_read_scores(lazy, 0, s)
                    se, pe = mkv.mkv_read_scores(eager, 0, s)
                    assert np.array_equal(pl, pe), f"step {t} seq {s}: retained tokens differ"
                    assert np.allclose(sl, se, rtol=1e-5, atol=1e-9)
                    for g in range(wl.n_kv_heads):
                        kl, vl = mkv.mkv_read_kv(lazy, 0, s, 0, g, 128, mkv.MKV_BF16)
                        ke, ve = mkv.mkv_read_kv(eager, 0, s, 0, g, 128, mkv.MKV_BF16)
                        assert np.array_equal(kl, ke) and np.array_equal(vl, ve)
        assert seen_holes >= 5
    finally:
        mkv.mkv_destroy(lazy)
        mkv.mkv_destroy(eager)


@pytest.mark.slow
def test_cfg4_qwen_layer_deferred_compaction_from_an_empty_pool(mkv, capsys):
    """The Qwen-shaped layer at full size in the configuration the bench times (default capacity:
    64 spare slots), all 8 sequences active, 1500 steps from an empty pool; sequences 2 and 7 are
    followed, the readers look every 200 steps.  MKV_TEST_CFG4_STEPS=16384 in the environment makes
    it the workload's whole run (about seven minutes, the oracle's)."""
    import os
    wl = WL["cfg4"]
    steps = int(os.environ.get("MKV_TEST_CFG4_STEPS", "1500"))
    dr = DeferredRun(mkv, wl, seqs=[2, 7], active=range(wl.batch))
    alive = Progress(capsys, "cfg4 deferred")
    try:
        dr.prefill()
        for t in range(steps):
            dr.step(t, read=(t % 200 == 199 or t == steps - 1), check_abar=(t % 50 == 0))
            alive.tick(f"step {t} of {steps}, {dr.evictions} evictions")
        assert dr.evictions == 2 * (steps - 512) and dr.max_holes >= 60
    finally:
        dr.close()
    spread = np.percentile(dr.evicted_slots, [0, 25, 50, 75, 100]).astype(int).tolist()
    print(f"cfg4 deferred: {dr.evictions} evictions, {dr.near_ties} near-ties, up to {dr.max_holes} holes, "
          f"evicted-slot quartiles {spread}, max |out err| {dr.max_out_err:.2e}, max score rel {dr.max_score_rel:.2e}")
