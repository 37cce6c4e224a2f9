"""GPU parity of the path a caller runs: contexts that evict by themselves (the library's own
capacity check inside mkv_decode_step), followed by the oracle without score injection.

At the paper's cadence (trigger = budget, Algorithm 1 as printed: one token leaves per step once
the pool is full) the selection of Eq. 8 is the arg-min the finishing kernel takes over the scores
it has just written, merged across its slot blocks, and Eq. 9 is a one-row shift; these cases put
exactly that path under the oracle's selection, run on the device's own float32 score bits."""
import numpy as np
import pytest
import torch

from oracle import momentkv_oracle as O
from paper_2605_29873_amd import inputs as X
from tests.harness import FreeRun, Progress, to_device

pytestmark = pytest.mark.gpu

WL = X.workloads()


def _cadence_wl(G, Hkv, D, dtype, budget, W, alpha=0.8, M=(60, 260), batch=3):
    return X.Workload("cadence", batch=batch, n_layers=1, n_q_heads=G * Hkv, n_kv_heads=Hkv, head_dim=D,
                      dtype=dtype, prefill_min=M[0], prefill_max=M[1], decode_budget=budget,
                      evict_trigger=budget, recent_window=W, alpha=alpha, steps=0, hh_prob=0.02,
                      dip_period=32, dip_len=4)


@pytest.mark.parametrize("G,Hkv,D,dtype,budget,W,per_head,variant", [
    (4, 2, 128, "bf16", 300, 0, False, 0),      # matrix-core kernels, two slot blocks, the paper's W = 0
    (4, 2, 128, "bf16", 300, 24, False, 0),
    (7, 2, 128, "bf16", 600, 32, False, 0),     # Qwen grouping, three slot blocks
    (4, 2, 128, "bf16", 300, 24, True, 0),      # one score vector and one retained set per KV head
    (12, 4, 128, "bf16", 130, 10, False, 0),    # 48 heads: the general finishing kernel, 64-slot blocks
    (4, 2, 64, "f32", 300, 24, False, 0),       # vector-ALU kernels, fp32
    (2, 2, 64, "f32", 300, 0, True, 0),
    (4, 2, 128, "bf16", 300, 24, False, 15),    # vector-ALU kernels on a bf16 x 128 layer
])
def test_paper_cadence_free_run_under_the_oracle(mkv, G, Hkv, D, dtype, budget, W, per_head, variant):
    wl = _cadence_wl(G, Hkv, D, dtype, budget, W)
    fr = FreeRun(mkv, wl, seqs=[0, 2], active=[0, 2], per_head=per_head, attn_variant=variant)
    try:
        fr.prefill()
        steps = budget + 90
        for t in range(steps):
            fr.step(t, check_rows=(t % 37 == 0 or t >= steps - 3))
        assert fr.evictions == 2 * 90
    finally:
        fr.close()
    print(f"cadence G={G} D={D} {dtype} B_d={budget} W={W} per_head={per_head}: {fr.evictions} one-token evictions, "
          f"{fr.near_ties} near-ties, evicted slots {min(fr.evicted_slots)}..{max(fr.evicted_slots)}, "
          f"max |out err| {fr.max_out_err:.2e}, max score rel {fr.max_score_rel:.2e}")


def _planted_scores(n, low_slots, level=5.0):
    sc = np.full(n, level, dtype=np.float32)
    sc[list(low_slots)] = 0.0
    return sc


@pytest.mark.parametrize("G,Hkv,D,dtype,variant", [
    (4, 2, 128, "bf16", 0),     # single-row finishing kernel: 256-slot blocks
    (12, 4, 128, "bf16", 0),    # general finishing kernel: 64-slot blocks
    (4, 2, 64, "f32", 0),       # vector-ALU path
])
@pytest.mark.parametrize("budget,W", [(300, 1), (600, 40), (1500, 7)])
def test_paper_cadence_minimum_planted_in_every_slot_block(mkv, G, Hkv, D, dtype, variant, budget, W):
    """One step from a budget-full pool whose previous scores are 5 everywhere except at planted
    slots (0): the step's arg-min must land there -- first, middle and last slot block, the last
    candidate before the protected window, and exact ties across blocks (zero K rows: logit 0 for
    every head, hence identical probabilities), where the older token goes.  1500 slots: the
    row shift takes two rounds and the score shift two items per thread.  (W >= 1 keeps the
    appended token, whose score is its own attention only, out of the candidates; W = 0 runs in
    the free-run cases.)"""
    n = budget
    last_cand = n - W                      # slot n is the appended token; candidates are [0, n + 1 - W), W >= 1
    cases = [[0], [n // 2], [last_cand], [3, n // 2 + 1], [n // 2, last_cand], [0, 255, 256, last_cand]]
    if W:
        cases.append([n - 1, 5])           # a planted slot inside the window is no candidate
    wl = _cadence_wl(G, Hkv, D, dtype, budget, W, batch=len(cases), M=(30, 90))
    fr = FreeRun(mkv, wl, attn_variant=variant)
    try:
        fr.prefill()
        t_now = 4 * n
        fr.load_snapshot(n, t_now, scores={s: _planted_scores(n, c) for s, c in enumerate(cases)})
        # exact ties: the planted slots of a case with several get all-zero K rows
        for s, c in enumerate(cases):
            if len(c) < 2:
                continue
            k, v, _, pos = X.decode_snapshot(wl, 0, s, n, t_now)
            k[c] = 0.0
            dk, dv = to_device(k, dtype), to_device(v, dtype)
            for ctx in (fr.auto, fr.twin):
                mkv.mkv_load_decode(ctx, 0, s, dk.data_ptr(), dv.data_ptr(), _planted_scores(n, c), pos, t_now)
            fr.oracles[s].load_decode(k, v, _planted_scores(n, c), pos, t_now)
        fr.step(t_now, check_rows=True)
        assert fr.evictions == len(cases)
        for s, c in enumerate(cases):
            cand = [j for j in c if j < n + 1 - W]
            assert fr.evicted_slots[s] == min(cand), f"case {c}: slot {fr.evicted_slots[s]} left"
        fr.step(t_now + 1, check_rows=True)        # and the pool is consistent for the next step
    finally:
        fr.close()


def test_tied_minimum_is_an_exact_tie_on_the_device(mkv):
    # the planted-tie cases above mean something only if the tie is exact in the device's scores
    from tests.harness import make_ctx
    wl = _cadence_wl(4, 2, 128, "bf16", 300, 0, batch=1, M=(50, 50))
    ctx = make_ctx(mkv, wl, manual_evict=True)
    try:
        k, v = X.prefill_kv(wl, 0, 0)
        dk, dv = to_device(k, "bf16"), to_device(v, "bf16")
        mkv.mkv_prefill_append(ctx, 0, 0, dk.data_ptr(), dv.data_ptr(), k.shape[0])
        n, c = 300, [7, 270]
        k, v, _, pos = X.decode_snapshot(wl, 0, 0, n, 4 * n)
        k[c] = 0.0
        dk, dv = to_device(k, "bf16"), to_device(v, "bf16")
        mkv.mkv_load_decode(ctx, 0, 0, dk.data_ptr(), dv.data_ptr(), _planted_scores(n, c), pos, 4 * n)
        q, kn, vn = (to_device(a, "bf16") for a in X.step_batch(wl, 0, 4 * n))
        out = torch.zeros((1, wl.n_q_heads, 128), dtype=torch.bfloat16, device="cuda")
        mkv.mkv_decode_step(ctx, 0, q.data_ptr(), kn.data_ptr(), vn.data_ptr(), out.data_ptr())
        sc, _ = mkv.mkv_read_scores(ctx, 0, 0)
        assert sc[7] == sc[270] and 0 < sc[7] < sc[8]
    finally:
        mkv.mkv_destroy(ctx)


@pytest.mark.parametrize("name,changes,steps", [
    ("cfg1", {}, 200),                                    # fp32, evicts 9 whenever the pool exceeds 72
    ("cfg2", dict(prefill_min=500, prefill_max=500, decode_budget=128, evict_trigger=128 + 31,
                  recent_window=16, burst_period=96, burst_keys=12, burst_len=8), 400),
])
def test_chunked_auto_eviction_free_run_under_the_oracle(mkv, name, changes, steps):
    # the library's own trigger with chunked eviction (selection kernel + row mover launched by
    # mkv_decode_step), never stopping at a near-tie
    wl = X.scaled(WL[name], **changes)
    fr = FreeRun(mkv, wl)
    try:
        fr.prefill()
        for t in range(steps):
            fr.step(t, check_rows=(t % 50 == 0))
        chunk = wl.evict_trigger - wl.decode_budget + 1
        assert fr.evictions == (steps - wl.decode_budget) // chunk
    finally:
        fr.close()
    print(f"{name} free run: {fr.evictions} evictions, {fr.near_ties} near-ties, max |out err| {fr.max_out_err:.2e}, "
          f"max score rel {fr.max_score_rel:.2e}")


@pytest.mark.slow
def test_cfg4_qwen_layer_from_an_empty_pool_2048_steps(mkv, capsys):
    """The Qwen-shaped layer at full size (8 sequences x 8192 prompt tokens, 28/4 heads, budget 512,
    window 32, alpha 0.8), all sequences active, from an empty decode pool through 2048 steps:
    1536 one-token evictions per sequence through the finishing kernel's arg-min and the one-row
    shift, with the query dips (8 of every 128 steps) the workload was drawn with.  Sequence 5 is
    followed from step 0; four windows of 48 steps start from the device's own mid-run state of
    other sequences (pools and scores read back through the ABI)."""
    wl = WL["cfg4"]
    fr = FreeRun(mkv, wl, seqs=[5], active=range(wl.batch), device_fill_unfollowed=True)
    windows = {560: 1, 900: 6, 1400: 3, 1900: 0}        # first step of the window -> sequence
    closing = {}
    alive = Progress(capsys, "cfg4 free run")
    try:
        fr.prefill()
        for t in range(2048):
            if t in windows:
                fr.follow_from_gpu(windows[t])
                closing[t + 48] = windows[t]
            if t in closing:
                fr.unfollow(closing[t])
            fr.step(t, check_rows=(t % 256 == 0 or t in closing or t == 2047))
            alive.tick(f"step {t} of 2048, {fr.evictions} evictions")
        assert fr.evictions == (2048 - 512) + 4 * 48
    finally:
        fr.close()
    spread = np.percentile(fr.evicted_slots, [0, 25, 50, 75, 100]).astype(int).tolist()
    print(f"cfg4 free run: {fr.evictions} one-token evictions, {fr.near_ties} near-ties, evicted-slot quartiles {spread}, "
          f"max |out err| {fr.max_out_err:.2e}, max score rel {fr.max_score_rel:.2e}")
