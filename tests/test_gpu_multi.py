"""GPU parity of the multi-query step (q_len tokens per call on the matrix cores) against the CPU
oracle taking the same tokens one Algorithm-1 step at a time, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2605_29873_amd import inputs as X
from tests.harness import Lockstep, make_ctx

pytestmark = pytest.mark.gpu

WL = X.workloads()


def _chunks(ls, tokens, q_lens, t0=0, **kw):
    """Feeds `tokens` tokens in calls of the given lengths (cycled)."""
    try:
        t, i = t0, 0
        while t < t0 + tokens:
            n = q_lens[i % len(q_lens)]
            if n == 0:
                ls.step(t, **kw)
                t += 1
            else:
                ls.step_multi(t, n, **kw)
                t += n
            i += 1
        for s in ls.seqs:
            ls.check_prefill_untouched(s)
    finally:
        ls.close()


def _small(G, Hkv, **kw):
    base = dict(batch=2, n_layers=1, n_q_heads=G * Hkv, n_kv_heads=Hkv, head_dim=128, dtype="bf16",
                prefill_min=50, prefill_max=333, decode_budget=20, evict_trigger=27, recent_window=3,
                alpha=0.65, steps=0, hh_prob=0.05)
    base.update(kw)
    return X.Workload("multi", **base)


@pytest.mark.parametrize("G,Hkv,Q", [
    (4, 2, 4),     # Llama grouping: 16 rows, one pass
    (4, 2, 1),     # single query on the matrix-core kernel: 4 of 16 rows used
    (7, 1, 2),     # Qwen grouping: 14 rows
    (7, 2, 1),
    (8, 1, 2),     # exactly 16 rows
    (1, 2, 16),    # no grouping, 16 query positions
    (2, 2, 8),
    (4, 1, 8),     # 32 rows: two row blocks, one pass
    (3, 2, 5),     # 15 rows
    (12, 1, 3),    # 36 rows: ten heads per pass in two row blocks, two passes, the last with two heads
    (7, 1, 4),     # Qwen grouping, 28 rows in two row blocks
    (4, 2, 16),    # two heads per pass, two passes of 32 rows
    (4, 1, 5),     # 20 rows: the second row block has four
    (20, 1, 1),    # single query, more heads per KV head than one row block holds
    (12, 4, 1),    # 48 heads: the finishing kernel's general instantiation with one query row
    (6, 8, 2),     # 48 heads, two rows
])
@pytest.mark.parametrize("split_keys", [0, 64])
def test_chunked_decode_matches_token_by_token_oracle(mkv, G, Hkv, Q, split_keys):
    wl = _small(G, Hkv)
    ls = Lockstep(mkv, wl, split_keys=split_keys, max_q_len=Q)
    ls.prefill()
    _chunks(ls, 70 if Q > 1 else 40, [Q], check_abar=True)
    assert ls.evictions >= 4


def test_call_lengths_may_vary_and_mix_with_single_steps(mkv):
    # 0 = the single-query entry point; the pool crosses the trigger at different offsets
    wl = _small(4, 2, decode_budget=33, evict_trigger=40, recent_window=0, alpha=0.9)
    ls = Lockstep(mkv, wl, split_keys=64, max_q_len=7)
    ls.prefill()
    _chunks(ls, 150, [3, 0, 7, 1, 0, 0, 5, 2], check_abar=True)
    assert ls.evictions >= 10


def test_empty_prefill_and_empty_pool(mkv):
    # the first call sees nothing but its own tokens: row i attends to tokens 0..i only
    wl = _small(4, 1, prefill_min=0, prefill_max=0, batch=1)
    ls = Lockstep(mkv, wl, max_q_len=4)
    ls.prefill()
    _chunks(ls, 48, [4], check_abar=True)


@pytest.mark.parametrize("G,Q,n_d", [(4, 4, 2400), (7, 2, 2700), (4, 8, 1300), (4, 16, 1300), (4, 4, 1000)])
def test_decode_pool_longer_than_one_logit_window(mkv, G, Q, n_d):
    # the kernel stages decode logits in LDS windows of 36864 floats: 2304 keys at 16 rows, 2624 at
    # 14, 1152 at 32 rows (two row blocks; sixteen query rows take two passes of 32); the last case
    # fits one window
    wl = _small(G, 2, decode_budget=n_d, evict_trigger=n_d + 5, recent_window=5, alpha=0.9, hh_prob=0.02)
    for split in (0, 64):
        ls = Lockstep(mkv, wl, split_keys=split, max_q_len=Q)
        ls.prefill()
        ls.load_snapshot(n_d - 1, 3 * n_d)
        _chunks(ls, 4 * Q, [Q], t0=3 * n_d, check_abar=True)
        assert ls.evictions >= 2


def test_cfg3_ragged_batch_full_size_sampled_chunks_of_4(mkv):
    # all 16 ragged sequences in the automatic launch configuration, three followed by the oracle
    wl = WL["cfg3"]
    ls = Lockstep(mkv, wl, seqs=[0, 7, 13], active=range(wl.batch), max_q_len=4)
    ls.prefill()
    ls.load_snapshot(wl.evict_trigger - 6, 5000)
    _chunks(ls, 12, [4], t0=5000)
    assert ls.evictions == 3
    print(f"cfg3 q_len 4: max |out err| {ls.max_out_err:.2e}, max score rel {ls.max_score_rel:.2e}")


def test_cfg4_qwen_single_query_on_matrix_cores(mkv):
    wl = WL["cfg4"]
    ls = Lockstep(mkv, wl, seqs=[2, 5], active=range(wl.batch), max_q_len=2)
    ls.prefill()
    ls.load_snapshot(wl.decode_budget - 2, 9000)
    _chunks(ls, 8, [1, 2], t0=9000)
    assert ls.evictions >= 2 * 4


def test_inactive_sequences_are_left_alone(mkv):
    wl = _small(4, 2, batch=3)
    ls = Lockstep(mkv, wl, seqs=[0, 2], max_q_len=4)
    ls.prefill()
    _chunks(ls, 24, [4])
    ctx = make_ctx(mkv, wl, manual_evict=True, max_q_len=4)
    try:
        assert mkv.mkv_get_lens(ctx, 0, 1) == (0, 0, 0)
    finally:
        mkv.mkv_destroy(ctx)


def test_argument_and_state_errors(mkv):
    wl = _small(4, 2)
    z = torch.zeros(2 * 16 * 8 * 128, dtype=torch.bfloat16, device="cuda")
    ctx = make_ctx(mkv, wl, manual_evict=True)            # max_q_len = 0
    try:
        with pytest.raises(mkv.MkvError) as e:
            mkv.mkv_decode_step_multi(ctx, 0, 2, z.data_ptr(), z.data_ptr(), z.data_ptr(), z.data_ptr())
        assert e.value.code == mkv.MKV_ERR_STATE
    finally:
        mkv.mkv_destroy(ctx)
    ctx = make_ctx(mkv, wl, manual_evict=True, max_q_len=4)
    try:
        for bad in (0, 5, -1):
            with pytest.raises(mkv.MkvError) as e:
                mkv.mkv_decode_step_multi(ctx, 0, bad, z.data_ptr(), z.data_ptr(), z.data_ptr(), z.data_ptr())
            assert e.value.code == mkv.MKV_ERR_ARG
        # capacity = 28 + 3 slots: seven calls of 4 fit, the eighth does not (no eviction here)
        for _ in range(7):
            mkv.mkv_decode_step_multi(ctx, 0, 4, z.data_ptr(), z.data_ptr(), z.data_ptr(), z.data_ptr())
        with pytest.raises(mkv.MkvError) as e:
            mkv.mkv_decode_step_multi(ctx, 0, 4, z.data_ptr(), z.data_ptr(), z.data_ptr(), z.data_ptr())
        assert e.value.code == mkv.MKV_ERR_CAPACITY
        assert mkv.mkv_get_lens(ctx, 0, 0)[1] == 28
    finally:
        mkv.mkv_destroy(ctx)
    with pytest.raises(mkv.MkvError):
        make_ctx(mkv, X.scaled(wl, dtype="f32"), manual_evict=True, max_q_len=2)
    with pytest.raises(mkv.MkvError):
        make_ctx(mkv, X.scaled(wl, head_dim=64), manual_evict=True, max_q_len=2)


def test_batch_beyond_the_inline_length_table(mkv):
    wl = _small(4, 2, batch=40, prefill_min=0, prefill_max=120)
    ls = Lockstep(mkv, wl, seqs=[0, 31, 32, 39], active=range(wl.batch), max_q_len=3)
    ls.prefill()
    _chunks(ls, 36, [3, 1, 2], check_abar=True)
    assert ls.evictions >= 4 * 2


@pytest.mark.parametrize("i", range(24))
def test_random_shapes_and_call_lengths(mkv, i):
    # seeded sweep over head groupings (one and two row blocks per pass, several passes), budgets,
    # chunks, windows and ragged prefills, with calls of mixed lengths; 64-key work-group ranges
    # cut the units into many pieces at odd places
    rng = np.random.default_rng(9000 + i)
    G = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12]))
    Hkv = int(rng.choice([1, 2, 4]))
    Q = int(rng.choice([2, 3, 4, 5, 8, 11, 16]))
    budget = int(rng.integers(Q, 90))
    chunk = int(rng.integers(1, 40))
    W = int(rng.integers(0, budget + 1)) if rng.random() < 0.5 else 0
    M = int(rng.choice([0, 1, 63, 64, 65, 200, 777]))
    wl = X.Workload(f"randmq{i}", batch=int(rng.integers(1, 5)), n_layers=1, n_q_heads=G * Hkv, n_kv_heads=Hkv,
                    head_dim=128, dtype="bf16", prefill_min=M // 2, prefill_max=M, decode_budget=budget,
                    evict_trigger=budget + chunk - 1, recent_window=W, alpha=float(rng.choice([0.2, 0.8, 0.98])),
                    steps=0, hh_prob=0.05, seed=3000 + i)
    q_lens = [int(x) for x in rng.integers(0, Q + 1, size=6)] + [Q]
    ls = Lockstep(mkv, wl, split_keys=int(rng.choice([0, 64, 128])), max_q_len=Q)
    ls.prefill()
    tokens = min(wl.evict_trigger + 2 * chunk + Q, 150)
    _chunks(ls, tokens, q_lens, check_abar=True)
