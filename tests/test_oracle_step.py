"""Pins for the oracle's whole step (Algorithm 1): with the budget never reached it is plain
attention over the concatenated cache (the paper's "Full Cache" baseline) and the score is the
discounted sum of library-softmax probabilities.  Also the input generators' contracts.  CPU only."""
import math

import numpy as np
import pytest
import torch

from oracle import momentkv_oracle as O
from paper_2605_29873_amd import inputs as X


def _torch_probs(q, K, scale, G):
    # library softmax over the pool, per query head, fp64
    tk = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(G, 0)          # [H,N,D]
    logits = torch.einsum("hd,hnd->hn", torch.from_numpy(q), tk) * scale
    return torch.softmax(logits, dim=-1)


@pytest.mark.parametrize("alpha", [0.2, 0.9, 0.98])
def test_full_cache_run_equals_library_attention_and_discounted_sum(alpha):
    rng = np.random.default_rng(3)
    H, Hkv, D, M, T = 8, 2, 16, 23, 17
    G = H // Hkv
    st = O.MomentKVState(H, Hkv, D, decode_budget=10 ** 6, alpha=alpha)
    Kp, Vp = rng.standard_normal((M, Hkv, D)), rng.standard_normal((M, Hkv, D))
    st.prefill_append(Kp[:10], Vp[:10])
    st.prefill_append(Kp[10:], Vp[10:])                    # appends concatenate in order
    Ks, Vs = [Kp], [Vp]
    expect_I = np.zeros(0)
    for t in range(T):
        q, k, v = rng.standard_normal((H, D)), rng.standard_normal((Hkv, D)), rng.standard_normal((Hkv, D))
        Ks.append(k[None]); Vs.append(v[None])
        Kall, Vall = np.concatenate(Ks), np.concatenate(Vs)
        out, abar = st.decode_step(q, k, v)
        P = _torch_probs(q, Kall, 1 / math.sqrt(D), G)
        tv = torch.from_numpy(Vall).permute(1, 0, 2).repeat_interleave(G, 0)
        ref_out = torch.einsum("hn,hnd->hd", P, tv).numpy()
        assert np.allclose(out, ref_out, rtol=1e-12, atol=1e-13)
        ref_abar = P.mean(dim=0).numpy()[M:]
        assert np.allclose(abar, ref_abar, rtol=1e-12, atol=1e-16)
        expect_I = np.concatenate([alpha * expect_I, [0.0]]) + ref_abar
        assert np.allclose(st.I[0], expect_I, rtol=1e-12)
        assert st.pos[0].tolist() == list(range(t + 1))
    assert st.n_decode == T and st.n_prefill == M


def test_attention_sees_the_cache_before_this_steps_eviction():
    # budget 2, trigger 2: at the third step three decode keys are attended, then one leaves
    rng = np.random.default_rng(4)
    st = O.MomentKVState(2, 1, 4, decode_budget=2, alpha=0.5)
    for t in range(3):
        _, abar = st.decode_step(rng.standard_normal((2, 4)), rng.standard_normal((1, 4)),
                                 rng.standard_normal((1, 4)))
    assert abar.shape == (3,) and st.n_decode == 2
    assert abar.sum() == pytest.approx(1.0, rel=1e-13)     # empty prefill: decode slice is everything


def test_per_kv_head_variant_reduces_to_layer_mean_for_one_kv_head():
    rng = np.random.default_rng(5)
    a = O.MomentKVState(4, 1, 8, decode_budget=5, alpha=0.7, recent_window=1)
    b = O.MomentKVState(4, 1, 8, decode_budget=5, alpha=0.7, recent_window=1, score_mode="per_kv_head")
    for t in range(15):
        q, k, v = rng.standard_normal((4, 8)), rng.standard_normal((1, 8)), rng.standard_normal((1, 8))
        oa, _ = a.decode_step(q, k, v)
        ob, _ = b.decode_step(q, k, v)
        assert np.array_equal(oa, ob)
        assert np.array_equal(a.I[0], b.I[0]) and np.array_equal(a.pos[0], b.pos[0])


def test_heavy_hitters_outlive_ordinary_tokens():
    # the behaviour the method is for: keys aligned with what every query carries keep a high score
    # and survive; shifts scaled so the logit gap is pronounced (the literal cfg1 gap is mild)
    wl = X.scaled(X.workloads()["cfg1"], hh_shift=3.0 * 64 ** 0.25 * 2, q_align=0.5 * 64 ** 0.25 * 2)
    st = O.MomentKVState(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.decode_budget, wl.alpha,
                         wl.evict_trigger, wl.recent_window)
    st.prefill_append(*X.prefill_kv(wl, 0, 0))
    for t in range(wl.steps):
        st.decode_step(*X.step_inputs(wl, 0, 0, t))
    hh = set(X.heavy_hitter_steps(wl, 0, 0).tolist())
    assert hh <= set(st.pos[0].tolist())
    assert st.n_decode <= wl.evict_trigger


# ---------------------------------------------------------------------------------------------
# generators
# ---------------------------------------------------------------------------------------------

def test_generators_are_deterministic_and_storage_exact():
    wl = X.workloads()["cfg2"]
    a = X.step_inputs(wl, 0, 0, 77)
    b = X.step_inputs(wl, 0, 0, 77)
    c = X.step_inputs(wl, 0, 0, 78)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    assert not np.array_equal(a[0], c[0])
    for x in a:
        assert x.dtype == np.float32
        assert np.array_equal(X.bf16_from_bits(X.bf16_bits(x)).reshape(x.shape), x)


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -7, -3.14159], dtype=np.float32)
    r = X.round_bf16(x)
    assert r[0] == 1.0
    assert r[1] == 1.0                      # tie -> even mantissa
    assert r[2] == np.float32(1.0 + 2 ** -6)  # tie -> even mantissa (rounds up)
    assert r[3] == np.float32(1.0 + 2 ** -7)
    assert abs(r[4] - x[4]) <= abs(x[4]) * 2 ** -8
    t = torch.from_numpy(np.random.default_rng(0).standard_normal(4096).astype(np.float32))
    assert np.array_equal(X.round_bf16(t.numpy()), t.to(torch.bfloat16).to(torch.float32).numpy())


def test_workload_table_matches_the_configs():
    w = X.workloads()
    assert (w["cfg1"].evict_trigger, w["cfg1"].capacity) == (72, 73)
    assert (w["cfg2"].evict_trigger, w["cfg2"].capacity) == (1087, 1088)
    assert w["cfg4"].evict_trigger == w["cfg4"].decode_budget == 512
    assert w["cfg4"].group == 7 and w["cfg3"].group == 4
    lens = [X.prefill_len(w["cfg3"], s) for s in range(16)]
    assert min(lens) >= 2048 and max(lens) <= 8192 and len(set(lens)) > 8
    assert len(X.heavy_hitter_steps(w["cfg1"], 0, 0)) == 4
    k, v, s, p = X.decode_snapshot(w["cfg2"], 0, 0, 100, 5000)
    assert k.shape == (100, 8, 128) and np.all(np.diff(p) > 0) and np.all(s >= 0)
