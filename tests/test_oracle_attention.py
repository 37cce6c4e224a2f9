"""Pins for the oracle's attention (Eq. 2) and head mean (Eq. 4): closed forms, invariants and a
library SDPA.  CPU only."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import momentkv_oracle as O


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_uniform_keys_give_equal_attention():
    # every key identical => every logit identical => p = 1/N exactly; Att = mean of V
    H, Hkv, D, N = 8, 2, 16, 37
    q = _rand((H, D), 0)
    K = np.broadcast_to(_rand((1, Hkv, D), 1), (N, Hkv, D)).copy()
    V = _rand((N, Hkv, D), 2)
    A = O.attention_weights(q, K, 1 / math.sqrt(D))
    assert np.allclose(A, 1.0 / N, rtol=0, atol=1e-15)
    out = O.attention_output(A, V)
    G = H // Hkv
    for h in range(H):
        assert np.allclose(out[h], V[:, h // G].mean(axis=0), atol=1e-13)


def test_probabilities_sum_to_one_and_are_positive():
    H, Hkv, D, N = 12, 4, 32, 301
    A = O.attention_weights(_rand((H, D), 3), _rand((N, Hkv, D), 4), 1 / math.sqrt(D))
    assert np.all(A > 0)
    assert np.max(np.abs(A.sum(axis=1) - 1.0)) < 1e-12


def test_dominant_key_takes_everything():
    # one key aligned with the query at logit ~ +60 over the rest: Att ~= its V row
    H, Hkv, D, N = 4, 4, 8, 50
    q = np.zeros((H, D)); q[:, 0] = 1.0
    K = np.zeros((N, Hkv, D)); K[17, :, 0] = 60.0
    V = _rand((N, Hkv, D), 5)
    A = O.attention_weights(q, K, 1.0)
    assert np.allclose(A[:, 17], 1.0, atol=1e-20 + N * math.exp(-60))
    assert np.allclose(O.attention_output(A, V), V[17], atol=1e-20 + 10 * N * math.exp(-60))


def test_two_key_closed_form_and_scale():
    # two keys, logits s0, s1: p0 = 1/(1+exp(s1-s0)) = logistic(s0 - s1); checks sign and scale
    D = 4
    q = np.array([[1.0, 2.0, -1.0, 0.5]])
    K = np.array([[[0.3, -0.2, 0.9, 1.0]], [[-1.0, 0.4, 0.1, 2.0]]])
    scale = 0.37
    s = [scale * sum(q[0, d] * K[j, 0, d] for d in range(D)) for j in range(2)]
    A = O.attention_weights(q, K, scale)
    assert A[0, 0] == pytest.approx(1.0 / (1.0 + math.exp(s[1] - s[0])), rel=1e-14)
    assert A[0, 1] == pytest.approx(1.0 / (1.0 + math.exp(s[0] - s[1])), rel=1e-14)


def test_slot_permutation_permutes_probabilities_and_keeps_output():
    H, Hkv, D, N = 6, 3, 16, 40
    q, K, V = _rand((H, D), 6), _rand((N, Hkv, D), 7), _rand((N, Hkv, D), 8)
    perm = np.random.default_rng(9).permutation(N)
    A = O.attention_weights(q, K, 0.25)
    Ap = O.attention_weights(q, K[perm], 0.25)
    assert np.allclose(Ap, A[:, perm], atol=1e-15)
    assert np.allclose(O.attention_output(Ap, V[perm]), O.attention_output(A, V), atol=1e-13)


@pytest.mark.parametrize("H,Hkv,D,N", [(8, 2, 64, 330), (28, 4, 128, 97), (4, 4, 32, 5), (7, 1, 16, 64)])
def test_matches_library_sdpa_with_repeated_kv_heads(H, Hkv, D, N):
    # a textbook routine: torch's fp64 CPU scaled_dot_product_attention, GQA by repeating KV heads
    q, K, V = _rand((H, D), 10), _rand((N, Hkv, D), 11), _rand((N, Hkv, D), 12)
    G = H // Hkv
    tq = torch.from_numpy(q)[None, :, None, :]                         # [1,H,1,D]
    tk = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(G, 0)[None]   # [1,H,N,D]
    tv = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(G, 0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0, :, 0, :].numpy()
    A = O.attention_weights(q, K, 1 / math.sqrt(D))
    assert np.allclose(O.attention_output(A, V), ref, rtol=1e-12, atol=1e-13)


def test_kv_head_mapping_is_blockwise_not_interleaved():
    # query head h must read KV head h // G: make KV head 1 carry a dominant key only
    H, Hkv, D, N = 4, 2, 4, 6
    q = np.ones((H, D))
    K = np.zeros((N, Hkv, D)); K[2, 1, :] = 20.0
    A = O.attention_weights(q, K, 1.0)
    assert np.allclose(A[0], 1 / N) and np.allclose(A[1], 1 / N)      # heads 0,1 -> KV head 0
    assert A[2, 2] > 0.999 and A[3, 2] > 0.999                        # heads 2,3 -> KV head 1


def test_head_mean_special_cases():
    a = np.random.default_rng(13).random((1, 9))
    assert np.array_equal(O.head_mean(a), a[0])                       # H = 1
    rep = np.repeat(a, 5, axis=0)
    assert np.allclose(O.head_mean(rep), a[0], atol=1e-16)            # replicated heads
    x = np.array([[0.1, 0.2], [0.5, 0.0], [0.3, 0.4]])
    assert np.allclose(O.head_mean(x), [0.3, 0.2])                    # (1/H) * column sums


def test_decode_slice_mass_with_equal_keys():
    # all keys equal: decode slice of the head mean sums to n_d/(M+n_d), not to 1 (no renormalising)
    st = O.MomentKVState(4, 2, 8, decode_budget=100, alpha=0.5)
    M = 11
    row = _rand((1, 2, 8), 14)
    st.prefill_append(np.repeat(row, M, axis=0), _rand((M, 2, 8), 15))
    for t in range(5):
        _, abar = st.decode_step(_rand((4, 8), 16 + t), row[0], _rand((2, 8), 30 + t))
        n_d = t + 1
        assert abar.shape == (n_d,)
        assert np.allclose(abar, 1.0 / (M + n_d), atol=1e-15)
        assert abar.sum() == pytest.approx(n_d / (M + n_d), rel=1e-13)


def test_kv_footprint_arithmetic_from_paper():
    # Introduction: 128 KB per token for Llama-3.1-8B in 16 bit, ~13 GB for 100K tokens
    path = os.path.join(os.path.dirname(__file__), "golden", "kv_footprint.txt")
    row = [ln for ln in open(path) if not ln.startswith("#")][0].split()
    layers, kvh, d, b, kb, tokens, gb = map(int, row)
    per_token = 2 * layers * kvh * d * b
    assert per_token == kb * 1024
    assert per_token // layers == 4096                                # bytes/token/layer used by bench
    assert round(per_token * tokens / 1e9) == gb


@pytest.mark.parametrize("H,Hkv,D,N", [(8, 2, 64, 330), (28, 4, 128, 97), (32, 8, 128, 2048)])
def test_float32_accumulation_switch_stays_close_to_the_library_sdpa(H, Hkv, D, N):
    # the rounding probe: same steps in float32.  Pinned to the same library routine as the fp64
    # path (torch's fp64 SDPA), within what float32 sums over N keys allow, and really float32
    q, K, V = _rand((H, D), 20), _rand((N, Hkv, D), 21), _rand((N, Hkv, D), 22)
    G = H // Hkv
    tq = torch.from_numpy(q)[None, :, None, :]
    tk = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(G, 0)[None]
    tv = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(G, 0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0, :, 0, :].numpy()
    A32 = O.attention_weights(q, K, 1 / math.sqrt(D), accumulate=np.float32)
    out32 = O.attention_output(A32, V, accumulate=np.float32)
    assert A32.dtype == np.float32 and out32.dtype == np.float32
    assert np.allclose(out32, ref, rtol=0, atol=1e-5)
    A64 = O.attention_weights(q, K, 1 / math.sqrt(D))
    assert np.allclose(A32, A64, rtol=1e-4, atol=1e-9)
    assert np.any(A32.astype(np.float64) != A64)          # the switch does change the arithmetic
    assert abs(float(A32.sum(axis=1, dtype=np.float64).max()) - 1.0) < 1e-5


def test_float32_accumulation_reaches_the_state_machine():
    rng = np.random.default_rng(23)
    a = O.MomentKVState(8, 2, 16, decode_budget=6, alpha=0.9)
    b = O.MomentKVState(8, 2, 16, decode_budget=6, alpha=0.9, accumulate=np.float32)
    Kp, Vp = rng.standard_normal((40, 2, 16)), rng.standard_normal((40, 2, 16))
    a.prefill_append(Kp, Vp); b.prefill_append(Kp, Vp)
    for t in range(12):
        q, k, v = rng.standard_normal((8, 16)), rng.standard_normal((2, 16)), rng.standard_normal((2, 16))
        oa, _ = a.decode_step(q, k, v)
        ob, _ = b.decode_step(q, k, v)
        assert ob.dtype == np.float32
        assert np.allclose(oa, ob, rtol=0, atol=1e-5)
    assert np.array_equal(a.pos[0], b.pos[0])
    assert np.allclose(a.I[0], b.I[0], rtol=1e-4)
