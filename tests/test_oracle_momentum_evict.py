"""Pins for the oracle's momentum update (Eq. 5-6), capacity check (Eq. 7), selection (Eq. 8) and
removal (Eq. 9): closed forms, exhaustive subset search, invariants.  CPU only."""
import itertools
import os

import numpy as np
import pytest

from oracle import momentkv_oracle as O

ALPHAS = [float(x) for x in [ln for ln in open(os.path.join(os.path.dirname(__file__), "golden",
                                                           "alpha_grid.txt"))
                             if not ln.startswith("#")][0].split()]


@pytest.mark.parametrize("alpha", ALPHAS)
def test_zero_input_decays_geometrically(alpha):
    I0 = np.array([1.0, 0.25, 3.5])
    I = I0.copy()
    for t in range(1, 40):
        I = O.momentum_update(I, np.zeros(3), alpha)
        assert np.allclose(I, I0 * alpha ** t, rtol=1e-13)


@pytest.mark.parametrize("alpha", ALPHAS)
def test_constant_input_follows_geometric_series_and_reaches_fixed_point(alpha):
    a = np.array([0.02, 0.5])
    I = np.zeros(2)
    for t in range(1, 2000):
        I = O.momentum_update(I, a, alpha)
        if t < 60:
            assert np.allclose(I, a * (1 - alpha ** t) / (1 - alpha), rtol=1e-12)
    assert np.allclose(I, a / (1 - alpha), rtol=1e-10)


def test_momentum_is_linear_in_its_inputs():
    rng = np.random.default_rng(0)
    a, b = rng.random((30, 7)), rng.random((30, 7))
    Ia = Ib = Iab = np.zeros(7)
    for t in range(30):
        Ia = O.momentum_update(Ia, a[t], 0.83)
        Ib = O.momentum_update(Ib, b[t], 0.83)
        Iab = O.momentum_update(Iab, a[t] + b[t], 0.83)
    assert np.allclose(Iab, Ia + Ib, rtol=1e-13)


def test_momentum_weights_old_score_by_alpha_not_new_input():
    # distinguishes alpha*I + a from I + alpha*a and from (1-alpha) blends
    assert O.momentum_update(np.array([2.0]), np.array([0.5]), 0.25)[0] == 2.0 * 0.25 + 0.5


def test_new_token_score_equals_its_own_attention_and_is_positive():
    # Eq. 6: the slot appended in this step holds exactly abar_self after the update
    rng = np.random.default_rng(1)
    st = O.MomentKVState(8, 2, 16, decode_budget=50, alpha=0.9)
    st.prefill_append(rng.standard_normal((20, 2, 16)), rng.standard_normal((20, 2, 16)))
    prev = np.zeros(0)
    for t in range(12):
        _, abar = st.decode_step(rng.standard_normal((8, 16)), rng.standard_normal((2, 16)),
                                 rng.standard_normal((2, 16)))
        assert st.I[0][-1] == abar[-1] > 0
        assert np.allclose(st.I[0][:-1], 0.9 * prev + abar[:-1], rtol=1e-15)
        prev = st.I[0].copy()


def test_overflow_is_clamped_difference():
    assert [O.overflow(n, 5) for n in (0, 4, 5, 6, 9)] == [0, 0, 0, 1, 4]


def _subset_cost(scores, pos, S):
    return (sum(scores[i] for i in S), sorted((scores[i], pos[i]) for i in S))


@pytest.mark.parametrize("seed", range(6))
def test_selection_is_the_minimum_sum_subset_exhaustively(seed):
    # Eq. 8 literally: among all subsets of the candidates with |S| = overflow take the one with
    # minimal score sum; among equal sums the pinned tie rule (older first)
    rng = np.random.default_rng(seed)
    n = 9
    scores = rng.integers(0, 4, n).astype(np.float64) / 4     # many ties on purpose
    pos = np.sort(rng.choice(100, n, replace=False))
    for window in (0, 2):
        cand = range(n - window)
        for k in range(0, n - window + 1):
            best = min(itertools.combinations(cand, k),
                       key=lambda S: _subset_cost(scores, pos, S))
            got = O.select_evict(scores, pos, k, window)
            assert list(got) == sorted(best)


def test_selection_equals_full_sort_with_ties_and_window():
    rng = np.random.default_rng(42)
    for n in (1, 2, 5, 16):
        for _ in range(20):
            scores = rng.integers(0, 3, n).astype(np.float32)
            pos = np.sort(rng.choice(1000, n, replace=False))
            for window in range(0, n + 1):
                for k in range(0, n - window + 1):
                    ranked = sorted(range(n - window), key=lambda i: (scores[i], pos[i]))
                    assert list(O.select_evict(scores, pos, k, window)) == sorted(ranked[:k])


def test_selection_refuses_more_evictions_than_candidates():
    with pytest.raises(ValueError):
        O.select_evict(np.zeros(5), np.arange(5), 4, window=2)


def test_selection_takes_low_scores_not_high():
    scores = np.array([5.0, 0.1, 3.0, 0.2, 4.0])
    assert list(O.select_evict(scores, np.arange(5), 2)) == [1, 3]


def test_eviction_invariants_over_a_run():
    rng = np.random.default_rng(7)
    H, Hkv, D, M, Bd, Te, W = 4, 2, 8, 13, 10, 14, 3
    st = O.MomentKVState(H, Hkv, D, decode_budget=Bd, alpha=0.8, evict_trigger=Te, recent_window=W)
    Kp, Vp = rng.standard_normal((M, Hkv, D)), rng.standard_normal((M, Hkv, D))
    st.prefill_append(Kp, Vp)
    appended = {}
    for t in range(60):
        k, v = rng.standard_normal((Hkv, D)), rng.standard_normal((Hkv, D))
        appended[t] = (k, v)
        before_n = st.n_decode + 1
        st.decode_step(rng.standard_normal((H, D)), k, v)
        if before_n > Te:
            assert st.n_decode == Bd                                   # back to exactly the budget
            assert len(st.last_evicted[0]) == before_n - Bd
            assert set(range(t - W + 1, t + 1)) <= set(st.pos[0].tolist())   # newest W survive
        else:
            assert st.n_decode == before_n                             # never fires at or below T_e
        assert st.n_decode <= Te
        assert st.n_prefill + st.n_decode <= M + Te                    # pool bound
        assert np.all(np.diff(st.pos[0]) > 0)                          # stable order of generation
        for slot, p in enumerate(st.pos[0]):                           # rows travel with their token
            assert np.array_equal(st.Kd[0][slot], appended[p][0])
            assert np.array_equal(st.Vd[0][slot], appended[p][1])
        assert np.array_equal(st.Kp, Kp) and np.array_equal(st.Vp, Vp)  # prefill never touched
    with pytest.raises(RuntimeError):
        st.prefill_append(Kp, Vp)


def test_paper_cadence_evicts_exactly_one_per_step_once_full():
    rng = np.random.default_rng(8)
    st = O.MomentKVState(2, 1, 4, decode_budget=6, alpha=0.5)           # T_e = B_d, W = 0
    for t in range(20):
        st.decode_step(rng.standard_normal((2, 4)), rng.standard_normal((1, 4)),
                       rng.standard_normal((1, 4)))
        assert st.n_decode == min(t + 1, 6)
        if t >= 6:
            assert len(st.last_evicted[0]) == 1


def test_scores_travel_with_survivors():
    st = O.MomentKVState(1, 1, 2, decode_budget=3, alpha=1.0)
    st.load_decode(np.arange(10.0).reshape(5, 1, 2), np.arange(10.0).reshape(5, 1, 2) + 100,
                   scores=[0.5, 0.1, 0.9, 0.1, 0.7], pos=[2, 5, 6, 8, 11], t=12)
    st.evict()
    assert st.pos[0].tolist() == [2, 6, 11]
    assert st.I[0].tolist() == [0.5, 0.9, 0.7]
    assert st.Kd[0][:, 0, 0].tolist() == [0.0, 4.0, 8.0]
    assert st.Vd[0][:, 0, 1].tolist() == [101.0, 105.0, 109.0]
    assert st.last_evicted[0].tolist() == [5, 8]


def test_decision_precision_is_the_callers():
    # two fp64 scores that collapse to one float32: the older token goes first in fp32
    st = O.MomentKVState(1, 1, 2, decode_budget=1, alpha=1.0, decision_dtype=np.float32)
    st.load_decode(np.zeros((2, 1, 2)), np.zeros((2, 1, 2)), scores=[1.0 + 1e-12, 1.0], pos=[3, 4], t=5)
    st.evict()
    assert st.pos[0].tolist() == [4]
    st = O.MomentKVState(1, 1, 2, decode_budget=1, alpha=1.0, decision_dtype=np.float64)
    st.load_decode(np.zeros((2, 1, 2)), np.zeros((2, 1, 2)), scores=[1.0 + 1e-12, 1.0], pos=[3, 4], t=5)
    st.evict()
    assert st.pos[0].tolist() == [3]


def test_remove_takes_exactly_the_given_slots_and_keeps_order():
    # Eq. 9 on a selection handed in: rows, scores and positions of the named slots leave together
    rng = np.random.default_rng(31)
    st = O.MomentKVState(4, 2, 8, decode_budget=5, alpha=0.5, evict_trigger=100)
    for t in range(9):
        st.decode_step(rng.standard_normal((4, 8)), rng.standard_normal((2, 8)), rng.standard_normal((2, 8)))
    K0, V0, I0, p0 = st.Kd[0].copy(), st.Vd[0].copy(), st.I[0].copy(), st.pos[0].copy()
    st.remove(0, np.array([1, 4, 8]))
    keep = [0, 2, 3, 5, 6, 7]
    assert st.pos[0].tolist() == p0[keep].tolist() == keep
    assert np.array_equal(st.I[0], I0[keep])
    assert np.array_equal(st.Kd[0], K0[keep]) and np.array_equal(st.Vd[0], V0[keep])
    assert st.last_evicted[0].tolist() == [1, 4, 8]
    # evict() is remove() of its own selection
    a = O.MomentKVState(4, 2, 8, decode_budget=3, alpha=0.5, evict_trigger=100)
    b = O.MomentKVState(4, 2, 8, decode_budget=3, alpha=0.5, evict_trigger=100)
    for t in range(7):
        x = (rng.standard_normal((4, 8)), rng.standard_normal((2, 8)), rng.standard_normal((2, 8)))
        a.decode_step(*x); b.decode_step(*x)
    a.evict()
    b.remove(0, O.select_evict(b.I[0].astype(np.float32), b.pos[0], 4, 0))
    assert np.array_equal(a.pos[0], b.pos[0]) and np.array_equal(a.I[0], b.I[0])
