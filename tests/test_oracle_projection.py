"""Pins of the oracle's key/value producer (linear maps + rotary encoding, rotate-half layout):
closed forms and properties that fix the sign of the rotation, the pairing i <-> i + D/2 and the
frequency ladder theta^(-2i/D)."""
import numpy as np

from oracle import momentkv_oracle as O


def test_position_zero_is_the_identity():
    k = np.random.default_rng(0).standard_normal((3, 16))
    assert np.array_equal(O.rotary(k, 0, 10000.0), k)


def test_two_dimensional_head_is_a_plane_rotation_by_pos_radians():
    # D = 2: one pair, exponent 0, angle = pos.  Counter-clockwise: (1, 0) -> (cos, sin)
    for pos in (1, 2, 7):
        out = O.rotary(np.array([1.0, 0.0]), pos, 500.0)
        assert np.allclose(out, [np.cos(pos), np.sin(pos)], atol=1e-15)
        out = O.rotary(np.array([0.0, 1.0]), pos, 500.0)
        assert np.allclose(out, [-np.sin(pos), np.cos(pos)], atol=1e-15)


def test_frequency_ladder_and_pairing_on_a_worked_case():
    # D = 4, theta = 10000: pair (0, 2) turns by pos * 1, pair (1, 3) by pos * 10000^(-1/2) = pos / 100
    k = np.array([1.0, 1.0, 0.0, 0.0])
    out = O.rotary(k, 100, 10000.0)
    assert np.allclose(out, [np.cos(100.0), np.cos(1.0), np.sin(100.0), np.sin(1.0)], atol=1e-12)
    assert abs(out[1] - 0.5403023058681398) < 1e-12 and abs(out[3] - 0.8414709848078965) < 1e-12


def test_agrees_with_the_complex_number_form():
    rng = np.random.default_rng(1)
    D, theta, pos = 64, 10000.0, 4321
    k = rng.standard_normal((5, D))
    z = (k[:, :D // 2] + 1j * k[:, D // 2:]) * np.exp(1j * pos * theta ** (-2.0 * np.arange(D // 2) / D))
    assert np.allclose(O.rotary(k, pos, theta), np.concatenate([z.real, z.imag], axis=-1), atol=1e-12)


def test_pair_norms_are_kept_and_dot_products_depend_on_the_position_difference_only():
    rng = np.random.default_rng(2)
    D = 32
    q, k = rng.standard_normal(D), rng.standard_normal(D)
    rq = O.rotary(q, 17, 10000.0)
    assert np.allclose(rq[:D // 2] ** 2 + rq[D // 2:] ** 2, q[:D // 2] ** 2 + q[D // 2:] ** 2)
    d0 = O.rotary(q, 17, 10000.0) @ O.rotary(k, 5, 10000.0)
    d1 = O.rotary(q, 1017, 10000.0) @ O.rotary(k, 1005, 10000.0)
    d2 = O.rotary(q, 12, 10000.0) @ k
    assert abs(d0 - d1) < 1e-9 and abs(d0 - d2) < 1e-9
    assert abs(d0 - O.rotary(q, 18, 10000.0) @ O.rotary(k, 5, 10000.0)) > 1e-3   # and it does depend on it


def test_projection_is_the_row_by_row_dot_product_with_heads_laid_out_blockwise():
    rng = np.random.default_rng(3)
    Hkv, D, hidden = 2, 4, 6
    Wk, Wv = rng.standard_normal((Hkv * D, hidden)), rng.standard_normal((Hkv * D, hidden))
    x = rng.standard_normal(hidden)
    k, v = O.project_kv(x, Wk, Wv, 0, 10000.0, Hkv)          # position 0: no rotation
    for g in range(Hkv):
        for i in range(D):
            assert abs(k[g, i] - sum(Wk[g * D + i, c] * x[c] for c in range(hidden))) < 1e-12
            assert abs(v[g, i] - sum(Wv[g * D + i, c] * x[c] for c in range(hidden))) < 1e-12
    k9, v9 = O.project_kv(x, Wk, Wv, 9, 10000.0, Hkv)        # the value is never rotated
    assert np.array_equal(v9, v) and np.allclose(k9, O.rotary(k, 9, 10000.0))
    assert not np.allclose(k9, k)
