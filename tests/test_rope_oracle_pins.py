"""Pins of oracle/zz_rope_oracle.py: what the mathematics of a plane rotation fixes, written
without the oracle's formula (closed forms, invariants, a one-hot probe of the pairing)."""
import numpy as np

from oracle import zz_rope_oracle as R


def angles(seed, rows, half):
    return np.random.default_rng(seed).uniform(-np.pi, np.pi, size=(rows, half))


def test_angle_zero_is_the_identity_and_a_quarter_turn_swaps_the_halves():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((3, 5, 2, 16))
    z = np.zeros((7, 8))
    assert np.array_equal(R.rotate_keys(x, np.arange(5), np.cos(z), np.sin(z)), x)
    q = np.full((7, 8), np.pi / 2)
    y = R.rotate_keys(x, np.arange(5), np.cos(q), np.sin(q))
    assert np.allclose(y[..., :8], -x[..., 8:], atol=1e-15) and np.allclose(y[..., 8:], x[..., :8], atol=1e-15)
    h = np.full((7, 8), np.pi)                                         # half a turn: the negative
    assert np.allclose(R.rotate_keys(x, np.arange(5), np.cos(h), np.sin(h)), -x, atol=1e-15)


def test_pairs_keep_their_norm_and_rotations_compose():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((2, 6, 3, 32))
    a, b = angles(3, 10, 16), angles(4, 10, 16)
    pos = np.array([0, 3, 4, 9, 9, 1])
    y = R.rotate_keys(x, pos, np.cos(a), np.sin(a))
    n_in = x[..., :16] ** 2 + x[..., 16:] ** 2
    n_out = y[..., :16] ** 2 + y[..., 16:] ** 2
    assert np.allclose(n_in, n_out, rtol=1e-13)
    two = R.rotate_keys(y, pos, np.cos(b), np.sin(b))
    once = R.rotate_keys(x, pos, np.cos(a + b), np.sin(a + b))
    assert np.allclose(two, once, atol=1e-13)
    back = R.rotate_keys(y, pos, np.cos(-a), np.sin(-a))
    assert np.allclose(back, x, atol=1e-13)


def test_the_partner_of_element_i_is_i_plus_half_and_the_sign_is_counter_clockwise():
    D, half = 16, 8
    ang = np.zeros((4, half))
    ang[2, 3] = 0.3                                   # only pair 3 of position 2 turns
    for i in range(D):
        x = np.zeros((1, 4, 1, D))
        x[0, :, 0, i] = 1.0
        y = R.rotate_keys(x, np.arange(4), np.cos(ang), np.sin(ang))
        for p in range(4):
            want = np.zeros(D)
            want[i] = 1.0
            if p == 2 and i == 3:
                want[3], want[3 + half] = np.cos(0.3), np.sin(0.3)        # e_lo -> cos e_lo + sin e_hi
            if p == 2 and i == 3 + half:
                want[3], want[3 + half] = -np.sin(0.3), np.cos(0.3)       # e_hi -> -sin e_lo + cos e_hi
            assert np.allclose(y[0, p, 0], want, atol=1e-15), (i, p)


def test_with_angles_linear_in_the_position_a_score_depends_on_the_distance_only():
    rng = np.random.default_rng(5)
    D, half, rows = 64, 32, 200
    freq = 10000.0 ** (-np.arange(half) / half)
    ang = np.arange(rows)[:, None] * freq[None, :]
    q = rng.standard_normal((1, 1, 1, D))
    k = rng.standard_normal((1, 1, 1, D))
    def score(pq, pk):
        a = R.rotate_keys(q, np.array([pq]), np.cos(ang), np.sin(ang))
        b = R.rotate_keys(k, np.array([pk]), np.cos(ang), np.sin(ang))
        return float((a * b).sum())
    assert abs(score(10, 3) - score(107, 100)) < 1e-9
    assert abs(score(50, 50) - float((q * k).sum())) < 1e-9          # distance 0: the plain product
    assert abs(score(10, 3) - score(3, 10)) > 1e-3                   # and the direction matters


def test_per_sequence_positions():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((2, 3, 1, 8))
    a = angles(7, 50, 4)
    pos = np.array([[0, 1, 2], [40, 41, 42]])
    y = R.rotate_keys(x, pos, np.cos(a), np.sin(a))
    for b in range(2):
        assert np.array_equal(y[b:b + 1], R.rotate_keys(x[b:b + 1], pos[b], np.cos(a), np.sin(a)))
