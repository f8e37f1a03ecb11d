"""Pins for the oracle's rotary embedding: hand-computable rotations and the group identities
of 2-D rotations (Section 3.4 uses the rotary embedding as its relative position encoding).
CPU only."""
import numpy as np
import pytest

import oracle


def test_hand_computed_rotations():
    # D = 2: one pair, theta_0 = 1; a quarter turn sends (1, 0) to (0, 1)  (counter-clockwise)
    out = oracle.rope(np.array([1.0, 0.0]), np.pi / 2)
    assert np.allclose(out, [0.0, 1.0], atol=1e-15)
    out = oracle.rope(np.array([0.0, 1.0]), np.pi / 2)
    assert np.allclose(out, [-1.0, 0.0], atol=1e-15)
    # D = 4, base 10000: theta_1 = 10000^(-2/4) = 1/100; dims (1, 3) form the second pair
    out = oracle.rope(np.array([0.0, 1.0, 0.0, 0.0]), 50.0 * np.pi)
    assert np.allclose(out, [0.0, 0.0, 0.0, 1.0], atol=1e-13)
    # first pair (0, 2) turns with theta_0 = 1: pos = pi flips its sign, second pair barely moves
    out = oracle.rope(np.array([1.0, 1.0, 0.0, 0.0]), np.pi)
    assert np.allclose(out, [-1.0, np.cos(np.pi / 100), 0.0, np.sin(np.pi / 100)], atol=1e-15)
    # interleaved style pairs (0, 1) and (2, 3)
    out = oracle.rope(np.array([1.0, 0.0, 1.0, 0.0]), np.pi / 2, style=1)
    assert np.allclose(out, [0.0, 1.0, np.cos(np.pi / 200), np.sin(np.pi / 200)], atol=1e-15)
    # another base: theta_1 = 100^(-1/2) = 1/10
    out = oracle.rope(np.array([0.0, 1.0, 0.0, 0.0]), 5.0 * np.pi, base=100.0)
    assert np.allclose(out, [0.0, 0.0, 0.0, 1.0], atol=1e-14)


def test_frequencies_follow_base_power_law():
    # rotate unit vectors e_i by pos = 1: angle of pair i must be base^(-2i/D)
    D, base = 16, 10000.0
    for i in range(D // 2):
        e = np.zeros(D); e[i] = 1.0
        out = oracle.rope(e, 1.0, base)
        ang = np.arctan2(out[i + D // 2], out[i])
        assert abs(ang - base ** (-2.0 * i / D)) <= 1e-15


@pytest.mark.parametrize("D", [2, 8, 64, 128])
def test_rotation_group_identities(D):
    rng = np.random.default_rng(D)
    x, y = rng.standard_normal(D), rng.standard_normal(D)
    half = D // 2
    assert np.array_equal(oracle.rope(x, 0.0), x)
    for p in (1.0, 17.0, 4095.0):
        r = oracle.rope(x, p)
        assert np.allclose(r[:half] ** 2 + r[half:] ** 2, x[:half] ** 2 + x[half:] ** 2, rtol=1e-13)
        # composition and inverse
        assert np.allclose(oracle.rope(r, 5.0), oracle.rope(x, p + 5.0), atol=1e-11)
        assert np.allclose(oracle.rope(r, -p), x, atol=1e-11)
    # scores depend on the position difference only
    m, n = 1234.0, 77.0
    lhs = oracle.rope(x, m) @ oracle.rope(y, n)
    assert abs(lhs - x @ oracle.rope(y, n - m)) <= 1e-10
    assert abs(lhs - oracle.rope(x, m - n) @ y) <= 1e-10
    # linear in x
    assert np.allclose(oracle.rope(2.0 * x + y, 9.0), 2.0 * oracle.rope(x, 9.0) + oracle.rope(y, 9.0),
                       atol=1e-13)
