"""Pins for the checker's positional re-encoding of stored keys (paper Sec. 4.1.1, last
paragraph: keys are stored without positional encoding and are encoded at inference by their
global position in the concatenated sequence).  None of these re-types the checker's formula:
they use complex multiplication, group properties and the relative-position invariance that
defines a rotary encoding."""
import numpy as np
import pytest

import oracle

THETA = 1.0e6


def _rand(n, H, D, seed):
    return np.random.default_rng(seed).standard_normal((n, H, D))


def test_equals_complex_rotation():
    """Pair (i, i + D/2) of a key is the complex number k_i + j k_{i+D/2}; encoding multiplies it
    by exp(j pos theta^(-2i/D))."""
    n, H, D = 37, 3, 16
    k = _rand(n, H, D, 1)
    pos = np.random.default_rng(2).integers(0, 50000, size=n)
    got = oracle.reencode_keys(k, pos, THETA)
    z = k[..., :D // 2] + 1j * k[..., D // 2:]
    w = THETA ** (-2.0 * np.arange(D // 2) / D)
    zr = z * np.exp(1j * pos[:, None, None] * w[None, None, :])
    np.testing.assert_allclose(got[..., :D // 2], zr.real, rtol=0, atol=1e-12)
    np.testing.assert_allclose(got[..., D // 2:], zr.imag, rtol=0, atol=1e-12)


def test_head_size_two_is_a_plane_rotation_by_the_position():
    k = np.array([[[1.0, 0.0]], [[0.0, 2.0]], [[3.0, 4.0]]])
    pos = np.array([1, 2, 0])
    got = oracle.reencode_keys(k, pos, 10000.0)
    np.testing.assert_allclose(got[0, 0], [np.cos(1.0), np.sin(1.0)], atol=1e-15)
    np.testing.assert_allclose(got[1, 0], [-2 * np.sin(2.0), 2 * np.cos(2.0)], atol=1e-15)
    np.testing.assert_array_equal(got[2, 0], [3.0, 4.0])          # position 0: identity, exactly


def test_group_properties():
    """Position 0 is the identity; encoding at a then at b (as if position-free again) equals
    encoding at a + b; pair norms are preserved."""
    n, H, D = 20, 2, 32
    k = _rand(n, H, D, 3)
    a = np.random.default_rng(4).integers(0, 3000, size=n)
    b = np.random.default_rng(5).integers(0, 3000, size=n)
    np.testing.assert_array_equal(oracle.reencode_keys(k, np.zeros(n, dtype=int), THETA), k)
    ab = oracle.reencode_keys(oracle.reencode_keys(k, a, THETA), b, THETA)
    np.testing.assert_allclose(ab, oracle.reencode_keys(k, a + b, THETA), atol=1e-11)
    r = oracle.reencode_keys(k, a, THETA)
    np.testing.assert_allclose(r[..., :D // 2] ** 2 + r[..., D // 2:] ** 2,
                               k[..., :D // 2] ** 2 + k[..., D // 2:] ** 2, rtol=1e-12)


def test_scores_depend_on_relative_position_only():
    """<R(m) q, R(n) k> is unchanged when both positions move by the same amount: the property
    that lets a table's keys be encoded wherever the table lands in the prompt."""
    H, D = 2, 64
    q = _rand(9, H, D, 6)
    k = _rand(9, H, D, 7)
    m = np.arange(100, 109)
    nn = np.array([3, 50, 7, 99, 0, 64, 12, 77, 31])
    s0 = np.einsum("thd,thd->th", oracle.reencode_keys(q, m, THETA), oracle.reencode_keys(k, nn, THETA))
    for shift in (1, 17, 4096):
        s1 = np.einsum("thd,thd->th", oracle.reencode_keys(q, m + shift, THETA),
                       oracle.reencode_keys(k, nn + shift, THETA))
        np.testing.assert_allclose(s1, s0, atol=1e-9)
    # and it does change when only one side moves
    s2 = np.einsum("thd,thd->th", oracle.reencode_keys(q, m + 1, THETA), oracle.reencode_keys(k, nn, THETA))
    assert np.abs(s2 - s0).max() > 1e-3


def test_lowest_frequency_pair_turns_slowest():
    """Pair D/2 - 1 has frequency theta^(-(D-2)/D): after `pos` steps it has turned by exactly that
    many radians (checked through the angle of the rotated unit vector)."""
    D = 8
    k = np.zeros((1, 1, D))
    k[0, 0, D // 2 - 1] = 1.0
    pos = 1000
    got = oracle.reencode_keys(k, [pos], 10000.0)
    ang = np.arctan2(got[0, 0, D - 1], got[0, 0, D // 2 - 1])
    assert ang == pytest.approx(pos * 10000.0 ** (-(D - 2) / D), abs=1e-12)


def test_rejects_bad_arguments():
    with pytest.raises(ValueError):
        oracle.reencode_keys(np.zeros((1, 1, 3)), [0], THETA)        # odd head size
    with pytest.raises(ValueError):
        oracle.reencode_keys(np.zeros((1, 1, 4)), [0], 0.0)
