"""Pins of the oracle's projection + rotary embedding (lckv_oracle_project; Section 2.1: the step either side of
the attention) against things other than itself: a library matrix product, the rotation written as a complex
multiplication, closed forms at D=2 and D=4, and the properties a rotary embedding must have (identity at
position 0, norms kept, additivity of positions, scores that depend on the distance only)."""
import math

import numpy as np
import pytest

from oracle import lckv_oracle as orc


def rng(seed):
    return np.random.default_rng(seed)


def rope_only(v, pos, base=10000.0):
    """Rotary embedding of v [B][H][D] alone: the projection with identity weights."""
    B, H, D = v.shape
    return orc.project(v.reshape(B, H * D), np.eye(H * D, dtype=np.float32), H, pos=pos, rope_base=base)


@pytest.mark.parametrize("B,hidden,H,D", [(1, 1, 1, 2), (3, 8, 2, 4), (5, 96, 3, 64), (2, 300, 2, 128)])
def test_projection_is_the_library_matrix_product(B, hidden, H, D):
    r = rng(B * 1000 + hidden)
    x = r.standard_normal((B, hidden)).astype(np.float32)
    W = r.standard_normal((H * D, hidden)).astype(np.float32)
    got = orc.project(x, W, H)                                           # values: no rotation
    want = x.astype(np.float64) @ W.astype(np.float64).T
    np.testing.assert_allclose(got.reshape(B, H * D), want, rtol=1e-12, atol=1e-12)
    # a weight matrix that is not square catches a transposed operand; single hot entries catch swapped indices
    W1 = np.zeros((H * D, hidden), np.float32)
    W1[H * D - 1, 0] = 2.0
    y = orc.project(x, W1, H).reshape(B, H * D)
    assert np.all(y[:, :-1] == 0) and np.allclose(y[:, -1], 2.0 * x[:, 0].astype(np.float64))


def test_rotation_at_position_zero_is_the_identity_and_values_are_never_rotated():
    r = rng(1)
    x = r.standard_normal((4, 32)).astype(np.float32)
    W = r.standard_normal((2 * 16, 32)).astype(np.float32)
    plain = orc.project(x, W, 2)
    assert np.array_equal(orc.project(x, W, 2, pos=[0, 0, 0, 0]), plain)
    moved = orc.project(x, W, 2, pos=[0, 3, 0, 9])
    assert np.array_equal(moved[0], plain[0]) and np.array_equal(moved[2], plain[2])
    assert not np.allclose(moved[1], plain[1]) and not np.allclose(moved[3], plain[3])   # per-sequence positions


def test_two_channels_rotate_by_the_position_in_radians():
    # D = 2: one pair, frequency base^0 = 1 whatever the base
    for pos in (1, 2, 7, 1000):
        for base in (10000.0, 3.0):
            got = rope_only(np.array([[[1.0, 0.0]], [[0.0, 1.0]]], np.float32), [pos, pos], base)
            assert got[0, 0] == pytest.approx([math.cos(pos), math.sin(pos)], abs=1e-12)
            assert got[1, 0] == pytest.approx([-math.sin(pos), math.cos(pos)], abs=1e-12)


def test_four_channels_pairs_are_half_a_head_apart_and_the_second_turns_a_hundred_times_slower():
    # D = 4, base 10000: frequencies 1 and 10000^(-2/4) = 1/100; channel 1 is paired with channel 3, not with 0 or 2
    pos = 50
    e = np.zeros((4, 1, 4), np.float32)
    for i in range(4):
        e[i, 0, i] = 1.0
    got = rope_only(e, [pos] * 4)[:, 0]
    c0, s0, c1, s1 = math.cos(pos), math.sin(pos), math.cos(pos / 100), math.sin(pos / 100)
    want = np.array([[c0, 0, s0, 0], [0, c1, 0, s1], [-s0, 0, c0, 0], [0, -s1, 0, c1]])
    np.testing.assert_allclose(got, want, atol=1e-12)


@pytest.mark.parametrize("D,base", [(8, 10000.0), (64, 10000.0), (128, 500000.0)])
def test_rotation_equals_a_complex_multiplication(D, base):
    # (lo + i*hi) * exp(i * pos * base^(-2k/D)) for the pairs (k, k + D/2), in numpy's complex arithmetic
    r = rng(D)
    v = r.standard_normal((3, 2, D)).astype(np.float32)
    pos = np.array([0, 5, 4097])
    got = rope_only(v, pos, base)
    z = v[..., :D // 2].astype(np.float64) + 1j * v[..., D // 2:].astype(np.float64)
    freq = base ** (-np.arange(D // 2) * 2.0 / D)
    z = z * np.exp(1j * pos[:, None, None] * freq[None, None, :])
    np.testing.assert_allclose(got[..., :D // 2], z.real, atol=1e-9)
    np.testing.assert_allclose(got[..., D // 2:], z.imag, atol=1e-9)


def test_norms_are_kept_pair_by_pair_and_positions_add_up():
    r = rng(3)
    D = 32
    v = r.standard_normal((2, 3, D)).astype(np.float32)
    a = rope_only(v, [11, 2000])
    pair = lambda t: t[..., :D // 2] ** 2 + t[..., D // 2:] ** 2
    np.testing.assert_allclose(pair(a), pair(v.astype(np.float64)), rtol=1e-12)
    # rotating by 11 then by 6 is rotating by 17 (the second application sees float32-rounded input: 1e-6)
    b = rope_only(a.astype(np.float32), [6, 6])
    np.testing.assert_allclose(b, rope_only(v, [17, 2006]), atol=2e-6)


def test_scores_depend_on_the_distance_only():
    r = rng(4)
    D = 64
    q = r.standard_normal((1, 1, D)).astype(np.float32)
    k = r.standard_normal((1, 1, D)).astype(np.float32)
    dots = []
    for m, n in [(9, 4), (105, 100), (5, 0), (4101, 4096)]:
        dots.append(float((rope_only(q, [m]) * rope_only(k, [n])).sum()))
    assert max(dots) - min(dots) < 1e-9
    other = float((rope_only(q, [9]) * rope_only(k, [3])).sum())
    assert abs(other - dots[0]) > 1e-3


def test_heads_are_rotated_independently_and_linearly():
    r = rng(5)
    H, D, hidden = 3, 16, 40
    x1 = r.standard_normal((2, hidden)).astype(np.float32)
    x2 = r.standard_normal((2, hidden)).astype(np.float32)
    W = r.standard_normal((H * D, hidden)).astype(np.float32)
    pos = [3, 77]
    y = orc.project(x1, W, H, pos=pos)
    for h in range(H):                                       # one head alone gives the same numbers
        np.testing.assert_allclose(orc.project(x1, W[h * D:(h + 1) * D], 1, pos=pos)[:, 0], y[:, h], rtol=1e-12)
    s = orc.project((x1 + x2), W, H, pos=pos)
    np.testing.assert_allclose(s, y + orc.project(x2, W, H, pos=pos), atol=1e-5)


def test_bad_arguments():
    x = np.zeros((1, 4), np.float32)
    W = np.zeros((6, 4), np.float32)
    with pytest.raises(ValueError):
        orc.project(x, W, 2)                                 # D = 3 is odd
    with pytest.raises(ValueError):
        orc.project(x, np.zeros((4, 4), np.float32), 1, pos=[1], rope_base=0.0)
