"""Pins for the RoPE oracle (oracle/rope.py).  None of them re-uses its loop: closed forms from the
rotation matrix, group properties of rotations, the relative-position property that defines RoPE
(RoFormer section 3.2), complex-number arithmetic as an independent route, and the position rule of
the pruned sequence (paper section 3.3, sentence before Eq. 7)."""
import cmath
import math

import numpy as np

from oracle import pruned_positions, rope_gathered, rope_rotate


def _rng(seed):
    return np.random.Generator(np.random.Philox(key=seed))


def test_closed_form_d2_and_d4():
    # D = 2: theta_0 = 1, plain rotation of the plane by p radians (counter-clockwise)
    out = rope_rotate(np.array([[1.0, 0.0]]), [3], 10000.0)
    assert np.allclose(out, [[math.cos(3.0), math.sin(3.0)]], atol=1e-15)
    out = rope_rotate(np.array([[0.0, 1.0]]), [3], 10000.0)
    assert np.allclose(out, [[-math.sin(3.0), math.cos(3.0)]], atol=1e-15)
    # D = 4, base 10000: theta = (1, 10000^(-1/2)) = (1, 0.01).  Half layout pairs (0,2), (1,3).
    x = np.array([[1.0, 0.0, 0.0, 1.0]])
    out = rope_rotate(x, [3], 10000.0)
    want = [math.cos(3.0), -math.sin(0.03), math.sin(3.0), math.cos(0.03)]
    assert np.allclose(out, [want], atol=1e-15)
    # interleaved layout pairs (0,1), (2,3)
    out = rope_rotate(x, [3], 10000.0, interleaved=True)
    want = [math.cos(3.0), math.sin(3.0), -math.sin(0.03), math.cos(0.03)]
    assert np.allclose(out, [want], atol=1e-15)


def test_position_zero_is_identity_and_norms_are_kept():
    x = _rng(1).standard_normal((2, 3, 5, 16))
    assert np.array_equal(rope_rotate(x, [0] * 5, 500000.0), x)
    y = rope_rotate(x, [7, 100, 3, 4095, 1], 500000.0)
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)
    # each pair keeps its own norm (half layout: i, i + D/2)
    assert np.allclose(y[..., :8] ** 2 + y[..., 8:] ** 2, x[..., :8] ** 2 + x[..., 8:] ** 2, rtol=1e-12)


def test_rotations_compose_additively():
    x = _rng(2).standard_normal((4, 8))
    for il in (False, True):
        a = rope_rotate(rope_rotate(x, [5, 6, 7, 8], 10000.0, il), [11, 0, 3, 100], 10000.0, il)
        b = rope_rotate(x, [16, 6, 10, 108], 10000.0, il)
        assert np.allclose(a, b, atol=1e-12)


def test_relative_position_property():
    """<rope(q, m), rope(k, n)> depends on m - n only."""
    g = _rng(3)
    q, k = g.standard_normal((1, 32)), g.standard_normal((1, 32))
    for il in (False, True):
        d0 = (rope_rotate(q, [40], 10000.0, il) @ rope_rotate(k, [33], 10000.0, il).T).item()
        for shift in (1, 17, 1000):
            d1 = (rope_rotate(q, [40 + shift], 10000.0, il) @ rope_rotate(k, [33 + shift], 10000.0, il).T).item()
            assert abs(d0 - d1) < 1e-10
        # and it does change with m - n
        d2 = (rope_rotate(q, [41], 10000.0, il) @ rope_rotate(k, [33], 10000.0, il).T).item()
        assert abs(d0 - d2) > 1e-6


def test_against_complex_multiplication():
    """Independent route: pair (a, b) as the complex number a + ib times exp(i p theta)."""
    g = _rng(4)
    D, base = 12, 500000.0
    x = g.standard_normal((3, D))
    pos = [2, 77, 5000]
    for il in (False, True):
        got = rope_rotate(x, pos, base, il)
        for t in range(3):
            for i in range(D // 2):
                a, b = (2 * i, 2 * i + 1) if il else (i, i + D // 2)
                z = complex(x[t, a], x[t, b]) * cmath.exp(1j * pos[t] * base ** (-2.0 * i / D))
                assert abs(got[t, a] - z.real) < 1e-12 and abs(got[t, b] - z.imag) < 1e-12


def test_pruned_rows_keep_their_original_positions():
    # block of 4 at position 10, suffix of 8 of which rows 0, 1 and the trailing one (7) are kept
    assert pruned_positions(10, 4, [0, 1, 7]).tolist() == [10, 11, 12, 13, 14, 15, 21]
    g = _rng(5)
    xb, xs = g.standard_normal((1, 2, 4, 8)), g.standard_normal((1, 2, 8, 8))
    ob, os_ = rope_gathered(xb, xs, [0, 1, 7], 10, 10000.0)
    # the same rows rotated inside the full, unpruned sequence give the same values
    full = np.concatenate([xb, xs], axis=-2)
    fr = rope_rotate(full, 10 + np.arange(12), 10000.0)
    assert np.allclose(ob, fr[..., :4, :], atol=1e-14)
    assert np.allclose(os_, fr[..., [4, 5, 11], :], atol=1e-14)
    # a wrong rule (ids shifted by the pruning: trailing row at 10+4+2) is detectably different
    wrong = rope_rotate(xs[..., [7], :], [16], 10000.0)
    assert np.abs(wrong - os_[..., 2:, :]).max() > 1e-3
    # empty keep list
    ob2, os2 = rope_gathered(xb, xs, [], 10, 10000.0)
    assert np.array_equal(ob2, ob) and os2.shape == (1, 2, 0, 8)
