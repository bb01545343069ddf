"""Pins of the rotary-embedding oracle (oracle/rope.py): a hand-worked example, the
complex-number form computed by an independent routine, and the properties that define
the method (identity at position 0, norm per pair, additivity of positions, scores that
depend on relative position only)."""
import os

import numpy as np
import pytest

from oracle.rope import pass_positions, rope_rotate

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "rope_example.txt")


def test_hand_worked_example():
    x, pos = None, None
    n = 0
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        vals = [float(v) for v in vals]
        if key == "x":
            x = np.array(vals).reshape(1, 1, -1)
        elif key == "pos":
            pos = np.array(vals)
        else:
            got = rope_rotate(x, pos)[0, 0]
            assert np.allclose(got, vals, rtol=0, atol=2e-15), (got, vals)
            n += 1
    assert n == 2


def test_equals_complex_multiplication():
    rng = np.random.default_rng(3)
    n, H, D = 7, 3, 16
    x = rng.standard_normal((n, H, D))
    pos = rng.integers(0, 70000, n)
    base = 500000.0
    theta = base ** (-np.arange(D // 2) * 2.0 / D)
    z = (x[..., : D // 2] + 1j * x[..., D // 2:]) * np.exp(1j * pos[:, None, None] * theta[None, None, :])
    want = np.concatenate([z.real, z.imag], axis=-1)
    assert np.allclose(rope_rotate(x, pos, base), want, rtol=1e-12, atol=1e-12)


def test_defining_properties():
    rng = np.random.default_rng(4)
    n, H, D = 5, 2, 8
    q = rng.standard_normal((n, H, D))
    k = rng.standard_normal((n, H, D))
    zero = np.zeros(n)
    assert np.array_equal(rope_rotate(q, zero), q)
    pa, pb = rng.integers(0, 5000, n), rng.integers(0, 5000, n)
    # positions add
    assert np.allclose(rope_rotate(rope_rotate(q, pa), pb), rope_rotate(q, pa + pb), atol=1e-11)
    # each (i, i + D/2) pair keeps its length
    r = rope_rotate(q, pa)
    assert np.allclose(r[..., : D // 2] ** 2 + r[..., D // 2:] ** 2, q[..., : D // 2] ** 2 + q[..., D // 2:] ** 2, atol=1e-12)
    # a score depends on the difference of the two positions only
    s1 = np.einsum("nhd,nhd->nh", rope_rotate(q, pa), rope_rotate(k, pb))
    shift = 1234
    s2 = np.einsum("nhd,nhd->nh", rope_rotate(q, pa + shift), rope_rotate(k, pb + shift))
    s3 = np.einsum("nhd,nhd->nh", rope_rotate(q, pa - pb), k)
    assert np.allclose(s1, s2, atol=1e-9) and np.allclose(s1, s3, atol=1e-9)
    # a wrong pairing (neighbours instead of halves) would break this one: rotating the unit vector e_0
    # by a quarter turn of frequency 0 must land on e_{D/2}
    e = np.zeros((1, 1, D))
    e[0, 0, 0] = 1.0
    quarter = rope_rotate(e, np.array([np.pi / 2]))
    assert quarter[0, 0, D // 2] == pytest.approx(1.0) and abs(quarter[0, 0, 1]) < 1e-12


def test_pass_positions():
    assert pass_positions([5, 0, 9], [2, 0, 3]).tolist() == [5, 6, 9, 10, 11]
    assert pass_positions([], []).shape == (0,)
