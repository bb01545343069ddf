"""Pins of the projection oracle (oracle/projection.py): the definition written out as loops,
a hand-worked example, selector weights that fix the operand order and the head layout,
linearity, and the identity at position 0."""
import os

import numpy as np

from oracle import bf16_bits_to_f64, qkv_projection, qkv_projection_rope, rope_rotate
from paper_2509_25762_amd.workload import f32_to_bf16_bits


def bits(a):
    return f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def test_triple_loop_on_tiny_inputs():
    rng = np.random.default_rng(0)
    rows, hidden, Hq, Hkv, D = 5, 7, 3, 1, 4
    xb = bits(rng.standard_normal((rows, hidden)))
    wb = bits(rng.standard_normal(((Hq + 2 * Hkv) * D, hidden)))
    q, k, v = qkv_projection(xb, wb, Hq, Hkv, D)
    x, w = bf16_bits_to_f64(xb), bf16_bits_to_f64(wb)
    for m in range(rows):
        for n in range((Hq + 2 * Hkv) * D):
            acc = 0.0
            for kk in range(hidden):
                acc += float(x[m, kk]) * float(w[n, kk])
            head, d = divmod(n, D)
            got = q[m, head, d] if head < Hq else k[m, head - Hq, d] if head < Hq + Hkv else v[m, head - Hq - Hkv, d]
            assert abs(got - acc) <= 1e-12 * max(1.0, abs(acc))


def test_hand_worked_example(golden_dir):
    vals = {}
    for line in open(os.path.join(golden_dir, "qkv_projection_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, *nums = line.split()
        vals[name] = [float(t) for t in nums]
    xb = bits([[1, 2, 0], [0, -1, 4]])
    wb = bits([[1, 0, 0], [0, 1, 0], [2, 0, 1], [0, 0, -1], [1, 1, 1], [0.5, 0, 0]])
    q, k, v = qkv_projection_rope(xb, wb, np.array([0.0, vals["position_row1"][0]]), 1, 1, 2, base=10000.0)
    for r in (0, 1):
        np.testing.assert_allclose(q[r, 0], vals[f"q_row{r}"], atol=1e-12)
        np.testing.assert_allclose(k[r, 0], vals[f"k_row{r}"], atol=1e-12)
        np.testing.assert_allclose(v[r, 0], vals[f"v_row{r}"], atol=1e-12)


def test_selector_weights_fix_operand_order_and_head_layout():
    """Row n of w being the unit vector e_{c(n)} makes output column n a copy of input column c(n):
    a transposed operand, a head-major/row-major mix-up or a wrong q|k|v order all fail."""
    rng = np.random.default_rng(1)
    rows, hidden, Hq, Hkv, D = 4, 40, 2, 1, 8
    n_out = (Hq + 2 * Hkv) * D
    pick = rng.permutation(hidden)[:n_out]
    w = np.zeros((n_out, hidden), dtype=np.float32)
    w[np.arange(n_out), pick] = 1.0
    xb = bits(rng.standard_normal((rows, hidden)))
    x = bf16_bits_to_f64(xb)
    q, k, v = qkv_projection(xb, bits(w), Hq, Hkv, D)
    flat = np.concatenate([q.reshape(rows, -1), k.reshape(rows, -1), v.reshape(rows, -1)], axis=1)
    assert np.array_equal(flat, x[:, pick])
    assert q.shape == (rows, Hq, D) and k.shape == (rows, Hkv, D) and v.shape == (rows, Hkv, D)
    assert np.array_equal(k[:, 0, 3], x[:, pick[Hq * D + 3]])
    assert np.array_equal(v[:, 0, 0], x[:, pick[(Hq + Hkv) * D]])


def test_linearity_and_rotation_properties():
    rng = np.random.default_rng(2)
    rows, hidden, Hq, Hkv, D = 6, 16, 2, 2, 4
    # sums of bf16 values with few mantissa bits stay exact in bf16, so x1 + x2 is again an input
    x1 = rng.integers(-4, 5, size=(rows, hidden)).astype(np.float32)
    x2 = rng.integers(-4, 5, size=(rows, hidden)).astype(np.float32)
    wb = bits(rng.integers(-3, 4, size=((Hq + 2 * Hkv) * D, hidden)).astype(np.float32))
    a = qkv_projection(bits(x1), wb, Hq, Hkv, D)
    b = qkv_projection(bits(x2), wb, Hq, Hkv, D)
    c = qkv_projection(bits(x1 + x2), wb, Hq, Hkv, D)
    for u, w_, s in zip(a, b, c):
        assert np.array_equal(u + w_, s)
    pos = np.arange(rows, dtype=np.float64) * 3
    qr, kr, vr = qkv_projection_rope(bits(x1), wb, pos, Hq, Hkv, D)
    assert np.array_equal(vr, a[2])                                   # values pass through
    assert np.array_equal(qr[0], a[0][0]) and np.array_equal(kr[0], a[1][0])   # position 0: identity
    np.testing.assert_allclose(qr, rope_rotate(a[0], pos), atol=0)    # the rotation is the pinned one
    np.testing.assert_allclose(np.sum(qr ** 2, axis=-1), np.sum(a[0] ** 2, axis=-1), rtol=1e-12)   # a rotation keeps norms
