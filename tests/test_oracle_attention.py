"""Pins for the float64 attention oracle (CPU only).

Each test fails for a plausible mistake in the oracle: a dropped scale, a
transposed operand, an off-by-one mask, a wrong GQA head map, a missing
normalisation, or bottom-right vs top-left mask alignment.
"""
import math
import os

import numpy as np
import pytest

from oracle import attention_row, bf16_bits_to_f64, causal_attention, full_prefill
from paper_2509_25762_amd.workload import f32_to_bf16_bits


def brute_force(q, k, v, q_pos, scale):
    """Independent triple loop in plain Python floats (math.exp)."""
    Tq, Hq, D = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    out = np.zeros((Tq, Hq, D))
    for j in range(Tq):
        n = int(q_pos[j])
        for h in range(Hq):
            g = h // G
            scores = []
            for m in range(n + 1):
                acc = 0.0
                for d in range(D):
                    acc += float(q[j, h, d]) * float(k[m, g, d])
                scores.append(scale * acc)
            mx = max(scores)
            ex = [math.exp(x - mx) for x in scores]
            z = sum(ex)
            for d in range(D):
                acc = 0.0
                for m in range(n + 1):
                    acc += ex[m] / z * float(v[m, g, d])
                out[j, h, d] = acc
    return out


def rand_bf16(rng, shape):
    return bf16_bits_to_f64(f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32)))


@pytest.mark.parametrize("N,Hq,Hkv,D", [(12, 4, 2, 8), (7, 3, 3, 5), (9, 4, 1, 4), (1, 2, 1, 3)])
def test_brute_force_full_prefill(N, Hq, Hkv, D):
    rng = np.random.default_rng(100 + N)
    q, k, v = rand_bf16(rng, (N, Hq, D)), rand_bf16(rng, (N, Hkv, D)), rand_bf16(rng, (N, Hkv, D))
    s = 1.0 / math.sqrt(D)
    got = full_prefill(q, k, v, s)
    want = brute_force(q, k, v, np.arange(N), s)
    assert np.max(np.abs(got - want)) <= 1e-13


def test_brute_force_chunk_rows_bottom_right_alignment():
    """A chunk of 3 rows on a 9-token cache: rows sit at positions 6, 7, 8."""
    rng = np.random.default_rng(7)
    N, Hq, Hkv, D = 9, 4, 2, 6
    q, k, v = rand_bf16(rng, (3, Hq, D)), rand_bf16(rng, (N, Hkv, D)), rand_bf16(rng, (N, Hkv, D))
    pos = np.array([6, 7, 8])
    got = causal_attention(q, k, v, pos, 0.3)
    assert np.max(np.abs(got - brute_force(q, k, v, pos, 0.3))) <= 1e-13
    # a top-left aligned mask (row j sees keys <= j) would differ
    wrong = brute_force(q, k, v, np.array([0, 1, 2]), 0.3)
    assert np.max(np.abs(got - wrong)) > 1e-3


def _parse_golden(path):
    vals = {}
    names = {"LN3": math.log(3.0), "LN4": math.log(4.0)}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *rest = line.split()
            vals[key] = np.array([names[x] if x in names else float(x) for x in rest])
    return vals


def test_golden_three_token_rational(golden_dir):
    g = _parse_golden(os.path.join(golden_dir, "three_token_rational.txt"))
    k = g["k"].reshape(3, 1, 2)
    v = g["v"].reshape(3, 1, 2)
    q = np.stack([g["q_head0"].reshape(3, 2), g["q_head1"].reshape(3, 2)], axis=1)  # [3, 2, 2]
    out, w = causal_attention(q, k, v, np.arange(3), float(g["scale"][0]), return_weights=True)
    assert np.max(np.abs(out[:, 0, :] - g["out_head0"].reshape(3, 2))) <= 1e-14
    assert np.max(np.abs(out[:, 1, :] - g["out_head1"].reshape(3, 2))) <= 1e-14
    assert np.max(np.abs(w[0, 2, :] - g["weights_head0_row2"])) <= 1e-15
    # the masked weights of earlier rows are exactly zero
    assert w[0, 0, 1] == 0.0 and w[0, 0, 2] == 0.0 and w[0, 1, 2] == 0.0


def test_rows_of_softmax_sum_to_one_and_v_ones():
    rng = np.random.default_rng(3)
    N, Hq, Hkv, D = 40, 4, 2, 16
    q, k = rand_bf16(rng, (N, Hq, D)), rand_bf16(rng, (N, Hkv, D))
    v = np.ones((N, Hkv, D))
    out, w = causal_attention(q, k, v, np.arange(N), 0.25, return_weights=True)
    assert np.max(np.abs(w.sum(axis=2) - 1.0)) <= 1e-14
    assert np.max(np.abs(out - 1.0)) <= 1e-14
    # weights beyond the diagonal are exactly zero
    for n in range(N):
        assert np.all(w[:, n, n + 1:] == 0.0)
        assert np.all(w[:, n, : n + 1] > 0.0)


def test_zero_queries_give_running_mean():
    rng = np.random.default_rng(4)
    N, Hq, Hkv, D = 33, 2, 1, 8
    k, v = rand_bf16(rng, (N, Hkv, D)), rand_bf16(rng, (N, Hkv, D))
    q = np.zeros((N, Hq, D))
    out = full_prefill(q, k, v, 0.5)
    want = np.cumsum(v[:, 0, :], axis=0) / np.arange(1, N + 1)[:, None]
    for h in range(Hq):
        assert np.max(np.abs(out[:, h, :] - want)) <= 1e-13
    # identical keys do the same for any query
    k_same = np.broadcast_to(k[:1], k.shape).copy()
    out2 = full_prefill(rand_bf16(rng, (N, Hq, D)), k_same, v, 0.5)
    assert np.max(np.abs(out2[:, 0, :] - want)) <= 1e-12


def test_first_token_returns_its_value_exactly():
    rng = np.random.default_rng(5)
    N, Hq, Hkv, D = 5, 4, 2, 8
    q, k, v = rand_bf16(rng, (N, Hq, D)), rand_bf16(rng, (N, Hkv, D)), rand_bf16(rng, (N, Hkv, D))
    out = full_prefill(q, k, v, 0.35)
    for h in range(Hq):
        assert np.array_equal(out[0, h, :], v[0, h // 2, :])


def test_dominant_key_limit():
    rng = np.random.default_rng(6)
    N, D = 20, 8
    q, k, v = rand_bf16(rng, (N, 1, D)), rand_bf16(rng, (N, 1, D)), rand_bf16(rng, (N, 1, D))
    out = full_prefill(q, k, v, 1e4)
    for n in range(N):
        m = int(np.argmax(k[: n + 1, 0, :] @ q[n, 0, :]))
        assert np.max(np.abs(out[n, 0, :] - v[m, 0, :])) <= 1e-9


def test_causality_bitwise_under_future_perturbation():
    rng = np.random.default_rng(8)
    N, Hq, Hkv, D = 48, 4, 2, 16
    q, k, v = rand_bf16(rng, (N, Hq, D)), rand_bf16(rng, (N, Hkv, D)), rand_bf16(rng, (N, Hkv, D))
    base = full_prefill(q, k, v, 0.25)
    n = 29
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    q2[n + 1:] += 3.0
    k2[n + 1:] -= 5.0
    v2[n + 1:] *= -2.0
    pert = full_prefill(q2, k2, v2, 0.25)
    assert np.array_equal(base[: n + 1], pert[: n + 1])
    assert np.max(np.abs(base[n + 1:] - pert[n + 1:])) > 1e-3


def test_gqa_head_map_batch_and_linearity():
    rng = np.random.default_rng(9)
    N, Hq, Hkv, D = 24, 8, 2, 8
    q, k, v = rand_bf16(rng, (N, Hq, D)), rand_bf16(rng, (N, Hkv, D)), rand_bf16(rng, (N, Hkv, D))
    out = full_prefill(q, k, v, 0.3)
    # contiguous groups: heads 0..3 read kv-head 0, heads 4..7 read kv-head 1;
    # each q-head equals single-head attention on its kv-head
    for h in range(Hq):
        single = full_prefill(q[:, h:h + 1], k[:, h // 4:h // 4 + 1], v[:, h // 4:h // 4 + 1], 0.3)
        assert np.array_equal(out[:, h], single[:, 0])
    # siblings given the same query give the same output
    q_same = q.copy()
    q_same[:, 1] = q_same[:, 0]
    o2 = full_prefill(q_same, k, v, 0.3)
    assert np.array_equal(o2[:, 0], o2[:, 1])
    # linear in V
    v_b = rand_bf16(rng, (N, Hkv, D))
    lin = full_prefill(q, k, 2.0 * v - 3.0 * v_b, 0.3)
    assert np.max(np.abs(lin - (2.0 * out - 3.0 * full_prefill(q, k, v_b, 0.3)))) <= 1e-12


def test_against_library_float64_sdpa():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(10)
    Tq, Tk, Hq, Hkv, D = 13, 37, 4, 2, 16
    q, k, v = rand_bf16(rng, (Tq, Hq, D)), rand_bf16(rng, (Tk, Hkv, D)), rand_bf16(rng, (Tk, Hkv, D))
    pos = Tk - Tq + np.arange(Tq)
    got = causal_attention(q, k, v, pos, 0.2)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]                       # [1, Hq, Tq, D]
    tk = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(2, 0)[None]
    tv = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(2, 0)[None]
    mask = torch.from_numpy(np.arange(Tk)[None, :] <= pos[:, None])
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=0.2)
    ref = ref[0].permute(1, 0, 2).numpy()
    assert np.max(np.abs(got - ref)) <= 1e-12


def test_row_mode_matches_full_mode():
    rng = np.random.default_rng(11)
    N, Hq, Hkv, D = 50, 4, 2, 8
    q, k, v = rand_bf16(rng, (N, Hq, D)), rand_bf16(rng, (N, Hkv, D)), rand_bf16(rng, (N, Hkv, D))
    full = full_prefill(q, k, v, 0.3)
    for n, h in [(0, 0), (17, 3), (49, 2), (31, 1)]:
        row = attention_row(q[n, h], k, v, n, h, Hq, 0.3)
        assert np.max(np.abs(row - full[n, h])) <= 1e-14


def test_bf16_widening_is_exact():
    bits = np.array([0x0000, 0x3F80, 0xBF80, 0x4000, 0x3DCD, 0x7F7F, 0x0080], dtype=np.uint16)
    want = [0.0, 1.0, -1.0, 2.0, 0.10009765625, 3.3895313892515355e38, 1.1754943508222875e-38]
    assert np.array_equal(bf16_bits_to_f64(bits), np.array(want))
    # round trip through the generator's rounding is the identity on bf16 values
    x = bf16_bits_to_f64(np.arange(0x3000, 0x4800, dtype=np.uint16)).astype(np.float32)
    assert np.array_equal(f32_to_bf16_bits(x), np.arange(0x3000, 0x4800, dtype=np.uint16))
