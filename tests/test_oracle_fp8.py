"""Pins of the 8-bit cache oracle (oracle/fp8_cache.py): hand-derived codes of the format, the
exhaustive round trip over all codes, an independent library conversion, error bounds, the layout
written out element by element, and the streaming invariant of Sec. 3.1 through the 8-bit cache."""
import os

import numpy as np
import pytest

from oracle import bf16_bits_to_f64, causal_attention
from oracle.fp8_cache import (BLOCK, Fp8KVCacheOracle, dequantize, e4m3_decode, e4m3_encode, quantize,
                              stream_episode_fp8)
from paper_2509_25762_amd.workload import f32_to_bf16_bits


def test_hand_derived_codes(golden_dir):
    for line in open(os.path.join(golden_dir, "e4m3_codes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        value, code = line.split()[:2]
        got = int(e4m3_encode(np.array([float(value)], dtype=np.float32))[0])
        assert got == int(code, 16), f"{value}: {got:#04x} instead of 0x{code}"


def test_every_code_round_trips_and_the_grid_is_monotonic():
    codes = np.arange(256, dtype=np.uint8)
    vals = e4m3_decode(codes)
    nan = np.isnan(vals)
    assert nan.sum() == 2 and nan[0x7F] and nan[0xFF]
    ok = ~nan
    back = e4m3_encode(vals[ok].astype(np.float32))
    want = codes[ok].copy()
    want[want == 0x80] = 0x80                      # minus zero keeps its sign bit
    assert np.array_equal(back, want)
    pos = vals[:0x7F]
    assert np.all(np.diff(pos) > 0) and pos[0] == 0 and pos[-1] == 448.0
    assert np.array_equal(vals[0x80:0xFF], -pos)


def test_against_an_independent_library_conversion():
    torch = pytest.importorskip("torch")
    if not hasattr(torch, "float8_e4m3fn"):
        pytest.skip("this torch has no float8_e4m3fn")
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000) * s for s in (1e-3, 0.02, 1.0, 30.0, 300.0)]).astype(np.float32)
    x = np.clip(x, -448, 448)                       # (the library's own overflow rule is not the clamp used here)
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = e4m3_encode(x)
    same_value = e4m3_decode(got) == e4m3_decode(ref)     # (+0 / -0 of tiny negative inputs compare equal)
    assert same_value.all(), f"{(~same_value).sum()} of {x.size} differ"


def test_error_bounds_of_the_round_trip():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(50000) * 3).astype(np.float32)
    bits = f32_to_bf16_bits(x)
    xv = bf16_bits_to_f64(bits)
    for scale in (1.0, 0.25, 0.013):
        back = dequantize(quantize(bits, scale), scale)
        s = float(np.float32(scale))
        lim = 448.0 * s
        inside = np.abs(xv) <= lim
        err = np.abs(back - xv)
        # half a code step: 2^-4 relative for normal codes, 2^-10 * scale absolute below the smallest normal
        assert np.all(err[inside] <= np.maximum(2.0 ** -4 * np.abs(xv[inside]), 2.0 ** -10 * s) * (1 + 1e-6))
        assert np.all(np.abs(back[~inside]) == lim)


def test_layout_and_zero_fill_of_the_value_blocks():
    rng = np.random.default_rng(2)
    Hkv, D = 2, 8
    slot_begin = [0, 128, 320]
    cache = Fp8KVCacheOracle(slot_begin, Hkv, D, 0.5, 2.0)
    k1, v1 = f32_to_bf16_bits(rng.standard_normal((70 + 3, Hkv, D)).astype(np.float32)), f32_to_bf16_bits(rng.standard_normal((70 + 3, Hkv, D)).astype(np.float32))
    cache.append([0, 70, 73], k1, v1)
    kc, vc = quantize(k1, 0.5), quantize(v1, 2.0)
    for (i, j, row) in [(0, 0, 0), (0, 69, 69), (1, 2, 72)]:
        slot = slot_begin[i] + j
        for g in range(Hkv):
            for d in range(D):
                assert cache.k[slot, g, d] == kc[row, g, d]
                assert cache.v[slot // BLOCK, g, d, slot % BLOCK] == vc[row, g, d]
    assert np.all(cache.v[1, :, :, 6:] == 0)        # sequence 0: tokens 64..69 in block 1, the rest of it zero
    assert np.all(cache.v[2, :, :, 3:] == 0)        # sequence 1 (slab from slot 128 = block 2): 3 tokens
    assert np.all(cache.v[3:] == 0xFF)              # blocks never touched keep their bytes
    assert np.all(cache.k[70:128] == 0xFF) and np.all(cache.k[131:] == 0xFF)
    assert cache.kv_len.tolist() == [70, 3]
    k, v = cache.values(0)
    assert np.array_equal(k, dequantize(kc[:70], 0.5)) and np.array_equal(v, dequantize(vc[:70], 2.0))


def test_streaming_through_the_8_bit_cache_equals_one_shot():
    rng = np.random.default_rng(3)
    Hq, Hkv, D = 4, 2, 16
    n = [150, 70]
    draw = lambda shape: f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
    q = [draw((m, Hq, D)) for m in n]
    k = [draw((m, Hkv, D)) for m in n]
    v = [draw((m, Hkv, D)) for m in n]
    scale = 1.0 / np.sqrt(D)
    one, cache_one = stream_episode_fp8(q, k, v, [n], scale, 0.75, 1.5)
    for chunks in ([[100, 3], [50, 67]], [[1, 64], [63, 6], [86, 0]], [[64, 0], [64, 0], [22, 70]]):
        outs, cache = stream_episode_fp8(q, k, v, chunks, scale, 0.75, 1.5)
        for a, b in zip(outs, one):
            assert np.abs(a - b).max() <= 1e-12     # the same codes; float64 sums in another order at most
        assert np.array_equal(cache.k, cache_one.k) and np.array_equal(cache.v, cache_one.v)
    # and it is the plain definition over the values the codes stand for
    kd, vd = cache_one.values(1)
    ref = causal_attention(bf16_bits_to_f64(q[1]), kd, vd, np.arange(n[1]), scale)
    assert np.abs(one[1] - ref).max() <= 1e-12
    # close to the 16-bit result: the 8-bit rounding of K and V moves outputs by a few hundredths at most
    full = causal_attention(bf16_bits_to_f64(q[1]), bf16_bits_to_f64(k[1]), bf16_bits_to_f64(v[1]), np.arange(n[1]), scale)
    assert np.abs(one[1] - full).max() < 0.2 and np.abs(one[1] - full).mean() < 0.03
