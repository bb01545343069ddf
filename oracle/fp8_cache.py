"""The KV cache in 8-bit floating point (test oracle).

The scorer of Sec. 3.1 re-reads each sequence's whole cache at every pass, so on small chunks the
pass is bound by the bytes of K and V; storing them in 8 bits halves those bytes.  The paper says
nothing about the cache's format; this is the reading the library documents:

  * format: OCP FP8 E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; no infinities;
    S.1111.111 is NaN; largest finite value 448 = 1.75 * 2^8; smallest normal 2^-6; subnormals are
    multiples of 2^-9);
  * one positive scale per tensor (keys, values) of the layer, given by the caller:
        code = e4m3( clamp( fl32(x * inv_scale), -448, 448 ) ),  inv_scale = fl32(1 / scale),
    rounding to nearest, ties to even (fl32 = rounding to float32; x is a bf16 value, exact in
    float32).  The value a code stands for is  code_value * scale  exactly;
  * layout: keys token-major like the 16-bit cache, one byte per element: token m of sequence i
    at [slot_begin[i] + m][Hkv][D]; values in blocks of 64 tokens with the token index fastest:
    [(slot_begin[i] + m) / 64][Hkv][D][(slot_begin[i] + m) % 64], slabs starting on block
    boundaries - which is the order the second matrix product of attention contracts them in;
  * append writes the codes of the new tokens and zero bytes into what is left of the last
    value block it touches (so that block never holds anything but codes and zeros); no other
    byte changes;
  * attention is the plain definition over the values the codes stand for, in float64, with
    the queries as they are.

Streaming-equivalence (Sec. 3.1, Eq. 3) holds exactly: a token's codes do not depend on the
chunk it arrived in, and every pass sees every key and value through its codes.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np

from .attention import bf16_bits_to_f64, causal_attention

E4M3_MAX = 448.0
BLOCK = 64


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    """Value of each E4M3 code (uint8) as float64; the two NaN codes decode to NaN."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = c & 0x7
    normal = (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64))
    sub = (m / 8.0) * 2.0 ** -6
    val = np.where(e == 0, sub, normal)
    val = np.where((e == 15) & (m == 7), np.nan, val)
    return sign * val


def e4m3_encode(x: np.ndarray) -> np.ndarray:
    """Nearest E4M3 code of each float32 value (ties to the code with an even mantissa),
    values beyond +-448 clamped to +-448 first.  Written out on the value grid: in the binade
    [2^e, 2^(e+1)) with e >= -6 the codes are 2^(e-3) apart, below 2^-6 they are 2^-9 apart."""
    x = np.asarray(x, dtype=np.float32).astype(np.float64)
    assert np.isfinite(x).all(), "the cache holds finite values only"
    a = np.minimum(np.abs(x), E4M3_MAX)
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -6)))          # binade of |x|, at least the first normal one
    e = np.where(np.exp2(e + 1) <= a, e + 1, e)                # (guards log2's rounding at powers of two)
    e = np.where(np.exp2(e) > np.maximum(a, 2.0 ** -6), e - 1, e)
    step = np.exp2(e - 3)
    q = np.rint(a / step)                                      # numpy's rint rounds ties to even
    mag = q * step                                             # may be 2^(e+1): the next binade's first code
    # back to a code: magnitude -> exponent and mantissa fields
    e2 = np.floor(np.log2(np.maximum(mag, 2.0 ** -6)))
    e2 = np.where(np.exp2(e2 + 1) <= mag, e2 + 1, e2)
    e2 = np.where(np.exp2(e2) > np.maximum(mag, 2.0 ** -6), e2 - 1, e2)
    is_sub = mag < 2.0 ** -6
    m = np.where(is_sub, np.rint(mag / 2.0 ** -9), np.rint((mag / np.exp2(e2) - 1.0) * 8.0)).astype(np.int64)
    ef = np.where(is_sub, 0, (e2 + 7).astype(np.int64))
    code = (ef << 3) | m
    code = np.where(np.signbit(x), code | 0x80, code)
    return code.astype(np.uint8)


def quantize(bits: np.ndarray, scale: float) -> np.ndarray:
    """bf16 bit patterns -> E4M3 codes under the documented rule (the product with 1/scale is
    rounded to float32 before it is rounded to 8 bits)."""
    x = (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
    inv = np.float32(1.0) / np.float32(scale)
    with np.errstate(over="ignore"):                           # (a product beyond float32 is +-inf, which the clamp takes)
        y = (x * inv).astype(np.float32)
    return e4m3_encode(np.clip(y, np.float32(-E4M3_MAX), np.float32(E4M3_MAX)))


def dequantize(codes: np.ndarray, scale: float) -> np.ndarray:
    """What the codes stand for, float64 (code value times float32(scale), exactly)."""
    return e4m3_decode(codes) * np.float64(np.float32(scale))


class Fp8KVCacheOracle:
    """Slabs of codes in the documented layout; every slab starts on a 64-token block boundary."""

    def __init__(self, slot_begin: Sequence[int], num_kv_heads: int, head_dim: int, k_scale: float, v_scale: float,
                 fill: int = 0xFF):
        self.slot_begin = np.asarray(slot_begin, dtype=np.int64)
        assert np.all(np.diff(self.slot_begin) >= 0) and np.all(self.slot_begin % BLOCK == 0)
        self.batch = self.slot_begin.size - 1
        total = int(self.slot_begin[-1])
        self.Hkv, self.D = num_kv_heads, head_dim
        self.k_scale, self.v_scale = float(k_scale), float(v_scale)
        self.k = np.full((total, num_kv_heads, head_dim), fill, dtype=np.uint8)
        self.v = np.full((total // BLOCK, num_kv_heads, head_dim, BLOCK), fill, dtype=np.uint8)
        self.kv_len = np.zeros(self.batch, dtype=np.int64)

    def append(self, cu_q: Sequence[int], k_new_bits: np.ndarray, v_new_bits: np.ndarray) -> None:
        cu_q = np.asarray(cu_q, dtype=np.int64)
        q_len = np.diff(cu_q)
        for i in range(self.batch):
            assert self.kv_len[i] + q_len[i] <= self.slot_begin[i + 1] - self.slot_begin[i], "chunk does not fit"
        kc = quantize(k_new_bits, self.k_scale)
        vc = quantize(v_new_bits, self.v_scale)
        for i in range(self.batch):
            for j in range(int(q_len[i])):
                slot = int(self.slot_begin[i] + self.kv_len[i] + j)
                self.k[slot] = kc[cu_q[i] + j]
                self.v[slot // BLOCK, :, :, slot % BLOCK] = vc[cu_q[i] + j]
            if q_len[i] > 0:
                end = int(self.slot_begin[i] + self.kv_len[i] + q_len[i])
                if end % BLOCK:
                    self.v[end // BLOCK, :, :, end % BLOCK:] = 0          # the rest of the last block touched
        self.kv_len += q_len

    def values(self, i: int):
        """(K, V) of sequence i as float64 [kv_len, Hkv, D]: what the codes stand for."""
        b, n = int(self.slot_begin[i]), int(self.kv_len[i])
        k = dequantize(self.k[b:b + n], self.k_scale)
        blocks = self.v[b // BLOCK:(b + n + BLOCK - 1) // BLOCK]            # [nb, Hkv, D, 64]
        v = np.transpose(blocks, (0, 3, 1, 2)).reshape(-1, self.Hkv, self.D)[:n]
        return k, dequantize(v, self.v_scale)

    def attend(self, cu_q: Sequence[int], q_bits: np.ndarray, scale: float) -> np.ndarray:
        cu_q = np.asarray(cu_q, dtype=np.int64)
        q = bf16_bits_to_f64(q_bits)
        out = np.empty(q.shape, dtype=np.float64)
        for i in range(self.batch):
            lo, hi = int(cu_q[i]), int(cu_q[i + 1])
            if hi == lo:
                continue
            k, v = self.values(i)
            n_kv = k.shape[0]
            pos = n_kv - (hi - lo) + np.arange(hi - lo)
            out[lo:hi] = causal_attention(q[lo:hi], k, v, pos, scale)
        return out


def stream_episode_fp8(q_bits: List[np.ndarray], k_bits: List[np.ndarray], v_bits: List[np.ndarray],
                       chunks: List[List[int]], scale: float, k_scale: float, v_scale: float):
    """Like stream_episode, through an 8-bit cache.  Returns (outputs per sequence, the cache)."""
    B = len(q_bits)
    n = [int(x.shape[0]) for x in q_bits]
    slot_begin = np.zeros(B + 1, dtype=np.int64)
    for i in range(B):
        slot_begin[i + 1] = slot_begin[i] + (n[i] + BLOCK - 1) // BLOCK * BLOCK
    cache = Fp8KVCacheOracle(slot_begin, k_bits[0].shape[1], k_bits[0].shape[2], k_scale, v_scale)
    outs = [np.empty(q_bits[i].shape, dtype=np.float64) for i in range(B)]
    done = [0] * B
    for step in chunks:
        cu_q = np.concatenate([[0], np.cumsum(step)]).astype(np.int64)
        gather = lambda src: np.concatenate([src[i][done[i]:done[i] + step[i]] for i in range(B)], axis=0)
        cache.append(cu_q, gather(k_bits), gather(v_bits))
        o = cache.attend(cu_q, gather(q_bits), scale)
        for i in range(B):
            outs[i][done[i]:done[i] + step[i]] = o[cu_q[i]:cu_q[i + 1]]
            done[i] += step[i]
    assert done == n
    return outs, cache
