"""GPU parity of the fused QKV projection with its rotary / cache epilogue (oppo_qkv_proj_rope_append)
against the float64 oracle (oracle/projection.py), and of the layer path projection -> attention
against the oracle's projection -> rotation -> one-shot prefill.

Tolerance of the projection: the kernel accumulates bf16 products in fp32 (MFMA), rotates in fp32 and
rounds once to bf16, so |gpu - oracle| <= 2^-8 |oracle| (half a bf16 ulp at most) plus the fp32
accumulation and rotation error, bounded by 2^-19 * sum_k |x_k| |w_k| of the columns involved
(hidden <= 1024 here; a sum of n fp32-rounded terms is off by at most ~n 2^-24 of the sum of magnitudes).
Keys and values are compared where they land: in the cache, whose other slots must stay untouched."""
import numpy as np
import pytest

from oracle import bf16_bits_to_f64, full_prefill, pass_positions, qkv_projection, qkv_projection_rope
from paper_2509_25762_amd.workload import f32_to_bf16_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2509_25762_amd import binding
    binding.load()
    return binding, torch


def draw(rng, shape, scale=1.0):
    return f32_to_bf16_bits((rng.standard_normal(shape) * scale).astype(np.float32))


def run_projection(gpu, rng, Hq, Hkv, D, hidden, kv_before, q_len, base):
    binding, torch = gpu
    dev = torch.device("cuda:0")
    B = len(q_len)
    cu = np.concatenate([[0], np.cumsum(q_len)]).astype(np.int32)
    rows = int(cu[-1])
    xb = draw(rng, (rows, hidden))
    wb = draw(rng, ((Hq + 2 * Hkv) * D, hidden), 1.0 / np.sqrt(hidden))
    cap = np.asarray(kv_before, dtype=np.int64) + q_len + 2
    slot_begin = np.concatenate([[0], np.cumsum(cap)])
    ck = torch.full((int(slot_begin[-1]), Hkv, D), -1, dtype=torch.int16, device=dev)
    cv = torch.full_like(ck, -1)
    cache = binding.KVCache(ck, cv, slot_begin, np.asarray(kv_before, dtype=np.int32))
    desc = binding.make_desc(Hq, Hkv, D, 1.0 / np.sqrt(D))
    tx = torch.from_numpy(xb.view(np.int16)).to(dev)
    tw = torch.from_numpy(wb.view(np.int16)).to(dev)
    q_out = torch.full((rows + 2, Hq, D), 0x7FC0, dtype=torch.int16, device=dev)     # a spare row on either side
    ws = torch.empty(binding.oppo_qkv_proj_workspace_bytes(desc, rows), dtype=torch.uint8, device=dev)
    binding.oppo_qkv_proj_rope_append(desc, cache, cu, tx, hidden, tw, q_out[1:-1], ws, base)
    torch.cuda.synchronize()
    return xb, wb, cu, slot_begin, cache, q_out.cpu().numpy().view(np.uint16), ck.cpu().numpy().view(np.uint16), cv.cpu().numpy().view(np.uint16)


def bound_of(want, mag):
    return 2.0 ** -8 * np.abs(want) * 1.001 + 2.0 ** -19 * mag + 1e-30


@pytest.mark.parametrize("Hq,Hkv,D,hidden,base", [(8, 2, 128, 256, 10000.0), (4, 4, 64, 128, 500000.0), (3, 1, 64, 1024, 10000.0),
                                                   (16, 1, 128, 512, 1000000.0), (2, 1, 64, 64, 10000.0)])   # the last: one k tile
def test_projection_epilogue_matches_the_oracle_on_a_ragged_pass(gpu, Hq, Hkv, D, hidden, base):
    rng = np.random.default_rng(300 + Hq + D + hidden)
    q_len = np.array([0, 1, 7, 64, 130, 9, 0, 33, 129], dtype=np.int32)          # 373 rows: three row tiles, a ragged last one
    kv_before = np.array([17, 0, 60000, 123, 4095, 1, 5, 65536 * 4, 3], dtype=np.int32)
    xb, wb, cu, slot_begin, cache, gq, gk, gv = run_projection(gpu, rng, Hq, Hkv, D, hidden, kv_before, q_len, base)
    pos = pass_positions(kv_before, q_len)
    q_ref, k_ref, v_ref = qkv_projection_rope(xb, wb, pos, Hq, Hkv, D, base)
    # magnitudes sum_k |x||w| per output column, and per rotated pair
    mag = np.abs(bf16_bits_to_f64(xb)) @ np.abs(bf16_bits_to_f64(wb)).T
    qc, kc = Hq * D, Hkv * D
    half = D // 2

    def pair(m, heads):
        m = m.reshape(m.shape[0], heads, D)
        p = m[..., :half] + m[..., half:]
        return np.concatenate([p, p], axis=-1)

    assert (gq[0] == 0x7FC0).all() and (gq[-1] == 0x7FC0).all(), "rows outside the pass were written"
    got_q = bf16_bits_to_f64(gq[1:-1])
    assert (np.abs(got_q - q_ref) <= bound_of(q_ref, pair(mag[:, :qc], Hq))).all(), "queries"
    assert cache.kv_len.tolist() == (kv_before + q_len).tolist()
    for i in range(len(q_len)):
        b, n0, n1 = int(slot_begin[i]), int(kv_before[i]), int(kv_before[i] + q_len[i])
        r0, r1 = int(cu[i]), int(cu[i + 1])
        got_k, got_v = bf16_bits_to_f64(gk[b + n0:b + n1]), bf16_bits_to_f64(gv[b + n0:b + n1])
        assert (np.abs(got_k - k_ref[r0:r1]) <= bound_of(k_ref[r0:r1], pair(mag[r0:r1, qc:qc + kc], Hkv))).all(), f"keys of sequence {i}"
        assert (np.abs(got_v - v_ref[r0:r1]) <= bound_of(v_ref[r0:r1], mag[r0:r1, qc + kc:].reshape(r1 - r0, Hkv, D))).all(), f"values of sequence {i}"
        # slots before and after the appended rows are untouched
        assert (gk[b:b + n0] == 0xFFFF).all() and (gk[b + n1:int(slot_begin[i + 1])] == 0xFFFF).all()
        assert (gv[b:b + n0] == 0xFFFF).all() and (gv[b + n1:int(slot_begin[i + 1])] == 0xFFFF).all()
    # almost every element is the oracle's value rounded to bf16 (fp32 noise crosses a rounding boundary rarely)
    differ = int((gq[1:-1] != f32_to_bf16_bits(q_ref.astype(np.float32))).sum())
    assert differ <= max(4, gq[1:-1].size // 200), f"{differ} of {gq[1:-1].size} query elements differ from the rounded oracle value"


@pytest.mark.parametrize("rows", [4091, 8155])
def test_larger_passes_take_the_larger_tiles(gpu, rows):
    """The launch picks the tile height from the pass's size: 64 rows for the thin passes above, 128 rows for
    ~4K rows x 6 column tiles and 256 rows for ~8K (the estimate in launch_qkv_proj); both with a ragged last
    row tile and sequences of uneven length, against the oracle as above."""
    Hq, Hkv, D, hidden, base = 8, 2, 128, 256, 10000.0
    rng = np.random.default_rng(900 + rows)
    q_len = np.array([rows // 2, 1, rows // 4 + 3, 0, 517], dtype=np.int32)
    q_len = np.append(q_len, rows - q_len.sum()).astype(np.int32)
    assert (q_len >= 0).all() and q_len.sum() == rows
    kv_before = np.array([3, 70000, 0, 9, 255, 1024], dtype=np.int32)
    xb, wb, cu, slot_begin, cache, gq, gk, gv = run_projection(gpu, rng, Hq, Hkv, D, hidden, kv_before, q_len, base)
    q_ref, k_ref, v_ref = qkv_projection_rope(xb, wb, pass_positions(kv_before, q_len), Hq, Hkv, D, base)
    mag = np.abs(bf16_bits_to_f64(xb)) @ np.abs(bf16_bits_to_f64(wb)).T
    qc, kc, half = Hq * D, Hkv * D, D // 2

    def pair(m, heads):
        m = m.reshape(m.shape[0], heads, D)
        p = m[..., :half] + m[..., half:]
        return np.concatenate([p, p], axis=-1)

    assert (gq[0] == 0x7FC0).all() and (gq[-1] == 0x7FC0).all(), "rows outside the pass were written"
    assert (np.abs(bf16_bits_to_f64(gq[1:-1]) - q_ref) <= bound_of(q_ref, pair(mag[:, :qc], Hq))).all(), "queries"
    assert cache.kv_len.tolist() == (kv_before + q_len).tolist()
    for i in range(len(q_len)):
        b, n0, n1 = int(slot_begin[i]), int(kv_before[i]), int(kv_before[i] + q_len[i])
        r0, r1 = int(cu[i]), int(cu[i + 1])
        got_k, got_v = bf16_bits_to_f64(gk[b + n0:b + n1]), bf16_bits_to_f64(gv[b + n0:b + n1])
        assert (np.abs(got_k - k_ref[r0:r1]) <= bound_of(k_ref[r0:r1], pair(mag[r0:r1, qc:qc + kc], Hkv))).all(), f"keys of sequence {i}"
        assert (np.abs(got_v - v_ref[r0:r1]) <= bound_of(v_ref[r0:r1], mag[r0:r1, qc + kc:].reshape(r1 - r0, Hkv, D))).all(), f"values of sequence {i}"
        assert (gk[b:b + n0] == 0xFFFF).all() and (gk[b + n1:int(slot_begin[i + 1])] == 0xFFFF).all()
        assert (gv[b:b + n0] == 0xFFFF).all() and (gv[b + n1:int(slot_begin[i + 1])] == 0xFFFF).all()


def test_values_are_the_rounded_fp32_sums_when_products_are_exact(gpu):
    """Small integers: every product and partial sum is exact in fp32, so value heads (no rotation) and
    the rows at position 0 (rotation by 0) must be bit-exact, whatever the order of accumulation."""
    binding, torch = gpu
    rng = np.random.default_rng(9)
    Hq, Hkv, D, hidden = 4, 2, 128, 128
    q_len = np.array([200, 1], dtype=np.int32)
    kv_before = np.array([0, 0], dtype=np.int32)
    cu = np.concatenate([[0], np.cumsum(q_len)]).astype(np.int32)
    rows = int(cu[-1])
    xb = f32_to_bf16_bits(rng.integers(-3, 4, size=(rows, hidden)).astype(np.float32))
    wb = f32_to_bf16_bits(rng.integers(-2, 3, size=((Hq + 2 * Hkv) * D, hidden)).astype(np.float32))
    dev = torch.device("cuda:0")
    slot_begin = np.array([0, 200, 201], dtype=np.int64)
    ck = torch.full((201, Hkv, D), -1, dtype=torch.int16, device=dev)
    cv = torch.full_like(ck, -1)
    cache = binding.KVCache(ck, cv, slot_begin, kv_before)
    desc = binding.make_desc(Hq, Hkv, D, 1.0 / np.sqrt(D))
    q_out = torch.zeros((rows, Hq, D), dtype=torch.int16, device=dev)
    ws = torch.empty(binding.oppo_qkv_proj_workspace_bytes(desc, rows), dtype=torch.uint8, device=dev)
    binding.oppo_qkv_proj_rope_append(desc, cache, cu, torch.from_numpy(xb.view(np.int16)).to(dev), hidden,
                                      torch.from_numpy(wb.view(np.int16)).to(dev), q_out, ws)
    torch.cuda.synchronize()
    q_ref, k_ref, v_ref = qkv_projection(xb, wb, Hq, Hkv, D)
    assert np.array_equal(cv.cpu().numpy().view(np.uint16), f32_to_bf16_bits(v_ref.astype(np.float32)))
    gq = q_out.cpu().numpy().view(np.uint16)
    for r in (0, 200):                                   # the two rows at position 0
        assert np.array_equal(gq[r], f32_to_bf16_bits(q_ref[r].astype(np.float32)))
        assert np.array_equal(ck.cpu().numpy().view(np.uint16)[r], f32_to_bf16_bits(k_ref[r].astype(np.float32)))


def test_layer_path_projection_then_attention_equals_one_shot(gpu):
    """Hidden rows streamed in ragged chunks: projection (+ rotation, + cache write) then oppo_chunk_prefill_attn,
    against the oracle's projection -> rotation of all rows -> one-shot prefill, to the attention's tolerance."""
    binding, torch = gpu
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(77)
    Hq, Hkv, D, hidden, base = 8, 2, 128, 256, 10000.0
    n_tok = np.array([150, 40, 300])
    B = len(n_tok)
    xs = [draw(rng, (int(n), hidden)) for n in n_tok]
    wb = draw(rng, ((Hq + 2 * Hkv) * D, hidden), 1.0 / np.sqrt(hidden))
    desc = binding.make_desc(Hq, Hkv, D, 1.0 / np.sqrt(D))
    slot_begin = np.concatenate([[0], np.cumsum(n_tok + 1)])
    ck = torch.full((int(slot_begin[-1]), Hkv, D), -1, dtype=torch.int16, device=dev)
    cv = torch.full_like(ck, -1)
    cache = binding.KVCache(ck, cv, slot_begin)
    tw = torch.from_numpy(wb.view(np.int16)).to(dev)
    outs = [np.zeros((int(n), Hq, D), dtype=np.uint16) for n in n_tok]
    done = np.zeros(B, dtype=np.int64)
    for chunk in ([70, 40, 1], [64, 0, 200], [16, 0, 99]):
        ql = np.array(chunk)
        cu = np.concatenate([[0], np.cumsum(ql)]).astype(np.int32)
        rows = int(cu[-1])
        xb = np.concatenate([xs[i][done[i]:done[i] + ql[i]] for i in range(B)])
        q_rot = torch.empty((rows, Hq, D), dtype=torch.int16, device=dev)
        out = torch.empty_like(q_rot)
        ws = torch.empty(binding.oppo_qkv_proj_workspace_bytes(desc, rows), dtype=torch.uint8, device=dev)
        binding.oppo_qkv_proj_rope_append(desc, cache, cu, torch.from_numpy(xb.view(np.int16)).to(dev), hidden, tw, q_rot, ws, base)
        binding.oppo_chunk_prefill_attn(desc, cache, cu, q_rot, out)
        torch.cuda.synchronize()
        o = out.cpu().numpy().view(np.uint16)
        for i in range(B):
            outs[i][done[i]:done[i] + ql[i]] = o[cu[i]:cu[i + 1]]
        done += ql
    assert done.tolist() == n_tok.tolist()
    errs = []
    for i in range(B):
        q, k, v = qkv_projection_rope(xs[i], wb, np.arange(int(n_tok[i]), dtype=np.float64), Hq, Hkv, D, base)
        # the attention sees what the projection stored: bf16-rounded queries, keys and values
        rq, rk, rv = (bf16_bits_to_f64(f32_to_bf16_bits(t.astype(np.float32))) for t in (q, k, v))
        ref = full_prefill(rq, rk, rv, 1.0 / np.sqrt(D))
        errs.append(np.abs(bf16_bits_to_f64(outs[i]) - ref).ravel())
    err = np.concatenate(errs)
    assert err.max() <= 3e-2 and err.mean() <= 2e-3, f"max {err.max():.3e} mean {err.mean():.3e}"
