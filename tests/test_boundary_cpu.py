"""CPU-side checks of the C ABI: the library loads, exports what the header
declares, validates arguments before touching the GPU, and its host logic
(chunk schedule, work planner) agrees with the oracle / with first principles.
No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import chunk_schedule as oracle_schedule
from paper_2509_25762_amd import binding as ob

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(ob.LIB_PATH):
        from paper_2509_25762_amd import build
        build.build(verbose=False)
    return ob.load()


def test_exports_match_header(lib):
    header = open(os.path.join(ROOT, "include", "oppo_attn.h")).read()
    declared = set(re.findall(r"\b(oppo_[a-z0-9_]+)\s*\(", header))
    assert declared == set(ob.EXPORTS), declared ^ set(ob.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), f"{name} not exported"
    assert ob.oppo_version() >= 100


def test_schedule_matches_oracle(lib):
    rng = np.random.default_rng(0)
    for _ in range(50):
        B = int(rng.integers(0, 40))
        P = rng.integers(0, 3000, size=B)
        R = rng.integers(0, 5000, size=B)
        C = int(rng.integers(1, 1200))
        t = int(rng.integers(0, 12))
        kvb, ql, cu = ob.oppo_chunk_schedule(P, R, C, t)
        okvb, oql, ocu = oracle_schedule(P, R, C, t)
        assert np.array_equal(kvb, okvb) and np.array_equal(ql, oql) and np.array_equal(cu, ocu)


def test_schedule_rejects_bad_arguments(lib):
    for args in ([[1], [1], 0, 0], [[1], [1], 4, -1], [[-1], [1], 4, 0], [[1], [-2], 4, 0]):
        with pytest.raises(ob.OppoError) as e:
            ob.oppo_chunk_schedule(*args)
        assert e.value.code == ob.OPPO_ERR_INVALID
    with pytest.raises(ob.OppoError):
        ob.oppo_chunk_schedule([2 ** 31 - 5], [100], 4, 0)          # P + R overflows int32
    assert ob.oppo_last_error() != ""


def _desc(Hq=32, Hkv=8, D=128, s=0.0884):
    return ob.make_desc(Hq, Hkv, D, s)


def _fake_cache(slot_begin, kv_len):
    """A cache whose device pointers are never dereferenced (validation fails first)."""
    return ob.KVCache(0x1000, 0x2000, np.asarray(slot_begin), np.asarray(kv_len))


def test_descriptor_validation(lib):
    cache = _fake_cache([0, 10], [0])
    for desc, code in [(_desc(D=96), ob.OPPO_ERR_UNSUPPORTED), (_desc(Hq=30), ob.OPPO_ERR_UNSUPPORTED),
                       (_desc(Hq=64, Hkv=2), ob.OPPO_ERR_UNSUPPORTED), (_desc(s=0.0), ob.OPPO_ERR_INVALID),
                       (_desc(s=float("nan")), ob.OPPO_ERR_INVALID), (_desc(Hq=0), ob.OPPO_ERR_INVALID)]:
        with pytest.raises(ob.OppoError) as e:
            ob.oppo_kv_append(desc, cache, [0, 1], 0x3000, 0x4000, stream=0)
        assert e.value.code == code
        assert ob.oppo_workspace_bytes(desc, 4, 100) == 0
    assert ob.oppo_workspace_bytes(_desc(), 4, 100) > 0
    assert ob.oppo_workspace_bytes(_desc(), -1, 100) == 0


def test_append_validation_leaves_lengths_untouched(lib):
    desc = _desc()
    cache = _fake_cache([0, 8, 20], [6, 0])
    cases = [([0, 3, 6], ob.OPPO_ERR_CAPACITY),      # 6 + 3 > 8
             ([1, 3, 6], ob.OPPO_ERR_INVALID),       # cu_q[0] != 0
             ([0, 3, 2], ob.OPPO_ERR_INVALID)]       # decreasing
    for cu, code in cases:
        with pytest.raises(ob.OppoError) as e:
            ob.oppo_kv_append(desc, cache, cu, 0x3000, 0x4000, stream=0)
        assert e.value.code == code
        assert cache.kv_len.tolist() == [6, 0]
    bad = _fake_cache([0, 8, 20], [9, 0])            # kv_len beyond the slab
    with pytest.raises(ob.OppoError) as e:
        ob.oppo_kv_append(desc, bad, [0, 0, 0], 0x3000, 0x4000, stream=0)
    assert e.value.code == ob.OPPO_ERR_INVALID
    dec = _fake_cache([0, 8, 4], [0, 0])             # slot_begin decreases
    with pytest.raises(ob.OppoError) as e:
        ob.oppo_kv_append(desc, dec, [0, 0, 0], 0x3000, 0x4000, stream=0)
    assert e.value.code == ob.OPPO_ERR_INVALID
    # a pass in which nobody has rows is legal and needs no device at all
    ob.oppo_kv_append(desc, cache, [0, 0, 0], None, None, stream=0)
    assert cache.kv_len.tolist() == [6, 0]


def test_attention_validation(lib):
    desc = _desc()
    cache = _fake_cache([0, 8, 20], [6, 2])
    with pytest.raises(ob.OppoError) as e:            # 3 query rows, only 2 cached tokens
        ob.oppo_chunk_prefill_attn(desc, cache, [0, 1, 4], 0x3000, 0x4000, stream=0)
    assert e.value.code == ob.OPPO_ERR_INVALID

    class FakeWs:                                      # unaligned / too small workspaces
        def __init__(self, ptr, n):
            self.ptr, self.n = ptr, n

        def is_contiguous(self):
            return True

        def data_ptr(self):
            return self.ptr

        def numel(self):
            return self.n

        def element_size(self):
            return 1

    for ws in (FakeWs(0x10001, 1 << 30), FakeWs(0x10000, 4096)):
        with pytest.raises(ob.OppoError) as e:
            ob.oppo_chunk_prefill_attn(desc, cache, [0, 1, 2], 0x3000, 0x4000, ws, stream=0)
        assert e.value.code == ob.OPPO_ERR_WORKSPACE
    # nothing to do: legal without any device pointer
    ob.oppo_chunk_prefill_attn(desc, cache, [0, 0, 0], None, None, stream=0)
    ob.oppo_full_prefill_ref(desc, [0, 0, 0], None, None, None, None, stream=0)
    with pytest.raises(ob.OppoError):
        ob.oppo_full_prefill_ref(desc, [0, 5, 3], 0x1, 0x2, 0x3, 0x4, stream=0)


def test_chunk_step_validation_leaves_lengths_untouched(lib):
    desc = _desc()
    cache = _fake_cache([0, 8, 20], [6, 0])
    cases = [([0, 3, 6], ob.OPPO_ERR_CAPACITY),      # 6 + 3 > 8
             ([1, 3, 6], ob.OPPO_ERR_INVALID),       # cu_q[0] != 0
             ([0, 3, 2], ob.OPPO_ERR_INVALID)]       # decreasing
    for cu, code in cases:
        with pytest.raises(ob.OppoError) as e:
            ob.oppo_chunk_step(desc, cache, cu, 0x3000, 0x4000, 0x5000, 0x6000, stream=0)
        assert e.value.code == code
        assert cache.kv_len.tolist() == [6, 0]
    with pytest.raises(ob.OppoError) as e:            # rows to do, but a null device pointer
        ob.oppo_chunk_step(desc, cache, [0, 1, 2], 0x3000, None, 0x5000, 0x6000, stream=0)
    assert e.value.code == ob.OPPO_ERR_INVALID and cache.kv_len.tolist() == [6, 0]
    with pytest.raises(ob.OppoError) as e:            # bad descriptor
        ob.oppo_chunk_step(_desc(D=96), cache, [0, 1, 2], 0x3000, 0x4000, 0x5000, 0x6000, stream=0)
    assert e.value.code == ob.OPPO_ERR_UNSUPPORTED
    # a pass in which nobody has rows is legal and needs no device at all
    ob.oppo_chunk_step(desc, cache, [0, 0, 0], None, None, None, None, stream=0)
    assert cache.kv_len.tolist() == [6, 0]


def test_options_validation(lib):
    with pytest.raises(ob.OppoError):
        ob.oppo_set_option(99, 1)
    with pytest.raises(ob.OppoError):
        ob.oppo_set_option(ob.OPT_ORDER, 7)
    with pytest.raises(ob.OppoError):
        ob.oppo_set_option(ob.OPT_SPLIT_KV, -1)
    ob.oppo_set_option(ob.OPT_SPLIT_KV, 0)
    ob.oppo_set_option(ob.OPT_ORDER, 0)


def _check_plan(desc, kv_before, q_len, items, TM):
    """Every (sequence, query tile) has its key range [0, keys) covered exactly
    once by pieces on 64-key boundaries; pieces of a split tile own distinct
    partial slots; whole tiles write final output."""
    by_tile = {}
    for seq, q_row0, n_tok, pos0, k0, k1, part, _ in items.tolist():
        by_tile.setdefault((seq, q_row0), []).append((k0, k1, part, n_tok, pos0))
    want = set()
    row = 0
    for i, (kvb, ql) in enumerate(zip(kv_before, q_len)):
        for j0 in range(0, ql, TM):
            want.add((i, row + j0))
        row += ql
    assert set(by_tile) == want
    parts = []
    row_of = np.concatenate([[0], np.cumsum(q_len)])
    for (seq, q_row0), pieces in by_tile.items():
        pieces.sort()
        n_tok, pos0 = pieces[0][3], pieces[0][4]
        j0 = q_row0 - row_of[seq]
        assert pos0 == kv_before[seq] + j0 and n_tok == min(TM, q_len[seq] - j0)
        assert pieces[0][0] == 0 and pieces[-1][1] == pos0 + n_tok
        for (a0, a1, _, _, _), (b0, _, _, _, _) in zip(pieces, pieces[1:]):
            assert a1 == b0 and a1 % 64 == 0
        if len(pieces) == 1:
            assert pieces[0][2] == -1
        else:
            parts += [p[2] for p in pieces]
            assert all(p[2] >= 0 for p in pieces)
    assert len(parts) == len(set(parts))
    return len(parts)


def test_planner_covers_every_key_exactly_once(lib):
    desc = _desc()
    ws = ob.oppo_workspace_bytes(desc, 64, 1 << 16)
    rng = np.random.default_rng(3)
    for trial in range(30):
        B = int(rng.integers(1, 70))
        kvb = rng.integers(0, 6000, size=B)
        ql = np.where(rng.random(B) < 0.3, 0, rng.integers(1, 300, size=B))
        for split in (0, 1, 2, 5):
            ob.oppo_set_option(ob.OPT_SPLIT_KV, split)
            items = ob.oppo_plan_debug(desc, kvb, ql, ws)
            n_parts = _check_plan(desc, kvb, ql, items, 256 // 4)
            if split == 1:
                assert n_parts == 0
            # pieces come grouped by queue, queues numbered without gaps
            queues = items[:, 7]
            assert np.all(np.diff(queues) >= 0) and queues[0] == 0 and queues[-1] < 256 // 8
            assert set(queues.tolist()) == set(range(int(queues[-1]) + 1))
            if split == 1:
                # whole query tiles: those of one sequence sit on different queues (they
                # read the same keys and are meant to run side by side) as long as the
                # sequence has no more of them than there are queues
                for sq in np.unique(items[:, 0]):
                    mine = queues[items[:, 0] == sq]
                    assert len(set(mine.tolist())) == min(len(mine), 256 // 8)
    ob.oppo_set_option(ob.OPT_SPLIT_KV, 0)
    # without a workspace nothing is ever split
    items = ob.oppo_plan_debug(desc, [5000], [256], 0)
    assert np.all(items[:, 6] == -1) and len(items) == 4


def test_planner_splits_a_thin_tail_but_not_a_full_batch(lib):
    desc = _desc()
    ws = ob.oppo_workspace_bytes(desc, 64, 1 << 16)
    tail = ob.oppo_plan_debug(desc, [3000], [256], ws)             # one straggler: 4 query tiles for 32 queues
    assert len(tail) > 4 and np.all(tail[:, 6] >= 0)
    assert len(set(tail[:, 7].tolist())) == 32                    # every queue gets a share ...
    keys = np.bincount(tail[:, 7], weights=tail[:, 5] - tail[:, 4])
    assert keys.max() - keys.min() <= 3 * 64                      # ... of about the same length
    full = ob.oppo_plan_debug(desc, np.full(64, 700), np.full(64, 256), ws)   # 8 query tiles per queue
    assert np.all(full[:, 6] == -1) and len(full) == 256
    assert np.all(np.bincount(full[:, 7]) == 8)


def test_planner_evens_out_the_ends_of_the_queues(lib):
    """40 query tiles of ~31 key tiles for 32 queues: whole tiles leave eight queues with two
    of them and the others with one, whatever the order.  The planner keeps most tiles
    whole and splits the last pieces of the long queues so that all queues end together."""
    desc = _desc()
    ws = ob.oppo_workspace_bytes(desc, 64, 1 << 16)
    rng = np.random.default_rng(11)
    kvb = rng.integers(1700, 1800, size=10)
    ql = np.full(10, 256)
    ob.oppo_set_option(ob.OPT_SPLIT_KV, 1)
    whole = ob.oppo_plan_debug(desc, kvb, ql, ws)
    ob.oppo_set_option(ob.OPT_SPLIT_KV, 0)
    auto = ob.oppo_plan_debug(desc, kvb, ql, ws)
    _check_plan(desc, kvb, ql, auto, 256 // 4)

    def loads(items):
        tiles = -(-(items[:, 5] - items[:, 4]) // 64)
        return np.bincount(items[:, 7], weights=tiles, minlength=32)

    lw, la = loads(whole), loads(auto)
    assert lw.max() - lw.min() > 25                       # the case is uneven to begin with
    assert la.max() <= lw.max() - 12                      # the longest queue got much shorter ...
    assert la.max() - la.min() <= 8                       # ... and all queues end about together
    split_tiles = len(set(map(tuple, auto[auto[:, 6] >= 0][:, :2].tolist())))
    assert 0 < split_tiles <= 31 and np.sum(auto[:, 6] == -1) >= 40 - 31   # the other tiles stay whole


def test_planner_balances_whole_tiles_by_exchanging_them(lib):
    """A full batch of ragged lengths: whole tiles only (nothing to merge), and after the
    exchange step the queues are within a few per cent of each other; the tiles of one
    sequence still sit on different queues."""
    desc = _desc()
    ws = ob.oppo_workspace_bytes(desc, 64, 1 << 16)
    rng = np.random.default_rng(12)
    kvb = rng.integers(300, 3000, size=60)
    ql = np.where(rng.random(60) < 0.2, rng.integers(1, 256, size=60), 256)
    items = ob.oppo_plan_debug(desc, kvb, ql, ws)
    _check_plan(desc, kvb, ql, items, 256 // 4)
    assert np.all(items[:, 6] == -1)
    tiles = -(-(items[:, 5] - items[:, 4]) // 64)
    load = np.bincount(items[:, 7], weights=tiles + 2.5, minlength=32)
    assert load.max() <= 1.03 * load.mean()
    for sq in np.unique(items[:, 0]):
        mine = items[items[:, 0] == sq][:, 7]
        assert len(set(mine.tolist())) == len(mine)


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: bench.py --gpus N with N > 1 exits with a message that says so,
    before anything touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_rope_validation(lib):
    desc = ob.make_desc(8, 2, 128, 0.1)
    kvb = np.array([3, 4], np.int32)
    cu = np.array([0, 2, 5], np.int32)
    f = lib.oppo_rope
    p = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    assert f(None, 2, p(kvb), p(cu), None, None, 10000.0, None) == ob.OPPO_ERR_INVALID
    assert f(ctypes.byref(desc), -1, p(kvb), p(cu), None, None, 10000.0, None) == ob.OPPO_ERR_INVALID
    assert f(ctypes.byref(desc), 2, None, p(cu), None, None, 10000.0, None) == ob.OPPO_ERR_INVALID
    assert f(ctypes.byref(desc), 2, p(kvb), None, None, None, 10000.0, None) == ob.OPPO_ERR_INVALID
    assert f(ctypes.byref(desc), 2, p(kvb), p(np.array([0, 3, 2], np.int32)), None, None, 10000.0, None) == ob.OPPO_ERR_INVALID
    assert f(ctypes.byref(desc), 2, p(np.array([3, -1], np.int32)), p(cu), None, None, 10000.0, None) == ob.OPPO_ERR_INVALID
    assert f(ctypes.byref(desc), 2, p(np.array([3, 2 ** 31 - 2], np.int32)), p(cu), None, None, 10000.0, None) == ob.OPPO_ERR_INVALID
    for bad in (1.0, 0.0, -5.0, float("nan"), float("inf")):
        assert f(ctypes.byref(desc), 2, p(kvb), p(cu), None, None, bad, None) == ob.OPPO_ERR_INVALID
    assert "theta_base" in ob.oppo_last_error()
    # nothing to rotate: no device is touched
    assert f(ctypes.byref(desc), 2, p(kvb), p(cu), None, None, 10000.0, None) == ob.OPPO_OK
    assert f(ctypes.byref(desc), 2, p(kvb), p(np.zeros(3, np.int32)), None, None, 10000.0, None) == ob.OPPO_OK


def test_qkv_epilogue_validation_leaves_lengths_untouched(lib):
    desc = _desc()
    cache = _fake_cache([0, 8, 20], [6, 0])
    cases = [([0, 3, 6], 10000.0, ob.OPPO_ERR_CAPACITY),   # 6 + 3 > 8
             ([1, 3, 6], 10000.0, ob.OPPO_ERR_INVALID),    # cu_q[0] != 0
             ([0, 3, 2], 10000.0, ob.OPPO_ERR_INVALID),    # decreasing
             ([0, 1, 2], 1.0, ob.OPPO_ERR_INVALID),        # theta_base must exceed 1
             ([0, 1, 2], float("nan"), ob.OPPO_ERR_INVALID)]
    for cu, base, code in cases:
        with pytest.raises(ob.OppoError) as e:
            ob.oppo_qkv_rope_append(desc, cache, cu, 0x3000, 0x4000, base, stream=0)
        assert e.value.code == code
        assert cache.kv_len.tolist() == [6, 0]
    with pytest.raises(ob.OppoError) as e:               # rows but no device arrays
        ob.oppo_qkv_rope_append(desc, cache, [0, 1, 2], None, 0x4000, stream=0)
    assert e.value.code == ob.OPPO_ERR_INVALID and cache.kv_len.tolist() == [6, 0]
    # nobody has rows: legal, no device needed
    ob.oppo_qkv_rope_append(desc, cache, [0, 0, 0], None, None, stream=0)
    assert cache.kv_len.tolist() == [6, 0]


def test_binding_refuses_undersized_or_host_buffers(lib):
    """The C ABI carries no sizes for device buffers; the binding knows them and refuses, before the
    library is called, a buffer smaller than the rows the call addresses or one that is not on the GPU."""
    import torch
    desc = _desc()
    rows, Hq, Hkv, D = 6, 32, 8, 128
    cu = [0, 2, 6]

    class Dev:
        """Stands in for a device tensor of n bytes (nothing dereferences it: every call below
        fails in the binding, or has nothing to do)."""
        def __init__(self, n, is_cuda=True):
            self.n, self.is_cuda = n, is_cuda

        def is_contiguous(self):
            return True

        def data_ptr(self):
            return 0x100000

        def numel(self):
            return self.n

        def element_size(self):
            return 1

    slabs = 30 * Hkv * D * 2
    cache = ob.KVCache(Dev(slabs), Dev(slabs), np.array([0, 10, 30]), np.array([2, 3]))
    q_ok, kv_ok = Dev(rows * Hq * D * 2), Dev(rows * Hkv * D * 2)
    q_small, kv_small = Dev(rows * Hq * D * 2 - 2), Dev(rows * Hkv * D * 2 - 2)
    with pytest.raises(ValueError, match="q holds"):
        ob.oppo_chunk_step(desc, cache, cu, q_small, kv_ok, kv_ok, q_ok, stream=0)
    with pytest.raises(ValueError, match="v_new holds"):
        ob.oppo_chunk_step(desc, cache, cu, q_ok, kv_ok, kv_small, q_ok, stream=0)
    with pytest.raises(ValueError, match="out holds"):
        ob.oppo_chunk_step_noalloc(desc, cache, cu, q_ok, kv_ok, kv_ok, q_small, stream=0)
    with pytest.raises(ValueError, match="k_new holds"):
        ob.oppo_kv_append(desc, cache, cu, kv_small, kv_ok, stream=0)
    with pytest.raises(ValueError, match="out holds"):
        ob.oppo_chunk_prefill_attn(desc, cache, cu, q_ok, q_small, stream=0)
    with pytest.raises(ValueError, match="qkv holds"):
        ob.oppo_qkv_rope_append(desc, cache, cu, Dev(rows * (Hq + 2 * Hkv) * D * 2 - 2), q_ok, stream=0)
    with pytest.raises(ValueError, match="k_new holds"):
        ob.oppo_rope(desc, [2, 3], cu, q_ok, kv_small, stream=0)
    with pytest.raises(ValueError, match="q holds"):
        ob.oppo_full_prefill_ref(desc, cu, q_small, kv_ok, kv_ok, q_ok, stream=0)
    short = ob.KVCache(Dev(slabs - 2), Dev(slabs), np.array([0, 10, 30]), np.array([2, 3]))
    with pytest.raises(ValueError, match=r"cache\.k holds"):
        ob.oppo_chunk_step(desc, short, cu, q_ok, kv_ok, kv_ok, q_ok, stream=0)
    with pytest.raises(ValueError, match="must be a device tensor"):
        ob.oppo_chunk_step(desc, cache, cu, Dev(rows * Hq * D * 2, is_cuda=False), kv_ok, kv_ok, q_ok, stream=0)
    host = torch.zeros((rows, Hq, D), dtype=torch.int16)                   # a real tensor in host memory
    with pytest.raises(ValueError, match="must be a device tensor"):
        ob.oppo_chunk_step(desc, cache, cu, host, kv_ok, kv_ok, q_ok, stream=0)
    with pytest.raises(ValueError, match="workspace must be a device tensor"):
        ob.oppo_chunk_prefill_attn(desc, cache, cu, q_ok, q_ok, torch.zeros(1 << 21, dtype=torch.uint8), stream=0)
    assert cache.kv_len.tolist() == [2, 3]


def test_noalloc_entry_point_validation(lib):
    """oppo_chunk_step_noalloc: the checks of oppo_chunk_step, plus the limit its built-in scratch
    buffer puts on the layer's width; all before any device is touched."""
    assert ob.oppo_static_scratch_bytes() == 64 << 20
    desc = _desc()
    cache = _fake_cache([0, 8, 20], [6, 0])
    for cu, code in [([0, 3, 6], ob.OPPO_ERR_CAPACITY), ([1, 3, 6], ob.OPPO_ERR_INVALID), ([0, 3, 2], ob.OPPO_ERR_INVALID)]:
        with pytest.raises(ob.OppoError) as e:
            ob.oppo_chunk_step_noalloc(desc, cache, cu, 0x3000, 0x4000, 0x5000, 0x6000, stream=0)
        assert e.value.code == code and cache.kv_len.tolist() == [6, 0]
    with pytest.raises(ob.OppoError) as e:                               # 16 kv-heads of 128: 16 x 130 > 2048
        ob.oppo_chunk_step_noalloc(_desc(Hq=64, Hkv=16), cache, [0, 1, 2], 0x3000, 0x4000, 0x5000, 0x6000, stream=0)
    assert e.value.code == ob.OPPO_ERR_UNSUPPORTED and "scratch" in e.value.message
    assert cache.kv_len.tolist() == [6, 0]
    with pytest.raises(ob.OppoError) as e:
        ob.oppo_chunk_step_noalloc(desc, cache, [0, 1, 2], 0x3000, None, 0x5000, 0x6000, stream=0)
    assert e.value.code == ob.OPPO_ERR_INVALID and cache.kv_len.tolist() == [6, 0]
    ob.oppo_chunk_step_noalloc(desc, cache, [0, 0, 0], None, None, None, None, stream=0)   # nobody has rows
    assert cache.kv_len.tolist() == [6, 0]


def test_workspace_size_follows_the_work(lib):
    """oppo_workspace_bytes honours its arguments, and a workspace smaller than it (but at least one
    slot) is accepted: it only bounds the number of partial pieces."""
    desc = _desc()
    slot = 8 * 256 * 130 * 4
    assert ob.oppo_workspace_bytes(desc, 1, 64) == 2 * 32 * slot          # one full tile + one ragged tile, 32 pieces each
    assert ob.oppo_workspace_bytes(desc, 64, 1 << 16) == (6 * 256 // 8 + 1) * slot   # bounded by the chip
    assert ob.oppo_workspace_bytes(desc, 0, 0) == 0
    full = ob.oppo_plan_debug(desc, [3000], [256], ob.oppo_workspace_bytes(desc, 1, 256))
    assert np.sum(full[:, 6] >= 0) > 20                                   # one straggler: cut for all 32 queues
    few = ob.oppo_plan_debug(desc, [3000], [256], 20 * slot)              # the same with twenty slots
    parts = few[few[:, 6] >= 0][:, 6]
    assert len(parts) <= 20 and (len(parts) == 0 or parts.max() < 20)
    _check_plan(desc, [3000], [256], few, 64)
    none = ob.oppo_plan_debug(desc, [3000], [256], slot)                  # one slot: nothing can be split
    assert np.all(none[:, 6] == -1) and len(none) == 4


def test_options_are_snapshotted_per_call_and_settable_from_threads(lib):
    """oppo_set_option from another thread while plans are being made: every plan is a valid plan of
    one of the two policies (no call sees a half-changed set), and nothing crashes."""
    import threading
    desc = _desc()
    ws = ob.oppo_workspace_bytes(desc, 64, 1 << 16)
    kvb, ql = np.array([3000, 1200, 40]), np.array([256, 256, 100])
    stop = threading.Event()

    def flip():
        i = 0
        while not stop.is_set():
            ob.oppo_set_option(ob.OPT_SPLIT_KV, 1 if i & 1 else 4)
            i += 1

    th = threading.Thread(target=flip)
    th.start()
    try:
        for _ in range(300):
            items = ob.oppo_plan_debug(desc, kvb, ql, ws)
            n_parts = _check_plan(desc, kvb, ql, items, 64)
            assert n_parts == 0 or n_parts >= 8
    finally:
        stop.set()
        th.join()
        ob.oppo_set_option(ob.OPT_SPLIT_KV, 0)


def test_projection_validation_leaves_lengths_untouched(lib):
    desc = _desc()
    cache = _fake_cache([0, 8, 20], [6, 0])
    ws = 0x100000

    class Ws:
        def __init__(self, ptr, n):
            self.ptr, self.n = ptr, n

        def is_contiguous(self):
            return True

        def data_ptr(self):
            return self.ptr

        def numel(self):
            return self.n

        def element_size(self):
            return 1

    need = ob.oppo_qkv_proj_workspace_bytes(desc, 2)
    assert need == 2 * (8 + 64 * 8) and ob.oppo_qkv_proj_workspace_bytes(_desc(D=96), 2) == 0
    cases = [([0, 3, 6], 128, 10000.0, Ws(ws, 1 << 20), ob.OPPO_ERR_CAPACITY),      # 6 + 3 > 8
             ([0, 3, 2], 128, 10000.0, Ws(ws, 1 << 20), ob.OPPO_ERR_INVALID),       # decreasing
             ([0, 1, 2], 100, 10000.0, Ws(ws, 1 << 20), ob.OPPO_ERR_UNSUPPORTED),   # hidden not a multiple of 64
             ([0, 1, 2], 0, 10000.0, Ws(ws, 1 << 20), ob.OPPO_ERR_INVALID),
             ([0, 1, 2], 128, 1.0, Ws(ws, 1 << 20), ob.OPPO_ERR_INVALID),           # theta_base must exceed 1
             ([0, 1, 2], 128, 10000.0, Ws(ws, need - 1), ob.OPPO_ERR_WORKSPACE),
             ([0, 1, 2], 128, 10000.0, Ws(ws + 1, 1 << 20), ob.OPPO_ERR_WORKSPACE),
             ([0, 1, 2], 128, 10000.0, None, ob.OPPO_ERR_WORKSPACE)]
    for cu, hidden, base, w_, code in cases:
        with pytest.raises(ob.OppoError) as e:
            ob.oppo_qkv_proj_rope_append(desc, cache, cu, 0x3000, hidden, 0x4000, 0x5000, w_, base, stream=0)
        assert e.value.code == code, (cu, hidden, base, code, e.value)
        assert cache.kv_len.tolist() == [6, 0]
    with pytest.raises(ob.OppoError) as e:               # rows but no weights
        ob.oppo_qkv_proj_rope_append(desc, cache, [0, 1, 2], 0x3000, 128, None, 0x5000, Ws(ws, 1 << 20), stream=0)
    assert e.value.code == ob.OPPO_ERR_INVALID and cache.kv_len.tolist() == [6, 0]
    ob.oppo_qkv_proj_rope_append(desc, cache, [0, 0, 0], None, 128, None, None, None, stream=0)   # nobody has rows
    assert cache.kv_len.tolist() == [6, 0]


def test_fp8_cache_validation_leaves_lengths_untouched(lib):
    """Argument checks of the 8-bit cache's two entry points (no device needed: every call fails
    before a launch, or has nothing to do)."""
    desc = _desc()

    def cache(slot_begin=(0, 128, 256), kv_len=(100, 0), ks=0.01, vs=0.02):
        return ob.KVCacheFp8(0x1000, 0x2000, np.asarray(slot_begin), ks, vs, np.asarray(kv_len))

    c = cache()
    for cu, code in (([0, 29, 30], ob.OPPO_ERR_CAPACITY), ([0, 3, 2], ob.OPPO_ERR_INVALID)):
        with pytest.raises(ob.OppoError) as e:
            ob.oppo_kv_append_fp8(desc, c, cu, 0x3000, 0x4000, stream=0)
        assert e.value.code == code
    for bad in (cache(ks=0.0), cache(vs=-1.0), cache(ks=float("nan")), cache(vs=float("inf")), cache(ks=1e-42),
                cache(slot_begin=(0, 100, 256)), cache(slot_begin=(0, 128, 250))):
        with pytest.raises(ob.OppoError) as e:
            ob.oppo_kv_append_fp8(desc, bad, [0, 1, 2], 0x3000, 0x4000, stream=0)
        assert e.value.code == ob.OPPO_ERR_INVALID
        with pytest.raises(ob.OppoError) as e:
            ob.oppo_chunk_prefill_attn_fp8(desc, bad, [0, 1, 0 + 1], 0x3000, 0x4000, stream=0)
        assert e.value.code == ob.OPPO_ERR_INVALID
        assert bad.kv_len.tolist() == [100, 0]
    with pytest.raises(ob.OppoError) as e:                       # a score factor the kernel cannot split
        ob.oppo_chunk_prefill_attn_fp8(desc, cache(ks=1e-36), [0, 1, 1], 0x3000, 0x4000, stream=0)
    assert e.value.code == ob.OPPO_ERR_INVALID
    with pytest.raises(ob.OppoError) as e:                       # rows that were never appended
        ob.oppo_chunk_prefill_attn_fp8(desc, c, [0, 101, 101], 0x3000, 0x4000, stream=0)
    assert e.value.code == ob.OPPO_ERR_INVALID
    assert c.kv_len.tolist() == [100, 0]
    ob.oppo_kv_append_fp8(desc, c, [0, 0, 0], None, None, stream=0)              # nobody has rows: legal
    ob.oppo_chunk_prefill_attn_fp8(desc, c, [0, 0, 0], None, None, stream=0)

    class Dev:
        def __init__(self, n):
            self.n, self.is_cuda = n, True

        def is_contiguous(self):
            return True

        def data_ptr(self):
            return 0x100000

        def numel(self):
            return self.n

        def element_size(self):
            return 1

    slab = 256 * 8 * 128                                          # one byte per element
    ok = ob.KVCacheFp8(Dev(slab), Dev(slab), np.array([0, 128, 256]), 1.0, 1.0, np.array([100, 0]))
    short = ob.KVCacheFp8(Dev(slab), Dev(slab - 1), np.array([0, 128, 256]), 1.0, 1.0, np.array([100, 0]))
    kv = Dev(2 * 8 * 128 * 2)
    with pytest.raises(ValueError, match=r"cache\.v holds"):
        ob.oppo_kv_append_fp8(desc, short, [0, 1, 2], kv, kv, stream=0)
    with pytest.raises(ValueError, match="v_new holds"):
        ob.oppo_kv_append_fp8(desc, ok, [0, 1, 2], kv, Dev(2 * 8 * 128 * 2 - 1), stream=0)
    with pytest.raises(ValueError, match="out holds"):
        ob.oppo_chunk_prefill_attn_fp8(desc, ok, [0, 1, 1], Dev(32 * 128 * 2), Dev(32 * 128 * 2 - 2), stream=0)
