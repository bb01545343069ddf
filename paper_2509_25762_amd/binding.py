"""ctypes binding of liboppo_attn.so: argument marshalling only.

Every function has the name and the semantics of its C entry point in
include/oppo_attn.h.  Device buffers are torch tensors (torch only allocates
device memory and provides the stream); length arrays are numpy int arrays in
host memory.  There is no fallback: if the library is missing or fails to
load, importing the symbols raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liboppo_attn.so")

OPPO_OK = 0
OPPO_ERR_INVALID = -1
OPPO_ERR_UNSUPPORTED = -2
OPPO_ERR_CAPACITY = -3
OPPO_ERR_WORKSPACE = -4
OPPO_ERR_HIP = -5

OPT_SPLIT_KV = 0
OPT_ORDER = 1
OPT_NUM_CUS = 2

EXPORTS = [
    "oppo_chunk_schedule", "oppo_kv_append", "oppo_chunk_prefill_attn", "oppo_chunk_step", "oppo_full_prefill_ref",
    "oppo_workspace_bytes", "oppo_set_option", "oppo_plan_debug", "oppo_last_error", "oppo_version", "oppo_rope", "oppo_qkv_rope_append", "oppo_qkv_proj_rope_append", "oppo_qkv_proj_workspace_bytes",
    "oppo_profile_enable", "oppo_profile_read", "oppo_profile_read_each", "oppo_profile_host", "oppo_chunk_step_noalloc", "oppo_static_scratch_bytes",
    "oppo_kv_append_fp8", "oppo_chunk_prefill_attn_fp8",
    "oppo_pool_create", "oppo_pool_destroy", "oppo_pool_acquire", "oppo_pool_release", "oppo_pool_slot_of",
    "oppo_pool_cache", "oppo_pool_pack", "oppo_pool_counts",
    "oppo_sched_create", "oppo_sched_destroy", "oppo_sched_set_delta", "oppo_sched_room", "oppo_sched_add",
    "oppo_sched_begin_pass", "oppo_sched_end_pass", "oppo_sched_end_iteration", "oppo_sched_counts",
    "oppo_tuner_create", "oppo_tuner_destroy", "oppo_tuner_chunk", "oppo_tuner_report", "oppo_overlap_timeline",
]

PASS_NONE, PASS_PROMPT, PASS_CHUNK = 0, 1, 2


class OppoError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"oppo status {code}: {message}")
        self.code = code
        self.message = message


class AttnDesc(ctypes.Structure):
    _fields_ = [("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("softmax_scale", ctypes.c_float)]


class KVCacheStruct(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("slot_begin", ctypes.POINTER(ctypes.c_int64)),
                ("kv_len", ctypes.POINTER(ctypes.c_int32)), ("batch", ctypes.c_int32)]


class KVCacheFp8Struct(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("slot_begin", ctypes.POINTER(ctypes.c_int64)),
                ("kv_len", ctypes.POINTER(ctypes.c_int32)), ("batch", ctypes.c_int32),
                ("k_scale", ctypes.c_float), ("v_scale", ctypes.c_float)]


_lib = None


def load() -> ctypes.CDLL:
    """Loads the shared library (built by paper_2509_25762_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2509_25762_amd.build`")
    try:
        # torch ships its own HIP runtime; it has to be the first one loaded into the process,
        # or the library's kernels and torch's buffers end up on two different runtimes
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(LIB_PATH)
    i32p = ctypes.POINTER(ctypes.c_int32)
    vp = ctypes.c_void_p
    lib.oppo_chunk_schedule.argtypes = [ctypes.c_int32, i32p, i32p, ctypes.c_int32, ctypes.c_int32, i32p, i32p, i32p]
    lib.oppo_chunk_schedule.restype = ctypes.c_int
    lib.oppo_kv_append.argtypes = [ctypes.POINTER(AttnDesc), ctypes.POINTER(KVCacheStruct), i32p, vp, vp, vp]
    lib.oppo_kv_append.restype = ctypes.c_int
    lib.oppo_qkv_rope_append.argtypes = [ctypes.POINTER(AttnDesc), ctypes.POINTER(KVCacheStruct), i32p, vp, vp,
                                         ctypes.c_double, vp]
    lib.oppo_qkv_rope_append.restype = ctypes.c_int
    lib.oppo_qkv_proj_rope_append.argtypes = [ctypes.POINTER(AttnDesc), ctypes.POINTER(KVCacheStruct), i32p, vp, ctypes.c_int32,
                                              vp, vp, ctypes.c_double, vp, ctypes.c_size_t, vp]
    lib.oppo_qkv_proj_rope_append.restype = ctypes.c_int
    lib.oppo_qkv_proj_workspace_bytes.argtypes = [ctypes.POINTER(AttnDesc), ctypes.c_int32]
    lib.oppo_qkv_proj_workspace_bytes.restype = ctypes.c_size_t
    lib.oppo_chunk_prefill_attn.argtypes = [ctypes.POINTER(AttnDesc), ctypes.POINTER(KVCacheStruct), i32p, vp, vp,
                                            vp, ctypes.c_size_t, vp]
    lib.oppo_chunk_prefill_attn.restype = ctypes.c_int
    lib.oppo_chunk_step.argtypes = [ctypes.POINTER(AttnDesc), ctypes.POINTER(KVCacheStruct), i32p, vp, vp, vp, vp,
                                    vp, ctypes.c_size_t, vp]
    lib.oppo_chunk_step.restype = ctypes.c_int
    lib.oppo_chunk_step_noalloc.argtypes = [ctypes.POINTER(AttnDesc), ctypes.POINTER(KVCacheStruct), i32p, vp, vp, vp, vp, vp]
    lib.oppo_chunk_step_noalloc.restype = ctypes.c_int
    lib.oppo_kv_append_fp8.argtypes = [ctypes.POINTER(AttnDesc), ctypes.POINTER(KVCacheFp8Struct), i32p, vp, vp, vp]
    lib.oppo_kv_append_fp8.restype = ctypes.c_int
    lib.oppo_chunk_prefill_attn_fp8.argtypes = [ctypes.POINTER(AttnDesc), ctypes.POINTER(KVCacheFp8Struct), i32p, vp, vp, vp,
                                                ctypes.c_size_t, vp]
    lib.oppo_chunk_prefill_attn_fp8.restype = ctypes.c_int
    lib.oppo_static_scratch_bytes.argtypes = []
    lib.oppo_static_scratch_bytes.restype = ctypes.c_size_t
    lib.oppo_profile_read_each.argtypes = [ctypes.POINTER(ctypes.c_double), i32p, ctypes.c_int32, i32p]
    lib.oppo_profile_read_each.restype = ctypes.c_int
    lib.oppo_profile_host.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    lib.oppo_profile_host.restype = ctypes.c_int
    lib.oppo_full_prefill_ref.argtypes = [ctypes.POINTER(AttnDesc), ctypes.c_int32, i32p, vp, vp, vp, vp, vp,
                                          ctypes.c_size_t, vp]
    lib.oppo_full_prefill_ref.restype = ctypes.c_int
    lib.oppo_workspace_bytes.argtypes = [ctypes.POINTER(AttnDesc), ctypes.c_int32, ctypes.c_int32]
    lib.oppo_workspace_bytes.restype = ctypes.c_size_t
    lib.oppo_set_option.argtypes = [ctypes.c_int, ctypes.c_int]
    lib.oppo_set_option.restype = ctypes.c_int
    lib.oppo_plan_debug.argtypes = [ctypes.POINTER(AttnDesc), ctypes.c_int32, i32p, i32p, ctypes.c_size_t, i32p,
                                    ctypes.c_int32, i32p]
    lib.oppo_plan_debug.restype = ctypes.c_int
    lib.oppo_profile_enable.argtypes = [ctypes.c_int]
    lib.oppo_profile_enable.restype = ctypes.c_int
    lib.oppo_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), i32p]
    lib.oppo_profile_read.restype = ctypes.c_int
    i64p = ctypes.POINTER(ctypes.c_int64)
    lib.oppo_pool_create.argtypes = [ctypes.c_int32, i32p, ctypes.POINTER(vp)]
    lib.oppo_pool_destroy.argtypes = [vp]
    lib.oppo_pool_acquire.argtypes = [vp, ctypes.c_int64, ctypes.c_int32, i32p]
    lib.oppo_pool_release.argtypes = [vp, ctypes.c_int64]
    lib.oppo_pool_slot_of.argtypes = [vp, ctypes.c_int64, i32p]
    lib.oppo_pool_cache.argtypes = [vp, vp, vp, ctypes.POINTER(KVCacheStruct)]
    lib.oppo_pool_pack.argtypes = [vp, ctypes.c_int32, i64p, i32p, i32p, i32p]
    lib.oppo_pool_counts.argtypes = [vp, i32p, i32p, i64p, i64p]
    u8p = ctypes.POINTER(ctypes.c_uint8)
    lib.oppo_sched_create.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(vp)]
    lib.oppo_sched_destroy.argtypes = [vp]
    lib.oppo_sched_set_delta.argtypes = [vp, ctypes.c_int32]
    lib.oppo_sched_room.argtypes = [vp, i32p]
    lib.oppo_sched_add.argtypes = [vp, ctypes.c_int64, ctypes.c_int32]
    lib.oppo_sched_begin_pass.argtypes = [vp, ctypes.c_int32, i64p, i32p, i32p, i32p, i32p]
    lib.oppo_sched_end_pass.argtypes = [vp, ctypes.c_int32, i64p, i32p, u8p]
    lib.oppo_sched_end_iteration.argtypes = [vp, ctypes.c_int32, i64p, i32p]
    lib.oppo_sched_counts.argtypes = [vp, i32p, i32p, i32p]
    lib.oppo_tuner_create.argtypes = [ctypes.c_int32, i32p, ctypes.c_int32, ctypes.POINTER(vp)]
    lib.oppo_tuner_destroy.argtypes = [vp]
    lib.oppo_tuner_chunk.argtypes = [vp, ctypes.c_int64, i32p]
    lib.oppo_tuner_report.argtypes = [vp, ctypes.c_int64, ctypes.c_double]
    lib.oppo_rope.argtypes = [ctypes.POINTER(AttnDesc), ctypes.c_int32, i32p, i32p, vp, vp, ctypes.c_double, vp]
    lib.oppo_rope.restype = ctypes.c_int
    lib.oppo_overlap_timeline.argtypes = [ctypes.c_int32, vp, vp, vp, vp, vp]
    lib.oppo_overlap_timeline.restype = ctypes.c_int
    for name in EXPORTS:
        if name.startswith(("oppo_pool_", "oppo_sched_", "oppo_tuner_")):
            getattr(lib, name).restype = ctypes.c_int
    lib.oppo_last_error.argtypes = []
    lib.oppo_last_error.restype = ctypes.c_char_p
    lib.oppo_version.argtypes = []
    lib.oppo_version.restype = ctypes.c_int
    _lib = lib
    return lib


def _check(rc: int) -> None:
    if rc != OPPO_OK:
        raise OppoError(rc, load().oppo_last_error().decode())


def _i32(a, n: Optional[int] = None) -> np.ndarray:
    arr = np.ascontiguousarray(a, dtype=np.int32)
    if n is not None and arr.shape != (n,):
        raise ValueError(f"expected int32 array of {n} entries, got shape {arr.shape}")
    return arr


def _i32p(arr: Optional[np.ndarray]):
    if arr is None:
        return None
    return arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _dev_ptr(t) -> Optional[int]:
    """Device address of a torch tensor (or None / a raw int address)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("device tensors must be contiguous")
    return t.data_ptr()


def _need(t, nbytes: int, name: str) -> None:
    """A device buffer handed to the library must hold at least `nbytes` and live on the GPU.
    The C ABI carries no sizes for device buffers, and an undersized one would be read or
    written out of bounds by a kernel, so it is refused here, where sizes are known.  Raw
    integer addresses cannot be checked and are taken as they are."""
    if t is None or isinstance(t, int) or nbytes <= 0:
        return
    have = t.numel() * t.element_size()
    if have < nbytes:
        raise ValueError(f"{name} holds {have} bytes, the call needs {nbytes}")
    if getattr(t, "is_cuda", True) is False:
        raise ValueError(f"{name} must be a device tensor")


def _need_cache(desc, cache, name: str = "cache") -> None:
    slots = int(cache.slot_begin[-1]) if len(cache.slot_begin) else 0
    nbytes = slots * desc.num_kv_heads * desc.head_dim * getattr(cache, "element_bytes", 2)
    _need(getattr(cache, "k", None), nbytes, f"{name}.k")
    _need(getattr(cache, "v", None), nbytes, f"{name}.v")


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def make_desc(num_q_heads: int, num_kv_heads: int, head_dim: int, softmax_scale: float) -> AttnDesc:
    return AttnDesc(num_q_heads, num_kv_heads, head_dim, softmax_scale)


class KVCache:
    """Caller-owned cache state: device slabs (torch tensors viewed as int16/bf16
    bit patterns [total_slots, Hkv, D]) plus the host length arrays the C struct
    points to.  kv_len is advanced by oppo_kv_append."""

    def __init__(self, k, v, slot_begin, kv_len=None):
        self.k = k
        self.v = v
        self.slot_begin = np.ascontiguousarray(slot_begin, dtype=np.int64)
        self.batch = self.slot_begin.shape[0] - 1
        self.kv_len = np.zeros(self.batch, dtype=np.int32) if kv_len is None else _i32(kv_len, self.batch).copy()
        self.struct = KVCacheStruct(_dev_ptr(k), _dev_ptr(v),
                                    self.slot_begin.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                    self.kv_len.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), self.batch)


class KVCacheFp8:
    """The cache in 8-bit codes: k is a byte tensor [total_slots, Hkv, D], v a byte tensor
    [total_slots / 64, Hkv, D, 64]; every slab starts on a multiple of 64 slots."""
    element_bytes = 1

    def __init__(self, k, v, slot_begin, k_scale: float, v_scale: float, kv_len=None):
        self.k = k
        self.v = v
        self.slot_begin = np.ascontiguousarray(slot_begin, dtype=np.int64)
        self.batch = self.slot_begin.shape[0] - 1
        self.kv_len = np.zeros(self.batch, dtype=np.int32) if kv_len is None else _i32(kv_len, self.batch).copy()
        self.k_scale, self.v_scale = float(k_scale), float(v_scale)
        self.struct = KVCacheFp8Struct(_dev_ptr(k), _dev_ptr(v),
                                       self.slot_begin.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                       self.kv_len.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), self.batch,
                                       self.k_scale, self.v_scale)


class SlotPool:
    """Handle of a library-owned slot pool (see oppo_pool_create)."""

    def __init__(self, handle: int, n_slots: int):
        self.handle = handle
        self.n_slots = n_slots


class PoolCache:
    """Cache view of a slot pool over caller-owned device slabs: usable wherever a
    KVCache is.  kv_len is the pool's own length array (not a copy)."""

    def __init__(self, k, v, struct: KVCacheStruct):
        self.k, self.v, self.struct = k, v, struct
        self.batch = struct.batch
        self.kv_len = np.ctypeslib.as_array(struct.kv_len, shape=(max(self.batch, 1),))[: self.batch]
        self.slot_begin = np.ctypeslib.as_array(struct.slot_begin, shape=(self.batch + 1,))


def oppo_pool_create(capacity) -> SlotPool:
    cap = _i32(capacity)
    h = ctypes.c_void_p()
    _check(load().oppo_pool_create(cap.shape[0], _i32p(cap), ctypes.byref(h)))
    return SlotPool(h.value, cap.shape[0])


def oppo_pool_destroy(pool: SlotPool) -> None:
    _check(load().oppo_pool_destroy(pool.handle))
    pool.handle = None


def oppo_pool_acquire(pool: SlotPool, seq_id: int, max_tokens: int) -> int:
    slot = ctypes.c_int32(-1)
    _check(load().oppo_pool_acquire(pool.handle, seq_id, max_tokens, ctypes.byref(slot)))
    return slot.value


def oppo_pool_release(pool: SlotPool, seq_id: int) -> None:
    _check(load().oppo_pool_release(pool.handle, seq_id))


def oppo_pool_slot_of(pool: SlotPool, seq_id: int) -> int:
    slot = ctypes.c_int32(-1)
    _check(load().oppo_pool_slot_of(pool.handle, seq_id, ctypes.byref(slot)))
    return slot.value


def oppo_pool_cache(pool: SlotPool, k, v) -> PoolCache:
    st = KVCacheStruct()
    _check(load().oppo_pool_cache(pool.handle, _dev_ptr(k), _dev_ptr(v), ctypes.byref(st)))
    return PoolCache(k, v, st)


def oppo_pool_pack(pool: SlotPool, seq_id, q_len):
    """Returns (cu_q[n_slots+1], row_begin[n]) as int32 numpy arrays."""
    ids = np.ascontiguousarray(seq_id, dtype=np.int64)
    ql = _i32(q_len, ids.shape[0])
    cu_q = np.empty(pool.n_slots + 1, dtype=np.int32)
    row_begin = np.empty(ids.shape[0], dtype=np.int32)
    _check(load().oppo_pool_pack(pool.handle, ids.shape[0], ids.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), _i32p(ql),
                                 _i32p(cu_q), _i32p(row_begin)))
    return cu_q, row_begin


def oppo_pool_counts(pool: SlotPool):
    """(n_slots, n_live, n_acquired, n_reused)."""
    a, b = ctypes.c_int32(0), ctypes.c_int32(0)
    c, d = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(load().oppo_pool_counts(pool.handle, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ctypes.byref(d)))
    return a.value, b.value, c.value, d.value


class Scheduler:
    """Handle of a library-owned Alg. 1 buffer (see oppo_sched_create)."""

    def __init__(self, handle: int, capacity: int):
        self.handle = handle
        self.max_n = capacity


def _i64p(arr: np.ndarray):
    return arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def oppo_sched_create(B: int, delta: int, C: int, max_capacity: Optional[int] = None) -> Scheduler:
    """max_capacity: the largest B + delta the handle's output arrays are sized for."""
    h = ctypes.c_void_p()
    _check(load().oppo_sched_create(B, delta, C, ctypes.byref(h)))
    return Scheduler(h.value, max(B + delta, max_capacity or 0))


def oppo_sched_destroy(s: Scheduler) -> None:
    _check(load().oppo_sched_destroy(s.handle))
    s.handle = None


def oppo_sched_set_delta(s: Scheduler, delta: int) -> None:
    _check(load().oppo_sched_set_delta(s.handle, delta))


def oppo_sched_room(s: Scheduler) -> int:
    n = ctypes.c_int32(0)
    _check(load().oppo_sched_room(s.handle, ctypes.byref(n)))
    return n.value


def oppo_sched_add(s: Scheduler, seq_id: int, prompt_len: int) -> None:
    _check(load().oppo_sched_add(s.handle, seq_id, prompt_len))


def oppo_sched_begin_pass(s: Scheduler):
    """Returns (kind, ids int64[n], kv_before int32[n], q_cap int32[n])."""
    ids = np.empty(s.max_n, dtype=np.int64)
    kvb = np.empty(s.max_n, dtype=np.int32)
    cap = np.empty(s.max_n, dtype=np.int32)
    n, kind = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(load().oppo_sched_begin_pass(s.handle, s.max_n, _i64p(ids), _i32p(kvb), _i32p(cap), ctypes.byref(n),
                                        ctypes.byref(kind)))
    return kind.value, ids[: n.value].copy(), kvb[: n.value].copy(), cap[: n.value].copy()


def oppo_sched_end_pass(s: Scheduler, ids, q_len, finished) -> None:
    i = np.ascontiguousarray(ids, dtype=np.int64)
    q = _i32(q_len, i.shape[0])
    f = np.ascontiguousarray(finished, dtype=np.uint8)
    if f.shape != i.shape:
        raise ValueError("finished must have one entry per sequence")
    _check(load().oppo_sched_end_pass(s.handle, i.shape[0], _i64p(i), _i32p(q),
                                      f.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))))


def oppo_sched_end_iteration(s: Scheduler) -> np.ndarray:
    """Ids that leave the buffer (the PPO batch), in finishing order."""
    out = np.empty(s.max_n, dtype=np.int64)
    n = ctypes.c_int32(0)
    _check(load().oppo_sched_end_iteration(s.handle, s.max_n, _i64p(out), ctypes.byref(n)))
    return out[: n.value].copy()


def oppo_sched_counts(s: Scheduler):
    """(sequences in the buffer, finished ones waiting, capacity B + delta)."""
    a, b, c = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int32(0)
    _check(load().oppo_sched_counts(s.handle, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
    return a.value, b.value, c.value


class ChunkTuner:
    """Handle of a library-owned chunk-size tuner (see oppo_tuner_create)."""

    def __init__(self, handle: int):
        self.handle = handle


def oppo_tuner_create(candidates, period: int) -> ChunkTuner:
    c = _i32(candidates)
    h = ctypes.c_void_p()
    _check(load().oppo_tuner_create(c.shape[0], _i32p(c), period, ctypes.byref(h)))
    return ChunkTuner(h.value)


def oppo_tuner_destroy(t: ChunkTuner) -> None:
    _check(load().oppo_tuner_destroy(t.handle))
    t.handle = None


def oppo_tuner_chunk(t: ChunkTuner, step: int) -> int:
    c = ctypes.c_int32(0)
    _check(load().oppo_tuner_chunk(t.handle, step, ctypes.byref(c)))
    return c.value


def oppo_tuner_report(t: ChunkTuner, step: int, seconds: float) -> None:
    _check(load().oppo_tuner_report(t.handle, step, seconds))


def oppo_rope(desc: AttnDesc, kv_before, cu_q, q, k_new, theta_base: float = 10000.0, stream=None) -> None:
    """Rotates the pass's query rows and new key rows in place (either may be None)."""
    cu = _i32(cu_q)
    kvb = _i32(kv_before, cu.shape[0] - 1)
    rows = int(cu[-1]) if cu.shape[0] else 0
    _need(q, rows * desc.num_q_heads * desc.head_dim * 2, "q")
    _need(k_new, rows * desc.num_kv_heads * desc.head_dim * 2, "k_new")
    _check(load().oppo_rope(ctypes.byref(desc), kvb.shape[0], _i32p(kvb), _i32p(cu), _dev_ptr(q), _dev_ptr(k_new),
                            float(theta_base), _stream_ptr(stream)))


def oppo_overlap_timeline(gen_s, score_s):
    """Returns (start_s, end_s, {"gen_end", "step_end", "exposed"}) of the scorer's work on each chunk."""
    g = np.ascontiguousarray(np.asarray(gen_s, dtype=np.float64))
    sc = np.ascontiguousarray(np.asarray(score_s, dtype=np.float64))
    if g.shape != sc.shape or g.ndim != 1:
        raise ValueError("gen_s and score_s must be 1-d arrays of one length")
    start, end, summary = np.zeros_like(g), np.zeros_like(g), np.zeros(3, dtype=np.float64)
    _check(load().oppo_overlap_timeline(g.shape[0], g.ctypes.data, sc.ctypes.data, start.ctypes.data,
                                        end.ctypes.data, summary.ctypes.data))
    return start, end, {"gen_end": float(summary[0]), "step_end": float(summary[1]), "exposed": float(summary[2])}


def oppo_version() -> int:
    return load().oppo_version()


def oppo_last_error() -> str:
    return load().oppo_last_error().decode()


def oppo_set_option(option: int, value: int) -> None:
    _check(load().oppo_set_option(option, value))


def oppo_profile_enable(on: bool) -> None:
    _check(load().oppo_profile_enable(1 if on else 0))


def oppo_profile_read():
    """({'attn','merge','append'} -> kernel milliseconds, same -> launch counts) since the last read."""
    ms = (ctypes.c_double * 3)()
    n = (ctypes.c_int32 * 3)()
    _check(load().oppo_profile_read(ms, n))
    names = ("attn", "merge", "append")
    return {k: ms[i] for i, k in enumerate(names)}, {k: n[i] for i, k in enumerate(names)}


def oppo_profile_read_each(max_n: int = 1 << 16):
    """(ms[n] float64, kind[n] int32: 0 attention, 1 merge, 2 append) of every launch since the last read, in launch order."""
    ms = np.zeros(max_n, dtype=np.float64)
    kind = np.zeros(max_n, dtype=np.int32)
    n = ctypes.c_int32(0)
    _check(load().oppo_profile_read_each(ms.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), _i32p(kind), max_n, ctypes.byref(n)))
    return ms[: n.value].copy(), kind[: n.value].copy()


def oppo_profile_host():
    """({'plan','launch'} -> host microseconds inside the attention entry points, number of calls) since the last read."""
    us = (ctypes.c_double * 2)()
    n = ctypes.c_int64(0)
    _check(load().oppo_profile_host(us, ctypes.byref(n)))
    return {"plan": us[0], "launch": us[1]}, n.value


def oppo_chunk_schedule(prompt_len, resp_len, C: int, t: int):
    """Returns (kv_before, q_len, cu_q) as int32 numpy arrays."""
    P = _i32(prompt_len)
    R = _i32(resp_len, P.shape[0])
    B = P.shape[0]
    kv_before = np.empty(B, dtype=np.int32)
    q_len = np.empty(B, dtype=np.int32)
    cu_q = np.empty(B + 1, dtype=np.int32)
    _check(load().oppo_chunk_schedule(B, _i32p(P), _i32p(R), C, t, _i32p(kv_before), _i32p(q_len), _i32p(cu_q)))
    return kv_before, q_len, cu_q


def oppo_workspace_bytes(desc: AttnDesc, max_batch: int, max_q_tokens: int) -> int:
    return int(load().oppo_workspace_bytes(ctypes.byref(desc), max_batch, max_q_tokens))


def _need_rows(desc: AttnDesc, cu: np.ndarray, **bufs) -> None:
    """q / out hold cu[-1] rows of Hq heads, k_new / v_new of Hkv heads, qkv of Hq + 2 Hkv."""
    rows = int(cu[-1]) if cu.shape[0] else 0
    heads = {"q": desc.num_q_heads, "out": desc.num_q_heads, "q_out": desc.num_q_heads, "k_new": desc.num_kv_heads,
             "v_new": desc.num_kv_heads, "qkv": desc.num_q_heads + 2 * desc.num_kv_heads}
    for name, t in bufs.items():
        _need(t, rows * heads[name] * desc.head_dim * 2, name)


def oppo_kv_append(desc: AttnDesc, cache: KVCache, cu_q, k_new, v_new, stream=None) -> None:
    cu = _i32(cu_q, cache.batch + 1)
    _need_rows(desc, cu, k_new=k_new, v_new=v_new)
    _need_cache(desc, cache)
    _check(load().oppo_kv_append(ctypes.byref(desc), ctypes.byref(cache.struct), _i32p(cu), _dev_ptr(k_new),
                                 _dev_ptr(v_new), _stream_ptr(stream)))


def oppo_qkv_rope_append(desc: AttnDesc, cache: KVCache, cu_q, qkv, q_out, theta_base: float = 10000.0, stream=None) -> None:
    """Epilogue of a fused QKV projection: rotated queries to q_out, rotated keys and values into the cache."""
    cu = _i32(cu_q, cache.batch + 1)
    _need_rows(desc, cu, qkv=qkv, q_out=q_out)
    _need_cache(desc, cache)
    _check(load().oppo_qkv_rope_append(ctypes.byref(desc), ctypes.byref(cache.struct), _i32p(cu), _dev_ptr(qkv),
                                       _dev_ptr(q_out), float(theta_base), _stream_ptr(stream)))


def oppo_qkv_proj_workspace_bytes(desc: AttnDesc, max_rows: int) -> int:
    return int(load().oppo_qkv_proj_workspace_bytes(ctypes.byref(desc), max_rows))


def oppo_qkv_proj_rope_append(desc: AttnDesc, cache: KVCache, cu_q, x, hidden: int, w, q_out, workspace,
                              theta_base: float = 10000.0, stream=None) -> None:
    """The fused QKV projection of a pass's hidden rows with the rotary embedding and the cache write as its epilogue."""
    cu = _i32(cu_q, cache.batch + 1)
    rows = int(cu[-1])
    _need(x, rows * hidden * 2, "x")
    _need(w, (desc.num_q_heads + 2 * desc.num_kv_heads) * desc.head_dim * hidden * 2, "w")
    _need_rows(desc, cu, q_out=q_out)
    _need_cache(desc, cache)
    _need(workspace, 1, "workspace")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().oppo_qkv_proj_rope_append(ctypes.byref(desc), ctypes.byref(cache.struct), _i32p(cu), _dev_ptr(x), hidden,
                                            _dev_ptr(w), _dev_ptr(q_out), float(theta_base), _dev_ptr(workspace), ws_bytes,
                                            _stream_ptr(stream)))


def oppo_chunk_prefill_attn(desc: AttnDesc, cache: KVCache, cu_q, q, out, workspace=None, stream=None) -> None:
    cu = _i32(cu_q, cache.batch + 1)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _need_rows(desc, cu, q=q, out=out)
    _need_cache(desc, cache)
    _need(workspace, 1, "workspace")
    _check(load().oppo_chunk_prefill_attn(ctypes.byref(desc), ctypes.byref(cache.struct), _i32p(cu), _dev_ptr(q),
                                          _dev_ptr(out), _dev_ptr(workspace), ws_bytes, _stream_ptr(stream)))


def oppo_chunk_step(desc: AttnDesc, cache: KVCache, cu_q, q, k_new, v_new, out, workspace=None, stream=None) -> None:
    cu = _i32(cu_q, cache.batch + 1)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _need_rows(desc, cu, q=q, k_new=k_new, v_new=v_new, out=out)
    _need_cache(desc, cache)
    _need(workspace, 1, "workspace")
    _check(load().oppo_chunk_step(ctypes.byref(desc), ctypes.byref(cache.struct), _i32p(cu), _dev_ptr(q),
                                  _dev_ptr(k_new), _dev_ptr(v_new), _dev_ptr(out), _dev_ptr(workspace), ws_bytes,
                                  _stream_ptr(stream)))


def oppo_kv_append_fp8(desc: AttnDesc, cache: KVCacheFp8, cu_q, k_new, v_new, stream=None) -> None:
    cu = _i32(cu_q, cache.batch + 1)
    _need_rows(desc, cu, k_new=k_new, v_new=v_new)
    _need_cache(desc, cache)
    _check(load().oppo_kv_append_fp8(ctypes.byref(desc), ctypes.byref(cache.struct), _i32p(cu), _dev_ptr(k_new),
                                     _dev_ptr(v_new), _stream_ptr(stream)))


def oppo_chunk_prefill_attn_fp8(desc: AttnDesc, cache: KVCacheFp8, cu_q, q, out, workspace=None, stream=None) -> None:
    cu = _i32(cu_q, cache.batch + 1)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _need_rows(desc, cu, q=q, out=out)
    _need_cache(desc, cache)
    _need(workspace, 1, "workspace")
    _check(load().oppo_chunk_prefill_attn_fp8(ctypes.byref(desc), ctypes.byref(cache.struct), _i32p(cu), _dev_ptr(q),
                                              _dev_ptr(out), _dev_ptr(workspace), ws_bytes, _stream_ptr(stream)))


def oppo_chunk_step_noalloc(desc: AttnDesc, cache: KVCache, cu_q, q, k_new, v_new, out, stream=None) -> None:
    """oppo_chunk_step with the library's built-in scratch buffer instead of a workspace."""
    cu = _i32(cu_q, cache.batch + 1)
    _need_rows(desc, cu, q=q, k_new=k_new, v_new=v_new, out=out)
    _need_cache(desc, cache)
    _check(load().oppo_chunk_step_noalloc(ctypes.byref(desc), ctypes.byref(cache.struct), _i32p(cu), _dev_ptr(q),
                                          _dev_ptr(k_new), _dev_ptr(v_new), _dev_ptr(out), _stream_ptr(stream)))


def oppo_static_scratch_bytes() -> int:
    return int(load().oppo_static_scratch_bytes())


def oppo_full_prefill_ref(desc: AttnDesc, cu_seq, q, k, v, out, workspace=None, stream=None) -> None:
    cu = _i32(cu_seq)
    B = cu.shape[0] - 1
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _need_rows(desc, cu, q=q, out=out, k_new=k, v_new=v)
    _need(workspace, 1, "workspace")
    _check(load().oppo_full_prefill_ref(ctypes.byref(desc), B, _i32p(cu), _dev_ptr(q), _dev_ptr(k), _dev_ptr(v),
                                        _dev_ptr(out), _dev_ptr(workspace), ws_bytes, _stream_ptr(stream)))


def oppo_plan_debug(desc: AttnDesc, kv_before, q_len, workspace_bytes: int, max_items: int = 1 << 16) -> np.ndarray:
    """Work list [n, 8] int32 the attention entry point would build (diagnostic)."""
    kvb = _i32(kv_before)
    ql = _i32(q_len, kvb.shape[0])
    items = np.zeros((max_items, 8), dtype=np.int32)
    n = ctypes.c_int32(0)
    _check(load().oppo_plan_debug(ctypes.byref(desc), kvb.shape[0], _i32p(kvb), _i32p(ql), workspace_bytes,
                                  items.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), max_items, ctypes.byref(n)))
    return items[: n.value].copy()
