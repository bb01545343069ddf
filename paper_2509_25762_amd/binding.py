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
    "oppo_workspace_bytes", "oppo_set_option", "oppo_plan_debug", "oppo_last_error", "oppo_version",
    "oppo_profile_enable", "oppo_profile_read",
]


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


_lib = None


def load() -> ctypes.CDLL:
    """Loads the shared library (built by paper_2509_25762_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2509_25762_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    i32p = ctypes.POINTER(ctypes.c_int32)
    vp = ctypes.c_void_p
    lib.oppo_chunk_schedule.argtypes = [ctypes.c_int32, i32p, i32p, ctypes.c_int32, ctypes.c_int32, i32p, i32p, i32p]
    lib.oppo_chunk_schedule.restype = ctypes.c_int
    lib.oppo_kv_append.argtypes = [ctypes.POINTER(AttnDesc), ctypes.POINTER(KVCacheStruct), i32p, vp, vp, vp]
    lib.oppo_kv_append.restype = ctypes.c_int
    lib.oppo_chunk_prefill_attn.argtypes = [ctypes.POINTER(AttnDesc), ctypes.POINTER(KVCacheStruct), i32p, vp, vp,
                                            vp, ctypes.c_size_t, vp]
    lib.oppo_chunk_prefill_attn.restype = ctypes.c_int
    lib.oppo_chunk_step.argtypes = [ctypes.POINTER(AttnDesc), ctypes.POINTER(KVCacheStruct), i32p, vp, vp, vp, vp,
                                    vp, ctypes.c_size_t, vp]
    lib.oppo_chunk_step.restype = ctypes.c_int
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


def oppo_kv_append(desc: AttnDesc, cache: KVCache, cu_q, k_new, v_new, stream=None) -> None:
    cu = _i32(cu_q, cache.batch + 1)
    _check(load().oppo_kv_append(ctypes.byref(desc), ctypes.byref(cache.struct), _i32p(cu), _dev_ptr(k_new),
                                 _dev_ptr(v_new), _stream_ptr(stream)))


def oppo_chunk_prefill_attn(desc: AttnDesc, cache: KVCache, cu_q, q, out, workspace=None, stream=None) -> None:
    cu = _i32(cu_q, cache.batch + 1)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().oppo_chunk_prefill_attn(ctypes.byref(desc), ctypes.byref(cache.struct), _i32p(cu), _dev_ptr(q),
                                          _dev_ptr(out), _dev_ptr(workspace), ws_bytes, _stream_ptr(stream)))


def oppo_chunk_step(desc: AttnDesc, cache: KVCache, cu_q, q, k_new, v_new, out, workspace=None, stream=None) -> None:
    cu = _i32(cu_q, cache.batch + 1)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().oppo_chunk_step(ctypes.byref(desc), ctypes.byref(cache.struct), _i32p(cu), _dev_ptr(q),
                                  _dev_ptr(k_new), _dev_ptr(v_new), _dev_ptr(out), _dev_ptr(workspace), ws_bytes,
                                  _stream_ptr(stream)))


def oppo_full_prefill_ref(desc: AttnDesc, cu_seq, q, k, v, out, workspace=None, stream=None) -> None:
    cu = _i32(cu_seq)
    B = cu.shape[0] - 1
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
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
