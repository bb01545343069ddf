"""Chunked-prefill attention with a persistent KV cache for MI355X (gfx950).

`binding` holds the ctypes wrappers of the C ABI (include/oppo_attn.h);
`workload` the seeded synthetic inputs; `build` compiles the library in-tree.
Nothing here computes attention on the host: without the built HIP library the
binding raises.
"""
from . import workload  # noqa: F401

__all__ = ["workload", "binding", "build"]
