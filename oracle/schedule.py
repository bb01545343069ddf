"""Which rows the scorer sees at each pass of the streaming loop (test oracle).

Alg. 1 (generation loop): every pass takes the unfinished sequences, the actor
produces up to C more tokens for each, and the scorer prefills the streamed
chunk on top of what it already processed (Sec. 3.1).  With final response
lengths R_i known, pass t therefore holds, for sequence i with prompt P_i,

    q_len_i     = min(C, max(0, R_i - t*C))      new rows (0 once finished)
    kv_before_i = P_i + min(R_i, t*C)            tokens already in its cache
"""
from __future__ import annotations

import numpy as np


def chunk_schedule(prompt_len, resp_len, chunk: int, t: int):
    """Returns (kv_before[B], q_len[B], cu_q[B+1]) as int64 arrays."""
    assert chunk >= 1 and t >= 0
    P = np.asarray(prompt_len, dtype=np.int64)
    R = np.asarray(resp_len, dtype=np.int64)
    kv_before = np.empty_like(P)
    q_len = np.empty_like(P)
    for i in range(P.shape[0]):
        done = min(int(R[i]), t * chunk)
        kv_before[i] = int(P[i]) + done
        q_len[i] = min(chunk, int(R[i]) - done)
    cu_q = np.zeros(P.shape[0] + 1, dtype=np.int64)
    for i in range(P.shape[0]):
        cu_q[i + 1] = cu_q[i] + q_len[i]
    return kv_before, q_len, cu_q


def num_steps(resp_len, chunk: int) -> int:
    """Passes until every sequence has streamed its whole response."""
    R = np.asarray(resp_len, dtype=np.int64)
    return int(max((int(r) + chunk - 1) // chunk for r in R)) if R.size else 0
