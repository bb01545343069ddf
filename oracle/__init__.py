"""CPU oracle for ragged chunked-prefill attention with a persistent KV cache.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this
package: only tests, the smoke check and the benchmark's CPU-baseline leg use
it.  It shares no code with the HIP library and never imports it.

What it states (float64 throughout, inputs are bf16 bit patterns widened
exactly):
  * attention.py  - softmax(s * Q K^T + causal mask) V written out as the plain
                    definition, for arbitrary query positions (so one-shot
                    prefill, a streamed chunk, or single sampled rows are all
                    the same function with different position lists);
  * kv_cache.py   - the per-sequence cache that persists across chunks
                    (Sec. 3.1: the scorer processes chunk k-1 on top of the
                    chunks before it) and the streamed episode built on it;
  * schedule.py   - which rows exist at each pass of the streaming loop
                    (Alg. 1, generation loop; Sec. 3.1);
  * deferral.py   - Alg. 1's buffer of B + Delta sequences over several training
                    iterations (Sec. 3.2): which sequences enter, stream, sit
                    out, leave and carry their cache over, pass by pass;
  * tuner.py      - the periodic search over candidate chunk sizes (Sec. 3.1);
  * rope.py       - the rotary position embedding of a pass's query and key rows at
                    their absolute positions (the published definition; the paper is
                    silent on it), the step before append and attention in the scorer's
                    layers;
  * projection.py - the layer's fused QKV projection (y = x W^T, columns laid out as query,
                    key, value heads) and the rotary embedding that follows it: the step
                    of Alg. 1's prefill that produces what the cache and the attention take;
  * fp8_cache.py  - the cache in 8-bit floating point (OCP E4M3 codes under per-tensor scales, keys
                    token-major, values in blocks of 64 tokens), its append and the attention
                    over the values the codes stand for;
  * overlap.py    - the timeline of intra-step overlap (Sec. 3.1): when the scorer
                    works on which chunk while the actor decodes the next one, and
                    how much scoring time stays exposed at the end of the step.

Pins (tests/test_oracle_*.py): brute-force triple loop on tiny inputs, a
hand-derived two/three-token example with rational softmax weights
(tests/golden), closed forms (V==1, Q==0 -> running mean, first token,
dominant key), the streaming-equivalence invariant of Sec. 3.1 / Eq. 3 (any
chunking equals one-shot prefill, cache included), causality under
perturbation of future tokens, GQA / batch-permutation / V-linearity
invariants, and an independent float64 library routine.  The append is pinned
by a full-buffer compare against a numpy scatter with sentinels.  The buffer
model is pinned by a hand-worked trace of Alg. 1 (tests/golden), by its Delta = 0
case, which must be the plain streaming schedule, and by the invariants the
paper states (capacity, first B finishers leave, nobody starves, no token is
recomputed or skipped); the tuner by a hand-worked run and by the argmin
property over random step times; the overlap timeline by hand-worked cases
(tests/golden), a tick-by-tick simulation on integer durations and its closed
forms (a scorer that keeps up exposes only the last chunk; one that never
idles ends at gen[0] + sum(score)); the rotary embedding by a hand-worked row
(tests/golden), the complex-number form through an independent routine, and its
defining properties (identity at position 0, additivity, scores that depend on
relative position only); the projection by a triple loop on tiny inputs, a hand-worked
example (tests/golden), selector weights that must copy given input columns into given
heads (which pins the operand order and the head layout) and linearity; the 8-bit cache by
hand-derived codes of the format (tests/golden), the round trip over all 256 codes, an
independent library conversion, the half-step error bound, its layout written out element by
element and the streaming invariant through it.  No function here is "parity unpinned".
"""
from .attention import bf16_bits_to_f64, causal_attention, full_prefill, attention_row
from .kv_cache import KVCacheOracle, CapacityError, stream_episode
from .schedule import chunk_schedule, num_steps
from .deferral import simulate as simulate_alg1_buffer, dense_descriptor
from .tuner import ChunkTunerOracle, run_tuner
from .overlap import timeline as overlap_timeline, sequential_step
from .rope import rope_rotate, pass_positions
from .projection import qkv_projection, qkv_projection_rope

__all__ = [
    "bf16_bits_to_f64", "causal_attention", "full_prefill", "attention_row",
    "KVCacheOracle", "CapacityError", "stream_episode", "chunk_schedule", "num_steps",
    "simulate_alg1_buffer", "dense_descriptor", "ChunkTunerOracle", "run_tuner",
    "overlap_timeline", "sequential_step", "rope_rotate", "pass_positions",
    "qkv_projection", "qkv_projection_rope",
]
