/*
 * oppo_attn.h - C ABI of the chunked-prefill attention library for MI355X (gfx950).
 *
 * The computation is the scorer's side of OPPO's intra-step overlap (Sec. 3.1 of
 * arXiv 2509.25762): while the actor is still decoding, the reward/critic model
 * prefills the response chunk by chunk.  For one attention layer that is, per
 * pass of the streaming loop (Alg. 1, generation loop) and per unfinished
 * sequence:
 *   1. append the chunk's K/V rows to the sequence's persistent cache, and
 *   2. let the chunk's query rows attend causally to the cached prefix plus the
 *      chunk itself.
 * Streaming must not change any result (Sec. 3.1, Eq. 3): any chunking gives the
 * outputs and the cache of a one-shot prefill.
 *
 * Conventions shared by every entry point
 *   - bf16 tensors are raw 16-bit patterns; "device" pointers are HIP device
 *     memory valid on the current device, "host" pointers ordinary host memory.
 *   - Length arrays are HOST memory and are snapshotted during the call: the
 *     caller may overwrite them as soon as the call returns, although the
 *     kernels run later on the stream.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work; they never synchronise and never allocate device
 *     memory.  All device buffers, the workspace included, belong to the caller
 *     and must stay alive until the enqueued work has run.
 *   - Return value: OPPO_OK or a negative oppo_status.  Every argument check
 *     happens on the host before anything is enqueued, so a failed call has
 *     written nothing and changed no length.  oppo_last_error() gives a
 *     human-readable reason (thread-local storage, valid until the next failing
 *     call on the same thread).
 *   - GQA: q-head h reads kv-head h / (num_q_heads / num_kv_heads).
 *   - Token-major layouts: a tensor [rows][H][D] stores row r, head h, element d
 *     at (r * H + h) * D + d.
 */
#ifndef OPPO_ATTN_H
#define OPPO_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  OPPO_OK = 0,
  OPPO_ERR_INVALID = -1,     /* null pointer, negative size, inconsistent lengths   */
  OPPO_ERR_UNSUPPORTED = -2, /* head_dim not 64/128, heads not divisible, group>16  */
  OPPO_ERR_CAPACITY = -3,    /* a chunk does not fit its sequence's cache slab      */
  OPPO_ERR_WORKSPACE = -4,   /* workspace given but smaller than required           */
  OPPO_ERR_HIP = -5          /* a HIP runtime call failed                           */
} oppo_status;

/* One attention layer of the scoring model. */
typedef struct {
  int32_t num_q_heads;   /* Hq                                            */
  int32_t num_kv_heads;  /* Hkv, divides Hq; Hq/Hkv <= 16                  */
  int32_t head_dim;      /* D, 64 or 128                                   */
  float softmax_scale;   /* s > 0, finite; the configs use 1/sqrt(D)       */
} oppo_attn_desc;

/*
 * Per-sequence KV state that persists across chunks (Sec. 3.1) and, for
 * sequences deferred by inter-step overlap, across training iterations
 * (Sec. 3.2; Alg. 1, Buffer.remove keeps unfinished sequences).
 * Sequence i owns token slots [slot_begin[i], slot_begin[i+1]); its token m
 * lives in slot slot_begin[i] + m for m < kv_len[i].  The caller owns
 * everything; a snapshot of the state is a copy of the slabs plus kv_len.
 */
typedef struct {
  void* k;                   /* device bf16 [total_slots][Hkv][D]                       */
  void* v;                   /* device bf16 [total_slots][Hkv][D]                       */
  const int64_t* slot_begin; /* host [batch+1], non-decreasing, slot_begin[0] >= 0      */
  int32_t* kv_len;           /* host [batch]; tokens valid in each slab; oppo_kv_append
                                advances it on success                                  */
  int32_t batch;             /* number of sequences (B, or B+Delta slots)               */
} oppo_kv_cache;

/*
 * Ragged descriptor of pass t of the streaming loop (Alg. 1, generation loop;
 * Sec. 3.1): with prompt lengths P_i, final response lengths R_i and chunk size
 * C, sequence i contributes q_len[i] = min(C, max(0, R_i - t*C)) new rows on top
 * of kv_before[i] = P_i + min(R_i, t*C) cached tokens; cu_q is the exclusive
 * prefix sum of q_len (cu_q[0] = 0).  All arrays are host memory; kv_before may
 * be NULL.  Pure host arithmetic, no GPU needed.
 * Errors: OPPO_ERR_INVALID for null arrays, B < 0, C < 1, t < 0, negative
 * lengths or sums that overflow int32.
 */
int oppo_chunk_schedule(int32_t B, const int32_t* prompt_len, const int32_t* resp_len,
                        int32_t C, int32_t t, int32_t* kv_before /* [B] or NULL */,
                        int32_t* q_len /* [B] */, int32_t* cu_q /* [B+1] */);

/*
 * Append one chunk per sequence to the cache (step 1 above; byte semantics).
 * For every i and j < q_len_i = cu_q[i+1]-cu_q[i], row cu_q[i]+j of k_new/v_new
 * (device bf16 [cu_q[B]][Hkv][D]) is copied bit for bit to slot
 * slot_begin[i] + kv_len[i] + j of cache->k / cache->v; no other byte of the
 * cache changes.  On success kv_len[i] += q_len_i (host side, immediately).
 * q_len_i = 0 is legal (finished or deferred sequence) and costs nothing.
 * Errors: INVALID (nulls, batch < 0, cu_q not non-decreasing from 0, bad
 * slot_begin/kv_len), UNSUPPORTED (desc), CAPACITY if any kv_len[i]+q_len_i
 * exceeds the slab - then nothing is enqueued and kv_len is unchanged.
 */
int oppo_kv_append(const oppo_attn_desc* desc, oppo_kv_cache* cache,
                   const int32_t* cu_q /* host [batch+1] */,
                   const void* k_new, const void* v_new, void* stream);

/*
 * Rotary position embedding of a pass's rows, in place: the step of the scorer's
 * attention layers that comes before the append and the attention (the paper is
 * silent on it; this is the published definition - Su et al., "RoFormer", Sec. 3.2
 * and 3.4.2 - in the half-split pairing of the Llama / Qwen families the paper
 * trains, Sec. 4.1).  Row j of sequence i's chunk sits at absolute position
 * p = kv_before[i] + j; with theta_t = theta_base^(-2 t / D), every pair
 * (x_t, x_{t + D/2}), t = 0 .. D/2 - 1, of every head of that row turns by
 * p * theta_t:  x_t' = x_t cos - x_{t+D/2} sin,  x_{t+D/2}' = x_{t+D/2} cos + x_t sin.
 * Because the angle depends on the absolute position only, keys rotated when their
 * chunk arrived stay valid in the cache for every later chunk (Sec. 3.1).
 *   kv_before : HOST int32[batch], tokens of each sequence before this pass.
 *   cu_q      : HOST int32[batch + 1], prefix sums of the pass's rows per sequence.
 *   q         : DEVICE bf16 [cu_q[batch]][Hq][D], rotated in place; null: skipped.
 *   k_new     : DEVICE bf16 [cu_q[batch]][Hkv][D], rotated in place; null: skipped.
 *   theta_base: > 1 (10000 in the original formulation).
 * Angles are formed in double precision, the rotation is fp32 with one rounding
 * to bf16.  The call enqueues on `stream` and returns; the host arrays may be
 * reused at once.  INVALID for null / malformed host arrays, negative lengths,
 * positions beyond 2^31, theta_base <= 1; UNSUPPORTED as for the descriptor.
 */
int oppo_rope(const oppo_attn_desc* desc, int32_t batch, const int32_t* kv_before, const int32_t* cu_q, void* q,
              void* k_new, double theta_base, void* stream);

/*
 * The rotation above as the epilogue of the layer's fused QKV projection, in one
 * pass over the projection's output: row r of `qkv` holds the Hq query heads, then
 * the Hkv key heads, then the Hkv value heads of one new token.  For row j of
 * sequence i (position p = kv_len[i] + j) the call writes the rotated queries to
 * q_out, the rotated keys and the unchanged values into the sequence's cache slab at
 * slot kv_len[i] + j, and then advances kv_len like oppo_kv_append does; what
 * follows is oppo_chunk_prefill_attn on q_out.  Compared with rotating in place and
 * appending, every byte of the projection's output is read once and written once.
 *   qkv   : DEVICE bf16 [cu_q[batch]][Hq + 2 Hkv][D], read only.
 *   q_out : DEVICE bf16 [cu_q[batch]][Hq][D].
 *   cache : as for oppo_kv_append (HOST length arrays, DEVICE slabs).
 * Values are copied bit for bit; queries and keys as for oppo_rope.  Errors as for
 * oppo_kv_append (a failed call writes nothing and leaves the lengths untouched),
 * and INVALID for theta_base <= 1.
 */
int oppo_qkv_rope_append(const oppo_attn_desc* desc, oppo_kv_cache* cache, const int32_t* cu_q, const void* qkv,
                         void* q_out, double theta_base, void* stream);

/*
 * The layer's fused QKV projection itself, with the call above as its epilogue: what
 * the scorer runs on a chunk's hidden rows before the attention (Alg. 1: the scorer's
 * prefill of the rows that arrived; the paper names no layer internals, this is the
 * attention block of the decoder-only model families it trains, Sec. 4.1).
 *     y[m, n] = sum_k x[m, k] * w[n, k]          (fp32 accumulation of bf16 products)
 * with output column n = head * D + d over [Hq query heads | Hkv key heads | Hkv value
 * heads]; query and key heads are then rotated as in oppo_rope at the row's position
 * kv_len[i] + j, on the fp32 sums, and rounded once to bf16; value heads are rounded as
 * they are.  Queries go to q_out, keys and values straight into the sequence's cache
 * slab at slot kv_len[i] + j; kv_len advances as in oppo_kv_append; what follows is
 * oppo_chunk_prefill_attn on q_out.  The projection's output never exists in memory.
 *   x       : DEVICE bf16 [cu_q[batch]][hidden], rows packed like q.
 *   w       : DEVICE bf16 [(Hq + 2 Hkv) * D][hidden] (output-major: y = x W^T).
 *   hidden  : multiple of 64 (otherwise UNSUPPORTED).
 *   q_out   : DEVICE bf16 [cu_q[batch]][Hq][D].
 *   workspace: DEVICE, 256-byte aligned, at least oppo_qkv_proj_workspace_bytes(desc,
 *             cu_q[batch]) bytes (per-row cache slots and rotation angles, written and
 *             read by this call only); WORKSPACE if missing or smaller.
 * Errors otherwise as for oppo_qkv_rope_append; a failed call writes nothing and leaves
 * the lengths untouched.
 */
size_t oppo_qkv_proj_workspace_bytes(const oppo_attn_desc* desc, int32_t max_rows);
int oppo_qkv_proj_rope_append(const oppo_attn_desc* desc, oppo_kv_cache* cache, const int32_t* cu_q,
                              const void* x, int32_t hidden, const void* w, void* q_out, double theta_base,
                              void* workspace, size_t workspace_bytes, void* stream);

/*
 * Chunked-prefill attention (step 2 above).  cache->kv_len is the length AFTER
 * the chunk was appended.  Row j of sequence i (row cu_q[i]+j of q and out,
 * device bf16 [cu_q[B]][Hq][D]) is the token at absolute position
 * n = kv_len[i] - q_len_i + j and receives
 *     out = softmax_m( s * <q, K_i[m]> ) . V_i[m]   over keys m = 0..n
 * (causal mask aligned to the end of the cache).  Scores and both contractions
 * accumulate in fp32 from bf16 inputs; out is rounded once to bf16
 * (nearest-even).  A prompt is prefilled by the same call with q_len_i = P_i on
 * an empty cache.
 * workspace: device scratch for splitting long key ranges across workgroups
 * (partial results merged by a second kernel).  NULL / 0 bytes disables
 * splitting; otherwise it must be 256-byte aligned and hold at least one partial
 * slot (256 x (D + 2) x Hkv floats).  oppo_workspace_bytes(desc, batch,
 * cu_q[batch]) is the size beyond which more does not help; a smaller one only
 * limits how many pieces key ranges are cut into, never what is computed.
 * Errors: INVALID (nulls, bad cu_q, q_len_i > kv_len[i], kv_len[i] beyond the
 * slab), UNSUPPORTED, WORKSPACE (misaligned, or smaller than one slot), HIP.
 */
int oppo_chunk_prefill_attn(const oppo_attn_desc* desc, const oppo_kv_cache* cache,
                            const int32_t* cu_q /* host [batch+1] */,
                            const void* q, void* out,
                            void* workspace, size_t workspace_bytes, void* stream);

/*
 * Steps 1 and 2 in one call and one kernel launch: appends the chunk's keys and
 * values to the cache (exactly as oppo_kv_append would) and computes the
 * chunk's attention rows (exactly as oppo_chunk_prefill_attn would afterwards:
 * the same bits in out and in the cache).  For callers that have the chunk's
 * q, k and v together, as a scoring model's layer does after its projections
 * (Sec. 3.1): it saves a launch and a pass over k_new / v_new per layer and
 * chunk.  cache->kv_len is the length BEFORE the chunk; on success
 * kv_len[i] += q_len_i.  k_new, v_new: device bf16 [cu_q[B]][Hkv][D], rows as in
 * q; the attention reads the chunk's own keys and values from them, and the
 * kernel writes them to their cache slots, which nothing reads before the
 * call's work has completed on the stream.
 * Errors: those of the two calls; on any error nothing is enqueued and kv_len
 * is unchanged.
 */
int oppo_chunk_step(const oppo_attn_desc* desc, oppo_kv_cache* cache,
                    const int32_t* cu_q /* host [batch+1] */,
                    const void* q, const void* k_new, const void* v_new, void* out,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * oppo_chunk_step for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, checks, results and length updates as
 * oppo_chunk_step, but the partial results of split key ranges go to a scratch
 * buffer built into the library (a device array of oppo_static_scratch_bytes()
 * = 64 MiB in the library's code object; every GPU the library runs on holds
 * its own copy until the process ends).  The call allocates no device memory,
 * creates no events (oppo_profile_enable does not time it) and frees nothing;
 * the buffer's address on the current device is looked up on the first call
 * on that device.
 * Limit: the buffer must hold the partial results of one fully split query tile,
 * 32 x 256 x (D + 2) x Hkv floats, i.e. Hkv x (D + 2) <= 2048 (D = 128: up to 15
 * kv-heads, D = 64: up to 31); wider layers get OPPO_ERR_UNSUPPORTED and the
 * message says so.  Within the limit the buffer only bounds how finely key
 * ranges are cut (63 slots for Hkv = 8, D = 128).
 * All calls on one GPU share the one buffer and nothing in it needs clearing
 * (every partial row is written before it is read), but two calls whose work
 * overlaps in time on one GPU - different streams, or different host threads -
 * race on it: callers serialise them, e.g. by using one stream.
 */
int oppo_chunk_step_noalloc(const oppo_attn_desc* desc, oppo_kv_cache* cache,
                            const int32_t* cu_q /* host [batch+1] */,
                            const void* q, const void* k_new, const void* v_new, void* out,
                            void* stream);
size_t oppo_static_scratch_bytes(void);

/*
 * The KV cache in 8 bits per element.  The scorer re-reads every live sequence's whole
 * cache at each pass of the streaming loop (Sec. 3.1), so with small chunks a pass is bound
 * by the bytes of K and V; this variant halves them.  The paper does not say how the cache
 * is stored; what follows is this library's definition.
 *   format : OCP FP8 E4M3 (1 sign, 4 exponent bits of bias 7, 3 mantissa bits; no
 *            infinities; largest finite value 448; subnormals are multiples of 2^-9).
 *   scales : one positive finite float per tensor (k_scale, v_scale), chosen by the caller
 *            (e.g. the largest magnitude expected / 448).  A bf16 value x is stored as the
 *            code nearest (ties to even) to clamp(fl32(x * fl32(1 / scale)), -448, 448);
 *            a code stands for code_value * scale.  NaN inputs are not supported.
 *   layout : keys token-major like the 16-bit cache, one byte per element,
 *            k[slot][Hkv][D]; values in blocks of 64 tokens with the token index fastest,
 *            v[slot / 64][Hkv][D][slot % 64] (the order in which the second product of
 *            attention contracts them).  Every slot_begin[i] is a multiple of 64.
 */
typedef struct {
  void* k;                   /* device bytes [total_slots][Hkv][D]                      */
  void* v;                   /* device bytes [total_slots / 64][Hkv][D][64]             */
  const int64_t* slot_begin; /* host [batch+1], non-decreasing multiples of 64         */
  int32_t* kv_len;           /* host [batch], as in oppo_kv_cache                      */
  int32_t batch;
  float k_scale;             /* > 0, finite                                            */
  float v_scale;             /* > 0, finite                                            */
} oppo_kv_cache_fp8;

/*
 * oppo_kv_append into the 8-bit cache: rows of k_new / v_new (device bf16
 * [cu_q[B]][Hkv][D]) are turned into codes as defined above and written to the slots
 * slot_begin[i] + kv_len[i] + j.  Of the value blocks, the bytes of the new tokens are
 * written, the bytes of earlier tokens are kept, and what is left of the last block a
 * sequence's chunk touches is set to zero bytes (so a block never holds anything but
 * codes and zeros, whatever the memory held before); no other byte changes.  The codes
 * of a token do not depend on the chunk it arrived in, so streaming-equivalence
 * (Sec. 3.1, Eq. 3) holds for them bit for bit.  On success kv_len[i] += q_len_i.
 * Errors: as oppo_kv_append, and INVALID for scales that are not positive and finite or
 * a slot_begin entry that is not a multiple of 64.
 */
int oppo_kv_append_fp8(const oppo_attn_desc* desc, oppo_kv_cache_fp8* cache,
                       const int32_t* cu_q /* host [batch+1] */,
                       const void* k_new, const void* v_new, void* stream);

/*
 * oppo_chunk_prefill_attn over the 8-bit cache: out = causal attention of the chunk's
 * queries (device bf16, rows as in cu_q) over the values the cached codes stand for,
 * out device bf16.  Both matrix products run on the 8-bit matrix instructions with fp32
 * accumulation: the kernel rounds the queries and the softmax weights to E4M3 on the fly
 * (the weights relative to a per-row reference, so that they use the format's normal
 * range); keys and values enter exactly as stored.  The result therefore differs from
 * exact attention over the stored values by the rounding of queries and weights - a few
 * percent of a value's magnitude per element for short rows, less for long ones - on top
 * of the error of storing K and V in 8 bits.  Workspace rules as oppo_chunk_prefill_attn.
 * Errors: as oppo_chunk_prefill_attn; INVALID for bad scales (softmax_scale x k_scale must
 * lie within 2^-100 .. 2^100) or slab starts that are not multiples of 64.
 */
int oppo_chunk_prefill_attn_fp8(const oppo_attn_desc* desc, const oppo_kv_cache_fp8* cache,
                                const int32_t* cu_q /* host [batch+1] */,
                                const void* q, void* out,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * One-shot causal prefill of whole sequences, without a cache: the reference
 * side of the streaming-equivalence invariant (Sec. 3.1, Eq. 3) on the device.
 * Sequence i owns rows [cu_seq[i], cu_seq[i+1]) of q/out (device bf16
 * [cu_seq[B]][Hq][D]) and of k/v (device bf16 [cu_seq[B]][Hkv][D]); row n of a
 * sequence sees its keys 0..n.  Same arithmetic and workspace rules as
 * oppo_chunk_prefill_attn.
 */
int oppo_full_prefill_ref(const oppo_attn_desc* desc, int32_t B,
                          const int32_t* cu_seq /* host [B+1] */,
                          const void* q, const void* k, const void* v, void* out,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * Slot pool: which sequence owns which slab of the persistent cache (Sec. 3.2;
 * Alg. 1: the buffer holds B + Delta sequences, `Buffer.remove` takes out the B
 * that finished first, the unfinished ones keep their cached state for the next
 * iteration, and stage 1 fills the freed places with new sequences).
 * The pool is host-side bookkeeping only: it never touches device memory and
 * needs no GPU.  A pool has a fixed set of slots with capacities in tokens; the
 * slabs are laid out back to back in that order (slot s starts at token slot
 * capacity[0] + ... + capacity[s-1] of the caller's k / v arrays).  A slot is
 * free or owned by one sequence, named by a caller-chosen 64-bit id.
 * The pool object is owned by the library (create / destroy); it is not
 * thread-safe.  All arrays in these calls are HOST memory.
 *
 * oppo_pool_create   : n_slots >= 0 slots, capacity[s] >= 0 tokens each.
 * oppo_pool_destroy  : frees the pool (NULL is allowed).  A cache view made
 *                      from it (see oppo_pool_cache) dangles afterwards.
 * oppo_pool_acquire  : Buffer.add - gives `seq_id` the free slot with the smallest
 *                      capacity >= max_tokens (lowest index among equals), sets
 *                      its length to 0 and writes the slot index.  INVALID if the
 *                      id already owns a slot, CAPACITY if no free slot is large
 *                      enough; then nothing changes.
 * oppo_pool_release  : Buffer.remove - the sequence's slot becomes free, its
 *                      length 0.  The slab's bytes are left as they are: nothing
 *                      reads a slot beyond its length.  INVALID for an unknown id.
 * oppo_pool_slot_of  : the slot of a live sequence; INVALID for an unknown id.
 * oppo_pool_cache    : fills *cache with a view of the pool over the caller's
 *                      device arrays k, v (bf16 [sum of capacities][Hkv][D]):
 *                      slot_begin and kv_len point into the pool, batch =
 *                      n_slots.  oppo_kv_append / oppo_chunk_step advance the
 *                      pool's lengths through it.  Valid until oppo_pool_destroy.
 * oppo_pool_pack     : the ragged descriptor of one pass.  seq_id[n] are distinct
 *                      live sequences, q_len[n] >= 0 their new rows; sequences
 *                      that are not listed sit the pass out.  Writes cu_q
 *                      [n_slots+1] (prefix sums of the per-slot row counts: rows
 *                      are packed in slot order) and, if row_begin is not NULL,
 *                      row_begin[j] = first row of sequence seq_id[j] in q / k_new
 *                      / v_new / out.  INVALID for unknown or repeated ids,
 *                      negative lengths or more than INT32_MAX rows; CAPACITY if a
 *                      sequence's cached + new tokens exceed its slot.
 * oppo_pool_counts   : slots, live sequences, acquisitions so far and how many
 *                      of those took a slot that had an owner before (any pointer
 *                      may be NULL).
 */
typedef struct oppo_slot_pool oppo_slot_pool;
int oppo_pool_create(int32_t n_slots, const int32_t* capacity /* [n_slots] */, oppo_slot_pool** pool);
int oppo_pool_destroy(oppo_slot_pool* pool);
int oppo_pool_acquire(oppo_slot_pool* pool, int64_t seq_id, int32_t max_tokens, int32_t* slot);
int oppo_pool_release(oppo_slot_pool* pool, int64_t seq_id);
int oppo_pool_slot_of(const oppo_slot_pool* pool, int64_t seq_id, int32_t* slot);
int oppo_pool_cache(oppo_slot_pool* pool, void* k, void* v, oppo_kv_cache* cache);
int oppo_pool_pack(const oppo_slot_pool* pool, int32_t n, const int64_t* seq_id /* [n] */,
                   const int32_t* q_len /* [n] */, int32_t* cu_q /* [n_slots+1] */,
                   int32_t* row_begin /* [n] or NULL */);
int oppo_pool_counts(const oppo_slot_pool* pool, int32_t* n_slots, int32_t* n_live,
                     int64_t* n_acquired, int64_t* n_reused);

/*
 * The buffer of Alg. 1 (Sec. 3.2) as a host-side state machine: it decides which
 * sequences the scorer serves in which pass and which sequences leave after an
 * iteration.  It knows nothing about devices; together with a slot pool it
 * drives oppo_chunk_step.  One training iteration is
 *
 *   stage 1   oppo_sched_room, then oppo_sched_add for each new sequence;
 *   stage 2   loop { oppo_sched_begin_pass -> run the pass -> oppo_sched_end_pass }
 *             until begin_pass reports OPPO_PASS_NONE;
 *   stage 3   oppo_sched_end_iteration: the first B finished sequences leave.
 *
 * The buffer is first-in first-out and holds at most B + delta sequences.
 * begin_pass hands out, in buffer order,
 *   OPPO_PASS_PROMPT : the sequences added since the last pass, each with
 *                      kv_before 0 and q_cap = its prompt length (the scorer
 *                      prefills a prompt when the sequence enters);
 *   OPPO_PASS_CHUNK  : every unfinished sequence with kv_before = prompt +
 *                      response tokens streamed so far and q_cap = C - as long as
 *                      fewer than B sequences have finished and some sequence is
 *                      unfinished (Alg. 1, generation loop);
 *   OPPO_PASS_NONE   : stage 2 is over.
 * end_pass takes what the actor produced for exactly those sequences, in the
 * same order: q_len[j] new tokens (the whole prompt in a prompt pass; 0..C in a
 * chunk pass, and fewer than C only if the sequence ends) and finished[j] != 0 if
 * the sequence has ended.  Sequences are recorded as finished in pass order and,
 * within a pass, in buffer order; a finished sequence that is not among the B
 * removed ones stays in the buffer and is first in line at the next iteration.
 * end_iteration writes the ids that leave (at most B) and removes them; the
 * caller releases their slots.  oppo_sched_set_delta is Buffer.set_capacity: it
 * takes effect at the next stage 1 (a smaller capacity removes nobody).
 * Errors: INVALID for calls out of order, unknown or misordered ids, lengths out
 * of range; CAPACITY when adding to a full buffer.  A failed call changes nothing.
 * All arrays are HOST memory; the object is not thread-safe.
 */
typedef struct oppo_scheduler oppo_scheduler;
typedef enum { OPPO_PASS_NONE = 0, OPPO_PASS_PROMPT = 1, OPPO_PASS_CHUNK = 2 } oppo_pass_kind;
int oppo_sched_create(int32_t B, int32_t delta, int32_t C, oppo_scheduler** sched);
int oppo_sched_destroy(oppo_scheduler* sched);
int oppo_sched_set_delta(oppo_scheduler* sched, int32_t delta);
int oppo_sched_room(const oppo_scheduler* sched, int32_t* n);
int oppo_sched_add(oppo_scheduler* sched, int64_t seq_id, int32_t prompt_len);
int oppo_sched_begin_pass(oppo_scheduler* sched, int32_t max_n, int64_t* ids /* [max_n] */,
                          int32_t* kv_before /* [max_n] */, int32_t* q_cap /* [max_n] */,
                          int32_t* n, int32_t* kind);
int oppo_sched_end_pass(oppo_scheduler* sched, int32_t n, const int64_t* ids /* [n] */,
                        const int32_t* q_len /* [n] */, const uint8_t* finished /* [n] */);
int oppo_sched_end_iteration(oppo_scheduler* sched, int32_t max_n, int64_t* removed /* [max_n] */,
                             int32_t* n_removed);
int oppo_sched_counts(const oppo_scheduler* sched, int32_t* in_buffer, int32_t* finished_waiting,
                      int32_t* capacity);

/*
 * Periodic search for the chunk size C (Sec. 3.1, "Dynamic Control on Intra-step
 * Overlap"): training steps are numbered 0, 1, 2, ...; every `period` steps a
 * window starts whose first steps try the candidates, one step each, in the
 * order given (at most `period` of them); every later step of the window uses
 * the candidate whose trial step of this window was reported fastest (the first
 * listed among equals; a trial without a report counts as infinitely slow).
 * oppo_tuner_chunk  : the chunk size for training step `step`.
 * oppo_tuner_report : the wall time of a finished step, in seconds (>= 0).
 * Host-side state machine, no GPU; not thread-safe.  INVALID for null pointers,
 * no candidates, candidates < 1, period < 1, negative steps or times.
 */
typedef struct oppo_chunk_tuner oppo_chunk_tuner;
int oppo_tuner_create(int32_t n, const int32_t* candidates /* [n] */, int32_t period, oppo_chunk_tuner** tuner);
int oppo_tuner_destroy(oppo_chunk_tuner* tuner);
int oppo_tuner_chunk(const oppo_chunk_tuner* tuner, int64_t step, int32_t* chunk);
int oppo_tuner_report(oppo_chunk_tuner* tuner, int64_t step, double seconds);

/*
 * Timeline of intra-step overlap (Sec. 3.1): the actor decodes its chunks back to
 * back from time 0, chunk k taking gen_s[k]; the scorer takes the chunks in order,
 * one at a time, chunk k taking score_s[k], and starts chunk k once the actor has
 * completed it and chunk k-1 has been scored.  Writes when the scorer starts and
 * ends each chunk; summary[0] = end of generation, summary[1] = end of the step
 * (the later of the two sides), summary[2] = exposed scoring time (end of step
 * minus end of generation).  Feeding it measured pass times of the scorer and the
 * decode times of the generating side turns kernel time into the quantity the
 * technique is about: scoring latency hidden behind generation.
 * All arrays are HOST memory, n_chunks entries each (summary: 3), caller-owned;
 * start_s / end_s may be null.  n_chunks = 0 gives an all-zero summary.
 * INVALID for a negative count, null inputs or summary, negative or NaN times.
 */
int oppo_overlap_timeline(int32_t n_chunks, const double* gen_s, const double* score_s,
                          double* start_s, double* end_s, double* summary /* [3] */);

/*
 * Bytes of workspace beyond which the attention entry points have no use for
 * more, for any call with at most max_batch sequences and max_q_tokens query
 * rows in total: one partial slot per piece that the planner may cut (bounded
 * by the chip: a few per compute unit; and by the work: at most 32 pieces per
 * query tile of 256 / (Hq / Hkv) tokens).  Returns 0 for an unsupported desc,
 * negative sizes, or when there is nothing to split.
 */
size_t oppo_workspace_bytes(const oppo_attn_desc* desc, int32_t max_batch, int32_t max_q_tokens);

/*
 * Tuning knobs, process-wide.  Every entry point takes one snapshot of them when
 * it starts (under a lock), so setting them from another thread never changes a
 * call half-way.  They change how work is cut and ordered, never what is
 * computed; tests use them to show that results do not depend on the cut.
 *   OPPO_OPT_SPLIT_KV : 0 = automatic (default: key ranges are cut where that
 *                       evens out the load of the persistent workgroups),
 *                       1 = never split, n >= 2 = cut every key range into up
 *                       to n pieces when a workspace is given.
 *   OPPO_OPT_ORDER    : order of the pieces within a workgroup's queue:
 *                       0 = as scheduled (default: sequences with the most
 *                       work first), 1 = input order, 2 = shortest first.
 *   OPPO_OPT_NUM_CUS  : compute units the planner fills (default 256); the
 *                       attention launch has num_cus / Hkv workgroups (queues)
 *                       per kv-head, at least 1 and at most 256.
 * Returns OPPO_ERR_INVALID for an unknown option or a negative value.
 */
typedef enum {
  OPPO_OPT_SPLIT_KV = 0,
  OPPO_OPT_ORDER = 1,
  OPPO_OPT_NUM_CUS = 2
} oppo_option;
int oppo_set_option(int option, int value);

/*
 * Diagnostic: the work list oppo_chunk_prefill_attn would build for a pass whose
 * sequences have kv_before[i] cached tokens and q_len[i] new rows (host arrays
 * [B]), given workspace_bytes of workspace.  Nothing is enqueued; no GPU needed.
 * items receives 8 int32 per piece of work, grouped by queue and in the order
 * a queue's workgroup runs them:
 *   {sequence index, first q row, tokens in tile, position of first token,
 *    first key, one past last key, partial slot or -1, queue}
 * n_items receives the count; OPPO_ERR_INVALID if it exceeds max_items.
 * Every queue exists once per kv-head at launch.
 */
int oppo_plan_debug(const oppo_attn_desc* desc, int32_t B, const int32_t* kv_before, const int32_t* q_len,
                    size_t workspace_bytes, int32_t* items /* [max_items][8] */, int32_t max_items,
                    int32_t* n_items);

/*
 * Per-kernel timing for benchmarks.  While enabled, every kernel launch of the
 * library is bracketed by two HIP events recorded on the launch stream (this
 * costs a little, so leave it off in production).  oppo_profile_read waits for
 * the recorded events, writes the summed kernel time in milliseconds and the
 * number of launches since the last read into kernel_ms[3] / launches[3]
 * (host arrays; index 0 = attention kernel, 1 = split-KV merge kernel,
 * 2 = append kernel) and forgets them.  The list of events is shared by all
 * threads (guarded by a lock): a read collects every thread's launches.
 * oppo_profile_read_each does the same but hands out every launch's own duration
 * (each_ms[i], milliseconds) and kind (each_kind[i], numbered as above) in launch
 * order, *n of them; INVALID (after forgetting them all the same) if more than
 * max_n launches were recorded.
 * oppo_profile_host reports what the attention entry points cost on the host
 * while profiling was enabled, summed since the last read: host_us[0] =
 * microseconds spent planning (cutting the pass into pieces and queues),
 * host_us[1] = microseconds spent launching (argument marshalling and the
 * runtime's launch calls), *calls = number of entry-point calls counted.
 */
int oppo_profile_enable(int on);
int oppo_profile_read(double* kernel_ms /* [3] */, int32_t* launches /* [3] */);
int oppo_profile_read_each(double* each_ms /* [max_n] */, int32_t* each_kind /* [max_n] */, int32_t max_n, int32_t* n);
int oppo_profile_host(double* host_us /* [2] */, int64_t* calls);

/* Reason of the last failing call on this thread ("" if none). */
const char* oppo_last_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int oppo_version(void);

#ifdef __cplusplus
}
#endif
#endif /* OPPO_ATTN_H */
