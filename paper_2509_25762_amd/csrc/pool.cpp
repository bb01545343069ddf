// Slot pool: which sequence owns which slab of the persistent KV cache.
// Host-side bookkeeping only; the slabs are the caller's device memory.
// (Sec. 3.2, Alg. 1: the buffer holds B + Delta sequences; the B that finish
// first leave it, the others keep their cached state for the next iteration and
// new sequences take the places that were freed.)
#include <stdint.h>

#include <unordered_map>
#include <vector>

#include "../../include/oppo_attn.h"
#include "oppo_internal.h"

struct oppo_slot_pool {
  std::vector<int32_t> capacity;        // tokens per slot
  std::vector<int64_t> slot_begin;      // [n_slots + 1] prefix sums of capacity
  std::vector<int32_t> kv_len;          // [n_slots] tokens held; 0 for a free slot
  std::vector<int64_t> owner;           // [n_slots] sequence id, meaningful where live[slot]
  std::vector<uint8_t> live;            // [n_slots]
  std::vector<uint8_t> used_before;     // [n_slots] the slot has had an owner before
  std::unordered_map<int64_t, int32_t> slot_of;
  int64_t n_acquired = 0, n_reused = 0;
};

using oppo::fail;

extern "C" {

int oppo_pool_create(int32_t n_slots, const int32_t* capacity, oppo_slot_pool** pool) {
  if (!pool) return fail(OPPO_ERR_INVALID, "pool is null");
  *pool = nullptr;
  if (n_slots < 0) return fail(OPPO_ERR_INVALID, "n_slots=%d is negative", n_slots);
  if (n_slots > 0 && !capacity) return fail(OPPO_ERR_INVALID, "capacity is null");
  for (int32_t s = 0; s < n_slots; ++s)
    if (capacity[s] < 0) return fail(OPPO_ERR_INVALID, "capacity[%d]=%d is negative", s, capacity[s]);
  oppo_slot_pool* p = new oppo_slot_pool();
  p->capacity.assign(capacity, capacity + n_slots);
  p->slot_begin.assign((size_t)n_slots + 1, 0);
  for (int32_t s = 0; s < n_slots; ++s) p->slot_begin[s + 1] = p->slot_begin[s] + capacity[s];
  p->kv_len.reserve(1);   // (so that even an empty pool hands out a non-null length array)
  p->kv_len.assign((size_t)n_slots, 0);
  p->owner.assign((size_t)n_slots, 0);
  p->live.assign((size_t)n_slots, 0);
  p->used_before.assign((size_t)n_slots, 0);
  *pool = p;
  return OPPO_OK;
}

int oppo_pool_destroy(oppo_slot_pool* pool) {
  delete pool;
  return OPPO_OK;
}

int oppo_pool_acquire(oppo_slot_pool* pool, int64_t seq_id, int32_t max_tokens, int32_t* slot) {
  if (!pool || !slot) return fail(OPPO_ERR_INVALID, "pool or slot is null");
  if (max_tokens < 0) return fail(OPPO_ERR_INVALID, "max_tokens=%d is negative", max_tokens);
  if (pool->slot_of.count(seq_id)) return fail(OPPO_ERR_INVALID, "sequence %lld already owns slot %d", (long long)seq_id, pool->slot_of[seq_id]);
  int32_t best = -1;   // best fit: the smallest free slab that is large enough, the lowest index among equals
  for (int32_t s = 0; s < (int32_t)pool->capacity.size(); ++s)
    if (!pool->live[s] && pool->capacity[s] >= max_tokens && (best < 0 || pool->capacity[s] < pool->capacity[best])) best = s;
  if (best < 0) return fail(OPPO_ERR_CAPACITY, "no free slot holds %d tokens", max_tokens);
  pool->live[best] = 1;
  pool->owner[best] = seq_id;
  pool->kv_len[best] = 0;
  pool->slot_of[seq_id] = best;
  ++pool->n_acquired;
  if (pool->used_before[best]) ++pool->n_reused;
  pool->used_before[best] = 1;
  *slot = best;
  return OPPO_OK;
}

int oppo_pool_release(oppo_slot_pool* pool, int64_t seq_id) {
  if (!pool) return fail(OPPO_ERR_INVALID, "pool is null");
  auto it = pool->slot_of.find(seq_id);
  if (it == pool->slot_of.end()) return fail(OPPO_ERR_INVALID, "sequence %lld owns no slot", (long long)seq_id);
  pool->live[it->second] = 0;
  pool->kv_len[it->second] = 0;
  pool->slot_of.erase(it);
  return OPPO_OK;
}

int oppo_pool_slot_of(const oppo_slot_pool* pool, int64_t seq_id, int32_t* slot) {
  if (!pool || !slot) return fail(OPPO_ERR_INVALID, "pool or slot is null");
  auto it = pool->slot_of.find(seq_id);
  if (it == pool->slot_of.end()) return fail(OPPO_ERR_INVALID, "sequence %lld owns no slot", (long long)seq_id);
  *slot = it->second;
  return OPPO_OK;
}

int oppo_pool_cache(oppo_slot_pool* pool, void* k, void* v, oppo_kv_cache* cache) {
  if (!pool || !cache) return fail(OPPO_ERR_INVALID, "pool or cache is null");
  cache->k = k;
  cache->v = v;
  cache->slot_begin = pool->slot_begin.data();
  cache->kv_len = pool->kv_len.data();
  cache->batch = (int32_t)pool->capacity.size();
  return OPPO_OK;
}

int oppo_pool_pack(const oppo_slot_pool* pool, int32_t n, const int64_t* seq_id, const int32_t* q_len,
                   int32_t* cu_q, int32_t* row_begin) {
  if (!pool || !cu_q) return fail(OPPO_ERR_INVALID, "pool or cu_q is null");
  if (n < 0 || (n > 0 && (!seq_id || !q_len))) return fail(OPPO_ERR_INVALID, "bad sequence list (n=%d)", n);
  const int32_t S = (int32_t)pool->capacity.size();
  std::vector<int32_t> len((size_t)S, 0);
  std::vector<uint8_t> named((size_t)S, 0);
  std::vector<int32_t> where((size_t)n, 0);
  for (int32_t j = 0; j < n; ++j) {
    auto it = pool->slot_of.find(seq_id[j]);
    if (it == pool->slot_of.end()) return fail(OPPO_ERR_INVALID, "sequence %lld owns no slot", (long long)seq_id[j]);
    const int32_t s = it->second;
    if (named[s]) return fail(OPPO_ERR_INVALID, "sequence %lld is listed twice", (long long)seq_id[j]);
    if (q_len[j] < 0) return fail(OPPO_ERR_INVALID, "q_len[%d]=%d is negative", j, q_len[j]);
    if ((int64_t)pool->kv_len[s] + q_len[j] > pool->capacity[s])
      return fail(OPPO_ERR_CAPACITY, "sequence %lld: %d cached + %d new tokens exceed its slot of %d", (long long)seq_id[j],
                  pool->kv_len[s], q_len[j], pool->capacity[s]);
    named[s] = 1;
    len[s] = q_len[j];
    where[j] = s;
  }
  int64_t total = 0;
  for (int32_t s = 0; s < S; ++s) total += len[s];
  if (total > INT32_MAX) return fail(OPPO_ERR_INVALID, "%lld rows in one pass exceed the int32 range", (long long)total);
  cu_q[0] = 0;
  for (int32_t s = 0; s < S; ++s) cu_q[s + 1] = cu_q[s] + len[s];
  if (row_begin)
    for (int32_t j = 0; j < n; ++j) row_begin[j] = cu_q[where[j]];
  return OPPO_OK;
}

int oppo_pool_counts(const oppo_slot_pool* pool, int32_t* n_slots, int32_t* n_live, int64_t* n_acquired, int64_t* n_reused) {
  if (!pool) return fail(OPPO_ERR_INVALID, "pool is null");
  if (n_slots) *n_slots = (int32_t)pool->capacity.size();
  if (n_live) *n_live = (int32_t)pool->slot_of.size();
  if (n_acquired) *n_acquired = pool->n_acquired;
  if (n_reused) *n_reused = pool->n_reused;
  return OPPO_OK;
}

}  // extern "C"
