// Test program for the host half of the library (argument checks, work planner, slot
// pool, scheduler), built by paper_2509_25762_amd.build.build_host_checked() together
// with the host sources and launcher stand-ins under AddressSanitizer and
// UndefinedBehaviorSanitizer.  It needs no GPU: the stand-ins check every work list the
// entry points would launch and launch nothing.  Exit status 0 = every check passed and
// the sanitizers stayed silent.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <algorithm>
#include <map>
#include <random>
#include <set>
#include <vector>

#include "../include/oppo_attn.h"

static int g_failed = 0;
#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      fprintf(stderr, "%s:%d: check failed: %s (last error: %s)\n", __FILE__, __LINE__, #cond, oppo_last_error()); \
      ++g_failed;                                                          \
    }                                                                      \
  } while (0)

static void* fake(uintptr_t a) { return (void*)a; }   // a "device address" nothing dereferences on the host

// Every (sequence, query tile) has its key range covered exactly once by pieces on 64-key
// boundaries; pieces of a split tile own distinct partial slots below the number of slots the
// workspace has; whole tiles write final rows; queues are numbered without gaps.
static void check_plan(int G, const std::vector<int32_t>& kvb, const std::vector<int32_t>& ql,
                       const std::vector<int32_t>& items, int n, size_t slots, int queues_per_launch) {
  const int TM = 256 / G;
  struct P { int k0, k1, part, n_tok, pos0; };
  std::map<std::pair<int, int>, std::vector<P>> by_tile;
  int prev_queue = -1;
  for (int i = 0; i < n; ++i) {
    const int32_t* o = &items[8 * (size_t)i];
    by_tile[{o[0], o[1]}].push_back(P{o[4], o[5], o[6], o[2], o[3]});
    CHECK(o[7] == prev_queue || o[7] == prev_queue + 1);
    prev_queue = o[7];
  }
  (void)queues_per_launch;
  std::set<int> parts;
  size_t want_tiles = 0;
  int64_t row = 0;
  for (size_t s = 0; s < kvb.size(); ++s) {
    for (int j0 = 0; j0 < ql[s]; j0 += TM) {
      ++want_tiles;
      auto it = by_tile.find({(int)s, (int)(row + j0)});
      CHECK(it != by_tile.end());
      if (it == by_tile.end()) continue;
      std::vector<P>& v = it->second;
      std::sort(v.begin(), v.end(), [](const P& a, const P& b) { return a.k0 < b.k0; });
      const int n_tok = std::min(TM, ql[s] - j0);
      CHECK(v.front().k0 == 0 && v.back().k1 == kvb[s] + j0 + n_tok);
      for (size_t k = 0; k < v.size(); ++k) {
        CHECK(v[k].n_tok == n_tok && v[k].pos0 == kvb[s] + j0 && v[k].k1 > v[k].k0);
        if (k + 1 < v.size()) CHECK(v[k].k1 == v[k + 1].k0 && v[k].k1 % 64 == 0);
        if (v.size() == 1) CHECK(v[k].part == -1);
        else {
          CHECK(v[k].part >= 0 && (size_t)v[k].part < slots);
          CHECK(parts.insert(v[k].part).second);
        }
      }
      CHECK(v.size() <= 32);
    }
    row += ql[s];
  }
  CHECK(by_tile.size() == want_tiles);
}

static void planner_fuzz() {
  std::mt19937_64 rng(20250926);
  auto uni = [&](int lo, int hi) { return (int)(lo + rng() % (uint64_t)(hi - lo + 1)); };
  const int groups[] = {1, 3, 4, 5, 8, 16};
  const int kvheads[] = {1, 2, 4, 8};
  std::vector<int32_t> items((size_t)8 * 40000);
  for (int trial = 0; trial < 160; ++trial) {
    const int G = groups[trial % 6], Hkv = kvheads[(trial / 6) % 4], D = (trial & 1) ? 64 : 128;
    oppo_attn_desc d{G * Hkv, Hkv, D, 0.1f};
    const bool huge = trial % 10 == 9;   // work lists that need several launches
    const int B = huge ? uni(150, 300) : uni(1, 80);
    std::vector<int32_t> kvb((size_t)B), ql((size_t)B);
    int64_t rows = 0;
    for (int i = 0; i < B; ++i) {
      kvb[(size_t)i] = uni(0, huge ? 1500 : 9000);
      ql[(size_t)i] = (rng() % 4 == 0) ? 0 : uni(1, huge ? 700 : 300);
      rows += ql[(size_t)i];
    }
    for (int split : {0, 1, 2, 7, 32}) {
      CHECK(oppo_set_option(OPPO_OPT_SPLIT_KV, split) == OPPO_OK);
      CHECK(oppo_set_option(OPPO_OPT_ORDER, trial % 3) == OPPO_OK);
      for (int ws_kind = 0; ws_kind < 3; ++ws_kind) {
        // no workspace, a small one (3 slots), the recommended one
        const size_t slot_bytes = (size_t)Hkv * 256 * (size_t)(D + 2) * 4;
        const size_t ws = ws_kind == 0 ? 0 : ws_kind == 1 ? 3 * slot_bytes : oppo_workspace_bytes(&d, B, (int32_t)rows);
        int32_t n = 0;
        const int rc = oppo_plan_debug(&d, B, kvb.data(), ql.data(), ws, items.data(), 40000, &n);
        CHECK(rc == OPPO_OK);
        if (rc != OPPO_OK) continue;
        check_plan(G, kvb, ql, items, n, ws / slot_bytes, std::max(1, 256 / Hkv));
        // the same pass through the fused entry point: the launcher stand-ins check each list
        std::vector<int64_t> slot_begin((size_t)B + 1, 0);
        std::vector<int32_t> kv_len = kvb, cu((size_t)B + 1, 0);
        for (int i = 0; i < B; ++i) {
          slot_begin[(size_t)i + 1] = slot_begin[(size_t)i] + kvb[(size_t)i] + ql[(size_t)i] + 2;
          cu[(size_t)i + 1] = cu[(size_t)i] + ql[(size_t)i];
        }
        oppo_kv_cache cache{fake(0x10000), fake(0x20000), slot_begin.data(), kv_len.data(), B};
        const int rc2 = oppo_chunk_step(&d, &cache, cu.data(), fake(0x30000), fake(0x40000), fake(0x50000), fake(0x60000),
                                        ws ? fake(0x7000000) : nullptr, ws, nullptr);
        CHECK(rc2 == OPPO_OK);
        for (int i = 0; i < B; ++i) CHECK(kv_len[(size_t)i] == kvb[(size_t)i] + ql[(size_t)i]);
        const int rc3 = oppo_chunk_prefill_attn(&d, &cache, cu.data(), fake(0x30000), fake(0x60000),
                                                ws ? fake(0x7000000) : nullptr, ws, nullptr);
        CHECK(rc3 == OPPO_OK);
      }
    }
  }
  oppo_set_option(OPPO_OPT_SPLIT_KV, 0);
  oppo_set_option(OPPO_OPT_ORDER, 0);
  // fewer compute units: fewer queues
  oppo_attn_desc d{32, 8, 128, 0.1f};
  for (int cus : {1, 8, 100, 256, 4096}) {
    CHECK(oppo_set_option(OPPO_OPT_NUM_CUS, cus) == OPPO_OK);
    std::vector<int32_t> kvb = {5000, 100, 0}, ql = {256, 300, 17};
    int32_t n = 0;
    const size_t ws = oppo_workspace_bytes(&d, 3, 600);
    CHECK(oppo_plan_debug(&d, 3, kvb.data(), ql.data(), ws, items.data(), 40000, &n) == OPPO_OK);
    check_plan(4, kvb, ql, items, n, ws / ((size_t)8 * 256 * 130 * 4), std::max(1, cus / 8));
  }
  oppo_set_option(OPPO_OPT_NUM_CUS, 256);
}

static void abi_errors() {
  oppo_attn_desc d{32, 8, 128, 0.1f};
  int64_t slot_begin[3] = {0, 8, 20};
  int32_t kv_len[2] = {6, 0};
  oppo_kv_cache cache{fake(0x1000), fake(0x2000), slot_begin, kv_len, 2};
  int32_t cu_ok[3] = {0, 1, 2}, cu_over[3] = {0, 3, 6}, cu_dec[3] = {0, 3, 2};
  CHECK(oppo_kv_append(nullptr, &cache, cu_ok, fake(1), fake(2), nullptr) == OPPO_ERR_INVALID);
  CHECK(oppo_kv_append(&d, nullptr, cu_ok, fake(1), fake(2), nullptr) == OPPO_ERR_INVALID);
  CHECK(oppo_kv_append(&d, &cache, cu_over, fake(1), fake(2), nullptr) == OPPO_ERR_CAPACITY);
  CHECK(oppo_kv_append(&d, &cache, cu_dec, fake(1), fake(2), nullptr) == OPPO_ERR_INVALID);
  CHECK(kv_len[0] == 6 && kv_len[1] == 0);
  CHECK(oppo_chunk_step(&d, &cache, cu_over, fake(1), fake(2), fake(3), fake(4), nullptr, 0, nullptr) == OPPO_ERR_CAPACITY);
  CHECK(oppo_chunk_step(&d, &cache, cu_ok, fake(1), nullptr, fake(3), fake(4), nullptr, 0, nullptr) == OPPO_ERR_INVALID);
  CHECK(oppo_chunk_step(&d, &cache, cu_ok, fake(1), fake(2), fake(3), fake(4), nullptr, 0, nullptr) == OPPO_OK);
  CHECK(kv_len[0] == 7 && kv_len[1] == 1);
  CHECK(oppo_chunk_step_noalloc(&d, &cache, cu_over, fake(1), fake(2), fake(3), fake(4), nullptr) == OPPO_ERR_CAPACITY);
  oppo_attn_desc wide{16 * 4, 16, 128, 0.1f};
  CHECK(oppo_chunk_step_noalloc(&wide, &cache, cu_ok, fake(1), fake(2), fake(3), fake(4), nullptr) == OPPO_ERR_UNSUPPORTED);
  CHECK(kv_len[0] == 7 && kv_len[1] == 1);
  CHECK(oppo_chunk_step_noalloc(&d, &cache, cu_ok, fake(1), fake(2), fake(3), fake(4), nullptr) == OPPO_OK);
  CHECK(kv_len[0] == 8 && kv_len[1] == 2);
  CHECK(oppo_chunk_prefill_attn(&d, &cache, cu_ok, fake(1), fake(2), fake(0x10001), 1 << 30, nullptr) == OPPO_ERR_WORKSPACE);
  CHECK(oppo_chunk_prefill_attn(&d, &cache, cu_ok, fake(1), fake(2), fake(0x10000), 4096, nullptr) == OPPO_ERR_WORKSPACE);
  int32_t cu_many[3] = {0, 1, 4};
  CHECK(oppo_chunk_prefill_attn(&d, &cache, cu_many, fake(1), fake(2), nullptr, 0, nullptr) == OPPO_ERR_INVALID);
  oppo_attn_desc bad = d;
  bad.softmax_scale = 0.0f / 0.0f;
  CHECK(oppo_kv_append(&bad, &cache, cu_ok, fake(1), fake(2), nullptr) == OPPO_ERR_INVALID);
  bad = d;
  bad.head_dim = 96;
  CHECK(oppo_workspace_bytes(&bad, 4, 100) == 0);
  CHECK(oppo_workspace_bytes(&d, 4, 100) > 0 && oppo_workspace_bytes(&d, 4, 100) < oppo_workspace_bytes(&d, 64, 1 << 16));
  CHECK(oppo_workspace_bytes(&d, 0, 0) == 0);
}

static void fp8_cache_errors() {
  oppo_attn_desc d{32, 8, 128, 0.1f};
  int64_t slot_begin[3] = {0, 128, 1344};
  int32_t kv_len[2] = {100, 0};
  oppo_kv_cache_fp8 cache{fake(0x1000), fake(0x2000), slot_begin, kv_len, 2, 0.01f, 0.02f};
  int32_t cu_ok[3] = {0, 20, 1020}, cu_over[3] = {0, 29, 30}, cu_attn[3] = {0, 10, 700};
  CHECK(oppo_kv_append_fp8(&d, nullptr, cu_ok, fake(1), fake(2), nullptr) == OPPO_ERR_INVALID);
  CHECK(oppo_kv_append_fp8(&d, &cache, cu_over, fake(1), fake(2), nullptr) == OPPO_ERR_CAPACITY);
  CHECK(oppo_kv_append_fp8(&d, &cache, cu_ok, fake(1), nullptr, nullptr) == OPPO_ERR_INVALID);
  oppo_kv_cache_fp8 bad = cache;
  bad.k_scale = 0.0f;
  CHECK(oppo_kv_append_fp8(&d, &bad, cu_ok, fake(1), fake(2), nullptr) == OPPO_ERR_INVALID);
  bad.k_scale = 0.0f / 0.0f;
  CHECK(oppo_chunk_prefill_attn_fp8(&d, &bad, cu_ok, fake(1), fake(2), nullptr, 0, nullptr) == OPPO_ERR_INVALID);
  bad = cache;
  bad.v_scale = 1e-42f;   // its reciprocal is not finite
  CHECK(oppo_kv_append_fp8(&d, &bad, cu_ok, fake(1), fake(2), nullptr) == OPPO_ERR_INVALID);
  int64_t ragged[3] = {0, 100, 1316};
  bad = cache;
  bad.slot_begin = ragged;
  CHECK(oppo_kv_append_fp8(&d, &bad, cu_ok, fake(1), fake(2), nullptr) == OPPO_ERR_INVALID);
  CHECK(kv_len[0] == 100 && kv_len[1] == 0);
  CHECK(oppo_kv_append_fp8(&d, &cache, cu_ok, fake(1), fake(2), nullptr) == OPPO_OK);
  CHECK(kv_len[0] == 120 && kv_len[1] == 1000);
  // attention: rows must have been appended; with and without a workspace; head size 128 only
  CHECK(oppo_chunk_prefill_attn_fp8(&d, &cache, cu_ok, fake(1), fake(2), nullptr, 0, nullptr) == OPPO_OK);
  CHECK(oppo_chunk_prefill_attn_fp8(&d, &cache, cu_attn, fake(1), fake(2), fake(0x10000),
                                    oppo_workspace_bytes(&d, 2, 710), nullptr) == OPPO_OK);
  CHECK(oppo_chunk_prefill_attn_fp8(&d, &cache, cu_attn, fake(1), fake(2), fake(0x10001), 1 << 30, nullptr) == OPPO_ERR_WORKSPACE);
  int32_t cu_more[3] = {0, 121, 121};
  CHECK(oppo_chunk_prefill_attn_fp8(&d, &cache, cu_more, fake(1), fake(2), nullptr, 0, nullptr) == OPPO_ERR_INVALID);
  CHECK(oppo_chunk_prefill_attn_fp8(&d, &cache, cu_ok, nullptr, fake(2), nullptr, 0, nullptr) == OPPO_ERR_INVALID);
  oppo_attn_desc d64{8, 8, 64, 0.1f};
  CHECK(oppo_chunk_prefill_attn_fp8(&d64, &cache, cu_ok, fake(1), fake(2), nullptr, 0, nullptr) == OPPO_OK);
  int32_t cu_one[3] = {0, 1, 1};
  CHECK(oppo_kv_append_fp8(&d64, &cache, cu_one, fake(1), fake(2), nullptr) == OPPO_OK);
  CHECK(kv_len[0] == 121);
}

static void pool_and_scheduler() {
  std::mt19937_64 rng(7);
  int32_t caps[6] = {100, 50, 400, 50, 0, 1000};
  oppo_slot_pool* pool = nullptr;
  CHECK(oppo_pool_create(6, caps, &pool) == OPPO_OK);
  std::set<int64_t> live;
  for (int step = 0; step < 2000; ++step) {
    const int64_t id = (int64_t)(rng() % 12);
    int32_t slot = -1;
    if (rng() & 1) {
      const int rc = oppo_pool_acquire(pool, id, (int32_t)(rng() % 500), &slot);
      if (rc == OPPO_OK) CHECK(live.insert(id).second && slot >= 0 && slot < 6);
      else CHECK(rc == OPPO_ERR_INVALID || rc == OPPO_ERR_CAPACITY);
    } else {
      const int rc = oppo_pool_release(pool, id);
      CHECK((rc == OPPO_OK) == (live.erase(id) == 1));
    }
    int32_t n_live = 0;
    CHECK(oppo_pool_counts(pool, nullptr, &n_live, nullptr, nullptr) == OPPO_OK && (size_t)n_live == live.size());
  }
  std::vector<int64_t> ids(live.begin(), live.end());
  std::vector<int32_t> ql(ids.size(), 0), cu(7), row_begin(ids.size());
  CHECK(oppo_pool_pack(pool, (int32_t)ids.size(), ids.data(), ql.data(), cu.data(), row_begin.data()) == OPPO_OK);
  CHECK(oppo_pool_destroy(pool) == OPPO_OK);

  oppo_scheduler* s = nullptr;
  CHECK(oppo_sched_create(4, 2, 16, &s) == OPPO_OK);
  int64_t next_id = 0;
  std::map<int64_t, int> left;   // response tokens each sequence still has to produce
  for (int iter = 0; iter < 30; ++iter) {
    int32_t room = 0;
    CHECK(oppo_sched_room(s, &room) == OPPO_OK);
    for (int k = 0; k < room; ++k) {
      CHECK(oppo_sched_add(s, next_id, 1 + (int32_t)(rng() % 40)) == OPPO_OK);
      left[next_id++] = 1 + (int)(rng() % 70);
    }
    for (;;) {
      int64_t pid[8];
      int32_t kvb[8], cap[8], n = 0, kind = 0;
      CHECK(oppo_sched_begin_pass(s, 8, pid, kvb, cap, &n, &kind) == OPPO_OK);
      if (kind == OPPO_PASS_NONE) break;
      int32_t got[8];
      uint8_t fin[8];
      for (int j = 0; j < n; ++j) {
        if (kind == OPPO_PASS_PROMPT) got[j] = cap[j], fin[j] = 0;
        else {
          got[j] = std::min(cap[j], left[pid[j]]);
          left[pid[j]] -= got[j];
          fin[j] = left[pid[j]] == 0;
        }
      }
      CHECK(oppo_sched_end_pass(s, n, pid, got, fin) == OPPO_OK);
    }
    int64_t gone[8];
    int32_t n_gone = 0;
    CHECK(oppo_sched_end_iteration(s, 8, gone, &n_gone) == OPPO_OK && n_gone <= 4);
  }
  CHECK(oppo_sched_destroy(s) == OPPO_OK);
}

int main() {
  abi_errors();
  fp8_cache_errors();
  planner_fuzz();
  pool_and_scheduler();
  if (g_failed) {
    fprintf(stderr, "%d checks failed\n", g_failed);
    return 1;
  }
  printf("host checks passed\n");
  return 0;
}
