// Host side of the C ABI: argument checks, work planning, launches.
// Every check runs before anything is enqueued, so a failed call has no effect.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <functional>
#include <vector>

#include "../../include/oppo_attn.h"
#include "oppo_internal.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

struct Options {
  int split_kv = 0;   // 0 auto, 1 off, n>=2 forced
  int order = 0;      // 0 longest first, 1 input order, 2 shortest first
  int num_cus = 256;
};
Options g_opt;

// Cost model of the planner, in units of one 64-key tile of one workgroup:
// shortest piece worth a workgroup of its own, fixed start-up + drain share of a
// workgroup, extra cost of writing a partial result, cost of the merge kernel.
// (Measured on MI355X: a tile takes about 2.1 us; a workgroup's start-up and
// drain about 4 us; a partial result is 256 rows x (D + 2) floats per kv-head,
// whose write shares HBM with all other workgroups, about 8 us; the merge kernel
// is bound by reading those partials back, about 0.26 us per piece.)
constexpr int kMinSplitTiles = 4;
constexpr float kStartTiles = 2.0f;
constexpr float kPartialTiles = 4.0f;
constexpr float kMergeTiles = 2.0f;
constexpr float kMergeTilesPerPiece = 0.125f;
// Upper bound on partial slots the automatic planner may ask for, per CU.
constexpr int kSlotsPerCu = 6;

int check_desc(const oppo_attn_desc* d, oppo::LayerShape* ls) {
  if (!d) return fail(OPPO_ERR_INVALID, "desc is null");
  if (d->num_q_heads <= 0 || d->num_kv_heads <= 0)
    return fail(OPPO_ERR_INVALID, "head counts must be positive (Hq=%d, Hkv=%d)", d->num_q_heads, d->num_kv_heads);
  if (!(d->softmax_scale > 0.0f) || !isfinite(d->softmax_scale))
    return fail(OPPO_ERR_INVALID, "softmax_scale must be positive and finite");
  if (d->head_dim != 64 && d->head_dim != 128)
    return fail(OPPO_ERR_UNSUPPORTED, "head_dim %d not supported (64 or 128)", d->head_dim);
  if (d->num_q_heads % d->num_kv_heads != 0)
    return fail(OPPO_ERR_UNSUPPORTED, "Hq=%d is not a multiple of Hkv=%d", d->num_q_heads, d->num_kv_heads);
  const int G = d->num_q_heads / d->num_kv_heads;
  if (G > 16) return fail(OPPO_ERR_UNSUPPORTED, "group size Hq/Hkv=%d exceeds 16", G);
  ls->Hq = d->num_q_heads;
  ls->Hkv = d->num_kv_heads;
  ls->G = G;
  ls->D = d->head_dim;
  ls->TM = oppo::kTileRows / G;
  ls->c = d->softmax_scale * 1.4426950408889634f;
  return OPPO_OK;
}

int check_cu(const int32_t* cu, int32_t n, const char* name) {
  if (!cu) return fail(OPPO_ERR_INVALID, "%s is null", name);
  if (cu[0] != 0) return fail(OPPO_ERR_INVALID, "%s[0] must be 0", name);
  for (int32_t i = 0; i < n; ++i)
    if (cu[i + 1] < cu[i]) return fail(OPPO_ERR_INVALID, "%s decreases at %d", name, i);
  return OPPO_OK;
}

size_t workspace_need(const oppo::LayerShape& ls) {
  const size_t slots = (size_t)kSlotsPerCu * (size_t)g_opt.num_cus / (size_t)ls.Hkv + 1;
  return slots * oppo::part_slot_bytes(ls.Hkv, ls.D);
}

// One sequence as the attention sees it.
struct SeqView {
  int64_t kv_row0;  // row of token 0 in the k/v arrays
  int32_t q_row0;   // row of the chunk's first token in q/out
  int32_t q_len;
  int32_t kv_before;
};

struct Plan {
  std::vector<oppo::AttnItem> items;
  std::vector<oppo::CombineItem> combines;
};

// Cut every sequence's chunk into query tiles, split long key ranges when the
// launch would otherwise leave compute units idle (the thin tail passes of a
// long-tailed batch), and order the pieces longest first so that the hardware
// dispatcher, which hands workgroups out in index order, balances them.
void make_plan(const oppo::LayerShape& ls, const std::vector<SeqView>& seqs, size_t slots_avail, Plan* plan) {
  struct Tile { int seq; int32_t j0, n_tok, keys; };
  std::vector<Tile> tiles;
  int64_t total_keys = 0;
  for (size_t i = 0; i < seqs.size(); ++i) {
    const SeqView& s = seqs[i];
    for (int32_t j0 = 0; j0 < s.q_len; j0 += ls.TM) {
      Tile t;
      t.seq = (int)i;
      t.j0 = j0;
      t.n_tok = std::min(ls.TM, s.q_len - j0);
      t.keys = s.kv_before + j0 + t.n_tok;
      total_keys += t.keys;
      tiles.push_back(t);
    }
  }
  // Key-range length per workgroup, in 64-key tiles (0 = no splitting).  The
  // automatic choice compares a few candidate piece lengths - cut so that the
  // launch fills the compute units in one, two, three or four even rounds - and
  // no splitting at all, under a small cost model: a workgroup costs its tiles
  // plus a fixed start-up/drain share, a split piece also its partial-result
  // write, and any split adds the merge kernel.  The estimate is the makespan of
  // longest-first list scheduling, which is what the hardware dispatcher does
  // with a launch sorted by length.
  int piece_tiles = 0;
  int forced = 0;
  auto tiles_of = [](const Tile& t) { return (t.keys + oppo::kKeyTile - 1) / oppo::kKeyTile; };
  auto split_of = [&](int ntile, int piece) {
    if (piece <= 0 || ntile <= piece) return 1;
    return std::min((ntile + piece - 1) / piece, oppo::kMaxSplit);
  };
  if (slots_avail > 0 && g_opt.split_kv != 1) {
    if (g_opt.split_kv >= 2) {
      forced = g_opt.split_kv;
    } else {
      const int W = g_opt.num_cus;
      int64_t total_tiles = 0;
      for (const Tile& t : tiles) total_tiles += tiles_of(t);
      total_tiles *= ls.Hkv;
      auto makespan = [&](int piece) {
        std::vector<float> costs;
        size_t slots = 0;
        for (const Tile& t : tiles) {
          const int ntile = tiles_of(t);
          int ns = split_of(ntile, piece);
          if (ns > 1 && slots + ns > slots_avail) ns = 1;
          if (ns > 1) slots += ns;
          for (int p = 0; p < ns; ++p) {   // pieces as even as whole tiles allow
            const int n = ntile / ns + (p < ntile % ns ? 1 : 0);
            costs.push_back((float)n + kStartTiles + (ns > 1 ? kPartialTiles : 0.f));
          }
        }
        std::sort(costs.begin(), costs.end(), [](float a, float b) { return a > b; });
        // every piece exists once per kv-head: schedule the replicated list
        std::vector<float> load((size_t)W, 0.f);
        std::make_heap(load.begin(), load.end(), std::greater<float>());
        for (float cst : costs)
          for (int h = 0; h < ls.Hkv; ++h) {
            std::pop_heap(load.begin(), load.end(), std::greater<float>());
            load.back() += cst;
            std::push_heap(load.begin(), load.end(), std::greater<float>());
          }
        float ms = 0.f;
        for (float x : load) ms = std::max(ms, x);
        return ms + (slots ? kMergeTiles + kMergeTilesPerPiece * (float)slots : 0.f);
      };
      float best = makespan(0);
      for (int rounds = 1; rounds <= 4; ++rounds) {
        const int piece = (int)std::max<int64_t>(kMinSplitTiles, (total_tiles + (int64_t)rounds * W - 1) / ((int64_t)rounds * W));
        const float m = makespan(piece);
        if (m < best * 0.97f) best = m, piece_tiles = piece;   // split only for a clear gain
      }
    }
  }
  size_t next_slot = 0;
  for (const Tile& t : tiles) {
    const SeqView& s = seqs[t.seq];
    const int ntile = tiles_of(t);
    int nsplit = forced ? std::min(std::min(forced, ntile), oppo::kMaxSplit) : split_of(ntile, piece_tiles);
    if (nsplit > 1 && next_slot + (size_t)nsplit > slots_avail) nsplit = 1;
    oppo::AttnItem it;
    it.kv_row0 = s.kv_row0;
    it.q_row0 = s.q_row0 + t.j0;
    it.n_tok = t.n_tok;
    it.pos0 = s.kv_before + t.j0;
    if (nsplit == 1) {
      it.k_begin = 0;
      it.k_end = t.keys;
      it.part = -1;
      plan->items.push_back(it);
    } else {
      oppo::CombineItem ci;
      ci.q_row0 = it.q_row0;
      ci.n_tok = it.n_tok;
      ci.part0 = (int32_t)next_slot;
      ci.nsplit = nsplit;
      plan->combines.push_back(ci);
      int tile0 = 0;
      for (int p = 0; p < nsplit; ++p) {   // pieces as even as whole tiles allow
        const int n = ntile / nsplit + (p < ntile % nsplit ? 1 : 0);
        it.k_begin = tile0 * oppo::kKeyTile;
        it.k_end = std::min<int32_t>(t.keys, (tile0 + n) * oppo::kKeyTile);
        it.part = (int32_t)next_slot++;
        plan->items.push_back(it);
        tile0 += n;
      }
    }
  }
  auto keys_of = [](const oppo::AttnItem& a) { return a.k_end - a.k_begin; };
  if (g_opt.order == 0)
    std::stable_sort(plan->items.begin(), plan->items.end(),
                     [&](const oppo::AttnItem& a, const oppo::AttnItem& b) { return keys_of(a) > keys_of(b); });
  else if (g_opt.order == 2)
    std::stable_sort(plan->items.begin(), plan->items.end(),
                     [&](const oppo::AttnItem& a, const oppo::AttnItem& b) { return keys_of(a) < keys_of(b); });
}

int run_attention(const oppo::LayerShape& ls, const std::vector<SeqView>& seqs, const void* q, const void* k,
                  const void* v, void* out, void* workspace, size_t workspace_bytes, void* stream) {
  size_t slots = 0;
  float* part_o = nullptr;
  float* part_ml = nullptr;
  if (workspace && workspace_bytes > 0) {
    // slot s, kv-head g: O at part_o[((s*Hkv+g)*256 + row)*D], (m, l) at part_ml[((s*Hkv+g)*256 + row)*2]
    slots = workspace_bytes / oppo::part_slot_bytes(ls.Hkv, ls.D);
    part_o = (float*)workspace;
    part_ml = part_o + slots * (size_t)ls.Hkv * oppo::kTileRows * (size_t)ls.D;
  }
  Plan plan;
  make_plan(ls, seqs, slots, &plan);
  if (plan.items.empty()) return OPPO_OK;
  int e = oppo::launch_attention(ls, q, k, v, out, part_o, part_ml, plan.items.data(), (int)plan.items.size(), stream);
  if (e) return fail(OPPO_ERR_HIP, "attention launch failed: %s", oppo::hip_error_string(e));
  if (!plan.combines.empty()) {
    e = oppo::launch_combine(ls, out, part_o, part_ml, plan.combines.data(), (int)plan.combines.size(), stream);
    if (e) return fail(OPPO_ERR_HIP, "combine launch failed: %s", oppo::hip_error_string(e));
  }
  return OPPO_OK;
}

int check_workspace(const oppo::LayerShape& ls, const void* workspace, size_t workspace_bytes) {
  if (!workspace || workspace_bytes == 0) return OPPO_OK;
  if (((uintptr_t)workspace & 255) != 0) return fail(OPPO_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  const size_t need = workspace_need(ls);
  if (workspace_bytes < need)
    return fail(OPPO_ERR_WORKSPACE, "workspace has %zu bytes, %zu required", workspace_bytes, need);
  return OPPO_OK;
}

}  // namespace

extern "C" {

int oppo_chunk_schedule(int32_t B, const int32_t* prompt_len, const int32_t* resp_len, int32_t C, int32_t t,
                        int32_t* kv_before, int32_t* q_len, int32_t* cu_q) {
  if (B < 0) return fail(OPPO_ERR_INVALID, "B is negative");
  if (C < 1) return fail(OPPO_ERR_INVALID, "chunk size must be at least 1");
  if (t < 0) return fail(OPPO_ERR_INVALID, "pass index is negative");
  if (!prompt_len || !resp_len || !q_len || !cu_q) return fail(OPPO_ERR_INVALID, "null array");
  const int64_t streamed = (int64_t)t * (int64_t)C;
  int64_t sum = 0;
  for (int32_t i = 0; i < B; ++i) {
    if (prompt_len[i] < 0 || resp_len[i] < 0) return fail(OPPO_ERR_INVALID, "negative length at sequence %d", i);
    if ((int64_t)prompt_len[i] + resp_len[i] > INT32_MAX)
      return fail(OPPO_ERR_INVALID, "sequence %d is longer than int32", i);
    const int64_t done = std::min<int64_t>(resp_len[i], streamed);
    sum += std::min<int64_t>(C, resp_len[i] - done);
    if (sum > INT32_MAX) return fail(OPPO_ERR_INVALID, "total rows overflow int32");
  }
  cu_q[0] = 0;
  for (int32_t i = 0; i < B; ++i) {
    const int64_t done = std::min<int64_t>(resp_len[i], streamed);
    const int32_t ql = (int32_t)std::min<int64_t>(C, resp_len[i] - done);
    if (kv_before) kv_before[i] = (int32_t)(prompt_len[i] + done);
    q_len[i] = ql;
    cu_q[i + 1] = cu_q[i] + ql;
  }
  return OPPO_OK;
}

int oppo_kv_append(const oppo_attn_desc* desc, oppo_kv_cache* cache, const int32_t* cu_q, const void* k_new,
                   const void* v_new, void* stream) {
  oppo::LayerShape ls;
  int rc = check_desc(desc, &ls);
  if (rc) return rc;
  if (!cache) return fail(OPPO_ERR_INVALID, "cache is null");
  if (cache->batch < 0) return fail(OPPO_ERR_INVALID, "cache->batch is negative");
  if (!cache->slot_begin || !cache->kv_len) return fail(OPPO_ERR_INVALID, "cache length arrays are null");
  const int32_t B = cache->batch;
  rc = check_cu(cu_q, B, "cu_q");
  if (rc) return rc;
  if (cache->slot_begin[0] < 0) return fail(OPPO_ERR_INVALID, "slot_begin[0] is negative");
  for (int32_t i = 0; i < B; ++i) {
    const int64_t cap = cache->slot_begin[i + 1] - cache->slot_begin[i];
    if (cap < 0) return fail(OPPO_ERR_INVALID, "slot_begin decreases at %d", i);
    if (cache->kv_len[i] < 0 || cache->kv_len[i] > cap)
      return fail(OPPO_ERR_INVALID, "kv_len[%d]=%d outside its slab of %lld slots", i, cache->kv_len[i], (long long)cap);
  }
  for (int32_t i = 0; i < B; ++i) {
    const int64_t cap = cache->slot_begin[i + 1] - cache->slot_begin[i];
    const int64_t ql = cu_q[i + 1] - cu_q[i];
    if ((int64_t)cache->kv_len[i] + ql > cap)
      return fail(OPPO_ERR_CAPACITY, "sequence %d: %d cached + %lld new tokens exceed %lld slots", i,
                  cache->kv_len[i], (long long)ql, (long long)cap);
  }
  if (cu_q[B] == 0) return OPPO_OK;
  if (!cache->k || !cache->v || !k_new || !v_new) return fail(OPPO_ERR_INVALID, "null device pointer");
  std::vector<oppo::AppendItem> items;
  int max_tok = 0;
  for (int32_t i = 0; i < B; ++i) {
    const int32_t ql = cu_q[i + 1] - cu_q[i];
    if (ql == 0) continue;
    oppo::AppendItem it;
    it.dst_row = cache->slot_begin[i] + cache->kv_len[i];
    it.src_row = cu_q[i];
    it.n_tok = ql;
    items.push_back(it);
    max_tok = std::max(max_tok, ql);
  }
  int e = oppo::launch_append(ls, cache->k, cache->v, k_new, v_new, items.data(), (int)items.size(), max_tok, stream);
  if (e) return fail(OPPO_ERR_HIP, "append launch failed: %s", oppo::hip_error_string(e));
  for (int32_t i = 0; i < B; ++i) cache->kv_len[i] += cu_q[i + 1] - cu_q[i];
  return OPPO_OK;
}

int oppo_chunk_prefill_attn(const oppo_attn_desc* desc, const oppo_kv_cache* cache, const int32_t* cu_q,
                            const void* q, void* out, void* workspace, size_t workspace_bytes, void* stream) {
  oppo::LayerShape ls;
  int rc = check_desc(desc, &ls);
  if (rc) return rc;
  if (!cache) return fail(OPPO_ERR_INVALID, "cache is null");
  if (cache->batch < 0) return fail(OPPO_ERR_INVALID, "cache->batch is negative");
  if (!cache->slot_begin || !cache->kv_len) return fail(OPPO_ERR_INVALID, "cache length arrays are null");
  const int32_t B = cache->batch;
  rc = check_cu(cu_q, B, "cu_q");
  if (rc) return rc;
  if (cache->slot_begin[0] < 0) return fail(OPPO_ERR_INVALID, "slot_begin[0] is negative");
  std::vector<SeqView> seqs;
  for (int32_t i = 0; i < B; ++i) {
    const int64_t cap = cache->slot_begin[i + 1] - cache->slot_begin[i];
    if (cap < 0) return fail(OPPO_ERR_INVALID, "slot_begin decreases at %d", i);
    if (cache->kv_len[i] < 0 || cache->kv_len[i] > cap)
      return fail(OPPO_ERR_INVALID, "kv_len[%d]=%d outside its slab of %lld slots", i, cache->kv_len[i], (long long)cap);
    const int32_t ql = cu_q[i + 1] - cu_q[i];
    if (ql > cache->kv_len[i])
      return fail(OPPO_ERR_INVALID, "sequence %d: %d query rows but only %d cached tokens (append first)", i, ql,
                  cache->kv_len[i]);
    if (ql == 0) continue;
    SeqView s;
    s.kv_row0 = cache->slot_begin[i];
    s.q_row0 = cu_q[i];
    s.q_len = ql;
    s.kv_before = cache->kv_len[i] - ql;
    seqs.push_back(s);
  }
  rc = check_workspace(ls, workspace, workspace_bytes);
  if (rc) return rc;
  if (seqs.empty()) return OPPO_OK;
  if (!cache->k || !cache->v || !q || !out) return fail(OPPO_ERR_INVALID, "null device pointer");
  return run_attention(ls, seqs, q, cache->k, cache->v, out, workspace, workspace_bytes, stream);
}

int oppo_full_prefill_ref(const oppo_attn_desc* desc, int32_t B, const int32_t* cu_seq, const void* q, const void* k,
                          const void* v, void* out, void* workspace, size_t workspace_bytes, void* stream) {
  oppo::LayerShape ls;
  int rc = check_desc(desc, &ls);
  if (rc) return rc;
  if (B < 0) return fail(OPPO_ERR_INVALID, "B is negative");
  rc = check_cu(cu_seq, B, "cu_seq");
  if (rc) return rc;
  rc = check_workspace(ls, workspace, workspace_bytes);
  if (rc) return rc;
  std::vector<SeqView> seqs;
  for (int32_t i = 0; i < B; ++i) {
    const int32_t n = cu_seq[i + 1] - cu_seq[i];
    if (n == 0) continue;
    SeqView s;
    s.kv_row0 = cu_seq[i];
    s.q_row0 = cu_seq[i];
    s.q_len = n;
    s.kv_before = 0;
    seqs.push_back(s);
  }
  if (seqs.empty()) return OPPO_OK;
  if (!q || !k || !v || !out) return fail(OPPO_ERR_INVALID, "null device pointer");
  return run_attention(ls, seqs, q, k, v, out, workspace, workspace_bytes, stream);
}

size_t oppo_workspace_bytes(const oppo_attn_desc* desc, int32_t max_batch, int32_t max_q_tokens) {
  oppo::LayerShape ls;
  if (max_batch < 0 || max_q_tokens < 0) return 0;
  if (check_desc(desc, &ls) != OPPO_OK) return 0;
  return workspace_need(ls);
}

int oppo_set_option(int option, int value) {
  if (value < 0) return fail(OPPO_ERR_INVALID, "option value is negative");
  switch (option) {
    case OPPO_OPT_SPLIT_KV: g_opt.split_kv = value; return OPPO_OK;
    case OPPO_OPT_ORDER:
      if (value > 2) return fail(OPPO_ERR_INVALID, "unknown order %d", value);
      g_opt.order = value;
      return OPPO_OK;
    case OPPO_OPT_NUM_CUS:
      if (value < 1) return fail(OPPO_ERR_INVALID, "num_cus must be at least 1");
      g_opt.num_cus = value;
      return OPPO_OK;
    default: return fail(OPPO_ERR_INVALID, "unknown option %d", option);
  }
}

int oppo_plan_debug(const oppo_attn_desc* desc, int32_t B, const int32_t* kv_before, const int32_t* q_len,
                    size_t workspace_bytes, int32_t* items, int32_t max_items, int32_t* n_items) {
  oppo::LayerShape ls;
  int rc = check_desc(desc, &ls);
  if (rc) return rc;
  if (B < 0 || max_items < 0) return fail(OPPO_ERR_INVALID, "negative size");
  if (!kv_before || !q_len || !n_items || (!items && max_items > 0)) return fail(OPPO_ERR_INVALID, "null array");
  std::vector<SeqView> seqs;
  int64_t row = 0;
  for (int32_t i = 0; i < B; ++i) {
    if (kv_before[i] < 0 || q_len[i] < 0) return fail(OPPO_ERR_INVALID, "negative length at sequence %d", i);
    if (q_len[i] > 0) {
      SeqView s;
      s.kv_row0 = i;  // stands for the sequence index in the dump
      s.q_row0 = (int32_t)row;
      s.q_len = q_len[i];
      s.kv_before = kv_before[i];
      seqs.push_back(s);
    }
    row += q_len[i];
  }
  Plan plan;
  make_plan(ls, seqs, workspace_bytes / oppo::part_slot_bytes(ls.Hkv, ls.D), &plan);
  *n_items = (int32_t)plan.items.size();
  if ((int32_t)plan.items.size() > max_items) return fail(OPPO_ERR_INVALID, "plan has %zu items", plan.items.size());
  for (size_t i = 0; i < plan.items.size(); ++i) {
    const oppo::AttnItem& it = plan.items[i];
    int32_t* o = items + 8 * i;
    o[0] = (int32_t)it.kv_row0;
    o[1] = it.q_row0;
    o[2] = it.n_tok;
    o[3] = it.pos0;
    o[4] = it.k_begin;
    o[5] = it.k_end;
    o[6] = it.part;
    o[7] = 0;
  }
  return OPPO_OK;
}

int oppo_profile_enable(int on) { return oppo::profile_enable(on); }

int oppo_profile_read(double* kernel_ms, int32_t* launches) {
  if (!kernel_ms || !launches) return fail(OPPO_ERR_INVALID, "null array");
  const int e = oppo::profile_read(kernel_ms, launches);
  if (e) return fail(OPPO_ERR_HIP, "event timing failed: %s", oppo::hip_error_string(e));
  return OPPO_OK;
}

const char* oppo_last_error(void) { return g_err; }

int oppo_version(void) { return 100; }

}  // extern "C"
