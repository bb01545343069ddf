// Host side of the C ABI: argument checks, work planning, launches.
// Every check runs before anything is enqueued, so a failed call has no effect.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <mutex>
#include <vector>

#include "../../include/oppo_attn.h"
#include "oppo_internal.h"

namespace {
thread_local char g_err[512] = "";
}

namespace oppo {
int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}
}  // namespace oppo

namespace {
using oppo::fail;

struct Options {
  int split_kv = 0;   // 0 auto, 1 off, n>=2 forced
  int order = 0;      // within a queue: 0 as scheduled, 1 input order, 2 shortest first
  int num_cus = 256;
};
// The process-wide knobs of oppo_set_option.  Every entry point takes one snapshot of
// them under the lock when it starts and works on that copy, so a call sees one
// consistent set whatever other threads set meanwhile.
std::mutex g_opt_mu;
Options g_opt;
Options options_now() {
  std::lock_guard<std::mutex> lock(g_opt_mu);
  return g_opt;
}

// Host-side cost of the calls (planning, launching), summed while profiling is on.
std::mutex g_host_mu;
double g_host_plan_us = 0.0, g_host_launch_us = 0.0;
int64_t g_host_calls = 0;
double now_us() {
  return std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

// Cost model of the planner, in units of one 64-key tile of one workgroup
// (about 1.9 us on MI355X): what a piece costs beyond its tiles (draining the
// pipeline, writing the rows, switching over to the next piece), what a partial
// result costs on top (256 rows x (D + 2) floats per kv-head written out), and the
// merge kernel (a launch of its own plus reading the partials back: its measured
// duration fits 4 us + 0.17 us per piece).
constexpr float kPieceTiles = 2.5f;
constexpr float kPartialTiles = 1.0f;
constexpr float kMergeTiles = 2.5f;
constexpr float kMergeTilesPerPiece = 0.1f;
// Shortest piece the stream cut makes on purpose.
constexpr int kMinPieceTiles = 2;
// Upper bound on partial slots the automatic planner may ask for, per CU.
constexpr int kSlotsPerCu = 6;

int check_desc(const oppo_attn_desc* d, oppo::LayerShape* ls) {
  if (!d) return fail(OPPO_ERR_INVALID, "desc is null");
  if (d->num_q_heads <= 0 || d->num_kv_heads <= 0)
    return fail(OPPO_ERR_INVALID, "head counts must be positive (Hq=%d, Hkv=%d)", d->num_q_heads, d->num_kv_heads);
  if (!(d->softmax_scale > 0.0f) || !std::isfinite(d->softmax_scale))
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

// The cache's host arrays: non-null, slabs in order, lengths inside their slabs.
int check_cache(const oppo_kv_cache* cache) {
  if (!cache) return fail(OPPO_ERR_INVALID, "cache is null");
  if (cache->batch < 0) return fail(OPPO_ERR_INVALID, "cache->batch is negative");
  if (!cache->slot_begin || !cache->kv_len) return fail(OPPO_ERR_INVALID, "cache length arrays are null");
  if (cache->slot_begin[0] < 0) return fail(OPPO_ERR_INVALID, "slot_begin[0] is negative");
  for (int32_t i = 0; i < cache->batch; ++i) {
    const int64_t cap = cache->slot_begin[i + 1] - cache->slot_begin[i];
    if (cap < 0) return fail(OPPO_ERR_INVALID, "slot_begin decreases at %d", i);
    if (cache->kv_len[i] < 0 || cache->kv_len[i] > cap)
      return fail(OPPO_ERR_INVALID, "kv_len[%d]=%d outside its slab of %lld slots", i, cache->kv_len[i], (long long)cap);
  }
  return OPPO_OK;
}

// The 8-bit cache: the same host arrays (returned as a view of the 16-bit cache's type, for the
// shared checks), slabs on block boundaries, usable scales.
int check_cache_fp8(const oppo_kv_cache_fp8* cache, oppo_kv_cache* view) {
  if (!cache) return fail(OPPO_ERR_INVALID, "cache is null");
  view->k = cache->k;
  view->v = cache->v;
  view->slot_begin = cache->slot_begin;
  view->kv_len = cache->kv_len;
  view->batch = cache->batch;
  const int rc = check_cache(view);
  if (rc) return rc;
  for (int32_t i = 0; i <= cache->batch; ++i)
    if (cache->slot_begin[i] % oppo::kKeyTile != 0)
      return fail(OPPO_ERR_INVALID, "slot_begin[%d]=%lld is not a multiple of %d", i, (long long)cache->slot_begin[i],
                  oppo::kKeyTile);
  if (!(cache->k_scale > 0.0f) || !std::isfinite(cache->k_scale) || !(cache->v_scale > 0.0f) ||
      !std::isfinite(cache->v_scale))
    return fail(OPPO_ERR_INVALID, "k_scale and v_scale must be positive and finite");
  if (!std::isfinite(1.0f / cache->k_scale) || !std::isfinite(1.0f / cache->v_scale))
    return fail(OPPO_ERR_INVALID, "k_scale or v_scale is too small to invert");
  return OPPO_OK;
}

// Every sequence's new rows fit behind what its slab already holds.
int check_room(const oppo_kv_cache* cache, const int32_t* cu_q) {
  for (int32_t i = 0; i < cache->batch; ++i) {
    const int64_t cap = cache->slot_begin[i + 1] - cache->slot_begin[i];
    const int64_t ql = cu_q[i + 1] - cu_q[i];
    if ((int64_t)cache->kv_len[i] + ql > cap)
      return fail(OPPO_ERR_CAPACITY, "sequence %d: %d cached + %lld new tokens exceed %lld slots", i,
                  cache->kv_len[i], (long long)ql, (long long)cap);
  }
  return OPPO_OK;
}

int queue_count(const Options& opt, const oppo::LayerShape& ls) {
  return std::max(1, std::min(opt.num_cus / ls.Hkv, oppo::kMaxQueues));
}

// Partial slots beyond which the planner has no use for more: the automatic cuts
// make fewer than two partial pieces per queue, and no call cuts more than
// kMaxSplit pieces out of any of its query tiles.
size_t useful_slots(const Options& opt, const oppo::LayerShape& ls, int64_t max_batch, int64_t max_q_tokens) {
  const size_t by_chip = (size_t)kSlotsPerCu * (size_t)opt.num_cus / (size_t)ls.Hkv + 1;
  const int64_t tiles = max_q_tokens / ls.TM + max_batch;   // every sequence adds at most one ragged tile
  const size_t by_work = (size_t)std::max<int64_t>(0, tiles) * (size_t)oppo::kMaxSplit;
  return std::min(by_chip, by_work);
}

// One sequence as the attention sees it.
struct SeqView {
  int64_t kv_row0;  // row of token 0 in the k/v arrays
  int32_t q_row0;   // row of the chunk's first token in q/out
  int32_t q_len;
  int32_t kv_before;
};

// One launch of the attention kernel: pieces grouped by queue.
struct Plan {
  std::vector<oppo::AttnItem> pieces;
  std::vector<uint16_t> first;   // queue j runs pieces first[j] .. first[j+1]-1
  std::vector<oppo::CombineItem> combines;
};

// A query tile: TM tokens of one sequence against all keys it may see.
struct QTile { int seq; int32_t j0, n_tok, keys, ntile; };

// Key tiles [t0, t1) of query tile `tile`, run by `queue`; rank = place in the scheduling order.
struct Piece { int tile; int t0, t1; int queue; int rank; };

// Plans one launch for the query tiles [lo, hi).
//
// The kernel runs one persistent workgroup per (queue, kv-head); the planner
// decides which pieces each queue runs.  Three ways of filling the queues are
// priced with the cost model above and the cheapest one is taken:
//   * whole tiles, sequence by sequence onto the least loaded group of queues (see
//     gang_schedule), then evened by moving and exchanging whole tiles (exchange) -
//     no partial results, but the longest tile bounds the makespan and with few
//     tiles per queue the loads are uneven (the thin tail passes of a long-tailed
//     batch);
//   * the same with the ends of the queues evened out (see even_out): a few tiles
//     are split, most stay whole;
//   * the tiles' key ranges laid end to end and cut into equal shares, one per
//     queue: a tile that straddles a cut is split there (on a 64-key boundary)
//     and its pieces are merged afterwards.  A cut that falls close to a tile
//     edge moves to the edge.
// All steps are linear or n log n in the number of pieces (a pass of a few hundred
// pieces plans in some tens of microseconds, well under the kernel time it plans).
class LaunchPlanner {
 public:
  LaunchPlanner(const Options& opt, const oppo::LayerShape& ls, const std::vector<SeqView>& seqs,
                const std::vector<QTile>& tiles, size_t lo, size_t hi)
      : opt_(opt), ls_(ls), seqs_(seqs), tiles_(tiles), lo_(lo), hi_(hi), Q_(queue_count(opt, ls)) {}

  // split_policy: the OPPO_OPT_SPLIT_KV value this launch is planned under.
  void run(int split_policy, size_t slots_avail, size_t* next_slot, Plan* plan) {
    const size_t slots_left = slots_avail > *next_slot ? slots_avail - *next_slot : 0;
    std::vector<Piece> chosen;
    if (split_policy >= 2 && slots_left > 0) {
      // forced: every tile in (up to) that many even pieces
      size_t used = 0;
      for (size_t i = lo_; i < hi_; ++i) {
        const int nt = tiles_[i].ntile;
        int ns = std::min(std::min(split_policy, nt), oppo::kMaxSplit);
        if (ns > 1 && used + (size_t)ns > slots_left) ns = 1;
        if (ns > 1) used += (size_t)ns;
        int t0 = 0;
        for (int p = 0; p < ns; ++p) {
          const int len = nt / ns + (p < nt % ns ? 1 : 0);
          chosen.push_back(Piece{(int)i, t0, t0 + len, 0, 0});
          t0 += len;
        }
      }
      gang_schedule(chosen);
    } else {
      chosen.reserve(hi_ - lo_ + (size_t)Q_);
      for (size_t i = lo_; i < hi_; ++i) chosen.push_back(Piece{(int)i, 0, tiles_[i].ntile, 0, 0});
      gang_schedule(chosen);
      exchange(chosen);
      if (split_policy == 0 && slots_left > 0) {
        float whole_cost = price(chosen, Q_, nullptr);
        {
          std::vector<Piece> evened = chosen;
          even_out(evened, slots_left);
          const float evened_cost = price(evened, Q_, nullptr);
          if (evened_cost < 0.97f * whole_cost) chosen.swap(evened), whole_cost = evened_cost;
        }
        std::vector<Piece> cut;
        int nq = 0;
        stream_cut(cut, &nq);
        size_t n_partial = 0;
        const float cut_cost = price(cut, nq, &n_partial);
        if (n_partial <= slots_left && cut_cost < 0.97f * whole_cost) chosen.swap(cut);
      }
    }
    emit(chosen, next_slot, plan);
  }

 private:
  static float cost(const Piece& pc) { return (float)(pc.t1 - pc.t0) + kPieceTiles; }
  int seq_of(const Piece& pc) const { return tiles_[pc.tile].seq; }

  float price(const std::vector<Piece>& pcs, int nq, size_t* n_partial) const {
    std::vector<float> load((size_t)std::max(nq, 1), 0.f);
    size_t np = 0;
    for (const Piece& pc : pcs) {
      const bool whole = pc.t0 == 0 && pc.t1 == tiles_[pc.tile].ntile;
      load[pc.queue] += cost(pc) + (whole ? 0.f : kPartialTiles);
      np += whole ? 0 : 1;
    }
    float ms = 0.f;
    for (float x : load) ms = std::max(ms, x);
    if (n_partial) *n_partial = np;
    return ms + (np ? kMergeTiles + kMergeTilesPerPiece * (float)np : 0.f);
  }

  // Whole pieces onto queues.  The pieces of one sequence (its query tiles of this
  // pass) read the same keys and values, and the workgroups of one kv-head share a
  // level-2 cache: scheduled side by side - on neighbouring queues, at about the
  // same time - they fetch every K/V tile from memory once instead of once per
  // query tile.  (Memory traffic matters beyond its bandwidth here: the chip runs
  // against its power limit, and traffic that is saved turns into clock rate.)
  // So sequences are taken in order of decreasing work, each one's pieces go as a
  // gang onto a group of consecutive queues - the group, among those starting at
  // multiples of the group size, that ends up least loaded - longest piece onto
  // the least loaded queue of the group, and every queue runs its pieces in the
  // order they were scheduled.
  void gang_schedule(std::vector<Piece>& pcs) const {
    const size_t ns = seqs_.size();
    std::vector<int32_t> off(ns + 1, 0);
    std::vector<int64_t> work(ns, 0);
    for (const Piece& pc : pcs) ++off[(size_t)seq_of(pc) + 1], work[(size_t)seq_of(pc)] += pc.t1 - pc.t0;
    for (size_t i = 0; i < ns; ++i) off[i + 1] += off[i];
    std::vector<int32_t> mem(pcs.size()), fill(off.begin(), off.end() - 1);
    for (size_t a = 0; a < pcs.size(); ++a) mem[(size_t)fill[(size_t)seq_of(pcs[a])]++] = (int32_t)a;
    std::vector<int32_t> order;
    order.reserve(ns);
    for (size_t i = 0; i < ns; ++i)
      if (off[i + 1] > off[i]) order.push_back((int32_t)i);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return work[(size_t)a] > work[(size_t)b]; });
    std::vector<float> load((size_t)Q_, 0.f);
    int rank = 0;
    auto len_of = [&](int32_t a) { return pcs[(size_t)a].t1 - pcs[(size_t)a].t0; };
    int qs[oppo::kMaxQueues];
    // the queues st, st+1, .. of a group of g, least loaded first (ties: lowest index)
    auto group_sorted = [&](int st, int g) {
      for (int m = 0; m < g; ++m) {
        const int qn = (st + m) % Q_;
        int k = m;
        for (; k > 0 && (load[(size_t)qs[k - 1]] > load[(size_t)qn] || (load[(size_t)qs[k - 1]] == load[(size_t)qn] && qs[k - 1] > qn)); --k)
          qs[k] = qs[k - 1];
        qs[k] = qn;
      }
    };
    for (int32_t sq : order) {
      int32_t* m_begin = mem.data() + off[(size_t)sq];
      int32_t* m_end = mem.data() + off[(size_t)sq + 1];
      if (m_end - m_begin > 1)
        std::stable_sort(m_begin, m_end, [&](int32_t a, int32_t b) { return len_of(a) > len_of(b); });
      for (int32_t* m0 = m_begin; m0 < m_end; m0 += Q_) {
        const int g = (int)std::min<ptrdiff_t>(Q_, m_end - m0);
        int best_start = 0;
        if (g == 1) {
          for (int st = 1; st < Q_; ++st)
            if (load[(size_t)st] < load[(size_t)best_start]) best_start = st;
        } else {
          int step = 1;   // largest divisor of Q that does not exceed the gang
          for (int d = 1; d <= g; ++d)
            if (Q_ % d == 0) step = d;
          float best = 0.f;
          best_start = -1;
          for (int st = 0; st < Q_; st += step) {
            group_sorted(st, g);
            float mx = 0.f;
            for (int m = 0; m < g; ++m) mx = std::max(mx, load[(size_t)qs[m]] + (float)len_of(m0[m]));
            if (best_start < 0 || mx < best) best = mx, best_start = st;
          }
        }
        group_sorted(best_start, g);
        for (int m = 0; m < g; ++m) {
          Piece& pc = pcs[(size_t)m0[m]];
          pc.queue = qs[m];
          pc.rank = rank++;
          load[(size_t)pc.queue] += cost(pc);
        }
      }
    }
  }

  // Whole pieces change queues while that shortens the longest queue: the most loaded
  // queue gives a piece to the least loaded one, or the two exchange a pair.  (Greedy
  // placement of a handful of pieces per queue leaves the loads a few per cent apart.)
  // A piece keeps its place in the scheduling order, so on its new queue it still runs at
  // about the time its gang does; the pieces of one sequence stay on different queues.
  // Per round: the best partner of a piece x of the long queue is the piece y of the short
  // one whose cost is closest to cost(x) - gap / 2, found in the short queue's pieces
  // sorted by cost.
  void exchange(std::vector<Piece>& pcs) const {
    std::vector<float> load((size_t)Q_, 0.f);
    std::vector<std::vector<int>> on((size_t)Q_);
    std::vector<int> per_seq(seqs_.size(), 0);
    for (size_t x = 0; x < pcs.size(); ++x) {
      load[(size_t)pcs[x].queue] += cost(pcs[x]);
      on[(size_t)pcs[x].queue].push_back((int)x);
      ++per_seq[(size_t)seq_of(pcs[x])];
    }
    // does `queue` hold a piece of x's sequence other than `except`?  (only sequences with
    // several pieces need the scan)
    auto holds = [&](int queue, int x, int except) {
      if (per_seq[(size_t)seq_of(pcs[(size_t)x])] < 2) return false;
      for (int z : on[(size_t)queue])
        if (z != except && z != x && seq_of(pcs[(size_t)z]) == seq_of(pcs[(size_t)x])) return true;
      return false;
    };
    auto move = [&](int x, int from, int to) {
      std::vector<int>& f = on[(size_t)from];
      f.erase(std::find(f.begin(), f.end(), x));
      on[(size_t)to].push_back(x);
      pcs[(size_t)x].queue = to;
      load[(size_t)from] -= cost(pcs[(size_t)x]), load[(size_t)to] += cost(pcs[(size_t)x]);
    };
    std::vector<int> sorted_b;
    for (int round = 0; round < 4 * Q_; ++round) {
      int a = 0, b = 0;
      for (int j = 1; j < Q_; ++j) {
        if (load[(size_t)j] > load[(size_t)a]) a = j;
        if (load[(size_t)j] < load[(size_t)b]) b = j;
      }
      const float gap = load[(size_t)a] - load[(size_t)b];
      if (gap < 1.0f) break;   // nothing can gain the half tile a move has to gain
      float best = load[(size_t)a] - 0.5f;
      int bx = -1, by = -1;
      sorted_b = on[(size_t)b];
      std::sort(sorted_b.begin(), sorted_b.end(), [&](int p, int q) {
        const float cp = cost(pcs[(size_t)p]), cq = cost(pcs[(size_t)q]);
        return cp < cq || (cp == cq && p < q);
      });
      for (int x : on[(size_t)a]) {
        const float cx = cost(pcs[(size_t)x]);
        if (std::max(load[(size_t)a] - cx, load[(size_t)b] + cx) < best && !holds(b, x, -1))
          best = std::max(load[(size_t)a] - cx, load[(size_t)b] + cx), bx = x, by = -1;
        if (sorted_b.empty() || cx <= 0.5f) continue;
        // partners around the ideal cost cx - gap / 2: the few pieces of the short queue on
        // either side of it in cost order (max(...) below is V-shaped in the partner's cost)
        const float want = cx - 0.5f * gap;
        const size_t mid = (size_t)(std::lower_bound(sorted_b.begin(), sorted_b.end(), want,
                                                     [&](int p, float w) { return cost(pcs[(size_t)p]) < w; }) - sorted_b.begin());
        const size_t from = mid >= 3 ? mid - 3 : 0, to = std::min(sorted_b.size(), mid + 3);
        for (size_t k = from; k < to; ++k) {
          const int y = sorted_b[k];
          const float cy = cost(pcs[(size_t)y]);
          const float m = std::max(load[(size_t)a] - cx + cy, load[(size_t)b] + cx - cy);
          if (m < best && !holds(b, x, y) && !holds(a, y, x)) best = m, bx = x, by = y;
        }
      }
      if (bx < 0) break;
      move(bx, a, b);
      if (by >= 0) move(by, b, a);
    }
  }

  // Evening out a schedule of whole tiles: as long as it pays, the most loaded
  // queue hands the end of its day to the least loaded one - its last piece as a
  // whole if that fits into the gap, otherwise the rear part of that piece's key
  // range, sized so that both queues end together (the tile is then merged from
  // partial results).  Only the ends of the queues change, so the gangs further
  // up keep running side by side.  Adds fewer than Q pieces.
  void even_out(std::vector<Piece>& pcs, size_t max_partial) const {
    const size_t n = hi_ - lo_;
    std::vector<float> load((size_t)Q_, 0.f);
    std::vector<int> n_of_tile(n, 0);
    std::vector<std::vector<int>> on((size_t)Q_);   // pieces of each queue, by rank
    for (size_t k = 0; k < pcs.size(); ++k) {
      load[(size_t)pcs[k].queue] += cost(pcs[k]);
      ++n_of_tile[(size_t)pcs[k].tile - lo_];
      on[(size_t)pcs[k].queue].push_back((int)k);
    }
    for (std::vector<int>& v : on)
      std::sort(v.begin(), v.end(), [&](int p, int q) { return pcs[(size_t)p].rank < pcs[(size_t)q].rank; });
    size_t n_partial = 0;
    int rank = (int)pcs.size();
    for (int added = 0, moves = 0; added + 1 < Q_ && moves < 8 * Q_; ++moves) {
      int a = 0, b = 0;
      for (int j = 1; j < Q_; ++j) {
        if (load[(size_t)j] > load[(size_t)a]) a = j;
        if (load[(size_t)j] < load[(size_t)b]) b = j;
      }
      const float gap = load[(size_t)a] - load[(size_t)b];
      if (on[(size_t)a].empty()) break;
      const int last = on[(size_t)a].back();   // the piece queue a runs last
      const int len = pcs[(size_t)last].t1 - pcs[(size_t)last].t0;
      const bool whole = n_of_tile[(size_t)pcs[(size_t)last].tile - lo_] == 1;
      const float own = (float)len + kPieceTiles + (whole ? 0.f : kPartialTiles);
      if (own < gap) {   // the whole piece moves
        load[(size_t)a] -= own;
        load[(size_t)b] += own;
        on[(size_t)a].pop_back();
        on[(size_t)b].push_back(last);
        pcs[(size_t)last].queue = b;
        pcs[(size_t)last].rank = rank++;
        continue;
      }
      // x key tiles move: a ends at load[a] - x (+ a partial write, if the tile was whole),
      // b at load[b] + x + a piece boundary + a partial write
      const float fresh = whole ? kPartialTiles : 0.f;
      const int x = std::min((int)((gap - kPieceTiles - kPartialTiles + fresh) * 0.5f), len - kMinPieceTiles);
      if (x < kMinPieceTiles || n_of_tile[(size_t)pcs[(size_t)last].tile - lo_] >= oppo::kMaxSplit) break;
      if (n_partial + (whole ? 2 : 1) > max_partial) break;
      n_partial += whole ? 2 : 1;
      ++n_of_tile[(size_t)pcs[(size_t)last].tile - lo_];
      const int t1 = pcs[(size_t)last].t1;
      pcs[(size_t)last].t1 = t1 - x;
      load[(size_t)a] += fresh - (float)x;
      load[(size_t)b] += (float)x + kPieceTiles + kPartialTiles;
      on[(size_t)b].push_back((int)pcs.size());
      pcs.push_back(Piece{pcs[(size_t)last].tile, t1 - x, t1, b, rank++});
      ++added;
    }
  }

  // The tiles' key ranges laid end to end and cut into equal shares.
  void stream_cut(std::vector<Piece>& cut, int* nq_out) const {
    int64_t total = 0;
    int longest = 0;
    for (size_t i = lo_; i < hi_; ++i) total += tiles_[i].ntile, longest = std::max(longest, tiles_[i].ntile);
    const int min_piece = std::max(kMinPieceTiles, (longest + oppo::kMaxSplit - 2) / (oppo::kMaxSplit - 1));
    const int nq = (int)std::max<int64_t>(1, std::min<int64_t>(Q_, total / min_piece));
    int64_t off = 0;      // stream position of the current tile's first key tile
    int64_t prev = 0;     // previous cut
    size_t i = lo_;
    for (int j = 0; j < nq; ++j) {
      int64_t b = (j + 1 == nq) ? total : (total * (j + 1)) / nq;
      // find the tile the cut falls into and move the cut to an edge that is close
      {
        int64_t o2 = off;
        size_t i2 = i;
        while (i2 < hi_ && o2 + tiles_[i2].ntile <= b) o2 += tiles_[i2].ntile, ++i2;
        if (i2 < hi_) {
          const int64_t into = b - o2, rest = o2 + tiles_[i2].ntile - b;
          if (into > 0 && into < min_piece) b = o2;
          else if (into > 0 && rest < min_piece) b = o2 + tiles_[i2].ntile;
        }
      }
      b = std::max(b, prev);
      // hand [prev, b) to queue j
      int64_t pos = prev;
      while (pos < b) {
        const int64_t end = std::min<int64_t>(b, off + tiles_[i].ntile);
        cut.push_back(Piece{(int)i, (int)(pos - off), (int)(end - off), j, (int)cut.size()});
        pos = end;
        if (end == off + tiles_[i].ntile) off += tiles_[i].ntile, ++i;
      }
      prev = b;
    }
    *nq_out = nq;
  }

  // Pieces in launch order (grouped by queue), partial slots, merge items.
  void emit(const std::vector<Piece>& chosen, size_t* next_slot, Plan* plan) const {
    const size_t n = hi_ - lo_;
    std::vector<size_t> idx(chosen.size());
    for (size_t i = 0; i < idx.size(); ++i) idx[i] = i;
    auto len_of = [&](size_t a) { return chosen[a].t1 - chosen[a].t0; };
    std::stable_sort(idx.begin(), idx.end(), [&](size_t a, size_t b) {
      if (chosen[a].queue != chosen[b].queue) return chosen[a].queue < chosen[b].queue;
      if (opt_.order == 1) return a < b;
      if (opt_.order == 2) return len_of(a) < len_of(b);
      return chosen[a].rank < chosen[b].rank;
    });
    // partial slots: the pieces of a split tile take consecutive slots in key order
    std::vector<int32_t> slot_of(chosen.size(), -1);
    {
      std::vector<int32_t> count(n, 0);
      for (const Piece& pc : chosen) ++count[(size_t)pc.tile - lo_];
      std::vector<size_t> split;   // pieces of split tiles
      for (size_t a = 0; a < chosen.size(); ++a)
        if (count[(size_t)chosen[a].tile - lo_] > 1) split.push_back(a);
      std::sort(split.begin(), split.end(), [&](size_t a, size_t b) {
        return chosen[a].tile != chosen[b].tile ? chosen[a].tile < chosen[b].tile : chosen[a].t0 < chosen[b].t0;
      });
      for (size_t s = 0; s < split.size();) {
        const int tile = chosen[split[s]].tile;
        const QTile& qt = tiles_[(size_t)tile];
        oppo::CombineItem ci;
        ci.q_row0 = seqs_[(size_t)qt.seq].q_row0 + qt.j0;
        ci.n_tok = qt.n_tok;
        ci.part0 = (int32_t)*next_slot;
        ci.nsplit = count[(size_t)tile - lo_];
        plan->combines.push_back(ci);
        for (; s < split.size() && chosen[split[s]].tile == tile; ++s) slot_of[split[s]] = (int32_t)(*next_slot)++;
      }
    }
    plan->pieces.reserve(chosen.size());
    int queue_prev = -1;
    for (size_t a : idx) {
      const Piece& pc = chosen[a];
      const QTile& qt = tiles_[(size_t)pc.tile];
      const SeqView& s = seqs_[(size_t)qt.seq];
      if (pc.queue != queue_prev) plan->first.push_back((uint16_t)plan->pieces.size());   // empty queues vanish
      queue_prev = pc.queue;
      oppo::AttnItem it;
      it.kv_row0 = s.kv_row0;
      it.q_row0 = s.q_row0 + qt.j0;
      it.n_tok = oppo::pack_tokens(qt.n_tok, qt.j0 / ls_.TM);
      it.pos0 = s.kv_before + qt.j0;
      it.k_begin = pc.t0 * oppo::kKeyTile;
      it.k_end = std::min<int32_t>(qt.keys, pc.t1 * oppo::kKeyTile);
      it.part = slot_of[a];
      plan->pieces.push_back(it);
    }
    plan->first.push_back((uint16_t)plan->pieces.size());
  }

  const Options& opt_;
  const oppo::LayerShape& ls_;
  const std::vector<SeqView>& seqs_;
  const std::vector<QTile>& tiles_;
  const size_t lo_, hi_;
  const int Q_;
};

// Cut every sequence's chunk into query tiles and plan the launches (one, unless
// the work list outgrows the kernel-argument segment).
void make_plans(const Options& opt, const oppo::LayerShape& ls, const std::vector<SeqView>& seqs, size_t slots_avail,
                std::vector<Plan>* plans) {
  std::vector<QTile> tiles;
  for (size_t i = 0; i < seqs.size(); ++i) {
    const SeqView& s = seqs[i];
    for (int32_t j0 = 0; j0 < s.q_len; j0 += ls.TM) {
      QTile t;
      t.seq = (int)i;
      t.j0 = j0;
      t.n_tok = std::min(ls.TM, s.q_len - j0);
      t.keys = s.kv_before + j0 + t.n_tok;
      t.ntile = (t.keys + oppo::kKeyTile - 1) / oppo::kKeyTile;
      tiles.push_back(t);
    }
  }
  // a launch holds at most kMaxAttnItems pieces; cutting adds fewer than one piece per queue
  const size_t per_launch = (size_t)(oppo::kMaxAttnItems - queue_count(opt, ls));
  size_t next_slot = 0;
  for (size_t lo = 0; lo < tiles.size(); lo += per_launch) {
    plans->emplace_back();
    Plan* plan = &plans->back();
    const size_t hi = std::min(tiles.size(), lo + per_launch);
    LaunchPlanner planner(opt, ls, seqs, tiles, lo, hi);
    const size_t slot_mark = next_slot;
    planner.run(opt.split_kv, slots_avail, &next_slot, plan);
    if (plan->pieces.size() > (size_t)oppo::kMaxAttnItems) {
      // forced splitting made the list too long for one launch: this launch runs whole
      // tiles instead, and the slots the first attempt took are handed back
      next_slot = slot_mark;
      *plan = Plan();
      planner.run(1, slots_avail, &next_slot, plan);
    }
  }
}

// k_new / v_new non-null: the appending variant (the chunk's keys and values are
// read from there and written into k / v by the same kernel).
int run_attention(const Options& opt, const oppo::LayerShape& ls, const std::vector<SeqView>& seqs, const void* q,
                  void* k, void* v, const void* k_new, const void* v_new, void* out, void* workspace,
                  size_t workspace_bytes, void* stream, bool timed) {
  size_t slots = 0;
  float* part_o = nullptr;
  float* part_ml = nullptr;
  if (workspace && workspace_bytes > 0) {
    // slot s, kv-head g: O at part_o[((s*Hkv+g)*256 + row)*D], (m, l) at part_ml[((s*Hkv+g)*256 + row)*2]
    slots = workspace_bytes / oppo::part_slot_bytes(ls.Hkv, ls.D);
    part_o = (float*)workspace;
    part_ml = part_o + slots * (size_t)ls.Hkv * oppo::kTileRows * (size_t)ls.D;
  }
  for (const SeqView& s : seqs)
    if (s.q_len / ls.TM >= (1 << 22))
      return fail(OPPO_ERR_UNSUPPORTED, "%d rows of one sequence in one call exceed the work descriptor's range", s.q_len);
  const bool clocked = timed && oppo::profile_is_on();
  const double t0 = clocked ? now_us() : 0.0;
  std::vector<Plan> plans;
  make_plans(opt, ls, seqs, slots, &plans);
  const double t1 = clocked ? now_us() : 0.0;
  for (const Plan& plan : plans) {
    const int e = oppo::launch_attention(ls, q, k, v, k_new, v_new, out, part_o, part_ml, plan.pieces.data(),
                                         (int)plan.pieces.size(), plan.first.data(), (int)plan.first.size() - 1, stream,
                                         timed);
    if (e) return fail(OPPO_ERR_HIP, "attention launch failed: %s", oppo::hip_error_string(e));
  }
  for (const Plan& plan : plans) {
    if (plan.combines.empty()) continue;
    const int e = oppo::launch_combine(ls, out, part_o, part_ml, plan.combines.data(), (int)plan.combines.size(), stream,
                                       timed);
    if (e) return fail(OPPO_ERR_HIP, "combine launch failed: %s", oppo::hip_error_string(e));
  }
  if (clocked) {
    const double t2 = now_us();
    std::lock_guard<std::mutex> lock(g_host_mu);
    g_host_plan_us += t1 - t0;
    g_host_launch_us += t2 - t1;
    g_host_calls += 1;
  }
  return OPPO_OK;
}

// A workspace is optional.  One that is given must be aligned and hold at least one
// partial slot; beyond that its size only bounds how many pieces key ranges are cut into.
int check_workspace(const oppo::LayerShape& ls, const void* workspace, size_t workspace_bytes) {
  if (!workspace || workspace_bytes == 0) return OPPO_OK;
  if (((uintptr_t)workspace & 255) != 0) return fail(OPPO_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  const size_t one = oppo::part_slot_bytes(ls.Hkv, ls.D);
  if (workspace_bytes < one)
    return fail(OPPO_ERR_WORKSPACE, "workspace has %zu bytes, one partial slot takes %zu (pass none to disable splitting)",
                workspace_bytes, one);
  return OPPO_OK;
}

// The sequences of an attention-only pass: kv_len is the length after the append.
int views_after_append(const oppo_kv_cache* cache, const int32_t* cu_q, std::vector<SeqView>* seqs) {
  for (int32_t i = 0; i < cache->batch; ++i) {
    const int32_t ql = cu_q[i + 1] - cu_q[i];
    if (ql > cache->kv_len[i])
      return fail(OPPO_ERR_INVALID, "sequence %d: %d query rows but only %d cached tokens (append first)", i, ql,
                  cache->kv_len[i]);
    if (ql == 0) continue;
    seqs->push_back(SeqView{cache->slot_begin[i], cu_q[i], ql, cache->kv_len[i] - ql});
  }
  return OPPO_OK;
}

// The sequences of a fused pass: kv_len is the length before the append.
void views_before_append(const oppo_kv_cache* cache, const int32_t* cu_q, std::vector<SeqView>* seqs) {
  for (int32_t i = 0; i < cache->batch; ++i) {
    const int32_t ql = cu_q[i + 1] - cu_q[i];
    if (ql == 0) continue;
    seqs->push_back(SeqView{cache->slot_begin[i], cu_q[i], ql, cache->kv_len[i]});
  }
}

// Checks shared by oppo_chunk_step and its variant with the built-in scratch buffer.
int chunk_step_checks(const oppo_attn_desc* desc, const oppo_kv_cache* cache, const int32_t* cu_q, oppo::LayerShape* ls,
                      std::vector<SeqView>* seqs) {
  int rc = check_desc(desc, ls);
  if (rc) return rc;
  rc = check_cache(cache);
  if (rc) return rc;
  rc = check_cu(cu_q, cache->batch, "cu_q");
  if (rc) return rc;
  rc = check_room(cache, cu_q);
  if (rc) return rc;
  if ((int64_t)cu_q[cache->batch] * ls->Hq > INT32_MAX)
    return fail(OPPO_ERR_UNSUPPORTED, "%d query rows x %d heads exceed the 32-bit row index of the kernel",
                cu_q[cache->batch], ls->Hq);
  views_before_append(cache, cu_q, seqs);
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
  rc = check_cache(cache);
  if (rc) return rc;
  const int32_t B = cache->batch;
  rc = check_cu(cu_q, B, "cu_q");
  if (rc) return rc;
  rc = check_room(cache, cu_q);
  if (rc) return rc;
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

int oppo_kv_append_fp8(const oppo_attn_desc* desc, oppo_kv_cache_fp8* cache, const int32_t* cu_q, const void* k_new,
                       const void* v_new, void* stream) {
  oppo::LayerShape ls;
  int rc = check_desc(desc, &ls);
  if (rc) return rc;
  oppo_kv_cache view;
  rc = check_cache_fp8(cache, &view);
  if (rc) return rc;
  const int32_t B = view.batch;
  rc = check_cu(cu_q, B, "cu_q");
  if (rc) return rc;
  rc = check_room(&view, cu_q);
  if (rc) return rc;
  if (cu_q[B] == 0) return OPPO_OK;
  if (!view.k || !view.v || !k_new || !v_new) return fail(OPPO_ERR_INVALID, "null device pointer");
  std::vector<oppo::AppendItem> items;
  for (int32_t i = 0; i < B; ++i) {
    const int32_t ql = cu_q[i + 1] - cu_q[i];
    if (ql == 0) continue;
    oppo::AppendItem it;
    it.dst_row = view.slot_begin[i] + view.kv_len[i];
    it.src_row = cu_q[i];
    it.n_tok = ql;
    items.push_back(it);
  }
  const int e = oppo::launch_append_fp8(ls, view.k, view.v, k_new, v_new, 1.0f / cache->k_scale, 1.0f / cache->v_scale,
                                        items.data(), (int)items.size(), stream);
  if (e) return fail(OPPO_ERR_HIP, "append launch failed: %s", oppo::hip_error_string(e));
  for (int32_t i = 0; i < B; ++i) cache->kv_len[i] += cu_q[i + 1] - cu_q[i];
  return OPPO_OK;
}

int oppo_chunk_prefill_attn_fp8(const oppo_attn_desc* desc, const oppo_kv_cache_fp8* cache, const int32_t* cu_q,
                                const void* q, void* out, void* workspace, size_t workspace_bytes, void* stream) {
  const Options opt = options_now();
  oppo::LayerShape ls;
  int rc = check_desc(desc, &ls);
  if (rc) return rc;
  oppo_kv_cache view;
  rc = check_cache_fp8(cache, &view);
  if (rc) return rc;
  const int32_t B = view.batch;
  rc = check_cu(cu_q, B, "cu_q");
  if (rc) return rc;
  rc = check_workspace(ls, workspace, workspace_bytes);
  if (rc) return rc;
  if ((int64_t)cu_q[B] * ls.Hq > INT32_MAX)
    return fail(OPPO_ERR_UNSUPPORTED, "%d query rows x %d heads exceed the 32-bit row index of the kernel", cu_q[B],
                ls.Hq);
  std::vector<SeqView> seqs;
  rc = views_after_append(&view, cu_q, &seqs);
  if (rc) return rc;
  if (seqs.empty()) return OPPO_OK;
  if (!view.k || !view.v || !q || !out) return fail(OPPO_ERR_INVALID, "null device pointer");
  // the keys' scale goes into the score scale, the values' into the final normalisation
  ls.fp8 = 1;
  ls.c *= cache->k_scale;
  ls.out_scale = cache->v_scale;
  // (the kernel splits the score factor into a power of two, which it hands to the matrix instruction as a
  // block scale, and a factor in [4, 8): the exponent has to be representable there)
  if (!(ls.c >= 0x1p-100f) || !(ls.c <= 0x1p100f))
    return fail(OPPO_ERR_INVALID, "softmax_scale x k_scale = %g is outside 2^-100 .. 2^100", (double)ls.c / 1.4426950408889634);
  return run_attention(opt, ls, seqs, q, view.k, view.v, nullptr, nullptr, out, workspace, workspace_bytes, stream, true);
}

int oppo_rope(const oppo_attn_desc* desc, int32_t batch, const int32_t* kv_before, const int32_t* cu_q, void* q,
              void* k_new, double theta_base, void* stream) {
  oppo::LayerShape ls;
  int rc = check_desc(desc, &ls);
  if (rc) return rc;
  if (batch < 0) return fail(OPPO_ERR_INVALID, "batch is negative");
  if (!kv_before && batch > 0) return fail(OPPO_ERR_INVALID, "kv_before is null");
  rc = check_cu(cu_q, batch, "cu_q");
  if (rc) return rc;
  if (!(theta_base > 1.0) || !std::isfinite(theta_base))
    return fail(OPPO_ERR_INVALID, "theta_base must be finite and greater than 1 (got %g)", theta_base);
  std::vector<oppo::RopeItem> items;
  for (int32_t i = 0; i < batch; ++i) {
    const int32_t ql = cu_q[i + 1] - cu_q[i];
    if (kv_before[i] < 0) return fail(OPPO_ERR_INVALID, "kv_before[%d]=%d is negative", i, kv_before[i]);
    if ((int64_t)kv_before[i] + ql > INT32_MAX) return fail(OPPO_ERR_INVALID, "sequence %d: positions exceed 2^31", i);
    if (ql == 0) continue;
    oppo::RopeItem it;
    it.row0 = cu_q[i];
    it.n_tok = ql;
    it.pos0 = kv_before[i];
    items.push_back(it);
  }
  if (items.empty() || (!q && !k_new)) return OPPO_OK;
  int e = oppo::launch_rope(ls, q, k_new, items.data(), (int)items.size(), theta_base, stream);
  if (e) return fail(OPPO_ERR_HIP, "rope launch failed: %s", oppo::hip_error_string(e));
  return OPPO_OK;
}

int oppo_qkv_rope_append(const oppo_attn_desc* desc, oppo_kv_cache* cache, const int32_t* cu_q, const void* qkv,
                         void* q_out, double theta_base, void* stream) {
  oppo::LayerShape ls;
  int rc = check_desc(desc, &ls);
  if (rc) return rc;
  rc = check_cache(cache);
  if (rc) return rc;
  const int32_t B = cache->batch;
  rc = check_cu(cu_q, B, "cu_q");
  if (rc) return rc;
  if (!(theta_base > 1.0) || !std::isfinite(theta_base))
    return fail(OPPO_ERR_INVALID, "theta_base must be finite and greater than 1 (got %g)", theta_base);
  rc = check_room(cache, cu_q);
  if (rc) return rc;
  if (cu_q[B] == 0) return OPPO_OK;
  if (!cache->k || !cache->v || !qkv || !q_out) return fail(OPPO_ERR_INVALID, "null device pointer");
  std::vector<oppo::QkvItem> items;
  for (int32_t i = 0; i < B; ++i) {
    const int32_t ql = cu_q[i + 1] - cu_q[i];
    if (ql == 0) continue;
    oppo::QkvItem it;
    it.dst_row = cache->slot_begin[i] + cache->kv_len[i];
    it.src_row = cu_q[i];
    it.n_tok = ql;
    it.pos0 = cache->kv_len[i];
    it.pad_ = 0;
    items.push_back(it);
  }
  int e = oppo::launch_qkv_rope_append(ls, qkv, q_out, cache->k, cache->v, items.data(), (int)items.size(), theta_base,
                                       stream);
  if (e) return fail(OPPO_ERR_HIP, "qkv epilogue launch failed: %s", oppo::hip_error_string(e));
  for (int32_t i = 0; i < B; ++i) cache->kv_len[i] += cu_q[i + 1] - cu_q[i];
  return OPPO_OK;
}

size_t oppo_qkv_proj_workspace_bytes(const oppo_attn_desc* desc, int32_t max_rows) {
  oppo::LayerShape ls;
  if (max_rows < 0 || check_desc(desc, &ls) != OPPO_OK) return 0;
  return oppo::proj_workspace_bytes(ls.D, max_rows);
}

int oppo_qkv_proj_rope_append(const oppo_attn_desc* desc, oppo_kv_cache* cache, const int32_t* cu_q, const void* x,
                              int32_t hidden, const void* w, void* q_out, double theta_base, void* workspace,
                              size_t workspace_bytes, void* stream) {
  oppo::LayerShape ls;
  int rc = check_desc(desc, &ls);
  if (rc) return rc;
  rc = check_cache(cache);
  if (rc) return rc;
  const int32_t B = cache->batch;
  rc = check_cu(cu_q, B, "cu_q");
  if (rc) return rc;
  if (!(theta_base > 1.0) || !std::isfinite(theta_base))
    return fail(OPPO_ERR_INVALID, "theta_base must be finite and greater than 1 (got %g)", theta_base);
  if (hidden < 1) return fail(OPPO_ERR_INVALID, "hidden=%d must be positive", hidden);
  if (hidden % 64 != 0) return fail(OPPO_ERR_UNSUPPORTED, "hidden=%d is not a multiple of 64", hidden);
  rc = check_room(cache, cu_q);
  if (rc) return rc;
  const int32_t rows = cu_q[B];
  if (rows == 0) return OPPO_OK;
  if ((int64_t)rows * hidden > INT32_MAX || (int64_t)rows * ls.Hq * ls.D > INT32_MAX)
    return fail(OPPO_ERR_UNSUPPORTED, "%d rows x %d columns exceed the 32-bit element index of the kernel", rows,
                std::max(hidden, ls.Hq * ls.D));
  if (!cache->k || !cache->v || !x || !w || !q_out) return fail(OPPO_ERR_INVALID, "null device pointer");
  const size_t need = oppo::proj_workspace_bytes(ls.D, rows);
  if (!workspace || ((uintptr_t)workspace & 255) != 0)
    return fail(OPPO_ERR_WORKSPACE, "workspace is null or not 256-byte aligned");
  if (workspace_bytes < need)
    return fail(OPPO_ERR_WORKSPACE, "workspace has %zu bytes, %zu required for %d rows", workspace_bytes, need, rows);
  std::vector<oppo::QkvItem> items;
  for (int32_t i = 0; i < B; ++i) {
    const int32_t ql = cu_q[i + 1] - cu_q[i];
    if (ql == 0) continue;
    oppo::QkvItem it;
    it.dst_row = cache->slot_begin[i] + cache->kv_len[i];
    it.src_row = cu_q[i];
    it.n_tok = ql;
    it.pos0 = cache->kv_len[i];
    it.pad_ = 0;
    items.push_back(it);
  }
  int e = oppo::launch_qkv_proj(ls, x, w, hidden, rows, q_out, cache->k, cache->v, items.data(), (int)items.size(),
                                theta_base, workspace, stream);
  if (e) return fail(OPPO_ERR_HIP, "projection launch failed: %s", oppo::hip_error_string(e));
  for (int32_t i = 0; i < B; ++i) cache->kv_len[i] += cu_q[i + 1] - cu_q[i];
  return OPPO_OK;
}

int oppo_chunk_prefill_attn(const oppo_attn_desc* desc, const oppo_kv_cache* cache, const int32_t* cu_q,
                            const void* q, void* out, void* workspace, size_t workspace_bytes, void* stream) {
  oppo::LayerShape ls;
  int rc = check_desc(desc, &ls);
  if (rc) return rc;
  rc = check_cache(cache);
  if (rc) return rc;
  const int32_t B = cache->batch;
  rc = check_cu(cu_q, B, "cu_q");
  if (rc) return rc;
  std::vector<SeqView> seqs;
  rc = views_after_append(cache, cu_q, &seqs);
  if (rc) return rc;
  rc = check_workspace(ls, workspace, workspace_bytes);
  if (rc) return rc;
  if ((int64_t)cu_q[B] * ls.Hq > INT32_MAX)
    return fail(OPPO_ERR_UNSUPPORTED, "%d query rows x %d heads exceed the 32-bit row index of the kernel", cu_q[B], ls.Hq);
  if (seqs.empty()) return OPPO_OK;
  if (!cache->k || !cache->v || !q || !out) return fail(OPPO_ERR_INVALID, "null device pointer");
  return run_attention(options_now(), ls, seqs, q, cache->k, cache->v, nullptr, nullptr, out, workspace, workspace_bytes,
                       stream, true);
}

int oppo_chunk_step(const oppo_attn_desc* desc, oppo_kv_cache* cache, const int32_t* cu_q, const void* q,
                    const void* k_new, const void* v_new, void* out, void* workspace, size_t workspace_bytes,
                    void* stream) {
  oppo::LayerShape ls;
  std::vector<SeqView> seqs;
  int rc = chunk_step_checks(desc, cache, cu_q, &ls, &seqs);
  if (rc) return rc;
  rc = check_workspace(ls, workspace, workspace_bytes);
  if (rc) return rc;
  if (seqs.empty()) return OPPO_OK;
  if (!cache->k || !cache->v || !q || !k_new || !v_new || !out) return fail(OPPO_ERR_INVALID, "null device pointer");
  rc = run_attention(options_now(), ls, seqs, q, cache->k, cache->v, k_new, v_new, out, workspace, workspace_bytes, stream,
                     true);
  if (rc) return rc;
  for (int32_t i = 0; i < cache->batch; ++i) cache->kv_len[i] += cu_q[i + 1] - cu_q[i];
  return OPPO_OK;
}

size_t oppo_static_scratch_bytes(void) { return oppo::kStaticScratchBytes; }

int oppo_chunk_step_noalloc(const oppo_attn_desc* desc, oppo_kv_cache* cache, const int32_t* cu_q, const void* q,
                            const void* k_new, const void* v_new, void* out, void* stream) {
  oppo::LayerShape ls;
  std::vector<SeqView> seqs;
  int rc = chunk_step_checks(desc, cache, cu_q, &ls, &seqs);
  if (rc) return rc;
  // the built-in buffer has to hold the partial results of at least one fully split
  // query tile of this layer shape
  const size_t one = oppo::part_slot_bytes(ls.Hkv, ls.D);
  if (one * (size_t)oppo::kMaxSplit > oppo::kStaticScratchBytes)
    return fail(OPPO_ERR_UNSUPPORTED,
                "layer too wide for the built-in scratch buffer: Hkv x (D + 2) = %d exceeds %zu; use oppo_chunk_step "
                "with a workspace of the caller's",
                ls.Hkv * (ls.D + 2), oppo::kStaticScratchBytes / ((size_t)oppo::kMaxSplit * oppo::kTileRows * sizeof(float)));
  if (seqs.empty()) return OPPO_OK;
  if (!cache->k || !cache->v || !q || !k_new || !v_new || !out) return fail(OPPO_ERR_INVALID, "null device pointer");
  void* scratch = nullptr;
  const int e = oppo::static_scratch(&scratch);
  if (e) return fail(OPPO_ERR_HIP, "address of the built-in scratch buffer: %s", oppo::hip_error_string(e));
  // (no event pairs here: creating them would allocate)
  rc = run_attention(options_now(), ls, seqs, q, cache->k, cache->v, k_new, v_new, out, scratch,
                     oppo::kStaticScratchBytes, stream, false);
  if (rc) return rc;
  for (int32_t i = 0; i < cache->batch; ++i) cache->kv_len[i] += cu_q[i + 1] - cu_q[i];
  return OPPO_OK;
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
  if ((int64_t)cu_seq[B] * ls.Hq > INT32_MAX)
    return fail(OPPO_ERR_UNSUPPORTED, "%d rows x %d heads exceed the 32-bit row index of the kernel", cu_seq[B], ls.Hq);
  std::vector<SeqView> seqs;
  for (int32_t i = 0; i < B; ++i) {
    const int32_t n = cu_seq[i + 1] - cu_seq[i];
    if (n == 0) continue;
    seqs.push_back(SeqView{cu_seq[i], cu_seq[i], n, 0});
  }
  if (seqs.empty()) return OPPO_OK;
  if (!q || !k || !v || !out) return fail(OPPO_ERR_INVALID, "null device pointer");
  return run_attention(options_now(), ls, seqs, q, const_cast<void*>(k), const_cast<void*>(v), nullptr, nullptr, out,
                       workspace, workspace_bytes, stream, true);
}

size_t oppo_workspace_bytes(const oppo_attn_desc* desc, int32_t max_batch, int32_t max_q_tokens) {
  oppo::LayerShape ls;
  if (max_batch < 0 || max_q_tokens < 0) return 0;
  if (check_desc(desc, &ls) != OPPO_OK) return 0;
  return useful_slots(options_now(), ls, max_batch, max_q_tokens) * oppo::part_slot_bytes(ls.Hkv, ls.D);
}

int oppo_set_option(int option, int value) {
  if (value < 0) return fail(OPPO_ERR_INVALID, "option value is negative");
  std::lock_guard<std::mutex> lock(g_opt_mu);
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
    if (q_len[i] > 0) seqs.push_back(SeqView{i /* stands for the sequence index in the dump */, (int32_t)row, q_len[i], kv_before[i]});
    row += q_len[i];
  }
  std::vector<Plan> plans;
  make_plans(options_now(), ls, seqs, workspace_bytes / oppo::part_slot_bytes(ls.Hkv, ls.D), &plans);
  size_t total = 0;
  for (const Plan& plan : plans) total += plan.pieces.size();
  *n_items = (int32_t)total;
  if ((int64_t)total > max_items) return fail(OPPO_ERR_INVALID, "plan has %zu pieces", total);
  size_t w = 0;
  int32_t queue0 = 0;
  for (const Plan& plan : plans) {
    for (size_t j = 0; j + 1 < plan.first.size(); ++j)
      for (size_t i = plan.first[j]; i < plan.first[j + 1]; ++i, ++w) {
        const oppo::AttnItem& it = plan.pieces[i];
        int32_t* o = items + 8 * w;
        o[0] = (int32_t)it.kv_row0;
        o[1] = it.q_row0;
        o[2] = oppo::tokens_of(it);
        o[3] = it.pos0;
        o[4] = it.k_begin;
        o[5] = it.k_end;
        o[6] = it.part;
        o[7] = queue0 + (int32_t)j;
      }
    queue0 += (int32_t)plan.first.size() - 1;
  }
  return OPPO_OK;
}

int oppo_profile_enable(int on) { return oppo::profile_enable(on); }

int oppo_profile_read(double* kernel_ms, int32_t* launches) {
  if (!kernel_ms || !launches) return fail(OPPO_ERR_INVALID, "null array");
  const int e = oppo::profile_read(kernel_ms, launches, nullptr, nullptr, 0, nullptr);
  if (e) return fail(OPPO_ERR_HIP, "event timing failed: %s", oppo::hip_error_string(e));
  return OPPO_OK;
}

int oppo_profile_read_each(double* each_ms, int32_t* each_kind, int32_t max_n, int32_t* n) {
  if (!each_ms || !each_kind || !n || max_n < 0) return fail(OPPO_ERR_INVALID, "null array or negative size");
  double ms[3];
  int32_t launches[3];
  const int e = oppo::profile_read(ms, launches, each_ms, each_kind, max_n, n);
  if (e) return fail(OPPO_ERR_HIP, "event timing failed: %s", oppo::hip_error_string(e));
  if (launches[0] + launches[1] + launches[2] > max_n)
    return fail(OPPO_ERR_INVALID, "%d launches were recorded, room for %d", launches[0] + launches[1] + launches[2], max_n);
  return OPPO_OK;
}

int oppo_profile_host(double* host_us, int64_t* calls) {
  if (!host_us || !calls) return fail(OPPO_ERR_INVALID, "null array");
  std::lock_guard<std::mutex> lock(g_host_mu);
  host_us[0] = g_host_plan_us;
  host_us[1] = g_host_launch_us;
  *calls = g_host_calls;
  g_host_plan_us = g_host_launch_us = 0.0;
  g_host_calls = 0;
  return OPPO_OK;
}

const char* oppo_last_error(void) { return g_err; }

int oppo_version(void) { return 200; }

}  // extern "C"
