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
Options g_opt;

// Cost model of the planner, in units of one 64-key tile of one workgroup
// (about 1.9 us on MI355X): what a piece costs beyond its tiles (draining the
// pipeline, writing the rows, switching over to the next piece: measured 4 to 5
// us), what a partial result costs on top (256 rows x (D + 2) floats per kv-head
// written out), and the merge kernel (a launch of its own plus reading the
// partials back: its measured duration fits 4 us + 0.17 us per piece).
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

// One launch of the attention kernel: pieces grouped by queue.
struct Plan {
  std::vector<oppo::AttnItem> pieces;
  std::vector<uint16_t> first;   // queue j runs pieces first[j] .. first[j+1]-1
  std::vector<oppo::CombineItem> combines;
};

int queue_count(const oppo::LayerShape& ls) {
  return std::max(1, std::min(g_opt.num_cus / ls.Hkv, oppo::kMaxQueues));
}

// A query tile: TM tokens of one sequence against all keys it may see.
struct QTile { int seq; int32_t j0, n_tok, keys, ntile; };

// Plan one launch for the query tiles [lo, hi).
//
// The kernel runs one persistent workgroup per (queue, kv-head); the planner
// decides which pieces each queue runs.  Three ways of filling the queues are
// priced with the cost model above and the cheapest one is taken:
//   * whole tiles, sequence by sequence onto the least loaded group of queues (see
//     gang_schedule) - no partial results, but the longest tile bounds the
//     makespan and with few tiles per queue the loads are uneven (the thin tail
//     passes of a long-tailed batch);
//   * the same with the ends of the queues evened out (see even_out): a few tiles
//     are split, most stay whole;
//   * the tiles' key ranges laid end to end and cut into equal shares, one per
//     queue: a tile that straddles a cut is split there (on a 64-key boundary)
//     and its pieces are merged afterwards.  A cut that falls close to a tile
//     edge moves to the edge.
void plan_launch(const oppo::LayerShape& ls, const std::vector<SeqView>& seqs, const std::vector<QTile>& tiles,
                 size_t lo, size_t hi, size_t slots_avail, size_t* next_slot, Plan* plan) {
  const int Q = queue_count(ls);
  const size_t n = hi - lo;
  struct Piece { int tile; int t0, t1; int queue; int rank; };   // key tiles [t0, t1) of query tile `tile`; rank = order of scheduling
  auto price = [&](const std::vector<Piece>& pcs, int nq, size_t* n_partial) {
    std::vector<float> load((size_t)nq, 0.f);
    size_t np = 0;
    for (const Piece& pc : pcs) {
      const bool whole = pc.t0 == 0 && pc.t1 == tiles[pc.tile].ntile;
      load[pc.queue] += (float)(pc.t1 - pc.t0) + kPieceTiles + (whole ? 0.f : kPartialTiles);
      np += whole ? 0 : 1;
    }
    float ms = 0.f;
    for (float x : load) ms = std::max(ms, x);
    if (n_partial) *n_partial = np;
    return ms + (np ? kMergeTiles + kMergeTilesPerPiece * (float)np : 0.f);
  };
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
  auto gang_schedule = [&](std::vector<Piece>& pcs) {
    std::vector<std::vector<size_t>> of_seq(seqs.size());
    for (size_t a = 0; a < pcs.size(); ++a) of_seq[tiles[pcs[a].tile].seq].push_back(a);
    std::vector<int> order;
    std::vector<int64_t> work(seqs.size(), 0);
    for (size_t i = 0; i < seqs.size(); ++i) {
      for (size_t a : of_seq[i]) work[i] += pcs[a].t1 - pcs[a].t0;
      if (!of_seq[i].empty()) order.push_back((int)i);
    }
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return work[a] > work[b]; });
    std::vector<float> load((size_t)Q, 0.f);
    int rank = 0;
    std::vector<int> qs;
    for (int sq : order) {
      std::vector<size_t>& mem = of_seq[sq];
      std::stable_sort(mem.begin(), mem.end(), [&](size_t a, size_t b) {
        return pcs[a].t1 - pcs[a].t0 > pcs[b].t1 - pcs[b].t0;
      });
      for (size_t m0 = 0; m0 < mem.size(); m0 += (size_t)Q) {
        const int g = (int)std::min<size_t>((size_t)Q, mem.size() - m0);
        int step = 1;   // largest divisor of Q that does not exceed the gang
        for (int d = 1; d <= g; ++d)
          if (Q % d == 0) step = d;
        float best = 0.f;
        int best_start = -1;
        for (int st = 0; st < Q; st += step) {
          qs.clear();
          for (int m = 0; m < g; ++m) qs.push_back((st + m) % Q);
          std::sort(qs.begin(), qs.end(), [&](int a, int b) { return load[a] < load[b] || (load[a] == load[b] && a < b); });
          float mx = 0.f;
          for (int m = 0; m < g; ++m)
            mx = std::max(mx, load[qs[m]] + (float)(pcs[mem[m0 + m]].t1 - pcs[mem[m0 + m]].t0));
          if (best_start < 0 || mx < best) best = mx, best_start = st;
        }
        qs.clear();
        for (int m = 0; m < g; ++m) qs.push_back((best_start + m) % Q);
        std::sort(qs.begin(), qs.end(), [&](int a, int b) { return load[a] < load[b] || (load[a] == load[b] && a < b); });
        for (int m = 0; m < g; ++m) {
          Piece& pc = pcs[mem[m0 + m]];
          pc.queue = qs[m];
          pc.rank = rank++;
          load[qs[m]] += (float)(pc.t1 - pc.t0) + kPieceTiles;
        }
      }
    }
  };

  // Evening out a schedule of whole tiles: as long as it pays, the most loaded
  // queue hands the end of its day to the least loaded one - its last piece as a
  // whole if that fits into the gap, otherwise the rear part of that piece's key
  // range, sized so that both queues end together (the tile is then merged from
  // partial results).  Only the ends of the queues change, so the gangs further
  // up keep running side by side.  Adds fewer than Q pieces.
  auto even_out = [&](std::vector<Piece>& pcs, size_t max_partial) {
    std::vector<float> load((size_t)Q, 0.f);
    std::vector<int> n_of_tile(n, 0);
    for (const Piece& pc : pcs) {
      load[pc.queue] += (float)(pc.t1 - pc.t0) + kPieceTiles;
      ++n_of_tile[pc.tile - lo];
    }
    size_t n_partial = 0;
    int rank = (int)pcs.size();
    for (int added = 0, moves = 0; added + 1 < Q && moves < 8 * Q; ++moves) {
      int a = 0, b = 0;
      for (int j = 1; j < Q; ++j) {
        if (load[j] > load[a]) a = j;
        if (load[j] < load[b]) b = j;
      }
      const float gap = load[a] - load[b];
      int last = -1;   // the piece queue a runs last
      for (size_t k = 0; k < pcs.size(); ++k)
        if (pcs[k].queue == a && (last < 0 || pcs[k].rank > pcs[last].rank)) last = (int)k;
      if (last < 0) break;
      const int len = pcs[last].t1 - pcs[last].t0;
      const bool whole = n_of_tile[pcs[last].tile - lo] == 1;
      const float own = (float)len + kPieceTiles + (whole ? 0.f : kPartialTiles);
      if (own < gap) {   // the whole piece moves
        load[a] -= own;
        load[b] += own;
        pcs[last].queue = b;
        pcs[last].rank = rank++;
        continue;
      }
      // x key tiles move: a ends at load[a] - x (+ a partial write, if the tile was whole),
      // b at load[b] + x + a piece boundary + a partial write
      const float fresh = whole ? kPartialTiles : 0.f;
      const int x = std::min((int)((gap - kPieceTiles - kPartialTiles + fresh) * 0.5f), len - kMinPieceTiles);
      if (x < kMinPieceTiles || n_of_tile[pcs[last].tile - lo] >= oppo::kMaxSplit) break;
      if (n_partial + (whole ? 2 : 1) > max_partial) break;
      n_partial += whole ? 2 : 1;
      ++n_of_tile[pcs[last].tile - lo];
      const int t1 = pcs[last].t1;
      pcs[last].t1 = t1 - x;
      load[a] += fresh - (float)x;
      load[b] += (float)x + kPieceTiles + kPartialTiles;
      pcs.push_back(Piece{pcs[last].tile, t1 - x, t1, b, rank++});
      ++added;
    }
  };

  // Whole pieces change queues while that shortens the longest queue: the most loaded
  // queue gives a piece to the least loaded one, or the two exchange a pair.  (Greedy
  // placement of a handful of pieces per queue leaves the loads a few per cent apart.)
  // A piece keeps its place in the scheduling order, so on its new queue it still runs at
  // about the time its gang does.
  auto swap_pieces = [&](std::vector<Piece>& pcs) {
    std::vector<float> load((size_t)Q, 0.f);
    std::vector<std::vector<int>> on((size_t)Q);   // pieces of each queue
    for (size_t x = 0; x < pcs.size(); ++x) {
      load[pcs[x].queue] += (float)(pcs[x].t1 - pcs[x].t0) + kPieceTiles;
      on[pcs[x].queue].push_back((int)x);
    }
    auto cost = [&](int x) { return (float)(pcs[x].t1 - pcs[x].t0) + kPieceTiles; };
    // (the pieces of one sequence stay on different queues)
    auto holds = [&](int queue, int seq, int except) {
      for (int z : on[queue])
        if (z != except && tiles[pcs[z].tile].seq == seq) return true;
      return false;
    };
    auto move = [&](int x, int from, int to) {
      std::vector<int>& f = on[from];
      f.erase(std::find(f.begin(), f.end(), x));
      on[to].push_back(x);
      pcs[x].queue = to;
      load[from] -= cost(x), load[to] += cost(x);
    };
    for (int round = 0; round < 4 * Q; ++round) {
      int a = 0, b = 0;
      for (int j = 1; j < Q; ++j) {
        if (load[j] > load[a]) a = j;
        if (load[j] < load[b]) b = j;
      }
      float best = load[a] - 0.5f;   // a move has to gain at least half a tile
      int bx = -1, by = -1;
      for (int x : on[a]) {
        const float cx = cost(x);
        const int sx = tiles[pcs[x].tile].seq;
        if (std::max(load[a] - cx, load[b] + cx) < best && !holds(b, sx, -1))
          best = std::max(load[a] - cx, load[b] + cx), bx = x, by = -1;
        for (int y : on[b]) {
          const float cy = cost(y);
          const float m = std::max(load[a] - cx + cy, load[b] + cx - cy);
          if (m < best && !holds(b, sx, y) && !holds(a, tiles[pcs[y].tile].seq, x)) best = m, bx = x, by = y;
        }
      }
      if (bx < 0) break;
      move(bx, a, b);
      if (by >= 0) move(by, b, a);
    }
  };

  const size_t slots_left = slots_avail > *next_slot ? slots_avail - *next_slot : 0;
  std::vector<Piece> chosen;
  if (g_opt.split_kv >= 2 && slots_left > 0) {
    // forced: every tile in (up to) that many even pieces
    size_t used = 0;
    for (size_t i = lo; i < hi; ++i) {
      const int nt = tiles[i].ntile;
      int ns = std::min(std::min(g_opt.split_kv, nt), oppo::kMaxSplit);
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
    for (size_t i = lo; i < hi; ++i) chosen.push_back(Piece{(int)i, 0, tiles[i].ntile, 0, 0});
    gang_schedule(chosen);
    swap_pieces(chosen);
    if (g_opt.split_kv == 0 && slots_left > 0) {
      float whole_cost = price(chosen, Q, nullptr);
      {
        std::vector<Piece> evened = chosen;
        even_out(evened, slots_left);
        const float evened_cost = price(evened, Q, nullptr);
        if (evened_cost < 0.97f * whole_cost) chosen.swap(evened), whole_cost = evened_cost;
      }
      int64_t total = 0;
      int longest = 0;
      for (size_t i = lo; i < hi; ++i) total += tiles[i].ntile, longest = std::max(longest, tiles[i].ntile);
      const int min_piece = std::max(kMinPieceTiles, (longest + oppo::kMaxSplit - 2) / (oppo::kMaxSplit - 1));
      const int nq = (int)std::max<int64_t>(1, std::min<int64_t>(Q, total / min_piece));
      std::vector<Piece> cut;
      int64_t off = 0;      // stream position of the current tile's first key tile
      int64_t prev = 0;     // previous cut
      size_t i = lo;
      for (int j = 0; j < nq; ++j) {
        int64_t b = (j + 1 == nq) ? total : (total * (j + 1)) / nq;
        // find the tile the cut falls into and move the cut to an edge that is close
        {
          int64_t o2 = off;
          size_t i2 = i;
          while (i2 < hi && o2 + tiles[i2].ntile <= b) o2 += tiles[i2].ntile, ++i2;
          if (i2 < hi) {
            const int64_t into = b - o2, rest = o2 + tiles[i2].ntile - b;
            if (into > 0 && into < min_piece) b = o2;
            else if (into > 0 && rest < min_piece) b = o2 + tiles[i2].ntile;
          }
        }
        b = std::max(b, prev);
        // hand [prev, b) to queue j
        int64_t pos = prev;
        while (pos < b) {
          const int64_t end = std::min<int64_t>(b, off + tiles[i].ntile);
          cut.push_back(Piece{(int)i, (int)(pos - off), (int)(end - off), j, (int)cut.size()});
          pos = end;
          if (end == off + tiles[i].ntile) off += tiles[i].ntile, ++i;
        }
        prev = b;
      }
      size_t n_partial = 0;
      const float cut_cost = price(cut, nq, &n_partial);
      if (n_partial <= slots_left && cut_cost < 0.97f * whole_cost) chosen.swap(cut);
    }
  }

  // order within a queue: as scheduled, input order, or shortest first
  std::vector<size_t> idx(chosen.size());
  for (size_t i = 0; i < idx.size(); ++i) idx[i] = i;
  auto len_of = [&](size_t a) { return chosen[a].t1 - chosen[a].t0; };
  std::stable_sort(idx.begin(), idx.end(), [&](size_t a, size_t b) {
    if (chosen[a].queue != chosen[b].queue) return chosen[a].queue < chosen[b].queue;
    if (g_opt.order == 1) return a < b;
    if (g_opt.order == 2) return len_of(a) < len_of(b);
    return chosen[a].rank < chosen[b].rank;
  });
  // partial slots: the pieces of a tile take consecutive slots in key order
  std::vector<int32_t> slot_of(chosen.size(), -1);
  {
    std::vector<std::vector<size_t>> by_tile(n);
    for (size_t a = 0; a < chosen.size(); ++a) by_tile[chosen[a].tile - lo].push_back(a);
    for (size_t t = 0; t < n; ++t) {
      std::vector<size_t>& v = by_tile[t];
      if (v.size() < 2) continue;
      std::sort(v.begin(), v.end(), [&](size_t a, size_t b) { return chosen[a].t0 < chosen[b].t0; });
      const QTile& qt = tiles[lo + t];
      oppo::CombineItem ci;
      ci.q_row0 = seqs[qt.seq].q_row0 + qt.j0;
      ci.n_tok = qt.n_tok;
      ci.part0 = (int32_t)*next_slot;
      ci.nsplit = (int32_t)v.size();
      plan->combines.push_back(ci);
      for (size_t a : v) slot_of[a] = (int32_t)(*next_slot)++;
    }
  }
  int queue_prev = -1;
  for (size_t a : idx) {
    const Piece& pc = chosen[a];
    const QTile& qt = tiles[pc.tile];
    const SeqView& s = seqs[qt.seq];
    if (pc.queue != queue_prev) plan->first.push_back((uint16_t)plan->pieces.size());   // empty queues vanish
    queue_prev = pc.queue;
    oppo::AttnItem it;
    it.kv_row0 = s.kv_row0;
    it.q_row0 = s.q_row0 + qt.j0;
    it.n_tok = oppo::pack_tokens(qt.n_tok, qt.j0 / ls.TM);
    it.pos0 = s.kv_before + qt.j0;
    it.k_begin = pc.t0 * oppo::kKeyTile;
    it.k_end = std::min<int32_t>(qt.keys, pc.t1 * oppo::kKeyTile);
    it.part = slot_of[a];
    plan->pieces.push_back(it);
  }
  plan->first.push_back((uint16_t)plan->pieces.size());
}

// Cut every sequence's chunk into query tiles and plan the launches (one, unless
// the work list outgrows the kernel-argument segment).
void make_plans(const oppo::LayerShape& ls, const std::vector<SeqView>& seqs, size_t slots_avail,
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
  const size_t per_launch = (size_t)(oppo::kMaxAttnItems - queue_count(ls));
  size_t next_slot = 0;
  for (size_t lo = 0; lo < tiles.size(); lo += per_launch) {
    plans->emplace_back();
    Plan* plan = &plans->back();
    const size_t hi = std::min(tiles.size(), lo + per_launch);
    plan_launch(ls, seqs, tiles, lo, hi, slots_avail, &next_slot, plan);
    if (plan->pieces.size() > (size_t)oppo::kMaxAttnItems) {   // forced splitting of a long list
      const int keep = g_opt.split_kv;
      g_opt.split_kv = 1;
      *plan = Plan();
      plan_launch(ls, seqs, tiles, lo, hi, slots_avail, &next_slot, plan);
      g_opt.split_kv = keep;
    }
  }
}

// k_new / v_new non-null: the appending variant (the chunk's keys and values are
// read from there and written into k / v by the same kernel).
int run_attention(const oppo::LayerShape& ls, const std::vector<SeqView>& seqs, const void* q, void* k, void* v,
                  const void* k_new, const void* v_new, void* out, void* workspace, size_t workspace_bytes,
                  void* stream) {
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
  std::vector<Plan> plans;
  make_plans(ls, seqs, slots, &plans);
  for (const Plan& plan : plans) {
    const int e = oppo::launch_attention(ls, q, k, v, k_new, v_new, out, part_o, part_ml, plan.pieces.data(),
                                         (int)plan.pieces.size(), plan.first.data(), (int)plan.first.size() - 1, stream);
    if (e) return fail(OPPO_ERR_HIP, "attention launch failed: %s", oppo::hip_error_string(e));
  }
  for (const Plan& plan : plans) {
    if (plan.combines.empty()) continue;
    const int e = oppo::launch_combine(ls, out, part_o, part_ml, plan.combines.data(), (int)plan.combines.size(), stream);
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
  if (!cache) return fail(OPPO_ERR_INVALID, "cache is null");
  if (cache->batch < 0) return fail(OPPO_ERR_INVALID, "cache->batch is negative");
  if (!cache->slot_begin || !cache->kv_len) return fail(OPPO_ERR_INVALID, "cache length arrays are null");
  const int32_t B = cache->batch;
  rc = check_cu(cu_q, B, "cu_q");
  if (rc) return rc;
  if (!(theta_base > 1.0) || !std::isfinite(theta_base))
    return fail(OPPO_ERR_INVALID, "theta_base must be finite and greater than 1 (got %g)", theta_base);
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
  if ((int64_t)cu_q[B] * ls.Hq > INT32_MAX)
    return fail(OPPO_ERR_UNSUPPORTED, "%d query rows x %d heads exceed the 32-bit row index of the kernel", cu_q[B], ls.Hq);
  if (seqs.empty()) return OPPO_OK;
  if (!cache->k || !cache->v || !q || !out) return fail(OPPO_ERR_INVALID, "null device pointer");
  return run_attention(ls, seqs, q, cache->k, cache->v, nullptr, nullptr, out, workspace, workspace_bytes, stream);
}

int oppo_chunk_step(const oppo_attn_desc* desc, oppo_kv_cache* cache, const int32_t* cu_q, const void* q,
                    const void* k_new, const void* v_new, void* out, void* workspace, size_t workspace_bytes,
                    void* stream) {
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
  std::vector<SeqView> seqs;
  for (int32_t i = 0; i < B; ++i) {
    const int64_t cap = cache->slot_begin[i + 1] - cache->slot_begin[i];
    const int32_t ql = cu_q[i + 1] - cu_q[i];
    if ((int64_t)cache->kv_len[i] + ql > cap)
      return fail(OPPO_ERR_CAPACITY, "sequence %d: %d cached + %d new tokens exceed %lld slots", i, cache->kv_len[i], ql,
                  (long long)cap);
    if (ql == 0) continue;
    SeqView s;
    s.kv_row0 = cache->slot_begin[i];
    s.q_row0 = cu_q[i];
    s.q_len = ql;
    s.kv_before = cache->kv_len[i];
    seqs.push_back(s);
  }
  rc = check_workspace(ls, workspace, workspace_bytes);
  if (rc) return rc;
  if ((int64_t)cu_q[B] * ls.Hq > INT32_MAX)
    return fail(OPPO_ERR_UNSUPPORTED, "%d query rows x %d heads exceed the 32-bit row index of the kernel", cu_q[B], ls.Hq);
  if (seqs.empty()) return OPPO_OK;
  if (!cache->k || !cache->v || !q || !k_new || !v_new || !out) return fail(OPPO_ERR_INVALID, "null device pointer");
  rc = run_attention(ls, seqs, q, cache->k, cache->v, k_new, v_new, out, workspace, workspace_bytes, stream);
  if (rc) return rc;
  for (int32_t i = 0; i < B; ++i) cache->kv_len[i] += cu_q[i + 1] - cu_q[i];
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
    SeqView s;
    s.kv_row0 = cu_seq[i];
    s.q_row0 = cu_seq[i];
    s.q_len = n;
    s.kv_before = 0;
    seqs.push_back(s);
  }
  if (seqs.empty()) return OPPO_OK;
  if (!q || !k || !v || !out) return fail(OPPO_ERR_INVALID, "null device pointer");
  return run_attention(ls, seqs, q, const_cast<void*>(k), const_cast<void*>(v), nullptr, nullptr, out, workspace,
                       workspace_bytes, stream);
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
  std::vector<Plan> plans;
  make_plans(ls, seqs, workspace_bytes / oppo::part_slot_bytes(ls.Hkv, ls.D), &plans);
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
  const int e = oppo::profile_read(kernel_ms, launches);
  if (e) return fail(OPPO_ERR_HIP, "event timing failed: %s", oppo::hip_error_string(e));
  return OPPO_OK;
}

const char* oppo_last_error(void) { return g_err; }

int oppo_version(void) { return 100; }

}  // extern "C"
