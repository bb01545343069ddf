// The buffer of Alg. 1 as a host-side state machine: which sequences the scorer
// serves in which pass, which leave after the iteration and which carry over.
// (Sec. 3.2, Alg. 1 stages 1-3.  No device work, no GPU needed.)
#include <math.h>
#include <stdint.h>

#include <algorithm>
#include <iterator>
#include <unordered_map>
#include <vector>

#include "../../include/oppo_attn.h"
#include "oppo_internal.h"

namespace {
struct Seq {
  int64_t id;
  int32_t prompt_len;
  int32_t streamed = 0;      // response tokens the scorer has been given
  bool prompt_done = false;  // the prompt pass has happened
  bool finished = false;
};
}  // namespace

struct oppo_scheduler {
  int32_t B, delta, C;
  std::vector<Seq> buffer;                 // FIFO order
  std::vector<int64_t> finished_order;     // finished and still in the buffer, in finishing order
  std::unordered_map<int64_t, size_t> at;  // id -> index in buffer (rebuilt after removals)
  std::vector<int64_t> open_ids;           // the pass handed out by begin_pass and not yet ended
  std::vector<int32_t> open_cap;
  int32_t open_kind = 0;
  void reindex() {
    at.clear();
    for (size_t i = 0; i < buffer.size(); ++i) at[buffer[i].id] = i;
  }
};

using oppo::fail;

extern "C" {

int oppo_sched_create(int32_t B, int32_t delta, int32_t C, oppo_scheduler** sched) {
  if (!sched) return fail(OPPO_ERR_INVALID, "sched is null");
  *sched = nullptr;
  if (B < 1 || delta < 0 || C < 1) return fail(OPPO_ERR_INVALID, "need B >= 1, delta >= 0, C >= 1 (got %d, %d, %d)", B, delta, C);
  if ((int64_t)B + delta > INT32_MAX) return fail(OPPO_ERR_INVALID, "B + delta overflows");
  oppo_scheduler* s = new oppo_scheduler();
  s->B = B, s->delta = delta, s->C = C;
  *sched = s;
  return OPPO_OK;
}

int oppo_sched_destroy(oppo_scheduler* sched) {
  delete sched;
  return OPPO_OK;
}

int oppo_sched_set_delta(oppo_scheduler* s, int32_t delta) {
  if (!s) return fail(OPPO_ERR_INVALID, "sched is null");
  if (delta < 0 || (int64_t)s->B + delta > INT32_MAX) return fail(OPPO_ERR_INVALID, "delta=%d out of range", delta);
  s->delta = delta;
  return OPPO_OK;
}

int oppo_sched_room(const oppo_scheduler* s, int32_t* n) {
  if (!s || !n) return fail(OPPO_ERR_INVALID, "sched or n is null");
  *n = std::max<int32_t>(0, s->B + s->delta - (int32_t)s->buffer.size());
  return OPPO_OK;
}

int oppo_sched_add(oppo_scheduler* s, int64_t seq_id, int32_t prompt_len) {
  if (!s) return fail(OPPO_ERR_INVALID, "sched is null");
  if (s->open_kind) return fail(OPPO_ERR_INVALID, "a pass is open");
  if (prompt_len < 1) return fail(OPPO_ERR_INVALID, "prompt_len=%d must be positive", prompt_len);
  if ((int32_t)s->buffer.size() >= s->B + s->delta) return fail(OPPO_ERR_CAPACITY, "the buffer is full (%d sequences)", s->B + s->delta);
  if (s->at.count(seq_id)) return fail(OPPO_ERR_INVALID, "sequence %lld is already in the buffer", (long long)seq_id);
  Seq q;
  q.id = seq_id;
  q.prompt_len = prompt_len;
  s->at[seq_id] = s->buffer.size();
  s->buffer.push_back(q);
  return OPPO_OK;
}

int oppo_sched_begin_pass(oppo_scheduler* s, int32_t max_n, int64_t* ids, int32_t* kv_before, int32_t* q_cap,
                          int32_t* n, int32_t* kind) {
  if (!s || !n || !kind) return fail(OPPO_ERR_INVALID, "sched, n or kind is null");
  if (s->open_kind) return fail(OPPO_ERR_INVALID, "the previous pass has not been ended");
  std::vector<int64_t> oid;
  std::vector<int32_t> okv, ocap;
  int32_t k = OPPO_PASS_NONE;
  for (const Seq& q : s->buffer)
    if (!q.prompt_done) oid.push_back(q.id), okv.push_back(0), ocap.push_back(q.prompt_len);
  if (!oid.empty()) {
    k = OPPO_PASS_PROMPT;
  } else if ((int32_t)s->finished_order.size() < s->B) {
    for (const Seq& q : s->buffer)
      if (!q.finished) oid.push_back(q.id), okv.push_back(q.prompt_len + q.streamed), ocap.push_back(s->C);
    if (!oid.empty()) k = OPPO_PASS_CHUNK;
  }
  if ((int32_t)oid.size() > max_n) return fail(OPPO_ERR_INVALID, "the pass has %d sequences, room for %d", (int)oid.size(), max_n);
  if (!oid.empty() && (!ids || !kv_before || !q_cap)) return fail(OPPO_ERR_INVALID, "output arrays are null");
  for (size_t j = 0; j < oid.size(); ++j) ids[j] = oid[j], kv_before[j] = okv[j], q_cap[j] = ocap[j];
  *n = (int32_t)oid.size();
  *kind = k;
  s->open_kind = k;
  s->open_ids.swap(oid);
  s->open_cap.swap(ocap);
  return OPPO_OK;
}

int oppo_sched_end_pass(oppo_scheduler* s, int32_t n, const int64_t* ids, const int32_t* q_len, const uint8_t* finished) {
  if (!s) return fail(OPPO_ERR_INVALID, "sched is null");
  if (!s->open_kind) return fail(OPPO_ERR_INVALID, "no pass is open");
  if (n != (int32_t)s->open_ids.size() || (n > 0 && (!ids || !q_len || !finished)))
    return fail(OPPO_ERR_INVALID, "the open pass has %d sequences, %d reported", (int)s->open_ids.size(), n);
  for (int32_t j = 0; j < n; ++j) {
    if (ids[j] != s->open_ids[j]) return fail(OPPO_ERR_INVALID, "entry %d: sequence %lld reported, %lld expected", j, (long long)ids[j], (long long)s->open_ids[j]);
    if (s->open_kind == OPPO_PASS_PROMPT) {
      if (q_len[j] != s->open_cap[j]) return fail(OPPO_ERR_INVALID, "entry %d: a prompt pass takes the whole prompt (%d rows, %d reported)", j, s->open_cap[j], q_len[j]);
    } else {
      if (q_len[j] < 0 || q_len[j] > s->open_cap[j]) return fail(OPPO_ERR_INVALID, "entry %d: %d new tokens, at most %d allowed", j, q_len[j], s->open_cap[j]);
      if (q_len[j] < s->open_cap[j] && !finished[j]) return fail(OPPO_ERR_INVALID, "entry %d: a chunk shorter than C must end its sequence", j);
      const Seq& q = s->buffer[s->at[ids[j]]];
      if ((int64_t)q.prompt_len + q.streamed + q_len[j] > INT32_MAX) return fail(OPPO_ERR_INVALID, "entry %d: sequence length overflows", j);
    }
  }
  for (int32_t j = 0; j < n; ++j) {
    Seq& q = s->buffer[s->at[ids[j]]];
    if (s->open_kind == OPPO_PASS_PROMPT) q.prompt_done = true;
    else q.streamed += q_len[j];
    if (finished[j]) {
      q.finished = true;
      s->finished_order.push_back(q.id);
    }
  }
  s->open_kind = 0;
  s->open_ids.clear();
  s->open_cap.clear();
  return OPPO_OK;
}

int oppo_sched_end_iteration(oppo_scheduler* s, int32_t max_n, int64_t* removed, int32_t* n_removed) {
  if (!s || !n_removed) return fail(OPPO_ERR_INVALID, "sched or n_removed is null");
  if (s->open_kind) return fail(OPPO_ERR_INVALID, "a pass is open");
  const int32_t k = std::min<int32_t>(s->B, (int32_t)s->finished_order.size());
  if (k > max_n || (k > 0 && !removed)) return fail(OPPO_ERR_INVALID, "%d sequences leave, room for %d", k, max_n);
  for (int32_t j = 0; j < k; ++j) removed[j] = s->finished_order[j];
  std::vector<int64_t> gone(s->finished_order.begin(), s->finished_order.begin() + k);
  s->finished_order.erase(s->finished_order.begin(), s->finished_order.begin() + k);
  std::sort(gone.begin(), gone.end());
  std::vector<Seq> keep;
  for (const Seq& q : s->buffer)
    if (!std::binary_search(gone.begin(), gone.end(), q.id)) keep.push_back(q);
  s->buffer.swap(keep);
  s->reindex();
  *n_removed = k;
  return OPPO_OK;
}

int oppo_sched_counts(const oppo_scheduler* s, int32_t* in_buffer, int32_t* finished_waiting, int32_t* capacity) {
  if (!s) return fail(OPPO_ERR_INVALID, "sched is null");
  if (in_buffer) *in_buffer = (int32_t)s->buffer.size();
  if (finished_waiting) *finished_waiting = (int32_t)s->finished_order.size();
  if (capacity) *capacity = s->B + s->delta;
  return OPPO_OK;
}

// ---- periodic chunk-size search (Sec. 3.1, dynamic control on intra-step overlap) ----

}  // extern "C"

struct oppo_chunk_tuner {
  std::vector<int32_t> candidates;
  int32_t period;
  std::unordered_map<int64_t, double> seconds;   // training step -> reported step time
  int32_t trials() const { return std::min<int32_t>((int32_t)candidates.size(), period); }
};

extern "C" {

int oppo_tuner_create(int32_t n, const int32_t* candidates, int32_t period, oppo_chunk_tuner** tuner) {
  if (!tuner) return fail(OPPO_ERR_INVALID, "tuner is null");
  *tuner = nullptr;
  if (n < 1 || !candidates) return fail(OPPO_ERR_INVALID, "at least one candidate chunk size is needed");
  if (period < 1) return fail(OPPO_ERR_INVALID, "period=%d must be positive", period);
  for (int32_t j = 0; j < n; ++j)
    if (candidates[j] < 1) return fail(OPPO_ERR_INVALID, "candidate %d is %d", j, candidates[j]);
  oppo_chunk_tuner* t = new oppo_chunk_tuner();
  t->candidates.assign(candidates, candidates + n);
  t->period = period;
  *tuner = t;
  return OPPO_OK;
}

int oppo_tuner_destroy(oppo_chunk_tuner* tuner) {
  delete tuner;
  return OPPO_OK;
}

int oppo_tuner_chunk(const oppo_chunk_tuner* t, int64_t step, int32_t* chunk) {
  if (!t || !chunk) return fail(OPPO_ERR_INVALID, "tuner or chunk is null");
  if (step < 0) return fail(OPPO_ERR_INVALID, "step is negative");
  const int64_t start = (step / t->period) * t->period;
  const int64_t k = step - start;
  if (k < t->trials()) {
    *chunk = t->candidates[(size_t)k];
    return OPPO_OK;
  }
  int32_t best = 0;
  double best_s = INFINITY;
  for (int32_t j = 0; j < t->trials(); ++j) {
    auto it = t->seconds.find(start + j);
    const double sj = it == t->seconds.end() ? INFINITY : it->second;
    if (sj < best_s) best = j, best_s = sj;
  }
  *chunk = t->candidates[(size_t)best];
  return OPPO_OK;
}

int oppo_tuner_report(oppo_chunk_tuner* t, int64_t step, double seconds) {
  if (!t) return fail(OPPO_ERR_INVALID, "tuner is null");
  if (step < 0 || !(seconds >= 0.0)) return fail(OPPO_ERR_INVALID, "bad report (step %lld, %g s)", (long long)step, seconds);
  // only trial steps decide anything; older windows are forgotten
  const int64_t start = (step / t->period) * t->period;
  if (step - start < t->trials()) {
    for (auto it = t->seconds.begin(); it != t->seconds.end();)
      it = it->first < start - t->period ? t->seconds.erase(it) : std::next(it);
    t->seconds[step] = seconds;
  }
  return OPPO_OK;
}

// ---------------------------------------------------------------------------------------
// Intra-step overlap as a two-stage pipeline (Sec. 3.1): chunk k reaches the scorer when
// the actor has decoded it; the scorer works through the chunks in order.

int oppo_overlap_timeline(int32_t n, const double* gen_s, const double* score_s, double* start_s,
                          double* end_s, double* summary) {
  if (n < 0) return fail(OPPO_ERR_INVALID, "negative chunk count %d", n);
  if (!summary || (n > 0 && (!gen_s || !score_s))) return fail(OPPO_ERR_INVALID, "null argument");
  for (int32_t k = 0; k < n; ++k)
    if (!(gen_s[k] >= 0.0) || !(score_s[k] >= 0.0))
      return fail(OPPO_ERR_INVALID, "chunk %d: bad times (decode %g s, scoring %g s)", k, gen_s[k], score_s[k]);
  double decoded = 0.0;   // when the actor completes the current chunk
  double scored = 0.0;    // when the scorer completes the previous one
  for (int32_t k = 0; k < n; ++k) {
    decoded += gen_s[k];
    const double begin = decoded > scored ? decoded : scored;
    scored = begin + score_s[k];
    if (start_s) start_s[k] = begin;
    if (end_s) end_s[k] = scored;
  }
  summary[0] = decoded;
  summary[1] = scored > decoded ? scored : decoded;
  summary[2] = summary[1] - decoded;
  return OPPO_OK;
}

}  // extern "C"
