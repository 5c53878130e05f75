// Wave schedule generator and stash planner (host only, integer only).
//
// Placement follows Table 1 (W = S / 2P) and the description of wave-like
// pipelines: stages run down the devices and back, W times.  The task order is
// a greedy list schedule of the whole pipeline with the cost model of the
// theoretical analysis (T_B = 2 T_F, T_C = 0), generated event by event:
// finish events release successors into per-rank ordered ready sets, and every
// rank that is free takes the minimum of its set (backward first, then lowest
// micro-batch).
#include <cstdint>
#include <cstring>
#include <queue>
#include <set>
#include <vector>

#include "internal.h"

namespace hanayo {

int stage_rank(int P, int stage) {
  const int lap = stage / P, pos = stage % P;
  return (lap & 1) ? P - 1 - pos : pos;
}

int rank_stage(int P, int rank, int chunk) { return chunk * P + ((chunk & 1) ? P - 1 - rank : rank); }

namespace {

struct Finish {
  long t;
  int mb;
  int pos;  // position in the micro-batch's chain F0..F(S-1) B(S-1)..B0
  bool operator>(const Finish& o) const { return t > o.t; }
};

// Ready-set key: backward before forward, then micro-batch.
struct Ready {
  int not_backward;
  int mb;
  int pos;
  bool operator<(const Ready& o) const {
    if (not_backward != o.not_backward) return not_backward < o.not_backward;
    return mb < o.mb;
  }
};

}  // namespace

void generate(int P, int W, int M, int want_rank, std::vector<hanayo_task>& out) {
  const int S = 2 * W * P;
  const int chain_len = 2 * S;
  auto pos_kind = [&](int pos) { return pos < S ? HANAYO_F : HANAYO_B; };
  auto pos_stage = [&](int pos) { return pos < S ? pos : 2 * S - 1 - pos; };

  std::vector<std::set<Ready>> ready(P);
  std::vector<char> busy(P, 0);
  std::priority_queue<Finish, std::vector<Finish>, std::greater<Finish>> events;
  std::vector<char> last_forward_done(M, 0);
  int inject = 0;  // next micro-batch allowed to enter stage 0
  long remaining = (long)M * chain_len;
  out.clear();
  out.reserve((size_t)4 * W * M);

  auto gate_open = [&](int m) { return m < P || last_forward_done[m - P]; };
  auto offer_injection = [&]() {
    if (inject < M && gate_open(inject)) ready[0].insert(Ready{1, inject, 0});
  };
  auto start_ready_tasks = [&](long t) {
    for (int r = 0; r < P; ++r) {
      if (busy[r] || ready[r].empty()) continue;
      const Ready pick = *ready[r].begin();
      ready[r].erase(ready[r].begin());
      const int kind = pos_kind(pick.pos), stage = pos_stage(pick.pos);
      busy[r] = 1;
      events.push(Finish{t + (kind == HANAYO_F ? 1 : 2), pick.mb, pick.pos});
      if (r == want_rank) {
        hanayo_task tk;
        tk.kind = (uint8_t)kind;
        tk.chunk = (uint8_t)(stage / P);
        tk.rsvd = 0;
        tk.mb = (uint32_t)pick.mb;
        tk.stage = (uint32_t)stage;
        out.push_back(tk);
      }
      if (pick.pos == 0) {  // the next micro-batch may be injected from now on,
        ++inject;           // but cannot start before the next event: rank 0 is busy
        offer_injection();
      }
    }
  };

  offer_injection();
  start_ready_tasks(0);
  while (!events.empty()) {
    const long t = events.top().t;
    while (!events.empty() && events.top().t == t) {
      const Finish f = events.top();
      events.pop();
      --remaining;
      busy[stage_rank(P, pos_stage(f.pos))] = 0;
      if (f.pos == S - 1) {
        last_forward_done[f.mb] = 1;
        if (inject == f.mb + P) offer_injection();
      }
      if (f.pos + 1 < chain_len) {
        const int nstage = pos_stage(f.pos + 1);
        ready[stage_rank(P, nstage)].insert(Ready{pos_kind(f.pos + 1) == HANAYO_B ? 0 : 1, f.mb, f.pos + 1});
      }
    }
    start_ready_tasks(t);
  }
  (void)remaining;
}

int plan_stash(const hanayo_task* list, size_t n, int W, int* peak_total, int* per_chunk, int32_t* slot) {
  const int nchunk = 2 * W;
  std::vector<std::set<int>> free_ids(nchunk);  // ids below `high` that are free again
  std::vector<int> high(nchunk, 0), live_in_chunk(nchunk, 0), peak_chunk(nchunk, 0);
  // live entries keyed by (mb, chunk)
  std::set<std::pair<uint32_t, int>> live;
  std::vector<std::pair<std::pair<uint32_t, int>, int>> owner;  // small: linear map
  auto find_owner = [&](uint32_t mb, int c) -> int {
    for (size_t i = 0; i < owner.size(); ++i)
      if (owner[i].first.first == mb && owner[i].first.second == c) return (int)i;
    return -1;
  };
  int peak = 0;
  for (size_t i = 0; i < n; ++i) {
    const hanayo_task& tk = list[i];
    if (tk.chunk >= nchunk || tk.kind > HANAYO_B) return set_error(HANAYO_EINVAL, "stash_plan: task %zu: bad chunk or kind", i);
    const int c = tk.chunk;
    if (tk.kind == HANAYO_F) {
      if (find_owner(tk.mb, c) >= 0)
        return set_error(HANAYO_ESTATE, "stash_plan: task %zu: forward of a live entry (mb %u chunk %d)", i, tk.mb, c);
      int id;
      if (!free_ids[c].empty()) {
        id = *free_ids[c].begin();
        free_ids[c].erase(free_ids[c].begin());
      } else {
        id = high[c]++;
      }
      owner.push_back({{tk.mb, c}, id});
      ++live_in_chunk[c];
      if (live_in_chunk[c] > peak_chunk[c]) peak_chunk[c] = live_in_chunk[c];
      if ((int)owner.size() > peak) peak = (int)owner.size();
      if (slot) slot[i] = id;
    } else {
      const int at = find_owner(tk.mb, c);
      if (at < 0)
        return set_error(HANAYO_ESTATE, "stash_plan: task %zu: backward without a live forward (mb %u chunk %d)", i, tk.mb, c);
      const int id = owner[at].second;
      owner[at] = owner.back();
      owner.pop_back();
      free_ids[c].insert(id);
      --live_in_chunk[c];
      if (slot) slot[i] = id;
    }
  }
  if (!owner.empty()) return set_error(HANAYO_ESTATE, "stash_plan: %zu entries still live at the end", owner.size());
  if (peak_total) *peak_total = peak;
  if (per_chunk) std::memcpy(per_chunk, peak_chunk.data(), sizeof(int) * nchunk);
  return HANAYO_OK;
}

}  // namespace hanayo

extern "C" {

int hanayo_stage_rank(int P, int W, int stage, int* rank) {
  if (P < 1 || W < 1 || !rank || stage < 0 || stage >= 2 * W * P) return hanayo::set_error(HANAYO_EINVAL, "stage_rank: bad argument");
  *rank = hanayo::stage_rank(P, stage);
  return HANAYO_OK;
}

int hanayo_rank_stage(int P, int W, int rank, int chunk, int* stage) {
  if (P < 1 || W < 1 || !stage || rank < 0 || rank >= P || chunk < 0 || chunk >= 2 * W)
    return hanayo::set_error(HANAYO_EINVAL, "rank_stage: bad argument");
  *stage = hanayo::rank_stage(P, rank, chunk);
  return HANAYO_OK;
}

int hanayo_schedule(int P, int W, int M, int rank, hanayo_task* out, size_t cap, size_t* n) {
  if (!n) return hanayo::set_error(HANAYO_EINVAL, "schedule: n is NULL");
  if (P < 1 || W < 1 || M < 1 || rank < 0 || rank >= P || 2 * W > 255 || (cap && !out))
    return hanayo::set_error(HANAYO_EINVAL, "schedule: bad argument P=%d W=%d M=%d rank=%d", P, W, M, rank);
  const size_t need = (size_t)4 * W * M;
  *n = need;
  if (cap < need) return hanayo::set_error(HANAYO_EBUFSIZE, "schedule: need %zu records, capacity %zu", need, cap);
  std::vector<hanayo_task> v;
  hanayo::generate(P, W, M, rank, v);
  if (v.size() != need) return hanayo::set_error(HANAYO_ESTATE, "schedule: generated %zu of %zu tasks", v.size(), need);
  std::memcpy(out, v.data(), need * sizeof(hanayo_task));
  return HANAYO_OK;
}

// The rank's list at the granularity of the paper's runtime section: its tasks, each with the
// communication it needs around it (a receive in front of a compute whose input comes from another
// rank, a send behind a compute whose output goes to another rank).
int hanayo_actions(int P, int W, int M, int rank, hanayo_action* out, size_t cap, size_t* n) {
  if (!n) return hanayo::set_error(HANAYO_EINVAL, "actions: n is NULL");
  if (P < 1 || W < 1 || M < 1 || rank < 0 || rank >= P || 2 * W > 255 || (cap && !out))
    return hanayo::set_error(HANAYO_EINVAL, "actions: bad argument P=%d W=%d M=%d rank=%d", P, W, M, rank);
  std::vector<hanayo_task> tasks;
  hanayo::generate(P, W, M, rank, tasks);
  const int S = 2 * W * P;
  std::vector<hanayo_action> v;
  v.reserve(tasks.size() * 3);
  for (const hanayo_task& t : tasks) {
    const int stage = (int)t.stage;
    // the stage whose output this task reads, and the stage that reads this task's output
    const int from = t.kind == HANAYO_F ? stage - 1 : stage + 1, to = t.kind == HANAYO_F ? stage + 1 : stage - 1;
    const int src = (from >= 0 && from < S) ? hanayo::stage_rank(P, from) : rank;
    const int dst = (to >= 0 && to < S) ? hanayo::stage_rank(P, to) : rank;
    hanayo_action a = {t.kind, t.chunk, (uint16_t)rank, t.mb, t.stage};
    if (src != rank) {
      hanayo_action r = a;
      r.kind = t.kind == HANAYO_F ? HANAYO_RECV_ACT : HANAYO_RECV_GRAD;
      r.peer = (uint16_t)src;
      v.push_back(r);
    }
    v.push_back(a);
    if (dst != rank) {
      hanayo_action snd = a;
      snd.kind = t.kind == HANAYO_F ? HANAYO_SEND_ACT : HANAYO_SEND_GRAD;
      snd.peer = (uint16_t)dst;
      v.push_back(snd);
    }
  }
  *n = v.size();
  if (cap < v.size()) return hanayo::set_error(HANAYO_EBUFSIZE, "actions: need %zu records, capacity %zu", v.size(), cap);
  std::memcpy(out, v.data(), v.size() * sizeof(hanayo_action));
  return HANAYO_OK;
}

int hanayo_stash_plan(const hanayo_task* list, size_t n, int W, int* peak_total, int* per_chunk, int32_t* slot) {
  if ((!list && n) || W < 1 || 2 * W > 255) return hanayo::set_error(HANAYO_EINVAL, "stash_plan: bad argument");
  return hanayo::plan_stash(list, n, W, peak_total, per_chunk, slot);
}

}  // extern "C"
