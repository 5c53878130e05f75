// Per-rank task executor: the worker-side interpreter of the paper's runtime
// section, restricted to compute actions.  It validates the list against the
// rank's task set and the local dependencies, plans the stash, then walks the
// list once, enqueueing chunk_forward / chunk_backward.  Stage boundaries are
// buffers in HBM; the turn-around between two stages that share this rank is a
// pointer hand-off.
//
// hanayo_pipeline_run (end of the file) runs ALL ranks' lists on one device with true dataflow;
// hanayo_replay turns task durations into the makespan and idle time P devices would see.
//
// With one lane everything goes to the caller's stream in list order.  With
// more, tasks that do not depend on each other run side by side on HIP streams
// of the library's own (lane 0 is the caller's stream): a GEMM's store-heavy
// tail and the memory-bound kernels of one task then overlap another task's
// MFMA work.  Every true dependency becomes an event wait, every task still
// starts in list order on its lane, and the weight gradients of a chunk are
// still accumulated in list order, so the results do not depend on the lane
// count.
#include <hip/hip_runtime.h>

#include <array>
#include <mutex>
#include <vector>

#include "ends.h"
#include "internal.h"
#include "kernels.h"

namespace hanayo {
int prepare_call(const hanayo_chunk_desc* d, Shape& sh);
int chunk_forward(const Shape& sh, const void* weights, const void* x, const int32_t* valid_len, void* y, void* stash,
                  hipStream_t st);
int chunk_backward(const Shape& sh, const void* weights, float* grads, const void* dy, const int32_t* valid_len,
                   const void* stash, void* dx, void* workspace, hipStream_t st);

namespace {

struct Plan {
  std::vector<int32_t> slot;
  std::vector<int> per_chunk;
  std::vector<size_t> chunk_base;  // entry index where a chunk's slots start
  int peak = 0;
  size_t entries = 0;
};

int make_plan(const hanayo_task* list, size_t n, int W, Plan& pl) {
  pl.slot.assign(n, 0);
  pl.per_chunk.assign(chunks_per_rank(W), 0);
  const int rc = plan_stash(list, n, W, &pl.peak, pl.per_chunk.data(), pl.slot.data());
  if (rc) return rc;
  pl.chunk_base.assign(chunks_per_rank(W), 0);
  size_t at = 0;
  for (int c = 0; c < chunks_per_rank(W); ++c) {
    pl.chunk_base[c] = at;
    at += (size_t)pl.per_chunk[c];
  }
  pl.entries = at;
  return HANAYO_OK;
}

// What a task must wait for besides the tasks before it on its own lane.
enum { DEP_INPUT, DEP_FORWARD, DEP_SLOT, DEP_GRADS, DEP_ENDS, N_DEPS };
struct LanePlan {
  std::vector<int32_t> lane;
  std::vector<std::array<int32_t, N_DEPS>> dep;  // task indices, -1 = none
  std::vector<float> busy;                       // lanes the plan expects to be busy while the task runs (average, >= 1)
};

// Dependencies of each task on earlier tasks of the list, and a lane for each by list scheduling
// with the schedule's own cost model (forward 1, backward 2): a task goes to the lane on which it
// can start first.
//   DEP_INPUT    the local stage that produces its input activation / gradient
//   DEP_FORWARD  (backward) its own forward, which filled the stash entry
//   DEP_SLOT     (forward) the backward that last read the stash entry it is about to overwrite
//   DEP_GRADS    (backward) the previous backward of the same chunk: one accumulation at a time
//   DEP_ENDS     (with the model's ends: forward of the last stage, backward of stage 0) the previous task that
//                added to the gradients of the embedding tables and the head, which may be one table
// head_cost: with ends, what the head and loss add to the forward task of the last stage, in forward tasks.
void plan_lanes(const hanayo_task* list, size_t n, int P, int W, int M, int rank, int lanes, bool ends, double head_cost,
                const Plan& pl, LanePlan& lp) {
  const int nchunk = chunks_per_rank(W), S = nchunk * P;
  lp.lane.assign(n, 0);
  lp.dep.assign(n, {-1, -1, -1, -1, -1});
  int32_t last_ends = -1;
  std::vector<int32_t> f_at((size_t)M * nchunk, -1), b_at((size_t)M * nchunk, -1), last_b(nchunk, -1);
  std::vector<std::vector<int32_t>> slot_reader(nchunk);
  for (int c = 0; c < nchunk; ++c) slot_reader[c].assign(pl.per_chunk[c], -1);
  std::vector<double> done(n, 0.0), lane_free(lanes, 0.0), cost(n, 0.0);
  for (size_t i = 0; i < n; ++i)
    cost[i] = (list[i].kind == HANAYO_F ? 1.0 : 2.0) + (ends && list[i].kind == HANAYO_F && (int)list[i].stage == S - 1 ? head_cost : 0.0);
  for (size_t i = 0; i < n; ++i) {
    const hanayo_task& tk = list[i];
    const size_t at = (size_t)tk.mb * nchunk + tk.chunk;
    const int stage = (int)tk.stage;
    auto& d = lp.dep[i];
    if (tk.kind == HANAYO_F) {
      if (stage > 0 && stage_rank(P, stage - 1) == rank) d[DEP_INPUT] = f_at[at - 1];
      d[DEP_SLOT] = slot_reader[tk.chunk][pl.slot[i]];
      f_at[at] = (int32_t)i;
      if (ends && stage == S - 1) d[DEP_ENDS] = last_ends, last_ends = (int32_t)i;
    } else {
      if (stage < S - 1 && stage_rank(P, stage + 1) == rank) d[DEP_INPUT] = b_at[at + 1];
      d[DEP_FORWARD] = f_at[at];
      d[DEP_GRADS] = last_b[tk.chunk];
      b_at[at] = last_b[tk.chunk] = (int32_t)i;
      slot_reader[tk.chunk][pl.slot[i]] = (int32_t)i;
      if (ends && stage == 0) d[DEP_ENDS] = last_ends, last_ends = (int32_t)i;
    }
    double ready = 0.0;
    for (int32_t j : d)
      if (j >= 0 && done[j] > ready) ready = done[j];
    int best = 0;
    double best_start = 0.0;
    for (int l = 0; l < lanes; ++l) {
      const double start = lane_free[l] > ready ? lane_free[l] : ready;
      if (l == 0 || start < best_start) best = l, best_start = start;
    }
    lp.lane[i] = best;
    done[i] = lane_free[best] = best_start + cost[i];
  }
  // In the plan's own clock, how many lanes work during each task: the overlap of its interval
  // with every task's, over its length.
  lp.busy.assign(n, 1.0f);
  for (size_t i = 0; i < n; ++i) {
    const double ci = cost[i], si = done[i] - ci;
    double overlap = 0.0;
    for (size_t j = 0; j < n; ++j) {
      const double sj = done[j] - cost[j];
      const double lo = si > sj ? si : sj, hi = done[i] < done[j] ? done[i] : done[j];
      if (hi > lo) overlap += hi - lo;
    }
    lp.busy[i] = (float)(overlap / ci);
  }
}

// Side streams and events, made once per device and kept: default priority, non-blocking.
constexpr int kMaxLanes = 4;
struct LaneResources {
  int device = -1;
  hipStream_t side[kMaxLanes - 1] = {};
  std::vector<hipEvent_t> events;
};
std::mutex g_lane_mutex;
std::vector<LaneResources> g_lane_resources;

int lane_resources(int lanes, size_t n_events, LaneResources** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return set_error(HANAYO_EHIP, "executor: hipGetDevice failed");
  LaneResources* r = nullptr;
  for (auto& x : g_lane_resources)
    if (x.device == dev) r = &x;
  if (!r) {
    g_lane_resources.reserve(64);  // pointers handed out stay valid
    if (g_lane_resources.size() == g_lane_resources.capacity()) return set_error(HANAYO_ESTATE, "executor: too many devices");
    g_lane_resources.emplace_back();
    r = &g_lane_resources.back();
    r->device = dev;
  }
  for (int l = 0; l + 1 < lanes; ++l)
    if (!r->side[l] && hipStreamCreateWithFlags(&r->side[l], hipStreamNonBlocking) != hipSuccess)
      return set_error(HANAYO_EHIP, "executor: cannot create a stream: %s", hipGetErrorString(hipGetLastError()));
  while (r->events.size() < n_events) {
    hipEvent_t e;
    if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess)
      return set_error(HANAYO_EHIP, "executor: cannot create an event: %s", hipGetErrorString(hipGetLastError()));
    r->events.push_back(e);
  }
  *out = r;
  return HANAYO_OK;
}

// Timing events of one call: created on demand, destroyed when the call returns, also on an error path.
struct TimingEvents {
  std::vector<hipEvent_t> ev;
  ~TimingEvents() {
    for (hipEvent_t e : ev) (void)hipEventDestroy(e);
  }
  int create(size_t n) {
    ev.reserve(n);
    for (size_t i = 0; i < n; ++i) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess)
        return set_error(HANAYO_EHIP, "executor: cannot create an event: %s", hipGetErrorString(hipGetLastError()));
      ev.push_back(e);
    }
    return HANAYO_OK;
  }
  hipEvent_t operator[](size_t i) const { return ev[i]; }
};

#define HIP_TRY(call)                                                                                  \
  do {                                                                                                 \
    const hipError_t e_ = (call);                                                                      \
    if (e_ != hipSuccess) return set_error(HANAYO_EHIP, "executor: %s: %s", #call, hipGetErrorString(e_)); \
  } while (0)
// Inside the executor's task loop a failure must not return: the loop ends, and the run still resets the
// GEMM tile-choice state of the thread and joins the side lanes into the caller's stream.
#define HIP_NOTE(rc, call)                                                                             \
  do {                                                                                                 \
    const hipError_t e_ = (call);                                                                      \
    if (e_ != hipSuccess && !(rc)) (rc) = set_error(HANAYO_EHIP, "executor: %s: %s", #call, hipGetErrorString(e_)); \
  } while (0)

// The list must hold exactly this rank's tasks, once each, in an order in which
// every task's local predecessor has already run.
int validate(const hanayo_task* list, size_t n, int P, int W, int M, int rank) {
  const int nchunk = chunks_per_rank(W), S = nchunk * P;
  if (n != (size_t)2 * nchunk * M)
    return set_error(HANAYO_ESTATE, "executor: list has %zu tasks, rank needs %d", n, 2 * nchunk * M);
  std::vector<char> fdone((size_t)M * nchunk, 0), bdone((size_t)M * nchunk, 0);
  for (size_t i = 0; i < n; ++i) {
    const hanayo_task& tk = list[i];
    if (tk.kind > HANAYO_B || tk.chunk >= nchunk || tk.mb >= (uint32_t)M)
      return set_error(HANAYO_ESTATE, "executor: task %zu out of range", i);
    const int stage = rank_stage(P, rank, tk.chunk);
    if ((int)tk.stage != stage) return set_error(HANAYO_ESTATE, "executor: task %zu: stage %u is not chunk %d of rank %d", i, tk.stage, tk.chunk, rank);
    const size_t at = (size_t)tk.mb * nchunk + tk.chunk;
    if (tk.kind == HANAYO_F) {
      if (fdone[at]) return set_error(HANAYO_ESTATE, "executor: task %zu: forward repeated", i);
      if (stage > 0 && stage_rank(P, stage - 1) == rank && !fdone[at - 1])
        return set_error(HANAYO_ESTATE, "executor: task %zu: forward before the local stage that feeds it", i);
      fdone[at] = 1;
    } else {
      if (bdone[at]) return set_error(HANAYO_ESTATE, "executor: task %zu: backward repeated", i);
      if (!fdone[at]) return set_error(HANAYO_ESTATE, "executor: task %zu: backward before its forward", i);
      if (stage < S - 1 && stage_rank(P, stage + 1) == rank && !bdone[at + 1])
        return set_error(HANAYO_ESTATE, "executor: task %zu: backward before the local stage that feeds it", i);
      bdone[at] = 1;
    }
  }
  return HANAYO_OK;
}

int check_ends_args(const Shape& sh, const hanayo_ends_args* en, int M) {
  const int rc = check_ends(sh, &en->desc);
  if (rc) return rc;
  if (!en->wte || !en->d_wte || !en->wpe || !en->d_wpe || !en->head || !en->d_head || !en->tokens || !en->labels ||
      !en->loss || !en->loss_grad || !en->workspace || (en->desc.final_ln && (!en->lnf || !en->d_lnf)))
    return set_error(HANAYO_EINVAL, "ends: NULL argument");
  for (int m = 0; m < M; ++m)
    if (!en->tokens[m] || !en->labels[m] || !en->loss_grad[m])
      return set_error(HANAYO_EINVAL, "ends: micro-batch %d has no tokens, labels or loss-gradient buffer", m);
  return HANAYO_OK;
}

}  // namespace
}  // namespace hanayo

using namespace hanayo;

extern "C" {

size_t hanayo_stash_arena_bytes(const hanayo_task* list, size_t n, int W, const hanayo_chunk_desc* d) {
  Shape sh;
  if (make_shape(d, sh) || W < 0 || 2 * W > 255 || (!list && n)) return 0;
  Plan pl;
  if (make_plan(list, n, W, pl)) return 0;
  return pl.entries * (stash_layout(sh).block_bytes * sh.nb);
}

size_t hanayo_stash_arena_bytes_input(const hanayo_task* list, size_t n, int W, const hanayo_chunk_desc* d) {
  Shape sh;
  if (make_shape(d, sh) || W < 0 || 2 * W > 255 || (!list && n)) return 0;
  Plan pl;
  if (make_plan(list, n, W, pl)) return 0;
  return pl.entries * align_up((size_t)sh.T * sh.H * sh.esz, 256);
}

size_t hanayo_recompute_scratch_bytes(const hanayo_chunk_desc* d) {
  Shape sh;
  if (make_shape(d, sh)) return 0;
  return stash_layout(sh).block_bytes * sh.nb + align_up((size_t)sh.T * sh.H * sh.esz, 256);
}

size_t hanayo_ends_workspace_bytes(const hanayo_chunk_desc* d, const hanayo_ends_desc* e) {
  Shape sh;
  if (make_shape(d, sh) || check_ends(sh, e)) return 0;
  return align_up((size_t)sh.T * sh.H * sh.esz, 256) + head_workspace_bytes(sh, e->vocab);
}

namespace {
// The head's GEMM work (logits, d_head, d_hidden: 6 T H V flops) over a forward task's (2 T (4 H^2 + 2 H F) per block).
double head_cost_of(const Shape& sh, const hanayo_ends_desc& e) {
  return 3.0 * e.vocab / ((double)sh.nb * (4.0 * sh.H + 2.0 * sh.F));
}
}  // namespace

int hanayo_executor_plan(const hanayo_task* list, size_t n, int P, int W, int M, int rank, int lanes,
                         const hanayo_chunk_desc* d, const hanayo_ends_desc* e, int32_t* lane, int32_t* deps) {
  if (!list || !lane || !deps) return set_error(HANAYO_EINVAL, "executor_plan: NULL argument");
  if (P < 1 || W < 0 || M < 1 || rank < 0 || rank >= P || 2 * W > 255 || lanes < 1 || lanes > kMaxLanes)
    return set_error(HANAYO_EINVAL, "executor_plan: bad P=%d W=%d M=%d rank=%d lanes=%d", P, W, M, rank, lanes);
  if (e && W == 0 && P > 1)
    return set_error(HANAYO_EUNSUPPORTED, "executor_plan: the model's ends need the first and the last stage on one rank");
  int rc = validate(list, n, P, W, M, rank);
  if (rc) return rc;
  Plan pl;
  rc = make_plan(list, n, W, pl);
  if (rc) return rc;
  double head_cost = 0.0;
  if (e) {
    Shape sh;
    if (!d) return set_error(HANAYO_EINVAL, "executor_plan: the ends need the chunk descriptor");
    rc = make_shape(d, sh);
    if (!rc) rc = check_ends(sh, e);
    if (rc) return rc;
    head_cost = head_cost_of(sh, *e);
  }
  LanePlan lp;
  plan_lanes(list, n, P, W, M, rank, lanes, e != nullptr && rank == 0, head_cost, pl, lp);
  for (size_t i = 0; i < n; ++i) {
    lane[i] = lp.lane[i];
    for (int k = 0; k < N_DEPS; ++k) deps[i * N_DEPS + k] = lp.dep[i][k];
  }
  return HANAYO_OK;
}

int hanayo_executor_run(const hanayo_task* list, size_t n, const hanayo_exec_args* a, int* peak_seen) {
  if (!list || !a || !a->desc || !a->weights || !a->grads || !a->act_in || !a->grad_in || !a->act_out || !a->grad_out ||
      !a->stash_arena || !a->workspace)
    return set_error(HANAYO_EINVAL, "executor: NULL argument");
  const int P = a->P, W = a->W, M = a->M, rank = a->rank;
  if (P < 1 || W < 0 || M < 1 || rank < 0 || rank >= P || 2 * W > 255)
    return set_error(HANAYO_EINVAL, "executor: bad P=%d W=%d M=%d rank=%d", P, W, M, rank);
  Shape sh;
  int rc = prepare_call(a->desc, sh);
  if (rc) return rc;
  rc = validate(list, n, P, W, M, rank);
  if (rc) return rc;
  Plan pl;
  rc = make_plan(list, n, W, pl);
  if (rc) return rc;
  if (a->stash_mode != HANAYO_STASH_FULL && a->stash_mode != HANAYO_STASH_INPUT)
    return set_error(HANAYO_EINVAL, "executor: stash_mode %d", a->stash_mode);
  const bool recompute = a->stash_mode == HANAYO_STASH_INPUT;
  if (recompute && !a->recompute_scratch) return set_error(HANAYO_EINVAL, "executor: stash_mode input needs recompute_scratch");
  const size_t full_entry_bytes = stash_layout(sh).block_bytes * sh.nb;
  const size_t act_bytes = (size_t)sh.T * sh.H * sh.esz;
  const size_t entry_bytes = recompute ? align_up(act_bytes, 256) : full_entry_bytes;  // what a stash slot holds
  if (pl.entries * entry_bytes > a->stash_arena_bytes)
    return set_error(HANAYO_ESTATE, "executor: stash arena holds %zu bytes, plan needs %zu", a->stash_arena_bytes,
                     pl.entries * entry_bytes);
  const int nchunk = chunks_per_rank(W), S = nchunk * P;
  // the model's ends sit on rank 0: stage 0 and stage S - 1
  const hanayo_ends_args* en = rank == 0 ? a->ends : nullptr;
  if (a->ends && W == 0 && P > 1)
    return set_error(HANAYO_EUNSUPPORTED, "executor: the model's ends need the first and the last stage on one rank "
                     "(any wave placement); a straight placement splits them over ranks 0 and P-1");
  if (en) {
    rc = check_ends_args(sh, en, M);
    if (rc) return rc;
  }
  // every pointer the walk will dereference, checked before anything is enqueued
  for (size_t i = 0; i < n; ++i) {
    const hanayo_task& tk = list[i];
    const size_t at = (size_t)tk.mb * nchunk + tk.chunk;
    const int stage = (int)tk.stage;
    if (!a->weights[tk.chunk] || !a->grads[tk.chunk]) return set_error(HANAYO_EINVAL, "executor: chunk %d has no weights or grads", tk.chunk);
    if (tk.kind == HANAYO_F) {
      const bool given = (stage > 0 && stage_rank(P, stage - 1) == rank) || (en && stage == 0);
      if (!a->act_out[at] || (!given && !a->act_in[at]))
        return set_error(HANAYO_EINVAL, "executor: missing activation buffer for mb %u chunk %d", tk.mb, tk.chunk);
    } else {
      const bool given = (stage < S - 1 && stage_rank(P, stage + 1) == rank) || (en && stage == S - 1);
      if (!a->grad_out[at] || (!given && !a->grad_in[at]))
        return set_error(HANAYO_EINVAL, "executor: missing gradient buffer for mb %u chunk %d", tk.mb, tk.chunk);
    }
  }
  const int lanes = a->lanes < 1 ? 1 : a->lanes;
  if (lanes > kMaxLanes) return set_error(HANAYO_EINVAL, "executor: at most %d lanes", kMaxLanes);
  LanePlan lp;
  plan_lanes(list, n, P, W, M, rank, lanes, en != nullptr, en ? head_cost_of(sh, en->desc) : 0.0, pl, lp);
  // a task records an event if a task on another lane waits for it
  std::vector<char> signals(n, 0);
  for (size_t i = 0; i < n; ++i)
    for (int32_t j : lp.dep[i])
      if (j >= 0 && lp.lane[j] != lp.lane[i]) signals[j] = 1;

  std::unique_lock<std::mutex> lock(g_lane_mutex, std::defer_lock);
  hipStream_t stream[kMaxLanes] = {static_cast<hipStream_t>(a->hip_stream)};
  LaneResources* res = nullptr;
  if (lanes > 1) {
    lock.lock();  // the side streams and events are shared by every call on this device
    rc = lane_resources(lanes, n + kMaxLanes, &res);
    if (rc) return rc;
    // fork: the side lanes start after whatever the caller's stream holds so far
    HIP_TRY(hipEventRecord(res->events[n], stream[0]));
    for (int l = 1; l < lanes; ++l) {
      stream[l] = res->side[l - 1];
      HIP_TRY(hipStreamWaitEvent(stream[l], res->events[n], 0));
    }
  }
  const size_t work_bytes = work_layout(sh).bytes;
  const size_t ends_bytes = en ? align_up(act_bytes, 256) + head_workspace_bytes(sh, en->desc.vocab) : 0;
  char* arena = static_cast<char*>(a->stash_arena);
  int live = 0, peak = 0;
  for (size_t i = 0; i < n; ++i) {
    const hanayo_task& tk = list[i];
    const size_t at = (size_t)tk.mb * nchunk + tk.chunk;
    const int stage = (int)tk.stage;
    const int lane = lp.lane[i];
    hipStream_t st = stream[lane];
    for (int32_t j : lp.dep[i])
      if (j >= 0 && lp.lane[j] != lane) HIP_NOTE(rc, hipStreamWaitEvent(st, res->events[j], 0));
    if (rc) break;
    // Measured: next to one other busy lane the shortest GEMM launch still wins, next to three the
    // one with the least CU time does; the plan says how busy the other lanes are during this task.
    k::set_gemm_sharing((lp.busy[i] - 2.0f) * 0.5f);
    void* entry = arena + (pl.chunk_base[tk.chunk] + (size_t)pl.slot[i]) * entry_bytes;
    const int32_t* vl = a->valid_len ? a->valid_len[tk.mb] : nullptr;
    // input-only stash: the lane's scratch entry takes what the forward materialises, then an output scratch
    char* scratch = recompute ? static_cast<char*>(a->recompute_scratch) + (size_t)lane * (full_entry_bytes + align_up(act_bytes, 256))
                              : nullptr;
    if (tk.kind == HANAYO_F) {
      const bool local = stage > 0 && stage_rank(P, stage - 1) == rank;
      const void* x = local ? a->act_out[at - 1] : a->act_in[at];
      // the lane's share of the ends workspace: the embedding's output, then the head's scratch
      char* ends_ws = en ? static_cast<char*>(en->workspace) + (size_t)lane * ends_bytes : nullptr;
      if (en && stage == 0) {
        rc = embed_forward(sh, &en->desc, en->wte, en->wpe, en->tokens[tk.mb], ends_ws, st);
        x = ends_ws;  // the chunk's forward copies its input into the stash, so the buffer is free after the task
      }
      if (!rc && recompute) rc = k::copy_bytes(entry, x, act_bytes, st);
      if (!rc) rc = chunk_forward(sh, a->weights[tk.chunk], x, vl, a->act_out[at], recompute ? scratch : entry, st);
      if (!rc && en && stage == S - 1)
        rc = head_loss(sh, &en->desc, en->lnf, en->head, a->act_out[at], en->labels[tk.mb], en->loss_scale,
                       en->loss + tk.mb, en->loss_grad[tk.mb], en->d_lnf, en->d_head, ends_ws + align_up(act_bytes, 256), st);
      if (++live > peak) peak = live;
    } else {
      const bool local = stage < S - 1 && stage_rank(P, stage + 1) == rank;
      const void* dy = local ? a->grad_out[at + 1] : a->grad_in[at];
      if (en && stage == S - 1) dy = en->loss_grad[tk.mb];
      void* work = static_cast<char*>(a->workspace) + (size_t)lane * work_bytes;  // one workspace per lane
      const void* stash = entry;
      if (recompute) {  // the forward again, from the stashed input
        rc = chunk_forward(sh, a->weights[tk.chunk], entry, vl, scratch + full_entry_bytes, scratch, st);
        stash = scratch;
      }
      if (!rc) rc = chunk_backward(sh, a->weights[tk.chunk], a->grads[tk.chunk], dy, vl, stash, a->grad_out[at], work, st);
      if (!rc && en && stage == 0)
        rc = embed_backward(sh, &en->desc, en->tokens[tk.mb], a->grad_out[at], en->d_wte, en->d_wpe, st);
      --live;
    }
    if (rc) break;
    if (signals[i]) HIP_NOTE(rc, hipEventRecord(res->events[i], st));
    if (rc) break;
  }
  k::set_gemm_sharing(0.0);
  // join, also after a failed enqueue or a failed event call: the caller's stream ends after every side lane
  for (int l = 1; l < lanes; ++l) {
    int jrc = 0;
    HIP_NOTE(jrc, hipEventRecord(res->events[n + l], stream[l]));
    if (!jrc) HIP_NOTE(jrc, hipStreamWaitEvent(stream[0], res->events[n + l], 0));
    if (jrc && !rc) rc = jrc;
  }
  if (rc) return rc;
  if (peak_seen) *peak_seen = peak;
  return HANAYO_OK;
}

// ---------------------------------------------------------------------------------------------
// All P ranks of the pipeline on one device, with true dataflow: what synchronous pipeline training
// computes must equal the model run without a pipeline, and running every rank's list against the
// others' outputs is how that is checked here.  One stream; the global order is a dataflow merge of
// the lists (poll the ranks in turn, run a rank's head task once its producer has run).
int hanayo_pipeline_run(const hanayo_task* const* lists, const size_t* counts, const hanayo_pipeline_args* a,
                        int* peak_seen, float* const* task_ms) {
  if (!lists || !counts || !a || !a->desc || !a->weights || !a->grads || !a->act || !a->grad || !a->stash_arena ||
      !a->stash_arena_bytes || !a->workspace || (!a->ends && (!a->x || !a->dy)))
    return set_error(HANAYO_EINVAL, "pipeline: NULL argument");
  const int P = a->P, W = a->W, M = a->M;
  if (P < 1 || W < 0 || M < 1 || 2 * W > 255) return set_error(HANAYO_EINVAL, "pipeline: bad P=%d W=%d M=%d", P, W, M);
  Shape sh;
  int rc = prepare_call(a->desc, sh);
  if (rc) return rc;
  const int nchunk = chunks_per_rank(W), S = nchunk * P;
  const hanayo_ends_args* en = a->ends;
  if (en) {
    rc = check_ends_args(sh, en, M);
    if (rc) return rc;
  }
  std::vector<Plan> plans(P);
  const size_t entry_bytes = stash_layout(sh).block_bytes * sh.nb;
  for (int r = 0; r < P; ++r) {
    if (!lists[r]) return set_error(HANAYO_EINVAL, "pipeline: rank %d has no list", r);
    rc = validate(lists[r], counts[r], P, W, M, r);
    if (rc) return rc;
    rc = make_plan(lists[r], counts[r], W, plans[r]);
    if (rc) return rc;
    if (!a->stash_arena[r] || plans[r].entries * entry_bytes > a->stash_arena_bytes[r])
      return set_error(HANAYO_ESTATE, "pipeline: rank %d stash arena holds %zu bytes, plan needs %zu", r,
                       a->stash_arena[r] ? a->stash_arena_bytes[r] : (size_t)0, plans[r].entries * entry_bytes);
  }
  for (int s = 0; s < S; ++s)
    if (!a->weights[s] || !a->grads[s]) return set_error(HANAYO_EINVAL, "pipeline: stage %d has no weights or grads", s);
  for (int m = 0; m < M; ++m) {
    if (!en && (!a->x[m] || !a->dy[m]))
      return set_error(HANAYO_EINVAL, "pipeline: micro-batch %d has no input or loss gradient", m);
    for (int s = 0; s < S; ++s)
      if (!a->act[(size_t)m * S + s] || !a->grad[(size_t)m * S + s])
        return set_error(HANAYO_EINVAL, "pipeline: missing boundary buffer for mb %d stage %d", m, s);
  }
  // dataflow merge; nothing is enqueued unless every list runs to its end
  struct Step { int rank; size_t index; };
  std::vector<Step> order;
  {
    std::vector<char> fdone((size_t)M * S, 0), bdone((size_t)M * S, 0);
    std::vector<size_t> head(P, 0);
    bool progressed = true;
    while (progressed) {
      progressed = false;
      for (int r = 0; r < P; ++r) {
        while (head[r] < counts[r]) {
          const hanayo_task& tk = lists[r][head[r]];
          const size_t at = (size_t)tk.mb * S + tk.stage;
          if (tk.kind == HANAYO_F) {
            if (tk.stage > 0 && !fdone[at - 1]) break;
            fdone[at] = 1;
          } else {
            if (!fdone[at] || ((int)tk.stage < S - 1 && !bdone[at + 1])) break;
            bdone[at] = 1;
          }
          order.push_back({r, head[r]++});
          progressed = true;
        }
      }
    }
    for (int r = 0; r < P; ++r)
      if (head[r] != counts[r])
        return set_error(HANAYO_ESTATE, "pipeline: the lists deadlock (rank %d stops at task %zu)", r, head[r]);
  }
  hipStream_t st = static_cast<hipStream_t>(a->hip_stream);
  TimingEvents ev;
  if (task_ms) {
    for (int r = 0; r < P; ++r)
      if (!task_ms[r]) return set_error(HANAYO_EINVAL, "pipeline: task_ms[%d] is NULL", r);
    rc = ev.create(2 * order.size());
    if (rc) return rc;
  }
  for (size_t k = 0; k < order.size() && !rc; ++k) {
    const int r = order[k].rank;
    const size_t i = order[k].index;
    const hanayo_task& tk = lists[r][i];
    const size_t at = (size_t)tk.mb * S + tk.stage;
    void* entry = static_cast<char*>(a->stash_arena[r]) +
                  (plans[r].chunk_base[tk.chunk] + (size_t)plans[r].slot[i]) * entry_bytes;
    const int32_t* vl = a->valid_len ? a->valid_len[tk.mb] : nullptr;
    if (task_ms) HIP_TRY(hipEventRecord(ev[2 * k], st));
    char* ends_ws = en ? static_cast<char*>(en->workspace) : nullptr;  // embedding output, then the head's scratch
    if (tk.kind == HANAYO_F) {
      const void* x = tk.stage > 0 ? a->act[at - 1] : en ? ends_ws : a->x[tk.mb];
      if (en && tk.stage == 0) rc = embed_forward(sh, &en->desc, en->wte, en->wpe, en->tokens[tk.mb], ends_ws, st);
      if (!rc) rc = chunk_forward(sh, a->weights[tk.stage], x, vl, a->act[at], entry, st);
      if (!rc && en && (int)tk.stage == S - 1)
        rc = head_loss(sh, &en->desc, en->lnf, en->head, a->act[at], en->labels[tk.mb], en->loss_scale, en->loss + tk.mb,
                       en->loss_grad[tk.mb], en->d_lnf, en->d_head, ends_ws + align_up((size_t)sh.T * sh.H * sh.esz, 256), st);
    } else {
      const void* dy = (int)tk.stage < S - 1 ? a->grad[at + 1] : en ? en->loss_grad[tk.mb] : a->dy[tk.mb];
      rc = chunk_backward(sh, a->weights[tk.stage], a->grads[tk.stage], dy, vl, entry, a->grad[at], a->workspace, st);
      if (!rc && en && tk.stage == 0)
        rc = embed_backward(sh, &en->desc, en->tokens[tk.mb], a->grad[at], en->d_wte, en->d_wpe, st);
    }
    if (task_ms && !rc) HIP_TRY(hipEventRecord(ev[2 * k + 1], st));
  }
  if (task_ms) {
    if (!rc) {
      HIP_TRY(hipStreamSynchronize(st));
      for (size_t k = 0; k < order.size(); ++k)
        HIP_TRY(hipEventElapsedTime(&task_ms[order[k].rank][order[k].index], ev[2 * k], ev[2 * k + 1]));
    }
  }
  if (rc) return rc;
  if (peak_seen)
    for (int r = 0; r < P; ++r) peak_seen[r] = plans[r].peak;
  return HANAYO_OK;
}

// Replay of all P lists with given task durations: every rank runs its list strictly in order and a
// task starts when the rank is free and its producer has finished (transfers take no time).
int hanayo_replay(const hanayo_task* const* lists, const size_t* counts, int P, int W, int M, const float* const* cost,
                  double* makespan, double* idle) {
  if (!lists || !counts || !makespan) return set_error(HANAYO_EINVAL, "replay: NULL argument");
  if (P < 1 || W < 0 || M < 1 || 2 * W > 255) return set_error(HANAYO_EINVAL, "replay: bad P=%d W=%d M=%d", P, W, M);
  const int S = chunks_per_rank(W) * P;
  for (int r = 0; r < P; ++r) {
    if (!lists[r] || (cost && !cost[r])) return set_error(HANAYO_EINVAL, "replay: rank %d has no list or costs", r);
    const int rc = validate(lists[r], counts[r], P, W, M, r);
    if (rc) return rc;
  }
  std::vector<double> ffin((size_t)M * S, -1.0), bfin((size_t)M * S, -1.0), free_at(P, 0.0), busy(P, 0.0);
  std::vector<size_t> head(P, 0);
  bool progressed = true;
  while (progressed) {
    progressed = false;
    for (int r = 0; r < P; ++r) {
      while (head[r] < counts[r]) {
        const hanayo_task& tk = lists[r][head[r]];
        const size_t at = (size_t)tk.mb * S + tk.stage;
        double ready = 0.0;
        if (tk.kind == HANAYO_F) {
          if (tk.stage > 0) {
            if (ffin[at - 1] < 0.0) break;
            ready = ffin[at - 1];
          }
        } else {
          if (ffin[at] < 0.0) break;
          ready = ffin[at];
          if ((int)tk.stage < S - 1) {
            if (bfin[at + 1] < 0.0) break;
            if (bfin[at + 1] > ready) ready = bfin[at + 1];
          }
        }
        const double c = cost ? (double)cost[r][head[r]] : (tk.kind == HANAYO_F ? 1.0 : 2.0);
        if (!(c >= 0.0)) return set_error(HANAYO_EINVAL, "replay: negative or NaN duration");
        const double t0 = free_at[r] > ready ? free_at[r] : ready;
        (tk.kind == HANAYO_F ? ffin : bfin)[at] = free_at[r] = t0 + c;
        busy[r] += c;
        ++head[r];
        progressed = true;
      }
    }
  }
  double end = 0.0;
  for (int r = 0; r < P; ++r) {
    if (head[r] != counts[r]) return set_error(HANAYO_ESTATE, "replay: the lists deadlock (rank %d stops at task %zu)", r, head[r]);
    if (free_at[r] > end) end = free_at[r];
  }
  *makespan = end;
  if (idle)
    for (int r = 0; r < P; ++r) idle[r] = end - busy[r];
  return HANAYO_OK;
}

int hanayo_replay_actions(const hanayo_action* const* lists, const size_t* counts, int P, int W, int M, double t_f,
                          double t_b, double t_c, int prefetch, const float* const* cost, double* makespan,
                          double* idle, double* waited) {
  if (!lists || !counts || !makespan) return set_error(HANAYO_EINVAL, "replay_actions: NULL argument");
  if (P < 1 || W < 0 || M < 1 || 2 * W > 255 || !(t_f >= 0.0) || !(t_b >= 0.0) || !(t_c >= 0.0))
    return set_error(HANAYO_EINVAL, "replay_actions: bad P=%d W=%d M=%d or negative time", P, W, M);
  const int S = chunks_per_rank(W) * P;
  // structure: the compute actions are the rank's tasks; each communication action belongs to its neighbour
  for (int r = 0; r < P; ++r) {
    if (!lists[r] || (cost && !cost[r])) return set_error(HANAYO_EINVAL, "replay_actions: rank %d has no list or costs", r);
    std::vector<hanayo_task> tasks;
    for (size_t i = 0; i < counts[r]; ++i) {
      const hanayo_action& a = lists[r][i];
      if (a.kind <= HANAYO_B) {
        tasks.push_back({a.kind, a.chunk, 0, a.mb, a.stage});
        continue;
      }
      if (a.kind > HANAYO_RECV_GRAD) return set_error(HANAYO_ESTATE, "replay_actions: rank %d action %zu: kind %u", r, i, a.kind);
      const bool is_recv = a.kind == HANAYO_RECV_ACT || a.kind == HANAYO_RECV_GRAD;
      const bool is_act = a.kind == HANAYO_SEND_ACT || a.kind == HANAYO_RECV_ACT;
      const size_t j = is_recv ? i + 1 : i - 1;  // the compute it serves
      if ((is_recv && i + 1 >= counts[r]) || (!is_recv && i == 0) || lists[r][j].kind != (is_act ? HANAYO_F : HANAYO_B) ||
          lists[r][j].mb != a.mb || lists[r][j].stage != a.stage)
        return set_error(HANAYO_ESTATE, "replay_actions: rank %d action %zu is not next to the compute it serves", r, i);
      const int other = (int)a.stage + ((is_act == is_recv) ? -1 : 1);  // act recv / grad send: stage - 1
      if (other < 0 || other >= S || stage_rank(P, other) != (int)a.peer || (int)a.peer == r)
        return set_error(HANAYO_ESTATE, "replay_actions: rank %d action %zu: wrong peer", r, i);
    }
    const int rc = validate(tasks.data(), tasks.size(), P, W, M, r);
    if (rc) return rc;
  }
  // message id: activations and gradients of (mb, producing stage)
  auto message = [&](const hanayo_action& a) -> size_t {
    const bool is_act = a.kind == HANAYO_SEND_ACT || a.kind == HANAYO_RECV_ACT;
    const bool is_recv = a.kind == HANAYO_RECV_ACT || a.kind == HANAYO_RECV_GRAD;
    const int producer = (int)a.stage + (is_recv ? (is_act ? -1 : 1) : 0);
    return ((size_t)(is_act ? 0 : 1) * M + a.mb) * S + producer;
  };
  const size_t n_msg = (size_t)2 * M * S;
  std::vector<double> sent(n_msg, -1.0), posted(n_msg, -1.0), arrived(n_msg, -1.0);
  std::vector<double> ffin((size_t)M * S, -1.0), bfin((size_t)M * S, -1.0), now(P, 0.0), busy(P, 0.0), blocked(P, 0.0);
  std::vector<size_t> head(P, 0);
  auto try_arrive = [&](size_t m) {
    if (sent[m] >= 0.0 && posted[m] >= 0.0 && arrived[m] < 0.0) arrived[m] = (sent[m] > posted[m] ? sent[m] : posted[m]) + t_c;
  };
  bool progressed = true;
  while (progressed) {
    progressed = false;
    for (int r = 0; r < P; ++r) {
      while (head[r] < counts[r]) {
        const size_t i = head[r];
        const hanayo_action& a = lists[r][i];
        const size_t at = (size_t)a.mb * S + a.stage;
        if (a.kind <= HANAYO_B) {
          double ready = now[r];
          if (a.kind == HANAYO_F) {
            if (a.stage > 0 && stage_rank(P, (int)a.stage - 1) == r) {
              if (ffin[at - 1] < 0.0) break;
              if (ffin[at - 1] > ready) ready = ffin[at - 1];
            }
          } else {
            if (ffin[at] < 0.0) break;
            if (ffin[at] > ready) ready = ffin[at];
            if ((int)a.stage < S - 1 && stage_rank(P, (int)a.stage + 1) == r) {
              if (bfin[at + 1] < 0.0) break;
              if (bfin[at + 1] > ready) ready = bfin[at + 1];
            }
          }
          if (prefetch) {  // look ahead to the receive of the following compute action
            for (size_t j = i + 1; j < counts[r] && lists[r][j].kind > HANAYO_B; ++j) {
              const hanayo_action& nx = lists[r][j];
              if (nx.kind == HANAYO_RECV_ACT || nx.kind == HANAYO_RECV_GRAD) {
                const size_t m = message(nx);
                if (posted[m] < 0.0) {
                  posted[m] = now[r];
                  try_arrive(m);
                }
                break;
              }
            }
          }
          const double c = cost ? (double)cost[r][i] : (a.kind == HANAYO_F ? t_f : t_b);
          if (!(c >= 0.0)) return set_error(HANAYO_EINVAL, "replay_actions: negative or NaN duration");
          now[r] = ready + c;
          busy[r] += c;
          (a.kind == HANAYO_F ? ffin : bfin)[at] = now[r];
        } else if (a.kind == HANAYO_SEND_ACT || a.kind == HANAYO_SEND_GRAD) {
          const size_t m = message(a);
          if (sent[m] >= 0.0) return set_error(HANAYO_ESTATE, "replay_actions: message sent twice");
          sent[m] = now[r];
          try_arrive(m);
        } else {
          const size_t m = message(a);
          if (posted[m] < 0.0) {
            posted[m] = now[r];
            try_arrive(m);
          }
          if (arrived[m] < 0.0) break;  // the peer has not sent yet
          if (arrived[m] > now[r]) {
            blocked[r] += arrived[m] - now[r];
            now[r] = arrived[m];
          }
        }
        ++head[r];
        progressed = true;
      }
    }
  }
  double end = 0.0;
  for (int r = 0; r < P; ++r) {
    if (head[r] != counts[r])
      return set_error(HANAYO_ESTATE, "replay_actions: the lists deadlock (rank %d stops at action %zu)", r, head[r]);
    if (now[r] > end) end = now[r];
  }
  *makespan = end;
  for (int r = 0; r < P; ++r) {
    if (idle) idle[r] = end - busy[r];
    if (waited) waited[r] = blocked[r];
  }
  return HANAYO_OK;
}

// The whole pipeline from ACTION lists: every rank has receive buffers of its own and a send /
// receive pair is one device copy from the producer's output buffer into the consumer's receive
// buffer, the emulated link.  link->async = 0: the copy runs on the compute stream at the position of
// the receive (a blocking receive: nothing overlaps it).  link->async = 1: the copy runs on a second
// stream as soon as the message has been sent and its receive posted, with the paper's look-ahead
// (the receive of the following compute is posted before the current compute is enqueued), and only
// the consumer waits for it, so transfers overlap the computes enqueued in between.
int hanayo_pipeline_run_actions(const hanayo_action* const* lists, const size_t* counts, const hanayo_pipeline_args* a,
                                const hanayo_link_args* link, int* peak_seen, float* const* action_ms) {
  if (!lists || !counts || !a || !link || !a->desc || !a->weights || !a->grads || !a->x || !a->dy || !a->act || !a->grad ||
      !a->stash_arena || !a->stash_arena_bytes || !a->workspace || !link->act_recv || !link->grad_recv)
    return set_error(HANAYO_EINVAL, "pipeline_actions: NULL argument");
  if (a->ends) return set_error(HANAYO_EUNSUPPORTED, "pipeline_actions: the model's ends are not part of this call");
  const int P = a->P, W = a->W, M = a->M;
  if (P < 1 || W < 0 || M < 1 || 2 * W > 255 || link->link_workgroups < 0)
    return set_error(HANAYO_EINVAL, "pipeline_actions: bad P=%d W=%d M=%d or link", P, W, M);
  Shape sh;
  int rc = prepare_call(a->desc, sh);
  if (rc) return rc;
  const int nchunk = chunks_per_rank(W), S = nchunk * P;
  // the lists themselves (structure, matching, no deadlock) are checked by the interpreter simulation
  double dummy = 0.0;
  rc = hanayo_replay_actions(lists, counts, P, W, M, 1.0, 2.0, 0.0, 0, nullptr, &dummy, nullptr, nullptr);
  if (rc) return rc;
  const size_t entry_bytes = stash_layout(sh).block_bytes * sh.nb;
  const size_t act_bytes = (size_t)sh.T * sh.H * sh.esz;
  std::vector<Plan> plans(P);
  std::vector<std::vector<int32_t>> slot_of(P);  // stash slot per action (compute actions only)
  for (int r = 0; r < P; ++r) {
    std::vector<hanayo_task> tasks;
    std::vector<size_t> where;
    for (size_t i = 0; i < counts[r]; ++i)
      if (lists[r][i].kind <= HANAYO_B) {
        tasks.push_back({lists[r][i].kind, lists[r][i].chunk, 0, lists[r][i].mb, lists[r][i].stage});
        where.push_back(i);
      }
    rc = make_plan(tasks.data(), tasks.size(), W, plans[r]);
    if (rc) return rc;
    slot_of[r].assign(counts[r], -1);
    for (size_t k = 0; k < where.size(); ++k) slot_of[r][where[k]] = plans[r].slot[k];
    if (!a->stash_arena[r] || plans[r].entries * entry_bytes > a->stash_arena_bytes[r])
      return set_error(HANAYO_ESTATE, "pipeline_actions: rank %d stash arena too small", r);
    if (action_ms && !action_ms[r]) return set_error(HANAYO_EINVAL, "pipeline_actions: action_ms[%d] is NULL", r);
  }
  for (int s = 0; s < S; ++s)
    if (!a->weights[s] || !a->grads[s]) return set_error(HANAYO_EINVAL, "pipeline_actions: stage %d has no weights or grads", s);
  for (int m = 0; m < M; ++m) {
    if (!a->x[m] || !a->dy[m]) return set_error(HANAYO_EINVAL, "pipeline_actions: micro-batch %d has no input or loss gradient", m);
    for (int s = 0; s < S; ++s) {
      const size_t at = (size_t)m * S + s;
      if (!a->act[at] || !a->grad[at]) return set_error(HANAYO_EINVAL, "pipeline_actions: missing boundary buffer for mb %d stage %d", m, s);
      if (s < S - 1 && stage_rank(P, s + 1) != stage_rank(P, s) && !link->act_recv[at])
        return set_error(HANAYO_EINVAL, "pipeline_actions: missing activation receive buffer for mb %d stage %d", m, s);
      if (s > 0 && stage_rank(P, s - 1) != stage_rank(P, s) && !link->grad_recv[at])
        return set_error(HANAYO_EINVAL, "pipeline_actions: missing gradient receive buffer for mb %d stage %d", m, s);
    }
  }
  // message m of (type, mb, producing stage): index as in the simulation
  auto message = [&](const hanayo_action& x) -> size_t {
    const bool is_act = x.kind == HANAYO_SEND_ACT || x.kind == HANAYO_RECV_ACT;
    const bool is_recv = x.kind == HANAYO_RECV_ACT || x.kind == HANAYO_RECV_GRAD;
    const int producer = (int)x.stage + (is_recv ? (is_act ? -1 : 1) : 0);
    return ((size_t)(is_act ? 0 : 1) * M + x.mb) * S + producer;
  };
  const size_t n_msg = (size_t)2 * M * S;
  size_t n_actions = 0;
  for (int r = 0; r < P; ++r) n_actions += counts[r];

  std::unique_lock<std::mutex> lock(g_lane_mutex);  // the copy stream and the event pool are shared per device
  LaneResources* res = nullptr;
  rc = lane_resources(2, 2 * n_msg + 1, &res);
  if (rc) return rc;
  hipStream_t compute = static_cast<hipStream_t>(a->hip_stream), copy = res->side[0];
  TimingEvents tev;  // two per action
  if (action_ms) {
    rc = tev.create(2 * n_actions);
    if (rc) return rc;
  }
  HIP_TRY(hipEventRecord(res->events[2 * n_msg], compute));  // fork: the copy stream starts after the caller's work
  HIP_TRY(hipStreamWaitEvent(copy, res->events[2 * n_msg], 0));

  enum : char { NOT_YET = 0, YES = 1 };
  std::vector<char> was_sent(n_msg, NOT_YET), was_posted(n_msg, NOT_YET), copy_enqueued(n_msg, NOT_YET);
  std::vector<size_t> tslot(n_msg, 0);  // timing slot of the receive action of a message
  std::vector<char> fdone((size_t)M * S, 0), bdone((size_t)M * S, 0);
  std::vector<size_t> head(P, 0), base(P, 0);
  for (int r = 1; r < P; ++r) base[r] = base[r - 1] + counts[r - 1];
  // source and destination of a message
  auto endpoints = [&](size_t m, const void*& src, void*& dst) {
    const bool is_act = m < (size_t)M * S;
    const size_t at = is_act ? m : m - (size_t)M * S;  // mb * S + producing stage
    src = is_act ? a->act[at] : a->grad[at];
    dst = is_act ? link->act_recv[at] : link->grad_recv[at];
  };
  // enqueue the transfer once the message has been sent and its receive posted
  auto maybe_copy = [&](size_t m) -> int {
    if (!was_sent[m] || !was_posted[m] || copy_enqueued[m]) return HANAYO_OK;
    const void* src;
    void* dst;
    endpoints(m, src, dst);
    hipStream_t st = link->async ? copy : compute;
    if (link->async) HIP_TRY(hipStreamWaitEvent(copy, res->events[2 * m], 0));  // sent
    if (action_ms) HIP_TRY(hipEventRecord(tev[2 * tslot[m]], st));
    const int crc = k::copy_bytes(dst, src, act_bytes, st, link->link_workgroups);
    if (crc) return crc;
    if (action_ms) HIP_TRY(hipEventRecord(tev[2 * tslot[m] + 1], st));
    if (link->async) HIP_TRY(hipEventRecord(res->events[2 * m + 1], copy));  // arrived
    copy_enqueued[m] = YES;
    return HANAYO_OK;
  };
  // every receive action's timing slot is known up front
  for (int r = 0; r < P; ++r)
    for (size_t i = 0; i < counts[r]; ++i)
      if (lists[r][i].kind == HANAYO_RECV_ACT || lists[r][i].kind == HANAYO_RECV_GRAD) tslot[message(lists[r][i])] = base[r] + i;

  bool progressed = true;
  while (progressed && !rc) {
    progressed = false;
    for (int r = 0; r < P && !rc; ++r) {
      while (head[r] < counts[r] && !rc) {
        const size_t i = head[r];
        const hanayo_action& x = lists[r][i];
        const size_t at = (size_t)x.mb * S + x.stage;
        if (x.kind <= HANAYO_B) {
          const bool prev_local = x.stage > 0 && stage_rank(P, (int)x.stage - 1) == r;
          const bool next_local = (int)x.stage < S - 1 && stage_rank(P, (int)x.stage + 1) == r;
          if (x.kind == HANAYO_F && prev_local && !fdone[at - 1]) break;
          if (x.kind == HANAYO_B && (!fdone[at] || (next_local && !bdone[at + 1]))) break;
          if (link->async) {  // look ahead: post the receive of the following compute
            for (size_t j = i + 1; j < counts[r] && lists[r][j].kind > HANAYO_B; ++j)
              if (lists[r][j].kind == HANAYO_RECV_ACT || lists[r][j].kind == HANAYO_RECV_GRAD) {
                const size_t m = message(lists[r][j]);
                was_posted[m] = YES;
                rc = maybe_copy(m);
                break;
              }
            if (rc) break;
          }
          void* entry = static_cast<char*>(a->stash_arena[r]) +
                        (plans[r].chunk_base[x.chunk] + (size_t)slot_of[r][i]) * entry_bytes;
          const int32_t* vl = a->valid_len ? a->valid_len[x.mb] : nullptr;
          if (action_ms) HIP_TRY(hipEventRecord(tev[2 * (base[r] + i)], compute));
          if (x.kind == HANAYO_F) {
            const void* in = x.stage == 0 ? a->x[x.mb] : (prev_local ? a->act[at - 1] : link->act_recv[at - 1]);
            rc = chunk_forward(sh, a->weights[x.stage], in, vl, a->act[at], entry, compute);
            fdone[at] = 1;
          } else {
            const void* dy = (int)x.stage == S - 1 ? a->dy[x.mb] : (next_local ? a->grad[at + 1] : link->grad_recv[at + 1]);
            rc = chunk_backward(sh, a->weights[x.stage], a->grads[x.stage], dy, vl, entry, a->grad[at], a->workspace, compute);
            bdone[at] = 1;
          }
          if (rc) break;
          if (action_ms) HIP_TRY(hipEventRecord(tev[2 * (base[r] + i) + 1], compute));
        } else if (x.kind == HANAYO_SEND_ACT || x.kind == HANAYO_SEND_GRAD) {
          const size_t m = message(x);
          if (link->async) HIP_TRY(hipEventRecord(res->events[2 * m], compute));  // the message exists from here on
          was_sent[m] = YES;
          rc = maybe_copy(m);
          if (rc) break;
        } else {
          const size_t m = message(x);
          if (!was_sent[m]) break;  // the peer has not got there yet
          was_posted[m] = YES;
          rc = maybe_copy(m);
          if (rc) break;
          if (link->async) HIP_TRY(hipStreamWaitEvent(compute, res->events[2 * m + 1], 0));  // wait for the arrival
        }
        ++head[r];
        progressed = true;
      }
    }
  }
  // join: the caller's stream ends after the copy stream
  HIP_TRY(hipEventRecord(res->events[2 * n_msg], copy));
  HIP_TRY(hipStreamWaitEvent(compute, res->events[2 * n_msg], 0));
  if (action_ms) {
    if (!rc) {
      HIP_TRY(hipStreamSynchronize(compute));
      for (int r = 0; r < P; ++r)
        for (size_t i = 0; i < counts[r]; ++i) {
          const bool is_send = lists[r][i].kind == HANAYO_SEND_ACT || lists[r][i].kind == HANAYO_SEND_GRAD;
          action_ms[r][i] = 0.f;
          if (!is_send) HIP_TRY(hipEventElapsedTime(&action_ms[r][i], tev[2 * (base[r] + i)], tev[2 * (base[r] + i) + 1]));
        }
    }
  }
  if (rc) return rc;
  for (int r = 0; r < P; ++r)
    if (head[r] != counts[r]) return set_error(HANAYO_ESTATE, "pipeline_actions: stopped at rank %d action %zu", r, head[r]);
  if (peak_seen)
    for (int r = 0; r < P; ++r) peak_seen[r] = plans[r].peak;
  return HANAYO_OK;
}

}  // extern "C"
