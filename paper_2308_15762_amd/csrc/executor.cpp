// Per-rank task executor: the worker-side interpreter of the paper's runtime
// section, restricted to compute actions.  It validates the list against the
// rank's task set and the local dependencies, plans the stash, then walks the
// list once, enqueueing chunk_forward / chunk_backward on one stream.  Stage
// boundaries are buffers in HBM; the turn-around between two stages that share
// this rank is a pointer hand-off.
#include <hip/hip_runtime.h>

#include <vector>

#include "internal.h"

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
  pl.per_chunk.assign(2 * W, 0);
  const int rc = plan_stash(list, n, W, &pl.peak, pl.per_chunk.data(), pl.slot.data());
  if (rc) return rc;
  pl.chunk_base.assign(2 * W, 0);
  size_t at = 0;
  for (int c = 0; c < 2 * W; ++c) {
    pl.chunk_base[c] = at;
    at += (size_t)pl.per_chunk[c];
  }
  pl.entries = at;
  return HANAYO_OK;
}

// The list must hold exactly this rank's tasks, once each, in an order in which
// every task's local predecessor has already run.
int validate(const hanayo_task* list, size_t n, int P, int W, int M, int rank) {
  const int nchunk = 2 * W, S = 2 * W * P;
  if (n != (size_t)4 * W * M) return set_error(HANAYO_ESTATE, "executor: list has %zu tasks, rank needs %d", n, 4 * W * M);
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

}  // namespace
}  // namespace hanayo

using namespace hanayo;

extern "C" {

size_t hanayo_stash_arena_bytes(const hanayo_task* list, size_t n, int W, const hanayo_chunk_desc* d) {
  Shape sh;
  if (make_shape(d, sh) || W < 1 || 2 * W > 255 || (!list && n)) return 0;
  Plan pl;
  if (make_plan(list, n, W, pl)) return 0;
  return pl.entries * (stash_layout(sh).block_bytes * sh.nb);
}

int hanayo_executor_run(const hanayo_task* list, size_t n, const hanayo_exec_args* a, int* peak_seen) {
  if (!list || !a || !a->desc || !a->weights || !a->grads || !a->act_in || !a->grad_in || !a->act_out || !a->grad_out ||
      !a->stash_arena || !a->workspace)
    return set_error(HANAYO_EINVAL, "executor: NULL argument");
  const int P = a->P, W = a->W, M = a->M, rank = a->rank;
  if (P < 1 || W < 1 || M < 1 || rank < 0 || rank >= P || 2 * W > 255)
    return set_error(HANAYO_EINVAL, "executor: bad P=%d W=%d M=%d rank=%d", P, W, M, rank);
  Shape sh;
  int rc = prepare_call(a->desc, sh);
  if (rc) return rc;
  rc = validate(list, n, P, W, M, rank);
  if (rc) return rc;
  Plan pl;
  rc = make_plan(list, n, W, pl);
  if (rc) return rc;
  const size_t entry_bytes = stash_layout(sh).block_bytes * sh.nb;
  if (pl.entries * entry_bytes > a->stash_arena_bytes)
    return set_error(HANAYO_ESTATE, "executor: stash arena holds %zu bytes, plan needs %zu", a->stash_arena_bytes,
                     pl.entries * entry_bytes);
  const int nchunk = 2 * W, S = 2 * W * P;
  // every pointer the walk will dereference, checked before anything is enqueued
  for (size_t i = 0; i < n; ++i) {
    const hanayo_task& tk = list[i];
    const size_t at = (size_t)tk.mb * nchunk + tk.chunk;
    const int stage = (int)tk.stage;
    if (!a->weights[tk.chunk] || !a->grads[tk.chunk]) return set_error(HANAYO_EINVAL, "executor: chunk %d has no weights or grads", tk.chunk);
    if (tk.kind == HANAYO_F) {
      const bool local = stage > 0 && stage_rank(P, stage - 1) == rank;
      if (!a->act_out[at] || (!local && !a->act_in[at]))
        return set_error(HANAYO_EINVAL, "executor: missing activation buffer for mb %u chunk %d", tk.mb, tk.chunk);
    } else {
      const bool local = stage < S - 1 && stage_rank(P, stage + 1) == rank;
      if (!a->grad_out[at] || (!local && !a->grad_in[at]))
        return set_error(HANAYO_EINVAL, "executor: missing gradient buffer for mb %u chunk %d", tk.mb, tk.chunk);
    }
  }
  hipStream_t st = static_cast<hipStream_t>(a->hip_stream);
  char* arena = static_cast<char*>(a->stash_arena);
  int live = 0, peak = 0;
  for (size_t i = 0; i < n; ++i) {
    const hanayo_task& tk = list[i];
    const size_t at = (size_t)tk.mb * nchunk + tk.chunk;
    const int stage = (int)tk.stage;
    void* entry = arena + (pl.chunk_base[tk.chunk] + (size_t)pl.slot[i]) * entry_bytes;
    const int32_t* vl = a->valid_len ? a->valid_len[tk.mb] : nullptr;
    if (tk.kind == HANAYO_F) {
      const bool local = stage > 0 && stage_rank(P, stage - 1) == rank;
      const void* x = local ? a->act_out[at - 1] : a->act_in[at];
      rc = chunk_forward(sh, a->weights[tk.chunk], x, vl, a->act_out[at], entry, st);
      if (++live > peak) peak = live;
    } else {
      const bool local = stage < S - 1 && stage_rank(P, stage + 1) == rank;
      const void* dy = local ? a->grad_out[at + 1] : a->grad_in[at];
      rc = chunk_backward(sh, a->weights[tk.chunk], a->grads[tk.chunk], dy, vl, entry, a->grad_out[at], a->workspace, st);
      --live;
    }
    if (rc) return rc;
  }
  if (peak_seen) *peak_seen = peak;
  return HANAYO_OK;
}

}  // extern "C"
