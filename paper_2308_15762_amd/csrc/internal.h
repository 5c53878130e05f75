// Shared declarations of the library's translation units (host side).
#pragma once

#include <cstddef>
#include <cstdint>
#include <vector>

#include "../../include/hanayo.h"

namespace hanayo {

// Records a thread-local message and returns `code`.
int set_error(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// Placements.  W >= 1: the wave placement of Table 1 (S = 2WP stages, 2W chunks per device, a micro-batch runs
// down the devices and back W times).  W == 0: the straight placement of GPipe and 1F1B, one stage per device
// (S = P; in Table 1's notation W = S / 2P = 1/2).  stage_rank / rank_stage cover both: with S = P the first
// lap of the wave is the straight pipeline.
inline int chunks_per_rank(int W) { return W ? 2 * W : 1; }
int stage_rank(int P, int stage);
int rank_stage(int P, int rank, int chunk);
void generate(int P, int W, int M, int rank, std::vector<hanayo_task>& out);
int plan_stash(const hanayo_task* list, size_t n, int W, int* peak_total, int* per_chunk, int32_t* slot);

// ---------------------------------------------------------------- layouts

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Shape {
  int nb, H, heads, d, F, s, b, T;
  int norm, mask, dtype;
  float eps;
  size_t esz;  // bytes per stored element
};

// Validates a descriptor; fills `sh`.  Returns HANAYO_OK / error.
int make_shape(const hanayo_chunk_desc* d, Shape& sh);

// Element offsets of one block's parameters inside the packed array.
struct ParamOffsets {
  size_t off[HANAYO_N_PARAMS];
  size_t cnt[HANAYO_N_PARAMS];
  size_t block_elems;
};
ParamOffsets param_offsets(const Shape& sh);

// Byte offsets inside one block's part of a stash entry.  Every tensor the
// forward pass materialises is written straight into the entry, so stashing
// costs no extra traffic and the backward pass recomputes only the attention
// probabilities.
struct StashLayout {
  size_t x;       // [T][H]   block input
  size_t ln_a;    // [T][H]   pre-LN: LN1(x);            post-LN: x + Attn(x) (input of LN1)
  size_t qkv;     // [T][3H]
  size_t ctx;     // [T][H]   attention context before Wo
  size_t x1;      // [T][H]   pre-LN: x + Attn;          post-LN: LN1 output
  size_t ln_b;    // [T][H]   pre-LN: LN2(x1);           post-LN: x1 + MLP(x1) (input of LN2)
  size_t hpre;    // [T][F]   FFN pre-activation
  size_t act;     // [T][F]   GELU output
  size_t stats1;  // [T] float2 (mean, rstd) of LN1
  size_t stats2;  // [T] float2 of LN2
  size_t lse;     // [b][heads][s] float, log-sum-exp of the scaled masked scores
  size_t block_bytes;
};
StashLayout stash_layout(const Shape& sh);

// Byte offsets inside the workspace (backward scratch; forward uses none).
struct WorkLayout {
  size_t d_act;    // [T][F]  gradient w.r.t. FFN pre-activation
  size_t d_h0;     // [T][H]  scratch gradient tensors
  size_t d_h1;     // [T][H]
  size_t d_h2;     // [T][H]
  size_t d_h3;     // [T][H]
  size_t d_qkv;    // [T][3H]
  size_t d_ping;   // [T][H]  dy hand-off between blocks
  size_t d_pong;   // [T][H]
  size_t delta;    // [b][heads][s] float, rowsum(dC * C)
  size_t partial;  // [rows][2H] float, LayerNorm gamma/beta partial sums; also bias-grad partials
  size_t ln_partial, ln_slot_bytes;  // 2 * nb slots of [kLnPartialRows][2H] float: the partial gamma/beta sums of each
                                     // LayerNorm of the chunk, kept until one launch adds them all up
  size_t bytes;
};
WorkLayout work_layout(const Shape& sh);
constexpr int kMaxPartialRows = 512;
constexpr int kLnPartialRows = 256;  // partial rows one LayerNorm backward writes (one per workgroup, one workgroup per CU)

}  // namespace hanayo
