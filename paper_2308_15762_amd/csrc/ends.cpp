// The two ends of the model (token + position embedding in front of stage 0,
// head GEMM + softmax cross-entropy behind the last stage) and the optimizer
// step at the flush: the fixed kernel sequences and their C entry points.
//
// The head's forward and backward run back to back: the loss gradient needs
// nothing from another stage, so the logits never leave the workspace and the
// gradient w.r.t. the last stage's output is ready when that stage's backward
// task comes up.
#include <hip/hip_runtime.h>

#include "ends.h"
#include "kernels.h"

namespace hanayo {

int prepare_call(const hanayo_chunk_desc* d, Shape& sh);

namespace {

#define TRY(expr)           \
  do {                      \
    const int rc_ = (expr); \
    if (rc_) return rc_;    \
  } while (0)

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) != 0; }

struct HeadLayout {
  size_t hn;       // [T][H]  LN_f(y)
  size_t d_hn;     // [T][H]  gradient w.r.t. hn
  size_t stats;    // [T] float2
  size_t nll;      // [T] float
  size_t count;    // float
  size_t partial;  // [kMaxPartialRows][2H] float
  size_t logits;   // [T][V]
  size_t split;    // [kHeadSplit][T][H] float: partial products of the d_hn GEMM when its K (= V) is split
  size_t bytes;
};
constexpr int kHeadSplit = 4;

HeadLayout head_layout(const Shape& sh, int vocab) {
  HeadLayout L{};
  size_t at = 0;
  auto take = [&](size_t bytes) {
    const size_t here = at;
    at += align_up(bytes, 256);
    return here;
  };
  const size_t act = (size_t)sh.T * sh.H * sh.esz;
  L.hn = take(act);
  L.d_hn = take(act);
  L.stats = take((size_t)sh.T * sizeof(float2));
  L.nll = take((size_t)sh.T * sizeof(float));
  L.count = take(sizeof(float));
  L.partial = take((size_t)kMaxPartialRows * 2 * sh.H * sizeof(float));
  L.logits = take((size_t)sh.T * vocab * sh.esz);
  L.split = take((size_t)kHeadSplit * sh.T * sh.H * sizeof(float));
  L.bytes = at;
  return L;
}

}  // namespace

int check_ends(const Shape& sh, const hanayo_ends_desc* e) {
  if (!e) return set_error(HANAYO_EINVAL, "ends: NULL descriptor");
  if (e->vocab < 8 || e->vocab % 8) return set_error(HANAYO_EINVAL, "ends: vocab %d must be a positive multiple of 8", e->vocab);
  if (e->max_pos < sh.s) return set_error(HANAYO_EINVAL, "ends: position table has %d rows, sequences %d tokens", e->max_pos, sh.s);
  if (e->final_ln != 0 && e->final_ln != 1) return set_error(HANAYO_EINVAL, "ends: final_ln %d", e->final_ln);
  if ((size_t)sh.T * e->vocab * sh.esz >= ((size_t)1 << 40)) return set_error(HANAYO_EUNSUPPORTED, "ends: logits too large");
  return HANAYO_OK;
}

size_t head_workspace_bytes(const Shape& sh, int vocab) { return head_layout(sh, vocab).bytes; }

int embed_forward(const Shape& sh, const hanayo_ends_desc* e, const void* wte, const void* wpe, const int32_t* tokens,
                  void* x, hipStream_t st) {
  return k::embed_forward(sh.dtype, wte, wpe, tokens, x, sh.b, sh.s, sh.H, e->vocab, st);
}

int embed_backward(const Shape& sh, const hanayo_ends_desc* e, const int32_t* tokens, const void* dx, float* d_wte,
                   float* d_wpe, hipStream_t st) {
  return k::embed_backward(sh.dtype, tokens, dx, d_wte, d_wpe, sh.b, sh.s, sh.H, e->vocab, st);
}

int head_loss(const Shape& sh, const hanayo_ends_desc* e, const void* lnf, const void* head, const void* y,
              const int32_t* labels, float loss_scale, float* loss, void* dy, float* d_lnf, float* d_head,
              void* workspace, hipStream_t st) {
  const HeadLayout L = head_layout(sh, e->vocab);
  char* ws = static_cast<char*>(workspace);
  const int T = sh.T, H = sh.H, V = e->vocab;
  float* count = reinterpret_cast<float*>(ws + L.count);
  float* nll = reinterpret_cast<float*>(ws + L.nll);
  float2* stats = reinterpret_cast<float2*>(ws + L.stats);
  const void* hn = y;
  if (e->final_ln) {
    const char* gamma = static_cast<const char*>(lnf);
    TRY(k::ln_forward(sh.dtype, y, gamma, gamma + (size_t)H * sh.esz, ws + L.hn, stats, nullptr, T, H, sh.eps, st));
    hn = ws + L.hn;
  }
  TRY(k::count_labels(labels, T, V, count, st));
  // The vocabulary is rarely a multiple of the largest GEMM tile (256): for the logits the rows of the table up to
  // the last such multiple go out as one launch that may use it, the few rows left as a second, small one.
  const int v_main = V >= 512 ? V / 256 * 256 : V, v_rest = V - v_main;
  const char* head_rest = static_cast<const char*>(head) + (size_t)v_main * H * sh.esz;
  // logits[T][V] = hn[T][H] head[V][H]^T
  k::GemmArgs g{};
  g.A = hn; g.B = head; g.C = ws + L.logits;
  g.M = T; g.N = v_main; g.K = H; g.lda = H; g.ldb = H; g.ldc = V;
  g.a_t = false; g.b_t = false; g.epi = k::EPI_NONE;
  TRY(k::gemm(sh.dtype, g, st));
  if (v_rest) {
    g.B = head_rest; g.C = ws + L.logits + (size_t)v_main * sh.esz; g.N = v_rest;
    TRY(k::gemm(sh.dtype, g, st));
  }
  // in place: logits -> gradient of loss_scale * loss w.r.t. the logits
  TRY(k::softmax_xent(sh.dtype, ws + L.logits, labels, count, loss_scale, nll, T, V, st));
  TRY(k::loss_finish(nll, count, T, loss, st));
  // d_head[V][H] += dlogits[T][V]^T hn[T][H]
  k::GemmArgs gw{};
  gw.A = ws + L.logits; gw.B = hn; gw.C = d_head;
  gw.M = V; gw.N = H; gw.K = T; gw.lda = V; gw.ldb = H; gw.ldc = H;
  gw.a_t = true; gw.b_t = true; gw.epi = k::EPI_ACCUM_F32;
  // Alone on the chip one launch of small tiles is fastest here (measured: V / 256 x H / 256 large tiles leave a
  // quarter of the last round idle); next to other lanes' kernels idle CUs are not lost and the large tile's
  // better use of a CU wins, so the rows split as for the logits.
  if (v_rest && k::gemm_sharing() > 0.0) {
    gw.M = v_main;
    TRY(k::gemm(sh.dtype, gw, st));
    gw.A = ws + L.logits + (size_t)v_main * sh.esz; gw.C = d_head + (size_t)v_main * H; gw.M = v_rest;
  }
  TRY(k::gemm(sh.dtype, gw, st));
  // d_hn[T][H] = dlogits[T][V] head[V][H]
  k::GemmArgs gx{};
  gx.A = ws + L.logits; gx.B = head; gx.C = e->final_ln ? static_cast<void*>(ws + L.d_hn) : dy;
  gx.M = T; gx.N = H; gx.K = V; gx.lda = V; gx.ldb = H; gx.ldc = H;
  gx.a_t = false; gx.b_t = true; gx.epi = k::EPI_NONE;
  // The output has T H / 256^2 tiles (64 for 4096 x 1024) and the contraction runs over the whole vocabulary:
  // where the largest tile would leave most of the chip idle, K is cut into kHeadSplit slices that go out as one
  // grouped launch into fp32 partial products, summed by a small kernel.
  const int slice = (V / kHeadSplit) / 64 * 64;  // the last slice takes the rest
  const long tiles256 = (long)(T / 256) * (H / 256);
  bool split = sh.dtype == HANAYO_BF16 && slice >= 1024 && T % 256 == 0 && H % 256 == 0 && tiles256 * kHeadSplit <= 256;
  k::GemmArgs part[kHeadSplit];
  for (int i = 0; i < kHeadSplit && split; ++i) {
    const int k0 = i * slice, kn = i + 1 < kHeadSplit ? slice : V - k0;
    part[i] = gx;
    part[i].A = ws + L.logits + (size_t)k0 * sh.esz;
    part[i].B = static_cast<const char*>(head) + (size_t)k0 * H * sh.esz;
    part[i].C = ws + L.split + (size_t)i * T * H * sizeof(float);
    part[i].K = kn;
    part[i].epi = k::EPI_STORE_F32;
    split = k::gemm_dma_supported(part[i], 7);  // 256 x 256 tiles, 64-wide K tiles
  }
  if (split) {
    TRY(k::gemm_dma_group(part, kHeadSplit, 7, st));
    TRY(k::sum_slices(sh.dtype, reinterpret_cast<const float*>(ws + L.split), kHeadSplit, (size_t)T * H, gx.C, st));
  } else {
    TRY(k::gemm(sh.dtype, gx, st));
  }
  if (e->final_ln)
    TRY(k::ln_backward(sh.dtype, ws + L.d_hn, y, lnf, stats, nullptr, dy, d_lnf, d_lnf + H,
                       reinterpret_cast<float*>(ws + L.partial), T, H, st));
  return HANAYO_OK;
}

int chunk_adam_step(const hanayo_adam* o, const Shape& sh, void* weights, float* master, float* grads, float* m,
                    float* v, hipStream_t st) {
  const ParamOffsets po = param_offsets(sh);
  k::AdamArgs a{};
  a.params = weights; a.master = master; a.grads = grads; a.m = m; a.v = v;
  a.count = po.block_elems * sh.nb;
  a.lr = o->lr; a.beta1 = o->beta1; a.beta2 = o->beta2; a.eps = o->eps; a.weight_decay = o->weight_decay;
  a.step = o->step; a.zero_grads = o->zero_grads;
  a.block_elems = po.block_elems;
  static const int kMatrices[4] = {2, 4, 8, 10};  // Wqkv, Wo, W1, W2: the biases and LayerNorm parameters do not decay
  for (int r = 0; r < 4; ++r) {
    a.lo[r] = po.off[kMatrices[r]];
    a.hi[r] = po.off[kMatrices[r]] + po.cnt[kMatrices[r]];
  }
  return k::adam(sh.dtype, a, st);
}

}  // namespace hanayo

using namespace hanayo;

extern "C" {

int hanayo_embed_forward(const hanayo_chunk_desc* d, const hanayo_ends_desc* e, const void* wte, const void* wpe,
                         const int32_t* tokens, void* x, void* hip_stream) {
  Shape sh;
  TRY(prepare_call(d, sh));
  TRY(check_ends(sh, e));
  if (!wte || !wpe || !tokens || !x) return set_error(HANAYO_EINVAL, "embed_forward: NULL pointer");
  if (misaligned(wte) || misaligned(wpe) || misaligned(x))
    return set_error(HANAYO_EINVAL, "embed_forward: device pointers must be 256-byte aligned");
  return embed_forward(sh, e, wte, wpe, tokens, x, static_cast<hipStream_t>(hip_stream));
}

int hanayo_embed_backward(const hanayo_chunk_desc* d, const hanayo_ends_desc* e, const int32_t* tokens, const void* dx,
                          float* d_wte, float* d_wpe, void* hip_stream) {
  Shape sh;
  TRY(prepare_call(d, sh));
  TRY(check_ends(sh, e));
  if (!tokens || !dx || !d_wte || !d_wpe) return set_error(HANAYO_EINVAL, "embed_backward: NULL pointer");
  if (misaligned(dx) || misaligned(d_wte) || misaligned(d_wpe))
    return set_error(HANAYO_EINVAL, "embed_backward: device pointers must be 256-byte aligned");
  return embed_backward(sh, e, tokens, dx, d_wte, d_wpe, static_cast<hipStream_t>(hip_stream));
}

size_t hanayo_head_workspace_bytes(const hanayo_chunk_desc* d, const hanayo_ends_desc* e) {
  Shape sh;
  if (make_shape(d, sh) || check_ends(sh, e)) return 0;
  return head_workspace_bytes(sh, e->vocab);
}

int hanayo_head_loss(const hanayo_chunk_desc* d, const hanayo_ends_desc* e, const void* lnf, const void* head,
                     const void* y, const int32_t* labels, float loss_scale, float* loss, void* dy, float* d_lnf,
                     float* d_head, void* workspace, void* hip_stream) {
  Shape sh;
  TRY(prepare_call(d, sh));
  TRY(check_ends(sh, e));
  if (!head || !y || !labels || !loss || !dy || !d_head || !workspace || (e->final_ln && (!lnf || !d_lnf)))
    return set_error(HANAYO_EINVAL, "head_loss: NULL pointer");
  if (misaligned(head) || misaligned(y) || misaligned(dy) || misaligned(d_head) || misaligned(workspace) ||
      (e->final_ln && (misaligned(lnf) || misaligned(d_lnf))))
    return set_error(HANAYO_EINVAL, "head_loss: device pointers must be 256-byte aligned");
  if (y == dy) return set_error(HANAYO_EINVAL, "head_loss: dy aliases y");
  return head_loss(sh, e, lnf, head, y, labels, loss_scale, loss, dy, d_lnf, d_head, workspace,
                   static_cast<hipStream_t>(hip_stream));
}

int hanayo_adam_step(const hanayo_adam* o, int dtype, void* params, float* master, float* grads, float* m, float* v,
                     size_t count, void* hip_stream) {
  if (!o) return set_error(HANAYO_EINVAL, "adam_step: NULL argument");
  if (dtype != HANAYO_FP32 && dtype != HANAYO_BF16) return set_error(HANAYO_EINVAL, "adam_step: dtype %d", dtype);
  TRY(device_ok());
  k::AdamArgs a{};
  a.params = params; a.master = master; a.grads = grads; a.m = m; a.v = v; a.count = count;
  a.lr = o->lr; a.beta1 = o->beta1; a.beta2 = o->beta2; a.eps = o->eps; a.weight_decay = o->weight_decay;
  a.step = o->step; a.zero_grads = o->zero_grads;
  a.block_elems = 0;
  return k::adam(dtype, a, static_cast<hipStream_t>(hip_stream));
}

int hanayo_chunk_adam_step(const hanayo_adam* o, const hanayo_chunk_desc* d, void* weights, float* master, float* grads,
                           float* m, float* v, void* hip_stream) {
  if (!o) return set_error(HANAYO_EINVAL, "chunk_adam_step: NULL argument");
  Shape sh;
  TRY(prepare_call(d, sh));
  return chunk_adam_step(o, sh, weights, master, grads, m, v, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
