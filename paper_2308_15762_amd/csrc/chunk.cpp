// chunk_forward / chunk_backward: the fixed kernel sequence of n_blocks
// transformer blocks for one micro-batch (the paper's T_F / 2W and T_B / 2W
// units of work), plus the dispatch between the MFMA and the ALU kernels.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>

#include <vector>

#include "kernels.h"

namespace hanayo {

namespace {

// gfx950 check, cached per device.
int check_device() {
  static thread_local int ok_device = -1;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return set_error(HANAYO_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev == ok_device) return HANAYO_OK;
  hipDeviceProp_t prop;
  e = hipGetDeviceProperties(&prop, dev);
  if (e != hipSuccess) return set_error(HANAYO_EHIP, "hipGetDeviceProperties: %s", hipGetErrorString(e));
  if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0)
    return set_error(HANAYO_EUNSUPPORTED, "device %d is %s, this library is built for gfx950 only", dev, prop.gcnArchName);
  ok_device = dev;
  return HANAYO_OK;
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) != 0; }

struct BlockPtrs {
  const char* w[HANAYO_N_PARAMS];
  float* g[HANAYO_N_PARAMS];
};

BlockPtrs block_ptrs(const Shape& sh, const ParamOffsets& po, const void* weights, float* grads, int blk) {
  BlockPtrs bp;
  for (int i = 0; i < HANAYO_N_PARAMS; ++i) {
    const size_t e = (size_t)blk * po.block_elems + po.off[i];
    bp.w[i] = static_cast<const char*>(weights) + e * sh.esz;
    bp.g[i] = grads ? grads + e : nullptr;
  }
  return bp;
}

enum { P_LN1G, P_LN1B, P_WQKV, P_BQKV, P_WO, P_BO, P_LN2G, P_LN2B, P_W1, P_B1, P_W2, P_B2 };

#define TRY(expr)          \
  do {                     \
    const int rc_ = (expr); \
    if (rc_) return rc_;   \
  } while (0)

// y[T][N] = x[T][K] W[K][N] (+ epilogue)
int linear_fwd(const Shape& sh, const void* x, const void* W, const void* bias, void* y, int K, int N, k::Epilogue epi,
               const void* aux, void* aux_out, hipStream_t st) {
  k::GemmArgs g{};
  g.A = x; g.B = W; g.C = y; g.bias = bias; g.aux = aux; g.aux_out = aux_out;
  g.M = sh.T; g.N = N; g.K = K; g.lda = K; g.ldb = N; g.ldc = N;
  g.a_t = false; g.b_t = true; g.epi = epi;
  return k::gemm(sh.dtype, g, st);
}

// dx[T][K] = dy[T][N] W[K][N]^T (+ epilogue)
int linear_bwd_input(const Shape& sh, const void* dy, const void* W, void* dx, int K, int N, k::Epilogue epi,
                     const void* aux, hipStream_t st) {
  k::GemmArgs g{};
  g.A = dy; g.B = W; g.C = dx; g.aux = aux;
  g.M = sh.T; g.N = K; g.K = N; g.lda = N; g.ldb = N; g.ldc = K;
  g.a_t = false; g.b_t = false; g.epi = epi;
  return k::gemm(sh.dtype, g, st);
}

// dW[K][N] += x[T][K]^T dy[T][N];  db[N] += column sums of dy
k::GemmArgs bwd_params_gemm(const Shape& sh, const void* x, const void* dy, float* dW, float* db, int K, int N,
                            float* partial) {
  k::GemmArgs g{};
  g.A = x; g.B = dy; g.C = dW;
  g.M = K; g.N = N; g.K = sh.T; g.lda = K; g.ldb = N; g.ldc = N;
  g.a_t = true; g.b_t = true; g.epi = k::EPI_ACCUM_F32;
  g.colsum = db; g.colsum_scratch = partial;  // bias gradient rides along with the weight gradient
  return g;
}

}  // namespace

namespace k {

namespace {
thread_local int g_gemm_config = -1;  // measurement knob: of the calling thread only
thread_local double g_gemm_sharing = 0.0;
}
void set_gemm_config(int config) { g_gemm_config = config; }
double gemm_sharing() { return g_gemm_sharing; }
void set_gemm_sharing(double share) { g_gemm_sharing = share < 0.0 ? 0.0 : (share > 1.0 ? 1.0 : share); }

// Tile choice for the direct-to-LDS kernels by a cost model fitted to timings on MI355X: a launch
// runs ceil(tiles / 256 CUs) rounds; a round costs one K tile's time per 32 columns of K (0.84 us for
// 256 x 256 with 8 wavefronts, 0.53 us for 256 x 128 (one wavefront per SIMD, three-stage ring; measured on a chip in
// its sustained clock state with operands that do not stay in the Infinity Cache), 0.295 us for 128 x 128 with two workgroups
// sharing a CU) plus an epilogue, and the launch a fixed start-up (pipeline fill grows with the
// tile).  Large tiles reuse operands better; small ones waste less of the last round, which matters
// less the more the chip is shared with other streams' kernels (set_gemm_sharing).  Returns -1 if no
// configuration takes every problem.
int choose_dma_config(const GemmArgs* gs, int count) {
  if (g_gemm_config >= 0 && g_gemm_config != 3) {
    for (int i = 0; i < count; ++i)
      if (!gemm_dma_supported(gs[i], g_gemm_config)) return -1;
    return g_gemm_config;
  }
  if (g_gemm_config != -1) return -1;
  static const struct { int config; double per_ktile, epilogue, start; } kTiles[] = {
      {6, 0.79, 3.0, 7.0}, {2, 0.53, 2.0, 4.5}, {4, 0.295, 2.3, 3.3}};
  int best = -1;
  double best_cost = 0.0;
  for (const auto& t : kTiles) {
    int bm, bn;
    gemm_dma_tile(t.config, bm, bn);
    long tiles = 0;
    double ktiles = 0.0;  // summed over all tiles
    bool ok = true;
    for (int i = 0; i < count && ok; ++i) {
      ok = gemm_dma_supported(gs[i], t.config);
      const long ti = (long)(gs[i].M / bm) * (gs[i].N / bn);
      tiles += ti;
      ktiles += (double)ti * (gs[i].K / 32);
    }
    if (!ok || tiles == 0) continue;
    // Alone on the chip a launch pays for whole rounds; next to kernels of other lanes the CUs its
    // last round leaves idle are not lost, so the count moves towards tiles / 256.
    const double rounds = g_gemm_sharing * (double)tiles / 256.0 + (1.0 - g_gemm_sharing) * (double)((tiles + 255) / 256);
    const double cost = t.start + rounds * ((ktiles / tiles) * t.per_ktile + t.epilogue);
    if (best < 0 || cost < best_cost) best = t.config, best_cost = cost;
  }
  // The same tile with 64-wide K tiles (half the barriers per unit of work) where K allows it.  The 256 x 128 tile
  // and, for a launch of at most one tile per CU alone on the chip, the 128 x 128 tile take a ring of three such
  // stages: with one wavefront per SIMD nothing else covers a load that is late, and one more tile of look-ahead
  // is worth 11 - 21 % on the 2048 x 4096 outputs with K = 4096 .. 16384 (270 us instead of 338 for the input gradient
  // of FC1 at H = 4096) and 4 - 6 % on the 4096 x 1024 outputs.  The 128 x 128 tile with two stages only where a CU
  // holds two workgroups at a time (more than 256 tiles, or a chip shared with other lanes): measured alone on the
  // chip, 2048 x 2560 x 2560 takes 35 us instead of 44, but 4096 x 1024 x 4096, one workgroup per CU, 42 instead of 38.
  if (best == 6 || best == 2 || best == 4) {
    long tiles = 0;
    for (int i = 0; i < count; ++i) tiles += (long)(gs[i].M / 128) * (gs[i].N / 128);
    const bool one_per_cu = best == 4 && tiles <= 256 && g_gemm_sharing <= 0.0;
    const int wide_config = best == 6 ? 7 : best == 2 ? 10 : one_per_cu ? 11 : 9;
    bool wide = true;
    for (int i = 0; i < count; ++i) wide = wide && gemm_dma_supported(gs[i], wide_config);
    if (wide) best = wide_config;
  }
  return best;
}

int gemm(int dtype, const GemmArgs& g, hipStream_t stream) {
  if (g.M < 1 || g.N < 1 || g.K < 1) return set_error(HANAYO_EINVAL, "gemm: empty problem");
  if (g.colsum && (!g.b_t || !g.colsum_scratch)) return set_error(HANAYO_EINVAL, "gemm: colsum needs b_t and scratch");
  if (dtype == HANAYO_BF16) {
    // the direct-to-LDS kernels fold the column sums into the GEMM
    const int config = choose_dma_config(&g, 1);
    if (config >= 0) return gemm_dma(g, config, stream);
  }
  int rc;
  if (dtype == HANAYO_BF16 && gemm_mfma_supported(g)) rc = gemm_mfma(g, stream);
  else rc = gemm_alu(dtype, g, stream);
  if (rc || !g.colsum) return rc;
  return colsum_add(dtype, g.B, g.K, g.N, g.colsum, g.colsum_scratch, stream);  // B is stored [K][ldb = N]
}

int gemm_group(int dtype, const GemmArgs* gs, int count, hipStream_t stream) {
  if (count < 1 || count > 4) return set_error(HANAYO_EINVAL, "gemm_group: %d problems", count);
  bool alike = dtype == HANAYO_BF16;
  for (int i = 0; i < count; ++i) {
    const GemmArgs& g = gs[i];
    if (g.M < 1 || g.N < 1 || g.K < 1) return set_error(HANAYO_EINVAL, "gemm: empty problem");
    if (g.colsum && (!g.b_t || !g.colsum_scratch)) return set_error(HANAYO_EINVAL, "gemm: colsum needs b_t and scratch");
    alike = alike && g.a_t == gs[0].a_t && g.b_t == gs[0].b_t && g.epi == gs[0].epi;
  }
  if (alike) {
    const int config = choose_dma_config(gs, count);
    if (config >= 0) return gemm_dma_group(gs, count, config, stream);
  }
  for (int i = 0; i < count; ++i) {
    const int rc = gemm(dtype, gs[i], stream);
    if (rc) return rc;
  }
  return HANAYO_OK;
}

int attn_forward(int dtype, const AttnArgs& a, hipStream_t stream) {
  if (dtype == HANAYO_BF16 && attn_mfma_supported(a)) return attn_forward_mfma(a, stream);
  return attn_forward_alu(dtype, a, stream);
}

int attn_backward(int dtype, const AttnArgs& a, hipStream_t stream) {
  if (dtype == HANAYO_BF16 && attn_mfma_supported(a)) return attn_backward_mfma(a, stream);
  return attn_backward_alu(dtype, a, stream);
}

}  // namespace k

int chunk_forward(const Shape& sh, const void* weights, const void* x, const int32_t* valid_len, void* y, void* stash,
                  hipStream_t st) {
  const ParamOffsets po = param_offsets(sh);
  const StashLayout L = stash_layout(sh);
  const int T = sh.T, H = sh.H, F = sh.F;
  const size_t act_bytes = (size_t)T * H * sh.esz;
  for (int blk = 0; blk < sh.nb; ++blk) {
    char* sb = static_cast<char*>(stash) + (size_t)blk * L.block_bytes;
    const BlockPtrs p = block_ptrs(sh, po, weights, nullptr, blk);
    // block input: the caller's x for the first block (copied into the stash), else what the block before wrote
    const void* xin = blk == 0 ? x : sb + L.x;
    void* yout = blk == sh.nb - 1 ? y : sb + L.block_bytes + L.x;
    k::AttnArgs at{};
    at.qkv = sb + L.qkv; at.valid_len = valid_len; at.ctx = sb + L.ctx; at.lse = reinterpret_cast<float*>(sb + L.lse);
    at.b = sh.b; at.s = sh.s; at.heads = sh.heads; at.d = sh.d; at.causal = sh.mask == HANAYO_MASK_CAUSAL;
    if (sh.norm == HANAYO_PRE_LN) {
      TRY(k::ln_forward(sh.dtype, xin, p.w[P_LN1G], p.w[P_LN1B], sb + L.ln_a, reinterpret_cast<float2*>(sb + L.stats1),
                        blk == 0 ? sb + L.x : nullptr, T, H, sh.eps, st));
      TRY(linear_fwd(sh, sb + L.ln_a, p.w[P_WQKV], p.w[P_BQKV], sb + L.qkv, H, 3 * H, k::EPI_BIAS, nullptr, nullptr, st));
      TRY(k::attn_forward(sh.dtype, at, st));
      TRY(linear_fwd(sh, sb + L.ctx, p.w[P_WO], p.w[P_BO], sb + L.x1, H, H, k::EPI_BIAS_RES, xin, nullptr, st));
      TRY(k::ln_forward(sh.dtype, sb + L.x1, p.w[P_LN2G], p.w[P_LN2B], sb + L.ln_b, reinterpret_cast<float2*>(sb + L.stats2),
                        nullptr, T, H, sh.eps, st));
      TRY(linear_fwd(sh, sb + L.ln_b, p.w[P_W1], p.w[P_B1], sb + L.act, H, F, k::EPI_BIAS_GELU, nullptr, sb + L.hpre, st));
      TRY(linear_fwd(sh, sb + L.act, p.w[P_W2], p.w[P_B2], yout, F, H, k::EPI_BIAS_RES, sb + L.x1, nullptr, st));
    } else {
      if (blk == 0) TRY(k::copy_bytes(sb + L.x, x, act_bytes, st));
      TRY(linear_fwd(sh, xin, p.w[P_WQKV], p.w[P_BQKV], sb + L.qkv, H, 3 * H, k::EPI_BIAS, nullptr, nullptr, st));
      TRY(k::attn_forward(sh.dtype, at, st));
      TRY(linear_fwd(sh, sb + L.ctx, p.w[P_WO], p.w[P_BO], sb + L.ln_a, H, H, k::EPI_BIAS_RES, xin, nullptr, st));
      TRY(k::ln_forward(sh.dtype, sb + L.ln_a, p.w[P_LN1G], p.w[P_LN1B], sb + L.x1, reinterpret_cast<float2*>(sb + L.stats1),
                        nullptr, T, H, sh.eps, st));
      TRY(linear_fwd(sh, sb + L.x1, p.w[P_W1], p.w[P_B1], sb + L.act, H, F, k::EPI_BIAS_GELU, nullptr, sb + L.hpre, st));
      TRY(linear_fwd(sh, sb + L.act, p.w[P_W2], p.w[P_B2], sb + L.ln_b, F, H, k::EPI_BIAS_RES, sb + L.x1, nullptr, st));
      TRY(k::ln_forward(sh.dtype, sb + L.ln_b, p.w[P_LN2G], p.w[P_LN2B], yout, reinterpret_cast<float2*>(sb + L.stats2),
                        nullptr, T, H, sh.eps, st));
    }
  }
  return HANAYO_OK;
}

int chunk_backward(const Shape& sh, const void* weights, float* grads, const void* dy, const int32_t* valid_len,
                   const void* stash, void* dx, void* workspace, hipStream_t st) {
  const ParamOffsets po = param_offsets(sh);
  const StashLayout L = stash_layout(sh);
  const WorkLayout WL = work_layout(sh);
  char* ws = static_cast<char*>(workspace);
  const int T = sh.T, H = sh.H, F = sh.F;
  float* partial = reinterpret_cast<float*>(ws + WL.partial);
  // Every LayerNorm backward leaves its partial gamma/beta sums in a slot of its own; one launch after the
  // last block adds them all to the gradients.
  std::vector<k::FinalizeJob> ln_jobs;
  ln_jobs.reserve(2 * (size_t)sh.nb);
  auto ln_slot = [&]() { return reinterpret_cast<float*>(ws + WL.ln_partial + ln_jobs.size() * WL.ln_slot_bytes); };
  auto ln_bwd = [&](const void* dout, const void* x, const void* gamma, const void* stats, const void* addend, void* dz,
                    float* dgamma, float* dbeta) {
    k::FinalizeJob job;
    const int rc = k::ln_backward_deferred(sh.dtype, dout, x, gamma, reinterpret_cast<const float2*>(stats), addend, dz,
                                           dgamma, dbeta, ln_slot(), T, H, st, &job);
    if (rc == HANAYO_OK) ln_jobs.push_back(job);
    return rc;
  };
  const void* dy_blk = dy;
  for (int blk = sh.nb - 1; blk >= 0; --blk) {
    // The four weight-gradient GEMMs of a block wait until its end and go out as one group: every
    // activation and gradient they read stays untouched until then.
    k::GemmArgs dw[4];
    const char* sb = static_cast<const char*>(stash) + (size_t)blk * L.block_bytes;
    const BlockPtrs p = block_ptrs(sh, po, weights, grads, blk);
    // gradient w.r.t. this block's input: the caller's dx for block 0, else a ping-pong buffer
    void* dx_blk = blk == 0 ? dx : ws + ((blk & 1) ? WL.d_ping : WL.d_pong);
    k::AttnArgs at{};
    at.qkv = sb + L.qkv; at.valid_len = valid_len; at.ctx = const_cast<char*>(sb + L.ctx);
    at.lse = reinterpret_cast<float*>(const_cast<char*>(sb + L.lse));
    at.dqkv = ws + WL.d_qkv; at.delta = reinterpret_cast<float*>(ws + WL.delta);
    at.b = sh.b; at.s = sh.s; at.heads = sh.heads; at.d = sh.d; at.causal = sh.mask == HANAYO_MASK_CAUSAL;
    if (sh.norm == HANAYO_PRE_LN) {
      // y = x1 + W2 GELU(W1 LN2(x1))
      dw[0] = bwd_params_gemm(sh, sb + L.act, dy_blk, p.g[P_W2], p.g[P_B2], F, H, partial);
      TRY(linear_bwd_input(sh, dy_blk, p.w[P_W2], ws + WL.d_act, F, H, k::EPI_MUL_DGELU, sb + L.hpre, st));
      dw[1] = bwd_params_gemm(sh, sb + L.ln_b, ws + WL.d_act, p.g[P_W1], p.g[P_B1], H, F, partial);
      TRY(linear_bwd_input(sh, ws + WL.d_act, p.w[P_W1], ws + WL.d_h0, H, F, k::EPI_NONE, nullptr, st));
      // dx1 = dy + LN2'(d_h0)
      TRY(ln_bwd(ws + WL.d_h0, sb + L.x1, p.w[P_LN2G], sb + L.stats2,
                 dy_blk, ws + WL.d_h1, p.g[P_LN2G], p.g[P_LN2B]));
      // x1 = x + Wo ctx
      dw[2] = bwd_params_gemm(sh, sb + L.ctx, ws + WL.d_h1, p.g[P_WO], p.g[P_BO], H, H, partial);
      TRY(linear_bwd_input(sh, ws + WL.d_h1, p.w[P_WO], ws + WL.d_h0, H, H, k::EPI_NONE, nullptr, st));
      at.dctx = ws + WL.d_h0;
      TRY(k::attn_backward(sh.dtype, at, st));
      dw[3] = bwd_params_gemm(sh, sb + L.ln_a, ws + WL.d_qkv, p.g[P_WQKV], p.g[P_BQKV], H, 3 * H, partial);
      TRY(linear_bwd_input(sh, ws + WL.d_qkv, p.w[P_WQKV], ws + WL.d_h2, H, 3 * H, k::EPI_NONE, nullptr, st));
      // dx = dx1 + LN1'(d_h2)
      TRY(ln_bwd(ws + WL.d_h2, sb + L.x, p.w[P_LN1G], sb + L.stats1,
                 ws + WL.d_h1, dx_blk, p.g[P_LN1G], p.g[P_LN1B]));
    } else {
      // y = LN2(f), f = x1 + W2 GELU(W1 x1)
      TRY(ln_bwd(dy_blk, sb + L.ln_b, p.w[P_LN2G], sb + L.stats2,
                 nullptr, ws + WL.d_h0, p.g[P_LN2G], p.g[P_LN2B]));
      dw[0] = bwd_params_gemm(sh, sb + L.act, ws + WL.d_h0, p.g[P_W2], p.g[P_B2], F, H, partial);
      TRY(linear_bwd_input(sh, ws + WL.d_h0, p.w[P_W2], ws + WL.d_act, F, H, k::EPI_MUL_DGELU, sb + L.hpre, st));
      dw[1] = bwd_params_gemm(sh, sb + L.x1, ws + WL.d_act, p.g[P_W1], p.g[P_B1], H, F, partial);
      // dx1 = df + d_act W1^T
      TRY(linear_bwd_input(sh, ws + WL.d_act, p.w[P_W1], ws + WL.d_h1, H, F, k::EPI_ADD, ws + WL.d_h0, st));
      // x1 = LN1(a), a = x + Wo ctx
      TRY(ln_bwd(ws + WL.d_h1, sb + L.ln_a, p.w[P_LN1G], sb + L.stats1,
                 nullptr, ws + WL.d_h2, p.g[P_LN1G], p.g[P_LN1B]));
      dw[2] = bwd_params_gemm(sh, sb + L.ctx, ws + WL.d_h2, p.g[P_WO], p.g[P_BO], H, H, partial);
      TRY(linear_bwd_input(sh, ws + WL.d_h2, p.w[P_WO], ws + WL.d_h3, H, H, k::EPI_NONE, nullptr, st));
      at.dctx = ws + WL.d_h3;  // d_h0 still feeds the W2 gradient
      TRY(k::attn_backward(sh.dtype, at, st));
      dw[3] = bwd_params_gemm(sh, sb + L.x, ws + WL.d_qkv, p.g[P_WQKV], p.g[P_BQKV], H, 3 * H, partial);
      // dx = da + dqkv Wqkv^T
      TRY(linear_bwd_input(sh, ws + WL.d_qkv, p.w[P_WQKV], dx_blk, H, 3 * H, k::EPI_ADD, ws + WL.d_h2, st));
    }
    TRY(k::gemm_group(sh.dtype, dw, 4, st));
    dy_blk = dx_blk;
  }
  return k::finalize_group(ln_jobs.data(), (int)ln_jobs.size(), st);
}

int device_ok() { return check_device(); }

int prepare_call(const hanayo_chunk_desc* d, Shape& sh) {
  TRY(make_shape(d, sh));
  return check_device();
}

}  // namespace hanayo

using namespace hanayo;

extern "C" {

int hanayo_chunk_forward(const hanayo_chunk_desc* d, const void* weights, const void* x, const int32_t* valid_len,
                         void* y, void* stash_entry, void* workspace, void* hip_stream) {
  Shape sh;
  TRY(prepare_call(d, sh));
  (void)workspace;
  if (!weights || !x || !y || !stash_entry) return set_error(HANAYO_EINVAL, "chunk_forward: NULL pointer");
  if (misaligned(weights) || misaligned(x) || misaligned(y) || misaligned(stash_entry))
    return set_error(HANAYO_EINVAL, "chunk_forward: device pointers must be 256-byte aligned");
  if (x == y) return set_error(HANAYO_EINVAL, "chunk_forward: y aliases x");
  return chunk_forward(sh, weights, x, valid_len, y, stash_entry, static_cast<hipStream_t>(hip_stream));
}

int hanayo_chunk_backward(const hanayo_chunk_desc* d, const void* weights, float* grads, const void* dy,
                          const int32_t* valid_len, const void* stash_entry, void* dx, void* workspace,
                          void* hip_stream) {
  Shape sh;
  TRY(prepare_call(d, sh));
  if (!weights || !grads || !dy || !dx || !stash_entry || !workspace)
    return set_error(HANAYO_EINVAL, "chunk_backward: NULL pointer");
  if (misaligned(weights) || misaligned(grads) || misaligned(dy) || misaligned(dx) || misaligned(stash_entry) ||
      misaligned(workspace))
    return set_error(HANAYO_EINVAL, "chunk_backward: device pointers must be 256-byte aligned");
  if (dx == dy) return set_error(HANAYO_EINVAL, "chunk_backward: dx aliases dy");
  return chunk_backward(sh, weights, grads, dy, valid_len, stash_entry, dx, workspace,
                        static_cast<hipStream_t>(hip_stream));
}

int hanayo_device_info(char* buf, size_t cap) {
  if (!buf || !cap) return set_error(HANAYO_EINVAL, "device_info: no buffer");
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
    (void)hipGetLastError();
    return set_error(HANAYO_EHIP, "device_info: no HIP device");
  }
  std::snprintf(buf, cap, "%s %s CUs=%d clock_khz=%d", prop.name, prop.gcnArchName, prop.multiProcessorCount,
                prop.clockRate);
  return HANAYO_OK;
}

}  // extern "C"
