// Host-side launchers of the HIP kernels.  Every launcher validates what the
// kernel and its grid assume, enqueues on `stream`, and returns HANAYO_OK or an
// error code (nothing is enqueued on error).
#pragma once

#include <hip/hip_runtime.h>

#include "internal.h"

namespace hanayo {
namespace k {

// ---- LayerNorm (row-wise over H; wavefront reductions) ----------------------
// out = LN(x) * gamma + beta; stats[t] = (mean, rstd); copy_out (optional) = x.
int ln_forward(int dtype, const void* x, const void* gamma, const void* beta, void* out, float2* stats, void* copy_out,
               int T, int H, float eps, hipStream_t stream);
// dz = LN'(dout) (+ addend, optional); dgamma += sum_t dout*xhat; dbeta += sum_t dout.
// `partial` is scratch of at least kMaxPartialRows * 2H floats.
int ln_backward(int dtype, const void* dout, const void* x, const void* gamma, const float2* stats, const void* addend,
                void* dz, float* dgamma, float* dbeta, float* partial, int T, int H, hipStream_t stream);
// The same with the last step left to the caller: dz is written, the gamma/beta sums stay as partial rows in
// `partial` (kLnPartialRows * 2H floats, untouched until finalize_group has run) and *job says how to add them up.
// finalize_group runs any number of such jobs, eight to a launch: one launch for all the LayerNorms of a chunk's
// backward pass instead of one each.
constexpr int kMaxFinalizeJobs = 8;
struct FinalizeJob {
  const float* partial;  // [rows][ld]
  int rows, ld, n;       // columns c < n: (c < split ? out0[c] : out1[c - split]) += sum over rows of partial[r][c]
  float* out0;
  float* out1;
  int split;
};
int ln_backward_deferred(int dtype, const void* dout, const void* x, const void* gamma, const float2* stats,
                         const void* addend, void* dz, float* dgamma, float* dbeta, float* partial, int T, int H,
                         hipStream_t stream, FinalizeJob* job);
int finalize_group(const FinalizeJob* jobs, int count, hipStream_t stream);
// out[n] += sum_t in[t][n]
int colsum_add(int dtype, const void* in, int T, int N, float* out, float* partial, hipStream_t stream);

// ---- GEMM ---------------------------------------------------------------------
enum Epilogue {
  EPI_NONE = 0,       // C = acc
  EPI_BIAS,           // C = acc + bias[n]
  EPI_BIAS_GELU,      // aux_out = acc + bias[n];  C = GELU(aux_out)
  EPI_BIAS_RES,       // C = acc + bias[n] + aux[m][n]
  EPI_MUL_DGELU,      // C = acc * GELU'(aux[m][n])
  EPI_ADD,            // C = acc + aux[m][n]
  EPI_ACCUM_F32,      // C (fp32) += acc
  EPI_STORE_F32       // C (fp32) = acc   (partial products of a K split; !a_t && b_t only)
};

// C[M][N] = A[M][K] * B[K][N] with fp32 accumulation.
//   a_t = false: A stored [M][lda] (K contiguous);  true: stored [K][lda] (M contiguous)
//   b_t = false: B stored [N][ldb] (K contiguous);  true: stored [K][ldb] (N contiguous)
// C, aux, aux_out are row-major [M][ldc]; bias is the storage type, [N].
struct GemmArgs {
  const void* A;
  const void* B;
  void* C;
  const void* bias;
  const void* aux;
  void* aux_out;
  int M, N, K;
  int lda, ldb, ldc;
  bool a_t, b_t;
  Epilogue epi;
  // Optional, only with b_t: colsum[n] (fp32) += sum over k of B[k][n] (the bias gradient that
  // goes with a weight-gradient GEMM).  colsum_scratch: at least 64 * N floats, used by the
  // kernels that cannot fold the sums into the GEMM itself.
  float* colsum;
  float* colsum_scratch;
};
int gemm(int dtype, const GemmArgs& g, hipStream_t stream);
// Up to 4 independent problems of one layout and epilogue; one launch where the tiled kernels allow
// it (small problems then fill the chip together), otherwise one after the other.
int gemm_group(int dtype, const GemmArgs* gs, int count, hipStream_t stream);

// ---- attention ------------------------------------------------------------------
// qkv is [b*s][3H] (Q | K | V, head j in columns j*d..), ctx [b*s][H], lse [b][heads][s].
struct AttnArgs {
  const void* qkv;
  const int32_t* valid_len;  // device [b] or nullptr
  void* ctx;                 // forward: out; backward: in
  float* lse;                // forward: out; backward: in
  const void* dctx;          // backward in
  void* dqkv;                // backward out [b*s][3H]
  float* delta;              // backward scratch [b][heads][s]
  int b, s, heads, d;
  bool causal;
};
int attn_forward(int dtype, const AttnArgs& a, hipStream_t stream);
int attn_backward(int dtype, const AttnArgs& a, hipStream_t stream);

// Implementations behind the dispatchers above.
int gemm_alu(int dtype, const GemmArgs& g, hipStream_t stream);
int attn_forward_alu(int dtype, const AttnArgs& a, hipStream_t stream);
int attn_backward_alu(int dtype, const AttnArgs& a, hipStream_t stream);
int attn_delta(int dtype, const AttnArgs& a, hipStream_t stream);  // delta = rowsum(dctx * ctx)
bool gemm_mfma_supported(const GemmArgs& g);
int gemm_mfma(const GemmArgs& g, hipStream_t stream);  // bf16 only
// Direct-to-LDS multi-stage kernel for tile-aligned shapes; config 0 = 256x256, 1 = 128x128 (8-deep ring),
// 2 = 256x128, 4 = 128x128 (4-deep ring), 5 = 128x128 with 8 wavefronts, 6 = 256x256 with 8 wavefronts,
// 7 / 8 / 9 = 256x256 (8 wavefronts) / 256x128 / 128x128 with two stages of 64-wide K tiles (K a multiple of 64),
// 10 / 11 = 256x128 / 128x128 with three such stages.
bool gemm_dma_supported(const GemmArgs& g, int config);
void gemm_dma_tile(int config, int& bm, int& bn);
int gemm_dma(const GemmArgs& g, int config, hipStream_t stream);
int gemm_dma_group(const GemmArgs* gs, int count, int config, hipStream_t stream);
// -1 = automatic choice; 0, 1, 2, 4 .. 11 = force that direct-to-LDS configuration where it applies; 3 = staged kernel only
void set_gemm_config(int config);
// How much of the chip the calling thread's GEMM launches share with kernels of other streams: 0 = a launch
// runs alone (choose the tile for the shortest launch), 1 = idle CUs are always taken by other work (choose
// for the least CU time).  The executor sets it from its lane count while it enqueues a list.
void set_gemm_sharing(double share);
double gemm_sharing();
bool attn_mfma_supported(const AttnArgs& a);
int attn_forward_mfma(const AttnArgs& a, hipStream_t stream);
int attn_backward_mfma(const AttnArgs& a, hipStream_t stream);

// ---- the model's ends and the optimizer --------------------------------------------
// x[n][i][:] = wte[tokens[n][i]][:] + wpe[i][:]; tokens outside [0, vocab) contribute nothing.
int embed_forward(int dtype, const void* wte, const void* wpe, const int32_t* tokens, void* x, int b, int s, int H,
                  int vocab, hipStream_t stream);
// d_wte[tokens[n][i]][:] += dx[n][i][:] (fixed order, no atomics); d_wpe[i][:] += sum_n dx[n][i][:].
int embed_backward(int dtype, const int32_t* tokens, const void* dx, float* d_wte, float* d_wpe, int b, int s, int H,
                   int vocab, hipStream_t stream);
// count[0] = number of labels inside [0, vocab).
int count_labels(const int32_t* labels, int rows, int vocab, float* count, hipStream_t stream);
// In place on logits [rows][V]: the gradient of loss_scale * (mean over counted rows of the negative
// log-likelihood); nll[row] = the row's negative log-likelihood (0 if its label is outside [0, V)).
int softmax_xent(int dtype, void* logits, const int32_t* labels, const float* count, float loss_scale, float* nll,
                 int rows, int V, hipStream_t stream);
// loss[0] = sum(nll) / count[0] (0 if count is 0).
int loss_finish(const float* nll, const float* count, int rows, float* loss, hipStream_t stream);
struct AdamArgs {
  void* params;   // storage type, updated
  float* master;  // bf16 storage: fp32 copy of the parameters, updated; ignored for fp32 storage
  float* grads;
  float* m;
  float* v;
  size_t count;   // multiple of 4
  float lr, beta1, beta2, eps, weight_decay;
  int step;       // t >= 1
  int zero_grads;
  // weight decay applies everywhere (block_elems = 0) or only where (index mod block_elems) falls in one of
  // the four ranges [lo, hi)
  size_t block_elems;
  size_t lo[4], hi[4];
};
int adam(int dtype, const AdamArgs& a, hipStream_t stream);

// out[i] = sum over s < slices of parts[s * count + i]  (the partial products of a K split; count multiple of 8)
int sum_slices(int dtype, const float* parts, int slices, size_t count, void* out, hipStream_t stream);

// ---- misc ------------------------------------------------------------------------
// max_workgroups > 0 caps the grid: a copy that uses only a few CUs and so runs at a chosen fraction of the
// memory bandwidth (the emulated link of the pipeline runs).
int copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t stream, int max_workgroups = 0);

// Checks the last launch; returns HANAYO_EHIP with the HIP message on failure.
int check_launch(const char* what);

}  // namespace k
}  // namespace hanayo
