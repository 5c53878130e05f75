// C entry points for the single kernels of the chunk path.
#include <hip/hip_runtime.h>

#include "kernels.h"

using namespace hanayo;

namespace hanayo {
int prepare_call(const hanayo_chunk_desc* d, Shape& sh);
}

namespace {
int check_dtype(int dtype) {
  if (dtype != HANAYO_FP32 && dtype != HANAYO_BF16) return set_error(HANAYO_EINVAL, "dtype must be HANAYO_FP32 or HANAYO_BF16");
  return HANAYO_OK;
}
}  // namespace

extern "C" {

namespace {
int fill_gemm(const hanayo_gemm_problem& q, int a_t, int b_t, int epilogue, k::GemmArgs& g) {
  if (!q.A || !q.B || !q.C || q.M < 1 || q.N < 1 || q.K < 1)
    return set_error(HANAYO_EINVAL, "op_gemm: NULL operand or empty problem");
  if (epilogue < HANAYO_EPI_NONE || epilogue > HANAYO_EPI_ACCUM_F32) return set_error(HANAYO_EINVAL, "op_gemm: epilogue");
  if (q.lda < (a_t ? q.M : q.K) || q.ldb < (b_t ? q.N : q.K) || q.ldc < q.N)
    return set_error(HANAYO_EINVAL, "op_gemm: leading dimension too small");
  const bool need_bias = epilogue == HANAYO_EPI_BIAS || epilogue == HANAYO_EPI_BIAS_GELU || epilogue == HANAYO_EPI_BIAS_RES;
  const bool need_aux = epilogue == HANAYO_EPI_BIAS_RES || epilogue == HANAYO_EPI_MUL_DGELU || epilogue == HANAYO_EPI_ADD;
  if ((need_bias && !q.bias) || (need_aux && !q.aux) || (epilogue == HANAYO_EPI_BIAS_GELU && !q.aux_out))
    return set_error(HANAYO_EINVAL, "op_gemm: epilogue operand missing");
  if (q.colsum && (!b_t || !q.colsum_scratch || q.ldb != q.N))
    return set_error(HANAYO_EINVAL, "op_gemm: colsum needs b_t = 1, ldb = N and a scratch buffer");
  g = k::GemmArgs{};
  g.A = q.A; g.B = q.B; g.C = q.C; g.bias = q.bias; g.aux = q.aux; g.aux_out = q.aux_out;
  g.M = q.M; g.N = q.N; g.K = q.K; g.lda = q.lda; g.ldb = q.ldb; g.ldc = q.ldc;
  g.a_t = a_t != 0; g.b_t = b_t != 0; g.epi = static_cast<k::Epilogue>(epilogue);
  g.colsum = q.colsum; g.colsum_scratch = q.colsum_scratch;
  return HANAYO_OK;
}
}  // namespace

int hanayo_op_gemm(int dtype, const void* A, const void* B, void* C, int M, int N, int K, int lda, int ldb, int ldc,
                   int a_t, int b_t, int epilogue, const void* bias, const void* aux, void* aux_out, float* colsum,
                   float* colsum_scratch, void* hip_stream) {
  if (int rc = check_dtype(dtype)) return rc;
  const hanayo_gemm_problem q = {A, B, C, bias, aux, aux_out, M, N, K, lda, ldb, ldc, colsum, colsum_scratch};
  k::GemmArgs g;
  if (int rc = fill_gemm(q, a_t, b_t, epilogue, g)) return rc;
  return k::gemm(dtype, g, static_cast<hipStream_t>(hip_stream));
}

int hanayo_op_gemm_group(int dtype, int a_t, int b_t, int epilogue, const hanayo_gemm_problem* problems, int count,
                         void* hip_stream) {
  if (int rc = check_dtype(dtype)) return rc;
  if (!problems || count < 1 || count > 4) return set_error(HANAYO_EINVAL, "op_gemm_group: 1 to 4 problems");
  k::GemmArgs gs[4];
  for (int i = 0; i < count; ++i)
    if (int rc = fill_gemm(problems[i], a_t, b_t, epilogue, gs[i])) return rc;
  return k::gemm_group(dtype, gs, count, static_cast<hipStream_t>(hip_stream));
}

int hanayo_op_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
  if (!dst || !src) return set_error(HANAYO_EINVAL, "op_copy: NULL pointer");
  return k::copy_bytes(dst, src, bytes, static_cast<hipStream_t>(hip_stream));
}

int hanayo_op_gemm_config(int config) {
  if (config < -1 || config > 11) return set_error(HANAYO_EINVAL, "op_gemm_config: config must be -1..11");
  k::set_gemm_config(config);
  return HANAYO_OK;
}

int hanayo_op_layernorm_forward(int dtype, const void* x, const void* gamma, const void* beta, void* out, float* stats,
                                void* copy_out, int rows, int hidden, float eps, void* hip_stream) {
  if (int rc = check_dtype(dtype)) return rc;
  if (!x || !gamma || !beta || !out || !stats || rows < 1) return set_error(HANAYO_EINVAL, "op_layernorm_forward: bad argument");
  return k::ln_forward(dtype, x, gamma, beta, out, reinterpret_cast<float2*>(stats), copy_out, rows, hidden, eps,
                       static_cast<hipStream_t>(hip_stream));
}

int hanayo_op_layernorm_backward(int dtype, const void* dout, const void* x, const void* gamma, const float* stats,
                                 const void* addend, void* dz, float* dgamma, float* dbeta, float* scratch, int rows,
                                 int hidden, void* hip_stream) {
  if (int rc = check_dtype(dtype)) return rc;
  if (!dout || !x || !gamma || !stats || !dz || !dgamma || !dbeta || !scratch || rows < 1)
    return set_error(HANAYO_EINVAL, "op_layernorm_backward: bad argument");
  return k::ln_backward(dtype, dout, x, gamma, reinterpret_cast<const float2*>(stats), addend, dz, dgamma, dbeta, scratch,
                        rows, hidden, static_cast<hipStream_t>(hip_stream));
}

int hanayo_op_colsum_add(int dtype, const void* in, int rows, int n, float* out, float* scratch, void* hip_stream) {
  if (int rc = check_dtype(dtype)) return rc;
  if (!in || !out || !scratch) return set_error(HANAYO_EINVAL, "op_colsum_add: NULL pointer");
  return k::colsum_add(dtype, in, rows, n, out, scratch, static_cast<hipStream_t>(hip_stream));
}

static int attn_args(k::AttnArgs& a, int b, int s, int heads, int head_dim, int causal) {
  if (b < 1 || s < 1 || heads < 1 || head_dim < 8 || head_dim % 8 || head_dim > 128)
    return set_error(HANAYO_EINVAL, "op_attention: bad shape");
  a.b = b; a.s = s; a.heads = heads; a.d = head_dim; a.causal = causal != 0;
  return HANAYO_OK;
}

int hanayo_op_attention_forward(int dtype, const void* qkv, const int32_t* valid_len, void* ctx, float* lse, int b, int s,
                                int heads, int head_dim, int causal, void* hip_stream) {
  if (int rc = check_dtype(dtype)) return rc;
  if (!qkv || !ctx || !lse) return set_error(HANAYO_EINVAL, "op_attention_forward: NULL pointer");
  k::AttnArgs a{};
  if (int rc = attn_args(a, b, s, heads, head_dim, causal)) return rc;
  a.qkv = qkv; a.valid_len = valid_len; a.ctx = ctx; a.lse = lse;
  return k::attn_forward(dtype, a, static_cast<hipStream_t>(hip_stream));
}

int hanayo_op_attention_backward(int dtype, const void* qkv, const int32_t* valid_len, const void* ctx, const float* lse,
                                 const void* dctx, void* dqkv, float* delta, int b, int s, int heads, int head_dim,
                                 int causal, void* hip_stream) {
  if (int rc = check_dtype(dtype)) return rc;
  if (!qkv || !ctx || !lse || !dctx || !dqkv || !delta) return set_error(HANAYO_EINVAL, "op_attention_backward: NULL pointer");
  k::AttnArgs a{};
  if (int rc = attn_args(a, b, s, heads, head_dim, causal)) return rc;
  a.qkv = qkv; a.valid_len = valid_len; a.ctx = const_cast<void*>(ctx); a.lse = const_cast<float*>(lse);
  a.dctx = dctx; a.dqkv = dqkv; a.delta = delta;
  return k::attn_backward(dtype, a, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
