// ALU (non-MFMA) GEMM and attention kernels for any storage type and any shape.
// They carry the fp32 storage path (which has to stay in fp32 arithmetic to
// meet its 1e-4 bound) and the bf16 shapes the MFMA kernels do not cover.
#include "device_util.h"
#include "epilogue.h"
#include "kernels.h"

namespace hanayo {
namespace k {

namespace {

// ---------------------------------------------------------------- GEMM 64x64x16
template <typename T, int EPI>
__global__ __launch_bounds__(256) void gemm_alu_kernel(const T* __restrict__ A, const T* __restrict__ B, int M, int N,
                                                       int K, int lda, int ldb, bool a_t, bool b_t, EpiParams<T> ep) {
  __shared__ float As[16][64 + 4];
  __shared__ float Bs[16][64 + 4];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
  for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = threadIdx.x + i * 256;
      int mm, kk;
      if (a_t) { kk = idx >> 6; mm = idx & 63; } else { mm = idx >> 4; kk = idx & 15; }
      const int gm = m0 + mm, gk = k0 + kk;
      float v = 0.f;
      if (gm < M && gk < K) v = ld(A + (a_t ? (size_t)gk * lda + gm : (size_t)gm * lda + gk));
      As[kk][mm] = v;
      int nn;
      if (b_t) { kk = idx >> 6; nn = idx & 63; } else { nn = idx >> 4; kk = idx & 15; }
      const int gn = n0 + nn, gk2 = k0 + kk;
      v = 0.f;
      if (gn < N && gk2 < K) v = ld(B + (b_t ? (size_t)gk2 * ldb + gn : (size_t)gn * ldb + gk2));
      Bs[kk][nn] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < M && n < N) epilogue_one<T, EPI>(ep, m, n, acc[i][j]);
    }
}

// ---------------------------------------------------------------- attention
// One wavefront per (query row, head, sequence).  Scores of the row sit in LDS.
__device__ __forceinline__ bool key_allowed(int i, int j, int s, int len, bool causal) {
  return j < len && (!causal || j <= i);
}

template <typename T>
__global__ __launch_bounds__(64) void attn_fwd_alu_kernel(const T* __restrict__ qkv, const int32_t* __restrict__ valid_len,
                                                          T* __restrict__ ctx, float* __restrict__ lse, int s, int heads,
                                                          int d, bool causal) {
  extern __shared__ float sc[];  // [s] scores, then [d] q
  float* qs = sc + s;
  const int i = blockIdx.x, h = blockIdx.y, n = blockIdx.z, lane = threadIdx.x;
  const int H = heads * d;
  const size_t ld3 = (size_t)3 * H;
  const T* base = qkv + (size_t)n * s * ld3;
  const int len = valid_len ? valid_len[n] : s;
  const float scale = rsqrtf((float)d);
  for (int c = lane; c < d; c += 64) qs[c] = ld(base + (size_t)i * ld3 + h * d + c);
  __syncthreads();
  float mx = -INFINITY;
  for (int j = lane; j < s; j += 64) {
    float v = -INFINITY;
    if (key_allowed(i, j, s, len, causal)) {
      const T* kr = base + (size_t)j * ld3 + H + h * d;
      float t = 0.f;
      for (int c = 0; c < d; ++c) t += qs[c] * ld(kr + c);
      v = t * scale;
    }
    sc[j] = v;
    mx = fmaxf(mx, v);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int j = lane; j < s; j += 64) {
    const float e = sc[j] == -INFINITY ? 0.f : __expf(sc[j] - mx);
    sc[j] = e;
    sum += e;
  }
  sum = wave_sum(sum);
  __syncthreads();
  const float inv = 1.f / sum;
  for (int c = lane; c < d; c += 64) {
    float t = 0.f;
    for (int j = 0; j < s; ++j) {
      const float p = sc[j];
      if (p != 0.f) t += p * ld(base + (size_t)j * ld3 + 2 * H + h * d + c);
    }
    st(ctx + ((size_t)n * s + i) * H + h * d + c, t * inv);
  }
  if (lane == 0) lse[((size_t)n * heads + h) * s + i] = mx + __logf(sum);
}

// delta[n][h][i] = sum_c dctx[i][c] * ctx[i][c].  ctx and dctx are read as one stream of 8-element
// vectors (d / 8 consecutive vectors make one (row, head) group); a workgroup takes kDeltaGroups
// groups, parks the per-vector sums in LDS and adds each group up.
constexpr int kDeltaGroups = 64;
template <typename T>
__global__ __launch_bounds__(256) void attn_delta_kernel(const T* __restrict__ ctx, const T* __restrict__ dctx,
                                                         float* __restrict__ delta, long groups, int s, int heads, int d) {
  __shared__ float part[kDeltaGroups * 16];
  const int vpg = d / 8;  // vectors per group, at most 16
  const long g0 = (long)blockIdx.x * kDeltaGroups;
  const int ng = (int)(groups - g0 < kDeltaGroups ? groups - g0 : kDeltaGroups);
  for (int v = threadIdx.x; v < ng * vpg; v += 256) {
    float a[8], b[8];
    load8(ctx + (g0 * vpg + v) * 8, a);
    load8(dctx + (g0 * vpg + v) * 8, b);
    float t = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) t += a[e] * b[e];
    part[v] = t;
  }
  __syncthreads();
  if ((int)threadIdx.x < ng) {
    float t = 0.f;
    for (int j = 0; j < vpg; ++j) t += part[threadIdx.x * vpg + j];
    const long g = g0 + threadIdx.x;  // = row * heads + head
    const long row = g / heads;
    const int h = (int)(g - row * heads);
    delta[((row / s) * heads + h) * s + row % s] = t;
  }
}

// dQ of one query row: dS_j = P_ij (dP_ij - delta_i), dQ_i = scale * sum_j dS_j K_j
template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_dq_alu_kernel(const T* __restrict__ qkv, const int32_t* __restrict__ valid_len,
                                                             const T* __restrict__ dctx, const float* __restrict__ lse,
                                                             const float* __restrict__ delta, T* __restrict__ dqkv,
                                                             int s, int heads, int d, bool causal) {
  extern __shared__ float sc[];  // [s] dS, [d] q, [d] dctx row
  float* qs = sc + s;
  float* dc = qs + d;
  const int i = blockIdx.x, h = blockIdx.y, n = blockIdx.z, lane = threadIdx.x;
  const int H = heads * d;
  const size_t ld3 = (size_t)3 * H;
  const T* base = qkv + (size_t)n * s * ld3;
  const int len = valid_len ? valid_len[n] : s;
  const float scale = rsqrtf((float)d);
  const size_t st_at = ((size_t)n * heads + h) * s + i;
  const float l = lse[st_at], dl = delta[st_at];
  for (int c = lane; c < d; c += 64) {
    qs[c] = ld(base + (size_t)i * ld3 + h * d + c);
    dc[c] = ld(dctx + ((size_t)n * s + i) * H + h * d + c);
  }
  __syncthreads();
  for (int j = lane; j < s; j += 64) {
    float ds = 0.f;
    if (key_allowed(i, j, s, len, causal)) {
      const T* kr = base + (size_t)j * ld3 + H + h * d;
      const T* vr = base + (size_t)j * ld3 + 2 * H + h * d;
      float t = 0.f, dp = 0.f;
      for (int c = 0; c < d; ++c) {
        t += qs[c] * ld(kr + c);
        dp += dc[c] * ld(vr + c);
      }
      ds = __expf(t * scale - l) * (dp - dl);
    }
    sc[j] = ds;
  }
  __syncthreads();
  for (int c = lane; c < d; c += 64) {
    float t = 0.f;
    for (int j = 0; j < s; ++j) {
      const float ds = sc[j];
      if (ds != 0.f) t += ds * ld(base + (size_t)j * ld3 + H + h * d + c);
    }
    st(dqkv + ((size_t)n * s + i) * ld3 + h * d + c, t * scale);
  }
}

// dK and dV of one key row: loops over all query rows.
template <typename T>
__global__ __launch_bounds__(64) void attn_bwd_dkv_alu_kernel(const T* __restrict__ qkv, const int32_t* __restrict__ valid_len,
                                                              const T* __restrict__ dctx, const float* __restrict__ lse,
                                                              const float* __restrict__ delta, T* __restrict__ dqkv,
                                                              int s, int heads, int d, bool causal) {
  extern __shared__ float sc[];  // [s] dS, [s] P, [d] k, [d] v
  float* pr = sc + s;
  float* ks = pr + s;
  float* vs = ks + d;
  const int j = blockIdx.x, h = blockIdx.y, n = blockIdx.z, lane = threadIdx.x;
  const int H = heads * d;
  const size_t ld3 = (size_t)3 * H;
  const T* base = qkv + (size_t)n * s * ld3;
  const int len = valid_len ? valid_len[n] : s;
  const float scale = rsqrtf((float)d);
  for (int c = lane; c < d; c += 64) {
    ks[c] = ld(base + (size_t)j * ld3 + H + h * d + c);
    vs[c] = ld(base + (size_t)j * ld3 + 2 * H + h * d + c);
  }
  __syncthreads();
  for (int i = lane; i < s; i += 64) {
    float ds = 0.f, p = 0.f;
    if (key_allowed(i, j, s, len, causal)) {
      const T* qr = base + (size_t)i * ld3 + h * d;
      const T* dr = dctx + ((size_t)n * s + i) * H + h * d;
      float t = 0.f, dp = 0.f;
      for (int c = 0; c < d; ++c) {
        t += ld(qr + c) * ks[c];
        dp += ld(dr + c) * vs[c];
      }
      const size_t st_at = ((size_t)n * heads + h) * s + i;
      p = __expf(t * scale - lse[st_at]);
      ds = p * (dp - delta[st_at]);
    }
    sc[i] = ds;
    pr[i] = p;
  }
  __syncthreads();
  for (int c = lane; c < d; c += 64) {
    float tk = 0.f, tv = 0.f;
    for (int i = 0; i < s; ++i) {
      const float p = pr[i];
      if (p != 0.f) {
        tk += sc[i] * ld(base + (size_t)i * ld3 + h * d + c);
        tv += p * ld(dctx + ((size_t)n * s + i) * H + h * d + c);
      }
    }
    st(dqkv + ((size_t)n * s + j) * ld3 + H + h * d + c, tk * scale);
    st(dqkv + ((size_t)n * s + j) * ld3 + 2 * H + h * d + c, tv);
  }
}

template <typename T>
int gemm_alu_t(const GemmArgs& g, hipStream_t stream) {
  EpiParams<T> ep{(T*)g.C, (float*)g.C, (const T*)g.bias, (const T*)g.aux, (T*)g.aux_out, g.ldc};
  const dim3 grid((g.N + 63) / 64, (g.M + 63) / 64), block(256);
#define LAUNCH(E)                                                                                                    \
  case E:                                                                                                            \
    hipLaunchKernelGGL((gemm_alu_kernel<T, E>), grid, block, 0, stream, (const T*)g.A, (const T*)g.B, g.M, g.N, g.K, \
                       g.lda, g.ldb, g.a_t, g.b_t, ep);                                                              \
    break
  switch (g.epi) {
    LAUNCH(EPI_NONE);
    LAUNCH(EPI_BIAS);
    LAUNCH(EPI_BIAS_GELU);
    LAUNCH(EPI_BIAS_RES);
    LAUNCH(EPI_MUL_DGELU);
    LAUNCH(EPI_ADD);
    LAUNCH(EPI_ACCUM_F32);
    LAUNCH(EPI_STORE_F32);
  }
#undef LAUNCH
  return check_launch("gemm_alu");
}

template <typename T>
int attn_fwd_alu_t(const AttnArgs& a, hipStream_t stream) {
  const dim3 grid(a.s, a.heads, a.b);
  const size_t lds = (size_t)(a.s + a.d) * sizeof(float);
  hipLaunchKernelGGL((attn_fwd_alu_kernel<T>), grid, dim3(64), lds, stream, (const T*)a.qkv, a.valid_len, (T*)a.ctx,
                     a.lse, a.s, a.heads, a.d, a.causal);
  return check_launch("attn_fwd_alu");
}

template <typename T>
int attn_delta_t(const AttnArgs& a, hipStream_t stream) {
  if (a.d % 8 || a.d > 128) return set_error(HANAYO_EUNSUPPORTED, "attn_delta: head dim %d", a.d);
  const long groups = (long)a.b * a.s * a.heads;
  hipLaunchKernelGGL((attn_delta_kernel<T>), dim3((unsigned)((groups + kDeltaGroups - 1) / kDeltaGroups)), dim3(256), 0,
                     stream, (const T*)a.ctx, (const T*)a.dctx, a.delta, groups, a.s, a.heads, a.d);
  return check_launch("attn_delta");
}

template <typename T>
int attn_bwd_alu_t(const AttnArgs& a, hipStream_t stream) {
  int rc = attn_delta_t<T>(a, stream);
  if (rc) return rc;
  const dim3 grid(a.s, a.heads, a.b);
  hipLaunchKernelGGL((attn_bwd_dq_alu_kernel<T>), grid, dim3(64), (size_t)(a.s + 2 * a.d) * sizeof(float), stream,
                     (const T*)a.qkv, a.valid_len, (const T*)a.dctx, a.lse, a.delta, (T*)a.dqkv, a.s, a.heads, a.d,
                     a.causal);
  rc = check_launch("attn_bwd_dq_alu");
  if (rc) return rc;
  hipLaunchKernelGGL((attn_bwd_dkv_alu_kernel<T>), grid, dim3(64), (size_t)(2 * a.s + 2 * a.d) * sizeof(float), stream,
                     (const T*)a.qkv, a.valid_len, (const T*)a.dctx, a.lse, a.delta, (T*)a.dqkv, a.s, a.heads, a.d,
                     a.causal);
  return check_launch("attn_bwd_dkv_alu");
}

}  // namespace

int gemm_alu(int dtype, const GemmArgs& g, hipStream_t stream) {
  return dtype == HANAYO_BF16 ? gemm_alu_t<bf16>(g, stream) : gemm_alu_t<float>(g, stream);
}
int attn_forward_alu(int dtype, const AttnArgs& a, hipStream_t stream) {
  if ((size_t)(2 * a.s + 2 * a.d) * sizeof(float) > 60 * 1024)
    return set_error(HANAYO_EUNSUPPORTED, "attention (ALU path): seq %d too long", a.s);
  return dtype == HANAYO_BF16 ? attn_fwd_alu_t<bf16>(a, stream) : attn_fwd_alu_t<float>(a, stream);
}
int attn_backward_alu(int dtype, const AttnArgs& a, hipStream_t stream) {
  if ((size_t)(2 * a.s + 2 * a.d) * sizeof(float) > 60 * 1024)
    return set_error(HANAYO_EUNSUPPORTED, "attention (ALU path): seq %d too long", a.s);
  return dtype == HANAYO_BF16 ? attn_bwd_alu_t<bf16>(a, stream) : attn_bwd_alu_t<float>(a, stream);
}
int attn_delta(int dtype, const AttnArgs& a, hipStream_t stream) {
  return dtype == HANAYO_BF16 ? attn_delta_t<bf16>(a, stream) : attn_delta_t<float>(a, stream);
}

}  // namespace k
}  // namespace hanayo
