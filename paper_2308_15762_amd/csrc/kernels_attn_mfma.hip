// Fused attention forward / backward for bf16 on the gfx950 matrix cores
// (v_mfma_f32_32x32x16_bf16).  The probability matrix never reaches HBM: the
// forward pass keeps a running row maximum and row sum (online softmax) and
// stores only the context and the per-row log-sum-exp; the backward pass
// recomputes the probabilities of a tile from Q, K and the log-sum-exp.
//
// Orientation.  Every score tile is produced in the orientation in which the
// next contraction consumes it, so probabilities go from accumulator registers
// straight into MFMA operands without any cross-lane movement:
//   * a product that contracts over KEYS (forward P V, backward dS K) uses the
//     tile as S^T = K Q^T: a lane owns one query row and 16 of the 32 keys;
//   * a product that contracts over QUERIES (backward P^T dC, dS^T Q) uses the
//     tile as S = Q K^T: a lane owns one key and 16 of the 32 queries.
// The 8 contraction elements a lane feeds per MFMA are then accumulator
// registers 8t .. 8t+7, i.e. tile rows 16t + {0..3, 8..11} + 4 (lane / 32); the
// other operand is fetched from LDS with the transpose read using the same row
// numbering, which makes the pairing exact.  All outputs come out transposed
// (lane = row, registers = 4 consecutive columns), so stores are 8-byte vectors
// and per-row softmax statistics are per-lane scalars.
#include "device_util.h"
#include "kernels.h"

namespace hanayo {
namespace k {

namespace {

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kPad = 8;  // LDS row padding in elements

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int r = 0; r < 16; ++r) z[r] = 0.f;
  return z;
}

// Row of accumulator register r inside its 32-row tile.
__device__ __forceinline__ int acc_row(int r, int half) { return 8 * (r >> 2) + 4 * half + (r & 3); }

// 16-byte fragment: row (r0 + lane % 32), contraction elements 16 kk + 8 (lane / 32) .. +7,
// from a row-major LDS tile whose rows hold the contraction index contiguously.
template <int PITCH>
__device__ __forceinline__ bf16x8 frag_rows(const bf16* lds, int r0, int kk, int lane) {
  return *reinterpret_cast<const bf16x8*>(lds + (r0 + (lane & 31)) * PITCH + kk * 16 + 8 * (lane >> 5));
}

// The same fragment straight from global memory (row pointer given), zero outside [0, d).
__device__ __forceinline__ bf16x8 frag_global(const bf16* row, bool row_ok, int kk, int lane, int d) {
  const int c = kk * 16 + 8 * (lane >> 5);
  bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
  return (row_ok && c < d) ? *reinterpret_cast<const bf16x8*>(row + c) : z;
}

// Transposed fragment: this lane's "row" is column (c0 + lane % 32) of the LDS tile, its 8
// contraction elements are tile rows rbase + {0..3} and rbase + 8 + {0..3}, with
// rbase = r0 + 4 (lane / 32): the row numbering of accumulator registers 8t .. 8t+7.
template <int PITCH>
__device__ __forceinline__ bf16x8 frag_cols(const bf16* lds, int r0, int c0, int lane) {
  const int row = r0 + 4 * (lane >> 5) + ((lane & 15) >> 2);
  const int col = c0 + 16 * ((lane >> 4) & 1) + (lane & 3) * 4;
  const bf16* p = lds + row * PITCH + col;
  union {
    struct { s16x4 lo, hi; } s;
    bf16x8 v;
  } u;
  u.s.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
  u.s.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 8 * PITCH));
  return u.v;
}

// Accumulator registers 8t .. 8t+7 as a bf16 MFMA operand.
__device__ __forceinline__ bf16x8 pack_half(const f32x16& a, int t) {
  bf16x8 o;
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = (bf16)a[8 * t + j];
  return o;
}

// ROWS x DP tile (DP contiguous) from global rows row0.. with stride ld; zero outside rows < row_lim, cols < d.
template <int ROWS, int DP>
__device__ __forceinline__ void tile_to_lds(bf16* lds, const bf16* g, size_t ld, int row0, int row_lim, int d) {
  constexpr int VPR = DP / 8;
  for (int v = threadIdx.x; v < ROWS * VPR; v += 256) {
    const int r = v / VPR, c = (v % VPR) * 8;
    bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    const bf16x8 val = (row0 + r < row_lim && c < d) ? *reinterpret_cast<const bf16x8*>(g + (size_t)(row0 + r) * ld + c) : z;
    *reinterpret_cast<bf16x8*>(lds + r * (DP + kPad) + c) = val;
  }
}

struct AttnDev {
  const bf16* qkv;
  const int32_t* valid_len;
  bf16* ctx;
  float* lse;
  const bf16* dctx;
  bf16* dqkv;
  const float* delta;
  int s, heads, d, causal;
};

__device__ __forceinline__ int seq_len(const AttnDev& p, int n) {
  if (!p.valid_len) return p.s;
  const int v = p.valid_len[n];
  return v < 1 ? 1 : (v > p.s ? p.s : v);
}

// ------------------------------------------------------------------ forward
// Workgroup = 128 query rows of one (sequence, head); wavefront = 32 of them.
template <int DP>
__global__ __launch_bounds__(256) void attn_fwd_kernel(AttnDev p) {
  constexpr int PITCH = DP + kPad, BKV = 64, KS = DP / 16, DT = DP / 32;
  __shared__ __attribute__((aligned(16))) bf16 Ks[BKV * PITCH];
  __shared__ __attribute__((aligned(16))) bf16 Vs[BKV * PITCH];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5;
  const int qt = gridDim.x - 1 - blockIdx.x, h = blockIdx.y, n = blockIdx.z;
  const int H = p.heads * p.d;
  const size_t ld3 = (size_t)3 * H;
  const bf16* base = p.qkv + (size_t)n * p.s * ld3 + h * p.d;
  const int len = seq_len(p, n);
  const int q0 = qt * 128, qw0 = q0 + 32 * wave, q = qw0 + (lane & 31);
  const int kv_end = p.causal ? min(len, q0 + 128) : len;
  const float c2 = rsqrtf((float)p.d) * kLog2e;

  bf16x8 qf[KS];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) qf[kk] = frag_global(base + (size_t)q * ld3, q < p.s, kk, lane, p.d);
  f32x16 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) o[dt] = zero16();
  float m = -INFINITY, lsum = 0.f;

  for (int k0 = 0; k0 < kv_end; k0 += BKV) {
    __syncthreads();
    tile_to_lds<BKV, DP>(Ks, base + H, ld3, k0, p.s, p.d);
    tile_to_lds<BKV, DP>(Vs, base + 2 * H, ld3, k0, p.s, p.d);
    __syncthreads();
    if (p.causal && k0 > qw0 + 31) continue;  // every key of the tile is ahead of this wavefront's rows
    f32x16 sc[2];
    float mloc = -INFINITY;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      sc[c] = zero16();
#pragma unroll
      for (int kk = 0; kk < KS; ++kk)
        sc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<PITCH>(Ks, 32 * c, kk, lane), qf[kk], sc[c], 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = k0 + 32 * c + acc_row(r, half);
        const bool ok = key < len && (!p.causal || key <= q);
        const float v = ok ? sc[c][r] * c2 : -INFINITY;
        sc[c][r] = v;
        mloc = fmaxf(mloc, v);
      }
    }
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
    const float m_new = fmaxf(m, mloc);  // finite: key 0 is allowed for every row and comes first
    const float alpha = exp2f(m - m_new);
    float rs = 0.f;
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float e = exp2f(sc[c][r] - m_new);
        sc[c][r] = e;
        rs += e;
      }
    rs += __shfl_xor(rs, 32, 64);
    lsum = lsum * alpha + rs;
    m = m_new;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 pf = pack_half(sc[c], t);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols<PITCH>(Vs, 32 * c + 16 * t, 32 * dt, lane), pf, o[dt], 0, 0, 0);
      }
  }
  if (q < p.s) {
    const float inv = 1.f / lsum;
    bf16* out = p.ctx + ((size_t)n * p.s + q) * H + h * p.d;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = 32 * dt + 8 * g + 4 * half;
        if (col < p.d) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (bf16)(o[dt][4 * g + e] * inv);
          *reinterpret_cast<bf16x4*>(out + col) = v;
        }
      }
    if (half == 0) p.lse[((size_t)n * p.heads + h) * p.s + q] = (m + log2f(lsum)) * kLn2;
  }
}

// ------------------------------------------------------------------ backward: dK, dV
// Workgroup = 128 keys of one (sequence, head); wavefront = 32 keys; loops over 64-query tiles.
template <int DP>
__global__ __launch_bounds__(256) void attn_bwd_dkv_kernel(AttnDev p) {
  constexpr int PITCH = DP + kPad, BQ = 64, KS = DP / 16, DT = DP / 32;
  __shared__ __attribute__((aligned(16))) bf16 Qs[BQ * PITCH];
  __shared__ __attribute__((aligned(16))) bf16 Cs[BQ * PITCH];
  __shared__ float lse2[BQ];
  __shared__ float dlt[BQ];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5;
  const int kt = blockIdx.x, h = blockIdx.y, n = blockIdx.z;
  const int H = p.heads * p.d;
  const size_t ld3 = (size_t)3 * H;
  const bf16* base = p.qkv + (size_t)n * p.s * ld3 + h * p.d;
  const bf16* dcb = p.dctx + (size_t)n * p.s * H + h * p.d;
  const size_t stat0 = ((size_t)n * p.heads + h) * p.s;
  const int len = seq_len(p, n);
  const int k0 = kt * 128, kw0 = k0 + 32 * wave, key = kw0 + (lane & 31);
  const float scale = rsqrtf((float)p.d), c2 = scale * kLog2e;

  bf16x8 kf[KS], vf[KS];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) {
    kf[kk] = frag_global(base + H + (size_t)key * ld3, key < p.s, kk, lane, p.d);
    vf[kk] = frag_global(base + 2 * H + (size_t)key * ld3, key < p.s, kk, lane, p.d);
  }
  f32x16 dk[DT], dv[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) {
    dk[dt] = zero16();
    dv[dt] = zero16();
  }
  const int q_begin = (p.causal && k0 < len) ? (k0 / BQ) * BQ : 0;
  const int q_end = k0 < len ? p.s : 0;  // a tile of masked keys gets zero gradients
  for (int q0 = q_begin; q0 < q_end; q0 += BQ) {
    __syncthreads();
    tile_to_lds<BQ, DP>(Qs, base, ld3, q0, p.s, p.d);
    tile_to_lds<BQ, DP>(Cs, dcb, (size_t)H, q0, p.s, p.d);
    if (threadIdx.x < BQ) {
      const int qq = q0 + threadIdx.x;
      lse2[threadIdx.x] = qq < p.s ? p.lse[stat0 + qq] * kLog2e : 0.f;
      dlt[threadIdx.x] = qq < p.s ? p.delta[stat0 + qq] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      if (p.causal && q0 + 32 * c + 31 < kw0) continue;  // all these queries precede the wavefront's keys
      f32x16 sacc = zero16(), dp = zero16();
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<PITCH>(Qs, 32 * c, kk, lane), kf[kk], sacc, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<PITCH>(Cs, 32 * c, kk, lane), vf[kk], dp, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int ql = 32 * c + acc_row(r, half), qq = q0 + ql;
        const bool ok = qq < p.s && key < len && (!p.causal || key <= qq);
        const float pr = ok ? exp2f(sacc[r] * c2 - lse2[ql]) : 0.f;
        sacc[r] = pr;
        dp[r] = pr * (dp[r] - dlt[ql]);
      }
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 pf = pack_half(sacc, t), dsf = pack_half(dp, t);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols<PITCH>(Cs, 32 * c + 16 * t, 32 * dt, lane), pf, dv[dt], 0, 0, 0);
          dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols<PITCH>(Qs, 32 * c + 16 * t, 32 * dt, lane), dsf, dk[dt], 0, 0, 0);
        }
      }
    }
  }
  if (key < p.s) {
    bf16* out = p.dqkv + ((size_t)n * p.s + key) * ld3 + h * p.d;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = 32 * dt + 8 * g + 4 * half;
        if (col < p.d) {
          bf16x4 a, b;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            a[e] = (bf16)(dk[dt][4 * g + e] * scale);
            b[e] = (bf16)dv[dt][4 * g + e];
          }
          *reinterpret_cast<bf16x4*>(out + H + col) = a;
          *reinterpret_cast<bf16x4*>(out + 2 * H + col) = b;
        }
      }
  }
}

// ------------------------------------------------------------------ backward: dQ
// Workgroup = 128 query rows; wavefront = 32; loops over 64-key tiles.
template <int DP>
__global__ __launch_bounds__(256) void attn_bwd_dq_kernel(AttnDev p) {
  constexpr int PITCH = DP + kPad, BKV = 64, KS = DP / 16, DT = DP / 32;
  __shared__ __attribute__((aligned(16))) bf16 Ks[BKV * PITCH];
  __shared__ __attribute__((aligned(16))) bf16 Vs[BKV * PITCH];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5;
  const int qt = gridDim.x - 1 - blockIdx.x, h = blockIdx.y, n = blockIdx.z;
  const int H = p.heads * p.d;
  const size_t ld3 = (size_t)3 * H;
  const bf16* base = p.qkv + (size_t)n * p.s * ld3 + h * p.d;
  const int len = seq_len(p, n);
  const int q0 = qt * 128, qw0 = q0 + 32 * wave, q = qw0 + (lane & 31);
  const int kv_end = p.causal ? min(len, q0 + 128) : len;
  const float scale = rsqrtf((float)p.d), c2 = scale * kLog2e;
  const size_t stat = ((size_t)n * p.heads + h) * p.s + q;
  const float my_lse2 = q < p.s ? p.lse[stat] * kLog2e : 0.f;
  const float my_delta = q < p.s ? p.delta[stat] : 0.f;

  bf16x8 qf[KS], cf[KS];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) {
    qf[kk] = frag_global(base + (size_t)q * ld3, q < p.s, kk, lane, p.d);
    cf[kk] = frag_global(p.dctx + ((size_t)n * p.s + q) * H + h * p.d, q < p.s, kk, lane, p.d);
  }
  f32x16 dq[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) dq[dt] = zero16();

  for (int k0 = 0; k0 < kv_end; k0 += BKV) {
    __syncthreads();
    tile_to_lds<BKV, DP>(Ks, base + H, ld3, k0, p.s, p.d);
    tile_to_lds<BKV, DP>(Vs, base + 2 * H, ld3, k0, p.s, p.d);
    __syncthreads();
    if (p.causal && k0 > qw0 + 31) continue;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      f32x16 sacc = zero16(), dp = zero16();
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<PITCH>(Ks, 32 * c, kk, lane), qf[kk], sacc, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<PITCH>(Vs, 32 * c, kk, lane), cf[kk], dp, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = k0 + 32 * c + acc_row(r, half);
        const bool ok = key < len && (!p.causal || key <= q);
        const float pr = ok ? exp2f(sacc[r] * c2 - my_lse2) : 0.f;
        dp[r] = pr * (dp[r] - my_delta);
      }
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 dsf = pack_half(dp, t);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
          dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols<PITCH>(Ks, 32 * c + 16 * t, 32 * dt, lane), dsf, dq[dt], 0, 0, 0);
      }
    }
  }
  if (q < p.s) {
    bf16* out = p.dqkv + ((size_t)n * p.s + q) * ld3 + h * p.d;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = 32 * dt + 8 * g + 4 * half;
        if (col < p.d) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (bf16)(dq[dt][4 * g + e] * scale);
          *reinterpret_cast<bf16x4*>(out + col) = v;
        }
      }
  }
}

AttnDev to_dev(const AttnArgs& a) {
  AttnDev p;
  p.qkv = (const bf16*)a.qkv; p.valid_len = a.valid_len; p.ctx = (bf16*)a.ctx; p.lse = a.lse;
  p.dctx = (const bf16*)a.dctx; p.dqkv = (bf16*)a.dqkv; p.delta = a.delta;
  p.s = a.s; p.heads = a.heads; p.d = a.d; p.causal = a.causal ? 1 : 0;
  return p;
}

}  // namespace

bool attn_mfma_supported(const AttnArgs& a) { return a.d % 8 == 0 && a.d >= 8 && a.d <= 128; }

int attn_forward_mfma(const AttnArgs& a, hipStream_t stream) {
  if (!attn_mfma_supported(a)) return set_error(HANAYO_EUNSUPPORTED, "attn_mfma: head dim %d", a.d);
  const AttnDev p = to_dev(a);
  const dim3 grid((a.s + 127) / 128, a.heads, a.b), block(256);
  if (a.d <= 64) hipLaunchKernelGGL((attn_fwd_kernel<64>), grid, block, 0, stream, p);
  else if (a.d <= 96) hipLaunchKernelGGL((attn_fwd_kernel<96>), grid, block, 0, stream, p);
  else hipLaunchKernelGGL((attn_fwd_kernel<128>), grid, block, 0, stream, p);
  return check_launch("attn_fwd_mfma");
}

int attn_backward_mfma(const AttnArgs& a, hipStream_t stream) {
  if (!attn_mfma_supported(a)) return set_error(HANAYO_EUNSUPPORTED, "attn_mfma: head dim %d", a.d);
  int rc = attn_delta(HANAYO_BF16, a, stream);
  if (rc) return rc;
  const AttnDev p = to_dev(a);
  const dim3 grid((a.s + 127) / 128, a.heads, a.b), block(256);
  if (a.d <= 64) {
    hipLaunchKernelGGL((attn_bwd_dkv_kernel<64>), grid, block, 0, stream, p);
    hipLaunchKernelGGL((attn_bwd_dq_kernel<64>), grid, block, 0, stream, p);
  } else if (a.d <= 96) {
    hipLaunchKernelGGL((attn_bwd_dkv_kernel<96>), grid, block, 0, stream, p);
    hipLaunchKernelGGL((attn_bwd_dq_kernel<96>), grid, block, 0, stream, p);
  } else {
    hipLaunchKernelGGL((attn_bwd_dkv_kernel<128>), grid, block, 0, stream, p);
    hipLaunchKernelGGL((attn_bwd_dq_kernel<128>), grid, block, 0, stream, p);
  }
  return check_launch("attn_bwd_mfma");
}

}  // namespace k
}  // namespace hanayo
