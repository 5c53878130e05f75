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
  float* delta;  // written by attn_delta or by the pipelined dQ kernel, read by the others
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
  const int qt = gridDim.z - 1 - blockIdx.z, h = blockIdx.x, n = blockIdx.y;
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
  const int kt = blockIdx.z, h = blockIdx.x, n = blockIdx.y;
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
  const int qt = gridDim.z - 1 - blockIdx.z, h = blockIdx.x, n = blockIdx.y;
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

// ======================================================================================
// Direct-to-LDS variants for head dims 64 and 128 (DP == d; 80 and 96 as partly filled DP = 128 rows): K/V (forward, dQ) or Q/dC (dK/dV)
// tiles of 64 rows go global -> LDS with global_load_lds_dwordx4 through a ring of NST buffers,
// so the loads of tile t+NST-1 are in flight while tile t is used; one barrier per tile.
// LDS rows are unpadded and XOR-swizzled in 16-byte slots so that both access patterns are
// bank-conflict free:
//   16-byte fragment reads: 16 consecutive rows at one slot;
//   transpose reads: 4 consecutive rows x 4 consecutive slots per half wavefront.
// DP = 64 (8 slots/row, two rows per 256-byte bank line): slot' = slot ^ (r1<<2 | r3<<1 | r2)
// DP = 128 (16 slots/row, one row per bank line):         slot' = slot ^ (r1<<3 | r0<<2 | r3<<1 | r2)
// with r0..r3 the low bits of the row.
// Softmax arithmetic is kept to one fma and one v_exp_f32 per score (scores stay unscaled, the
// scale goes into the exponent), masks are applied only on tiles that cross the diagonal or the
// end of the valid keys, and the output accumulator is rescaled only when a row maximum moved.
// ======================================================================================

__device__ __forceinline__ void dma16(const void* base, unsigned voff, unsigned lds_byte_addr) {
  asm volatile(
      "s_mov_b32 m0, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %1"
      :
      : "v"(voff), "s"(base), "s"(lds_byte_addr)
      : "memory");
}
__device__ __forceinline__ void dma4(const void* base, unsigned voff, unsigned lds_byte_addr) {
  asm volatile(
      "s_mov_b32 m0, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dword %0, %1"
      :
      : "v"(voff), "s"(base), "s"(lds_byte_addr)
      : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
template <int LOADS>
__device__ __forceinline__ void wait_tiles(int tiles_in_flight) {
  if (tiles_in_flight <= 0) wait_vmcnt<0>();
  else if (tiles_in_flight == 1) wait_vmcnt<LOADS>();
  else wait_vmcnt<2 * LOADS>();
}

template <int DP>
struct SwTile {
  static_assert(DP == 64 || DP == 128, "swizzled tiles exist for head dims 64 and 128");
  static constexpr int SPR = DP / 8;
  static constexpr int kRowsPerInstr = 64 / SPR;
  static constexpr int kInstr = 64 / kRowsPerInstr;  // per 64-row tile
  static constexpr int kPerWave = kInstr / 4;
  static constexpr int kBytes = 64 * DP * 2;

  __device__ static int swz(int row) {
    return DP == 64 ? ((((row >> 1) & 1) << 2) | ((row >> 2) & 3)) : (((row & 3) << 2) | ((row >> 2) & 3));
  }
  // This wavefront's share of the tile whose first row is row0 (rows clamped to s-1).  D = the row
  // length actually present in memory: for D < DP the slots past it are left as they are (every
  // instruction still has active lanes, so the load counts per wavefront do not change); their
  // contents only ever reach output columns >= D, which are not stored.
  template <int D = DP>
  __device__ static void issue(const bf16* gbase, int ld, int row0, int s, unsigned lds_addr, int wave, int lane) {
    static_assert(D % 16 == 0 && D <= DP && D > DP / 2, "row length for this layout");
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
      const int q = wave * kPerWave + i;
      const int lr = q * kRowsPerInstr + lane / SPR, sp = lane % SPR;
      const int row = min(row0 + lr, s - 1);
      const int src = sp ^ swz(lr);  // the global slot that lands in LDS slot sp of this row
      if (D == DP || src < D / 8) dma16(gbase, (unsigned)((row * ld + (src << 3)) * 2), lds_addr + q * 1024);
    }
  }
  // Per-lane byte offsets of every fragment read inside a tile, computed once per kernel.  The swizzle
  // depends on the row's low four bits only, so a fragment that starts r0 rows further down (r0 a
  // multiple of 16) is the same offset plus r0 * SPR * 16, an immediate in the LDS instruction.
  struct Offsets {
    unsigned rows[DP / 16];     // 16-byte fragment of contraction step kk (rows = lane % 32)
    unsigned cols_lo[DP / 32];  // transpose reads of column tile dt: tile rows 4 (lane/32) + 0..3
    unsigned cols_hi[DP / 32];  //                                   and those rows + 8
  };
  __device__ static void init(Offsets& f, int lane) {
#pragma unroll
    for (int kk = 0; kk < DP / 16; ++kk) {
      const int row = lane & 31, slot = 2 * kk + (lane >> 5);
      f.rows[kk] = (unsigned)((row * SPR + (slot ^ swz(row))) * 16);
    }
#pragma unroll
    for (int dt = 0; dt < DP / 32; ++dt) {
      const int row = 4 * (lane >> 5) + ((lane & 15) >> 2);
      const int col = 32 * dt + 16 * ((lane >> 4) & 1) + (lane & 3) * 4;
      const int slot = col >> 3, sub = (col & 7) * 2;
      f.cols_lo[dt] = (unsigned)((row * SPR + (slot ^ swz(row))) * 16 + sub);
      f.cols_hi[dt] = (unsigned)(((row + 8) * SPR + (slot ^ swz(row + 8))) * 16 + sub);
    }
  }
  // rows r0 + lane % 32 (r0 multiple of 16), contraction step kk
  __device__ static bf16x8 frag_rows(const char* lds, const Offsets& f, int r0, int kk) {
    return *reinterpret_cast<const bf16x8*>(lds + f.rows[kk] + r0 * SPR * 16);
  }
  // columns 32 dt + lane % 32; contraction rows r0 + {0..3, 8..11} + 4 (lane / 32) (r0 multiple of 16)
  __device__ static bf16x8 frag_cols(const char* lds, const Offsets& f, int r0, int dt) {
    union {
      struct { s16x4 lo, hi; } s;
      bf16x8 v;
    } u;
    u.s.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds + f.cols_lo[dt] + r0 * SPR * 16));
    u.s.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds + f.cols_hi[dt] + r0 * SPR * 16));
    return u.v;
  }
};

template <int DP, int NST, int D = DP>
__global__ __launch_bounds__(256) void attn_fwd_dma_kernel(AttnDev p) {
  using Tile = SwTile<DP>;
  constexpr int BKV = 64, KS = D / 16, DT = (D + 31) / 32;  // D = head dim in memory, DP = LDS row layout
  constexpr int STAGE = 2 * Tile::kBytes, LOADS = 2 * Tile::kPerWave;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const unsigned lds0 = (unsigned)(unsigned long)((__attribute__((address_space(3))) char*)smem);
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), half = lane >> 5;
  typename Tile::Offsets fo;
  Tile::init(fo, lane);
  const int qt = gridDim.z - 1 - blockIdx.z, h = blockIdx.x, n = blockIdx.y;
  const int H = p.heads * p.d, ld3 = 3 * H;
  const bf16* base = p.qkv + (size_t)n * p.s * ld3 + h * p.d;
  const int len = seq_len(p, n);
  const int q0 = qt * 128, qw0 = q0 + 32 * wave, q = qw0 + (lane & 31);
  const int kv_end = p.causal ? min(len, q0 + 128) : len;
  const int nt = (kv_end + BKV - 1) / BKV;
  const float c2 = rsqrtf((float)p.d) * kLog2e;

  auto issue = [&](int t) {
    const unsigned st = lds0 + (unsigned)(t % NST) * STAGE;
    Tile::template issue<D>(base + H, ld3, t * BKV, p.s, st, wave, lane);
    Tile::template issue<D>(base + 2 * H, ld3, t * BKV, p.s, st + Tile::kBytes, wave, lane);
  };
#pragma unroll
  for (int t = 0; t < NST - 1; ++t)
    if (t < nt) issue(t);

  bf16x8 qf[KS];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) qf[kk] = frag_global(base + (size_t)q * ld3, q < p.s, kk, lane, p.d);
  f32x16 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) o[dt] = zero16();
  float m = -INFINITY, lsum = 0.f;  // m in units of raw (unscaled) scores

  for (int t = 0; t < nt; ++t) {
    wait_tiles<LOADS>(min(NST - 2, nt - 1 - t));
    __syncthreads();
    if (t + NST - 1 < nt) issue(t + NST - 1);
    const int k0 = t * BKV;
    if (p.causal && k0 > qw0 + 31) continue;  // all keys of the tile are ahead of this wavefront's rows
    const char* Ks = smem + (t % NST) * STAGE;
    const char* Vs = Ks + Tile::kBytes;
    f32x16 sc[2];
#pragma unroll
    for (int c = 0; c < 2; ++c) sc[c] = zero16();
#pragma unroll
    for (int kk = 0; kk < KS; ++kk)
#pragma unroll
      for (int c = 0; c < 2; ++c)
        sc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_rows(Ks, fo, 32 * c, kk), qf[kk], sc[c], 0, 0, 0);
    if ((p.causal && k0 + BKV - 1 > qw0) || k0 + BKV > len) {
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + 32 * c + acc_row(r, half);
          if (!(key < len && (!p.causal || key <= q))) sc[c][r] = -INFINITY;
        }
    }
    float mloc = -INFINITY;
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) mloc = fmaxf(mloc, sc[c][r]);
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
    const float m_new = fmaxf(m, mloc);  // finite: key 0 is allowed for every row and comes first
    const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c2);
    const float shift = -m_new * c2;
    float rs = 0.f;
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float e = __builtin_amdgcn_exp2f(fmaf(sc[c][r], c2, shift));
        sc[c][r] = e;
        rs += e;
      }
    rs += __shfl_xor(rs, 32, 64);
    lsum = lsum * alpha + rs;
    m = m_new;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f)) {  // the running maximum moved for some row
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
    }
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        const bf16x8 pf = pack_half(sc[c], tt);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_cols(Vs, fo, 32 * c + 16 * tt, dt), pf, o[dt], 0, 0, 0);
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
        if (D % 32 != 0 && col >= D) continue;  // the last column tile of a head dim like 80 is partly padding
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (bf16)(o[dt][4 * g + e] * inv);
        *reinterpret_cast<bf16x4*>(out + col) = v;
      }
    if (half == 0) p.lse[((size_t)n * p.heads + h) * p.s + q] = (m * c2 + log2f(lsum)) * kLn2;
  }
}

// Forward, software-pipelined over the key tiles: the score MFMAs of tile t+1 are issued in the same
// straight-line block as the softmax of tile t, so the matrix pipe works on the next scores while
// the VALU does this tile's exponentials (within one wavefront the two would otherwise take turns:
// the longest query tile's chain of key tiles sets the kernel's duration).  Two score registers
// sets alternate roles; tile t+1 must have landed when step t starts, hence NST >= 3 buffers and
// the loads of tile t+NST-1 issued at step t.  Arithmetic is that of attn_fwd_dma_kernel.
template <int DP, int NST, int D = DP>
__device__ __forceinline__ void attn_fwd_pipe_body(const AttnDev& p) {
  using Tile = SwTile<DP>;
  static_assert(NST >= 3, "tile t+1 is read while tile t+NST-1 is loaded");
  constexpr int BKV = 64, KS = D / 16, DT = (D + 31) / 32;  // D = head dim in memory, DP = LDS row layout
  constexpr int STAGE = 2 * Tile::kBytes, LOADS = 2 * Tile::kPerWave;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const unsigned lds0 = (unsigned)(unsigned long)((__attribute__((address_space(3))) char*)smem);
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), half = lane >> 5;
  typename Tile::Offsets fo;
  Tile::init(fo, lane);
  const int qt = gridDim.z - 1 - blockIdx.z, h = blockIdx.x, n = blockIdx.y;
  const int H = p.heads * p.d, ld3 = 3 * H;
  const bf16* base = p.qkv + (size_t)n * p.s * ld3 + h * p.d;
  const int len = seq_len(p, n);
  const int q0 = qt * 128, qw0 = q0 + 32 * wave, q = qw0 + (lane & 31);
  const int kv_end = p.causal ? min(len, q0 + 128) : len;
  const int nt = (kv_end + BKV - 1) / BKV;
  const float c2 = rsqrtf((float)p.d) * kLog2e;

  auto issue = [&](int t) {
    const unsigned st = lds0 + (unsigned)(t % NST) * STAGE;
    Tile::template issue<D>(base + H, ld3, t * BKV, p.s, st, wave, lane);
    Tile::template issue<D>(base + 2 * H, ld3, t * BKV, p.s, st + Tile::kBytes, wave, lane);
  };
#pragma unroll
  for (int t = 0; t < NST - 1; ++t)
    if (t < nt) issue(t);

  bf16x8 qf[KS];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) qf[kk] = frag_global(base + (size_t)q * ld3, q < p.s, kk, lane, p.d);
  f32x16 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) o[dt] = zero16();
  float m = -INFINITY, lsum = 0.f;  // m in units of raw (unscaled) scores

  auto scores = [&](int t, f32x16 (&sc)[2]) {
    const char* Ks = smem + (t % NST) * STAGE;
#pragma unroll
    for (int c = 0; c < 2; ++c) sc[c] = zero16();
#pragma unroll
    for (int kk = 0; kk < KS; ++kk)
#pragma unroll
      for (int c = 0; c < 2; ++c)
        sc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_rows(Ks, fo, 32 * c, kk), qf[kk], sc[c], 0, 0, 0);
  };
  // Step t: scores of tile t are in cur; those of tile t+1 (if MORE) go to nxt.  MORE is a
  // compile-time flag so that the score MFMAs and the softmax arithmetic share one basic block,
  // where the scheduling hints below spread the MFMAs between the VALU instructions.
  auto step = [&](auto more_tag, int t, f32x16 (&cur)[2], f32x16 (&nxt)[2]) {
    constexpr bool MORE = decltype(more_tag)::value;
    if (MORE) wait_tiles<LOADS>(min(NST - 3, nt - 2 - t));  // tile t+1 has landed (this wavefront's share)
    __syncthreads();  // everyone's share of it has; everyone is done with tile t-1
    if (t + NST - 1 < nt) issue(t + NST - 1);
    const int k0 = t * BKV;
    if (p.causal && k0 > qw0 + 31) return;  // this and all later tiles are ahead of this wavefront's rows
    if ((p.causal && k0 + BKV - 1 > qw0) || k0 + BKV > len) {
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + 32 * c + acc_row(r, half);
          if (!(key < len && (!p.causal || key <= q))) cur[c][r] = -INFINITY;
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    if (MORE) scores(t + 1, nxt);
    const char* Vs = smem + (t % NST) * STAGE + Tile::kBytes;
    float mloc = -INFINITY;
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) mloc = fmaxf(mloc, cur[c][r]);
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
    const float m_new = fmaxf(m, mloc);  // finite: key 0 is allowed for every row and comes first
    const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c2);
    const float shift = -m_new * c2;
    float rs = 0.f;
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float e = __builtin_amdgcn_exp2f(fmaf(cur[c][r], c2, shift));
        cur[c][r] = e;
        rs += e;
      }
    rs += __shfl_xor(rs, 32, 64);
    lsum = lsum * alpha + rs;
    m = m_new;
    __builtin_amdgcn_sched_barrier(0);
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f)) {  // the running maximum moved for some row
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
    }
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        const bf16x8 pf = pack_half(cur[c], tt);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_cols(Vs, fo, 32 * c + 16 * tt, dt), pf, o[dt], 0, 0, 0);
      }
  };
  const std::true_type more;
  const std::false_type last;

  wait_tiles<LOADS>(min(NST - 2, nt - 1));  // tile 0
  __syncthreads();
  f32x16 sa[2], sb[2];
  scores(0, sa);
  int t = 0;
  for (; t + 2 < nt; t += 2) {
    step(more, t, sa, sb);
    step(more, t + 1, sb, sa);
  }
  if (t + 1 < nt) {
    step(more, t, sa, sb);
    step(last, t + 1, sb, sa);
  } else {
    step(last, t, sa, sb);
  }
  if (q < p.s) {
    const float inv = 1.f / lsum;
    bf16* out = p.ctx + ((size_t)n * p.s + q) * H + h * p.d;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = 32 * dt + 8 * g + 4 * half;
        if (D % 32 != 0 && col >= D) continue;  // the last column tile of a head dim like 80 is partly padding
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (bf16)(o[dt][4 * g + e] * inv);
        *reinterpret_cast<bf16x4*>(out + col) = v;
      }
    if (half == 0) p.lse[((size_t)n * p.heads + h) * p.s + q] = (m * c2 + log2f(lsum)) * kLn2;
  }
}

// Head dim 64: capped at 256 registers so that two workgroups share a CU.  Head dim 128: the output
// accumulators and two score sets need more, one workgroup per CU.
template <int DP, int NST>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_fwd_pipe_kernel(AttnDev p) {
  attn_fwd_pipe_body<DP, NST>(p);
}
template <int DP, int NST, int D = DP>
__global__ __launch_bounds__(256) void attn_fwd_pipe_wide_kernel(AttnDev p) {
  attn_fwd_pipe_body<DP, NST, D>(p);
}

template <int DP, int NST, int D = DP>
__device__ __forceinline__ void attn_bwd_dkv_dma_body(const AttnDev& p) {
  using Tile = SwTile<DP>;
  constexpr int BQ = 64, KS = D / 16, DT = (D + 31) / 32;  // D = head dim in memory, DP = LDS row layout
  constexpr int STAGE = 2 * Tile::kBytes + 512;  // Q tile, dC tile, 64 lse, 64 delta
  constexpr int LOADS = 2 * Tile::kPerWave + 1;  // every wavefront also issues one 4-byte-per-lane load
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const unsigned lds0 = (unsigned)(unsigned long)((__attribute__((address_space(3))) char*)smem);
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), half = lane >> 5;
  typename Tile::Offsets fo;
  Tile::init(fo, lane);
  const int kt = blockIdx.z, h = blockIdx.x, n = blockIdx.y;
  const int H = p.heads * p.d, ld3 = 3 * H;
  const bf16* base = p.qkv + (size_t)n * p.s * ld3 + h * p.d;
  const bf16* dcb = p.dctx + (size_t)n * p.s * H + h * p.d;
  const size_t stat0 = ((size_t)n * p.heads + h) * p.s;
  const int len = seq_len(p, n);
  const int k0 = kt * 128, kw0 = k0 + 32 * wave, key = kw0 + (lane & 31);
  const float scale = rsqrtf((float)p.d), c2 = scale * kLog2e;

  const int q_begin = (p.causal && k0 < len) ? (k0 / BQ) * BQ : 0;
  const int q_end = k0 < len ? p.s : 0;  // a tile of masked keys gets zero gradients
  const int nt = q_end > q_begin ? (q_end - q_begin + BQ - 1) / BQ : 0;

  auto issue = [&](int t) {
    const unsigned st = lds0 + (unsigned)(t % NST) * STAGE;
    const int q0 = q_begin + t * BQ;
    Tile::template issue<D>(base, ld3, q0, p.s, st, wave, lane);
    Tile::template issue<D>(dcb, H, q0, p.s, st + Tile::kBytes, wave, lane);
    // wavefronts 0 / 1 fetch the 64 log-sum-exp / delta values; 2 / 3 repeat them (same data, keeps
    // every wavefront's load count equal)
    const int qq = min(q0 + lane, p.s - 1);
    const float* src = (wave & 1) ? p.delta + stat0 : p.lse + stat0;
    dma4(src, (unsigned)(qq * 4), st + 2 * Tile::kBytes + (wave & 1) * 256);
  };
#pragma unroll
  for (int t = 0; t < NST - 1; ++t)
    if (t < nt) issue(t);

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
  for (int t = 0; t < nt; ++t) {
    wait_tiles<LOADS>(min(NST - 2, nt - 1 - t));
    __syncthreads();
    if (t + NST - 1 < nt) issue(t + NST - 1);
    const int q0 = q_begin + t * BQ;
    const char* Qs = smem + (t % NST) * STAGE;
    const char* Cs = Qs + Tile::kBytes;
    const float* lse_s = reinterpret_cast<const float*>(Cs + Tile::kBytes);
    const float* dlt_s = lse_s + 64;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      if (p.causal && q0 + 32 * c + 31 < kw0) continue;  // all these queries precede the wavefront's keys
      f32x16 sacc = zero16(), dp = zero16();
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_rows(Qs, fo, 32 * c, kk), kf[kk], sacc, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_rows(Cs, fo, 32 * c, kk), vf[kk], dp, 0, 0, 0);
      }
      // P = 2^(c2 s - lse log2e), dS = P (dP - delta); lse and delta of this lane's 16 queries come as 4-vectors
      const bool need_mask = (p.causal && q0 + 32 * c < kw0 + 31) || kw0 + 31 >= len || q0 + 32 * c + 31 >= p.s;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int ql = 32 * c + 8 * g + 4 * half;
        const f32x4 l4 = *reinterpret_cast<const f32x4*>(lse_s + ql);
        const f32x4 d4 = *reinterpret_cast<const f32x4*>(dlt_s + ql);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = 4 * g + e;
          float pr = __builtin_amdgcn_exp2f(fmaf(sacc[r], c2, -l4[e] * kLog2e));
          if (need_mask) {
            const int qq = q0 + ql + e;
            if (!(qq < p.s && key < len && (!p.causal || key <= qq))) pr = 0.f;
          }
          sacc[r] = pr;
          dp[r] = pr * (dp[r] - d4[e]);
        }
      }
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        const bf16x8 pf = pack_half(sacc, tt), dsf = pack_half(dp, tt);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_cols(Cs, fo, 32 * c + 16 * tt, dt), pf, dv[dt], 0, 0, 0);
          dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_cols(Qs, fo, 32 * c + 16 * tt, dt), dsf, dk[dt], 0, 0, 0);
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
        if (D % 32 != 0 && col >= D) continue;
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

template <int DP, int NST, int D = DP>
__global__ __launch_bounds__(256) void attn_bwd_dkv_dma_kernel(AttnDev p) {
  attn_bwd_dkv_dma_body<DP, NST, D>(p);
}
// The same under a cap of 256 registers, so that two workgroups share a CU.
template <int DP, int NST, int D = DP>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_bwd_dkv_dma2_kernel(AttnDev p) {
  attn_bwd_dkv_dma_body<DP, NST, D>(p);
}

template <int DP, int NST, int D = DP>
__device__ __forceinline__ void attn_bwd_dq_dma_body(const AttnDev& p) {
  using Tile = SwTile<DP>;
  constexpr int BKV = 64, KS = D / 16, DT = (D + 31) / 32;  // D = head dim in memory, DP = LDS row layout
  constexpr int STAGE = 2 * Tile::kBytes, LOADS = 2 * Tile::kPerWave;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const unsigned lds0 = (unsigned)(unsigned long)((__attribute__((address_space(3))) char*)smem);
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), half = lane >> 5;
  typename Tile::Offsets fo;
  Tile::init(fo, lane);
  const int qt = gridDim.z - 1 - blockIdx.z, h = blockIdx.x, n = blockIdx.y;
  const int H = p.heads * p.d, ld3 = 3 * H;
  const bf16* base = p.qkv + (size_t)n * p.s * ld3 + h * p.d;
  const int len = seq_len(p, n);
  const int q0 = qt * 128, qw0 = q0 + 32 * wave, q = qw0 + (lane & 31);
  const int kv_end = p.causal ? min(len, q0 + 128) : len;
  const int nt = (kv_end + BKV - 1) / BKV;
  const float scale = rsqrtf((float)p.d), c2 = scale * kLog2e;

  auto issue = [&](int t) {
    const unsigned st = lds0 + (unsigned)(t % NST) * STAGE;
    Tile::template issue<D>(base + H, ld3, t * BKV, p.s, st, wave, lane);
    Tile::template issue<D>(base + 2 * H, ld3, t * BKV, p.s, st + Tile::kBytes, wave, lane);
  };
#pragma unroll
  for (int t = 0; t < NST - 1; ++t)
    if (t < nt) issue(t);

  const size_t stat = ((size_t)n * p.heads + h) * p.s + q;
  const float my_lse2 = q < p.s ? p.lse[stat] * kLog2e : 0.f;
  bf16x8 qf[KS], cf[KS];
  // delta = rowsum(dC * C) of this lane's query row: each half wavefront holds half of the row's
  // columns.  Written out for the dK/dV kernel, which runs after this one.
  float my_delta = 0.f;
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) {
    qf[kk] = frag_global(base + (size_t)q * ld3, q < p.s, kk, lane, p.d);
    cf[kk] = frag_global(p.dctx + ((size_t)n * p.s + q) * H + h * p.d, q < p.s, kk, lane, p.d);
    const bf16x8 of = frag_global(p.ctx + ((size_t)n * p.s + q) * H + h * p.d, q < p.s, kk, lane, p.d);
#pragma unroll
    for (int e = 0; e < 8; ++e) my_delta += (float)cf[kk][e] * (float)of[e];
  }
  my_delta += __shfl_xor(my_delta, 32, 64);
  if (q < p.s && half == 0) p.delta[stat] = my_delta;
  f32x16 dq[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) dq[dt] = zero16();

  for (int t = 0; t < nt; ++t) {
    wait_tiles<LOADS>(min(NST - 2, nt - 1 - t));
    __syncthreads();
    if (t + NST - 1 < nt) issue(t + NST - 1);
    const int k0 = t * BKV;
    if (p.causal && k0 > qw0 + 31) continue;
    const char* Ks = smem + (t % NST) * STAGE;
    const char* Vs = Ks + Tile::kBytes;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      f32x16 sacc = zero16(), dp = zero16();
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_rows(Ks, fo, 32 * c, kk), qf[kk], sacc, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_rows(Vs, fo, 32 * c, kk), cf[kk], dp, 0, 0, 0);
      }
      const bool need_mask = (p.causal && k0 + 32 * c + 31 > qw0) || k0 + 32 * c + 32 > len;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float pr = __builtin_amdgcn_exp2f(fmaf(sacc[r], c2, -my_lse2));
        if (need_mask) {
          const int key = k0 + 32 * c + acc_row(r, half);
          if (!(key < len && (!p.causal || key <= q))) pr = 0.f;
        }
        dp[r] = pr * (dp[r] - my_delta);
      }
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        const bf16x8 dsf = pack_half(dp, tt);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
          dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_cols(Ks, fo, 32 * c + 16 * tt, dt), dsf, dq[dt], 0, 0, 0);
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
        if (D % 32 != 0 && col >= D) continue;
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (bf16)(dq[dt][4 * g + e] * scale);
        *reinterpret_cast<bf16x4*>(out + col) = v;
      }
  }
}

template <int DP, int NST, int D = DP>
__global__ __launch_bounds__(256) void attn_bwd_dq_dma_kernel(AttnDev p) {
  attn_bwd_dq_dma_body<DP, NST, D>(p);
}
template <int DP, int NST, int D = DP>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_bwd_dq_dma2_kernel(AttnDev p) {
  attn_bwd_dq_dma_body<DP, NST, D>(p);
}

// dK / dV, software-pipelined in half tiles of 32 queries like attn_bwd_dq_pipe_kernel: the score
// MFMAs of the next half tile (and this half's dP MFMAs) share a block with the exponentials, dS and
// the dV / dK MFMAs of this one.  Arithmetic is that of attn_bwd_dkv_dma_kernel.
template <int DP, int NST>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_bwd_dkv_pipe_kernel(AttnDev p) {
  using Tile = SwTile<DP>;
  static_assert(NST >= 3, "tile t+1 is read while tile t+NST-1 is loaded");
  constexpr int BQ = 64, KS = DP / 16, DT = DP / 32;
  constexpr int STAGE = 2 * Tile::kBytes + 512;  // Q tile, dC tile, 64 lse, 64 delta
  constexpr int LOADS = 2 * Tile::kPerWave + 1;  // every wavefront also issues one 4-byte-per-lane load
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const unsigned lds0 = (unsigned)(unsigned long)((__attribute__((address_space(3))) char*)smem);
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), half = lane >> 5;
  typename Tile::Offsets fo;
  Tile::init(fo, lane);
  const int kt = blockIdx.z, h = blockIdx.x, n = blockIdx.y;
  const int H = p.heads * p.d, ld3 = 3 * H;
  const bf16* base = p.qkv + (size_t)n * p.s * ld3 + h * p.d;
  const bf16* dcb = p.dctx + (size_t)n * p.s * H + h * p.d;
  const size_t stat0 = ((size_t)n * p.heads + h) * p.s;
  const int len = seq_len(p, n);
  const int k0 = kt * 128, kw0 = k0 + 32 * wave, key = kw0 + (lane & 31);
  const float scale = rsqrtf((float)p.d), c2 = scale * kLog2e;

  const int q_begin = (p.causal && k0 < len) ? (k0 / BQ) * BQ : 0;
  const int q_end = k0 < len ? p.s : 0;  // a tile of masked keys gets zero gradients
  const int nt = q_end > q_begin ? (q_end - q_begin + BQ - 1) / BQ : 0;

  auto issue = [&](int t) {
    const unsigned st = lds0 + (unsigned)(t % NST) * STAGE;
    const int q0 = q_begin + t * BQ;
    Tile::issue(base, ld3, q0, p.s, st, wave, lane);
    Tile::issue(dcb, H, q0, p.s, st + Tile::kBytes, wave, lane);
    // wavefronts 0 / 1 fetch the 64 log-sum-exp / delta values; 2 / 3 repeat them (same data, keeps
    // every wavefront's load count equal)
    const int qq = min(q0 + lane, p.s - 1);
    const float* src = (wave & 1) ? p.delta + stat0 : p.lse + stat0;
    dma4(src, (unsigned)(qq * 4), st + 2 * Tile::kBytes + (wave & 1) * 256);
  };
#pragma unroll
  for (int t = 0; t < NST - 1; ++t)
    if (t < nt) issue(t);

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
  if (nt == 0) goto store;  // uniform over the workgroup
  {
    // S of the 32 queries of half c of tile t
    auto scores = [&](int t, int c, f32x16& sc) {
      const char* Qs = smem + (t % NST) * STAGE;
      sc = zero16();
#pragma unroll
      for (int kk = 0; kk < KS; ++kk)
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_rows(Qs, fo, 32 * c, kk), kf[kk], sc, 0, 0, 0);
    };
    // The scores of half c of tile t are in sc; NEXT: those of the following half (tn, cn) go to sc_n.
    // dP of this half is formed here as well: its MFMAs and the next scores' run under the exponentials.
    auto half_step = [&](auto next_tag, int t, int c, f32x16& sc, int tn, int cn, f32x16& sc_n) {
      constexpr bool NEXT = decltype(next_tag)::value;
      const int q0 = q_begin + t * BQ + 32 * c;
      const bool active = !(p.causal && q0 + 31 < kw0);  // else all these queries precede the wavefront's keys
      if (active && ((p.causal && q0 < kw0 + 31) || kw0 + 31 >= len || q0 + 31 >= p.s)) {  // masked scores give P = 0
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int qq = q0 + acc_row(r, half);
          if (!(qq < p.s && key < len && (!p.causal || key <= qq))) sc[r] = -INFINITY;
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      if (!active) {  // only keep the pipeline going
        if (NEXT) scores(tn, cn, sc_n);
        return;
      }
      const char* Qs = smem + (t % NST) * STAGE;
      const char* Cs = Qs + Tile::kBytes;
      const float* lse_s = reinterpret_cast<const float*>(Cs + Tile::kBytes);
      const float* dlt_s = lse_s + 64;
      f32x16 dp = zero16();
#pragma unroll
      for (int kk = 0; kk < KS; ++kk)
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_rows(Cs, fo, 32 * c, kk), vf[kk], dp, 0, 0, 0);
      if (NEXT) scores(tn, cn, sc_n);
      // P = 2^(c2 s - lse log2e), dS = P (dP - delta); lse and delta of this lane's 16 queries come as 4-vectors
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int ql = 32 * c + 8 * g + 4 * half;
        const f32x4 l4 = *reinterpret_cast<const f32x4*>(lse_s + ql);
        const f32x4 d4 = *reinterpret_cast<const f32x4*>(dlt_s + ql);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = 4 * g + e;
          const float pr = __builtin_amdgcn_exp2f(fmaf(sc[r], c2, -l4[e] * kLog2e));
          sc[r] = pr;
          dp[r] = pr * (dp[r] - d4[e]);
        }
      }
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        const bf16x8 pf = pack_half(sc, tt), dsf = pack_half(dp, tt);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_cols(Cs, fo, 32 * c + 16 * tt, dt), pf, dv[dt], 0, 0, 0);
          dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_cols(Qs, fo, 32 * c + 16 * tt, dt), dsf, dk[dt], 0, 0, 0);
        }
      }
    };
    const std::true_type next;
    const std::false_type none;

    wait_tiles<LOADS>(min(NST - 2, nt - 1));  // tile 0
    __syncthreads();
    f32x16 sa, sb;
    scores(0, 0, sa);
    for (int t = 0; t < nt; ++t) {
      half_step(next, t, 0, sa, t, 1, sb);
      if (t + 1 < nt) {
        wait_tiles<LOADS>(min(NST - 3, nt - 2 - t));  // tile t+1 has landed (this wavefront's share)
        __syncthreads();                              // everyone's share has; everyone is done with tile t-1
        if (t + NST - 1 < nt) issue(t + NST - 1);
        half_step(next, t, 1, sb, t + 1, 0, sa);
      } else {
        half_step(none, t, 1, sb, 0, 0, sa);
      }
    }
  }
store:
  if (key < p.s) {
    bf16* out = p.dqkv + ((size_t)n * p.s + key) * ld3 + h * p.d;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = 32 * dt + 8 * g + 4 * half;
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

// dQ, software-pipelined in half tiles of 32 keys: the S and dP MFMAs of the next half tile are
// issued in the block that does the exponentials, dS and the dQ MFMAs of this one.  Also forms
// delta = rowsum(dC * C) for its rows and stores it (the dK/dV kernel is launched after this one).  Two register
// sets alternate; the barrier that admits tile t+1 sits between the two halves of tile t.
// Arithmetic is that of attn_bwd_dq_dma_kernel.
template <int DP, int NST>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_bwd_dq_pipe_kernel(AttnDev p) {
  using Tile = SwTile<DP>;
  static_assert(NST >= 3, "tile t+1 is read while tile t+NST-1 is loaded");
  constexpr int BKV = 64, KS = DP / 16, DT = DP / 32;
  constexpr int STAGE = 2 * Tile::kBytes, LOADS = 2 * Tile::kPerWave;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const unsigned lds0 = (unsigned)(unsigned long)((__attribute__((address_space(3))) char*)smem);
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), half = lane >> 5;
  typename Tile::Offsets fo;
  Tile::init(fo, lane);
  const int qt = gridDim.z - 1 - blockIdx.z, h = blockIdx.x, n = blockIdx.y;
  const int H = p.heads * p.d, ld3 = 3 * H;
  const bf16* base = p.qkv + (size_t)n * p.s * ld3 + h * p.d;
  const int len = seq_len(p, n);
  const int q0 = qt * 128, qw0 = q0 + 32 * wave, q = qw0 + (lane & 31);
  const int kv_end = p.causal ? min(len, q0 + 128) : len;
  const int nt = (kv_end + BKV - 1) / BKV;
  const float scale = rsqrtf((float)p.d), c2 = scale * kLog2e;

  auto issue = [&](int t) {
    const unsigned st = lds0 + (unsigned)(t % NST) * STAGE;
    Tile::issue(base + H, ld3, t * BKV, p.s, st, wave, lane);
    Tile::issue(base + 2 * H, ld3, t * BKV, p.s, st + Tile::kBytes, wave, lane);
  };
#pragma unroll
  for (int t = 0; t < NST - 1; ++t)
    if (t < nt) issue(t);

  const size_t stat = ((size_t)n * p.heads + h) * p.s + q;
  const float my_lse2 = q < p.s ? p.lse[stat] * kLog2e : 0.f;
  bf16x8 qf[KS], cf[KS];
  // delta = rowsum(dC * C) of this lane's query row: each half wavefront holds half of the row's
  // columns.  Written out for the dK/dV kernel, which runs after this one.
  float my_delta = 0.f;
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) {
    qf[kk] = frag_global(base + (size_t)q * ld3, q < p.s, kk, lane, p.d);
    cf[kk] = frag_global(p.dctx + ((size_t)n * p.s + q) * H + h * p.d, q < p.s, kk, lane, p.d);
    const bf16x8 of = frag_global(p.ctx + ((size_t)n * p.s + q) * H + h * p.d, q < p.s, kk, lane, p.d);
#pragma unroll
    for (int e = 0; e < 8; ++e) my_delta += (float)cf[kk][e] * (float)of[e];
  }
  my_delta += __shfl_xor(my_delta, 32, 64);
  if (q < p.s && half == 0) p.delta[stat] = my_delta;
  f32x16 dq[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) dq[dt] = zero16();

  // S (sc) and dP (dp) of the 32 keys of half c of tile t
  auto products = [&](int t, int c, f32x16& sc, f32x16& dp) {
    const char* Ks = smem + (t % NST) * STAGE;
    const char* Vs = Ks + Tile::kBytes;
    sc = zero16();
    dp = zero16();
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_rows(Ks, fo, 32 * c, kk), qf[kk], sc, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_rows(Vs, fo, 32 * c, kk), cf[kk], dp, 0, 0, 0);
    }
  };
  // Half c of tile t is in (sc, dp); NEXT: the following half (tn, cn) goes to (sc_n, dp_n).
  auto half_step = [&](auto next_tag, int t, int c, f32x16& sc, f32x16& dp, int tn, int cn, f32x16& sc_n, f32x16& dp_n) {
    constexpr bool NEXT = decltype(next_tag)::value;
    const int k0 = t * BKV + 32 * c;
    if ((p.causal && k0 + 31 > qw0) || k0 + 32 > len) {  // masked scores give P = 0
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = k0 + acc_row(r, half);
        if (!(key < len && (!p.causal || key <= q))) sc[r] = -INFINITY;
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    if (NEXT) products(tn, cn, sc_n, dp_n);
    const char* Ks = smem + (t % NST) * STAGE;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float pr = __builtin_amdgcn_exp2f(fmaf(sc[r], c2, -my_lse2));
      dp[r] = pr * (dp[r] - my_delta);
    }
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const bf16x8 dsf = pack_half(dp, tt);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
        dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_cols(Ks, fo, 32 * c + 16 * tt, dt), dsf, dq[dt], 0, 0, 0);
    }
  };
  const std::true_type next;
  const std::false_type none;

  wait_tiles<LOADS>(min(NST - 2, nt - 1));  // tile 0
  __syncthreads();
  f32x16 sa, da, sb, db;
  products(0, 0, sa, da);
  for (int t = 0; t < nt; ++t) {
    const bool active = !(p.causal && t * BKV > qw0 + 31);  // false from some tile on: keys ahead of all rows
    if (active) half_step(next, t, 0, sa, da, t, 1, sb, db);
    if (t + 1 < nt) {
      wait_tiles<LOADS>(min(NST - 3, nt - 2 - t));  // tile t+1 has landed (this wavefront's share)
      __syncthreads();                              // everyone's share has; everyone is done with tile t-1
      if (t + NST - 1 < nt) issue(t + NST - 1);
      if (active) half_step(next, t, 1, sb, db, t + 1, 0, sa, da);
    } else if (active) {
      half_step(none, t, 1, sb, db, 0, 0, sa, da);
    }
  }
  if (q < p.s) {
    bf16* out = p.dqkv + ((size_t)n * p.s + q) * ld3 + h * p.d;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = 32 * dt + 8 * g + 4 * half;
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (bf16)(dq[dt][4 * g + e] * scale);
        *reinterpret_cast<bf16x4*>(out + col) = v;
      }
  }
}

template <typename K>
int raise_lds(K kern, size_t lds) {
  if (lds <= 64 * 1024) return HANAYO_OK;
  const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return set_error(HANAYO_EHIP, "attention: cannot raise LDS limit: %s", hipGetErrorString(e));
  return HANAYO_OK;
}

// 32-bit lane offsets: the largest byte offset inside one sequence's rows must stay below 2^31
bool dma_ok(const AttnArgs& a) {
  return (a.d == 64 || a.d == 80 || a.d == 96 || a.d == 128) && (long)a.s * 3 * a.heads * a.d * 2 < (1L << 31);
}

AttnDev to_dev(const AttnArgs& a) {
  AttnDev p;
  p.qkv = (const bf16*)a.qkv; p.valid_len = a.valid_len; p.ctx = (bf16*)a.ctx; p.lse = a.lse;
  p.dctx = (const bf16*)a.dctx; p.dqkv = (bf16*)a.dqkv; p.delta = a.delta;
  p.s = a.s; p.heads = a.heads; p.d = a.d; p.causal = a.causal ? 1 : 0;
  return p;
}

}  // namespace

// Grid = (head, sequence, 128-row tile).  Workgroup ids run head-fastest and the dispatcher deals them to
// the 8 XCDs in turn, so with a multiple of 8 (sequence, head) pairs every tile of a pair lands on one
// XCD and K and V are fetched into one L2 only; the tile index is slowest and the kernels count it from
// the causal mask's heavy end, so the long tiles start first and the short ones fill in behind them.
bool attn_mfma_supported(const AttnArgs& a) { return a.d % 8 == 0 && a.d >= 8 && a.d <= 128 && a.b <= 65535; }

int attn_forward_mfma(const AttnArgs& a, hipStream_t stream) {
  if (!attn_mfma_supported(a)) return set_error(HANAYO_EUNSUPPORTED, "attn_mfma: head dim %d", a.d);
  const AttnDev p = to_dev(a);
  const dim3 grid(a.heads, a.b, (a.s + 127) / 128), block(256);
  if (dma_ok(a)) {
    if (a.d == 64) {
      constexpr size_t lds = 4 * 2 * SwTile<64>::kBytes;
      hipLaunchKernelGGL((attn_fwd_pipe_kernel<64, 4>), grid, block, lds, stream, p);
    } else if (a.d == 80) {
      // one tile at a time, two stages, in the 128-wide LDS rows partly filled: 231 registers and 64 KiB, so two
      // workgroups share a CU.  (The pipelined body is no faster here alone, 39.2 against 39.8 us at s = 1024,
      // 64 (sequence, head) pairs, and with its 128 KiB and one workgroup per CU it leaves less room for the
      // kernels of the executor's other lanes: 573.5 against 570.6 ms per step of the eight-chunk workload.)
      constexpr size_t lds = 2 * 2 * SwTile<128>::kBytes;
      hipLaunchKernelGGL((attn_fwd_dma_kernel<128, 2, 80>), grid, block, lds, stream, p);
    } else {  // the pipelined body without the register cap (one workgroup per CU), four stages of K and V
              // (128 KiB); head dim 96 in the 128-wide LDS rows, partly filled
      constexpr size_t lds = 4 * 2 * SwTile<128>::kBytes;
#define LAUNCH_FWD(...)                                                                        \
  do {                                                                                         \
    const int rc = raise_lds(attn_fwd_pipe_wide_kernel<__VA_ARGS__>, lds);                     \
    if (rc) return rc;                                                                         \
    hipLaunchKernelGGL((attn_fwd_pipe_wide_kernel<__VA_ARGS__>), grid, block, lds, stream, p); \
  } while (0)
      if (a.d == 128) LAUNCH_FWD(128, 4);
      else LAUNCH_FWD(128, 4, 96);
#undef LAUNCH_FWD
    }
    return check_launch("attn_fwd_dma");
  }
  if (a.d <= 64) hipLaunchKernelGGL((attn_fwd_kernel<64>), grid, block, 0, stream, p);
  else if (a.d <= 96) hipLaunchKernelGGL((attn_fwd_kernel<96>), grid, block, 0, stream, p);
  else hipLaunchKernelGGL((attn_fwd_kernel<128>), grid, block, 0, stream, p);
  return check_launch("attn_fwd_mfma");
}

int attn_backward_mfma(const AttnArgs& a, hipStream_t stream) {
  if (!attn_mfma_supported(a)) return set_error(HANAYO_EUNSUPPORTED, "attn_mfma: head dim %d", a.d);
  int rc;
  const AttnDev p = to_dev(a);
  const dim3 grid(a.heads, a.b, (a.s + 127) / 128), block(256);
  if (dma_ok(a) && a.d == 64) {  // the dQ kernel forms delta itself and goes first
    constexpr size_t lds_dkv = 4 * (2 * SwTile<64>::kBytes + 512);
    rc = raise_lds(attn_bwd_dkv_pipe_kernel<64, 4>, lds_dkv);
    if (rc) return rc;
    hipLaunchKernelGGL((attn_bwd_dq_pipe_kernel<64, 4>), grid, block, 4 * 2 * SwTile<64>::kBytes, stream, p);
    hipLaunchKernelGGL((attn_bwd_dkv_pipe_kernel<64, 4>), grid, block, lds_dkv, stream, p);
    return check_launch("attn_bwd_pipe");
  }
  if (dma_ok(a)) {  // likewise: dQ first (it writes delta), then dK/dV
    {
      constexpr size_t lds_dkv = 2 * (2 * SwTile<128>::kBytes + 512), lds_dq = 2 * 2 * SwTile<128>::kBytes;
#define LAUNCH_BWD(...)                                                                              \
  do {                                                                                               \
    rc = raise_lds(attn_bwd_dkv_dma_kernel<__VA_ARGS__>, lds_dkv);                                   \
    if (rc) return rc;                                                                               \
    hipLaunchKernelGGL((attn_bwd_dq_dma_kernel<__VA_ARGS__>), grid, block, lds_dq, stream, p);       \
    hipLaunchKernelGGL((attn_bwd_dkv_dma_kernel<__VA_ARGS__>), grid, block, lds_dkv, stream, p);     \
  } while (0)
      // Head dims 80 and 96 fit 256 registers (218 - 255, nothing spilled), so two workgroups share a CU: 118 -> 103 us
      // at d = 80, s = 1024, 64 (sequence, head) pairs.  Head dim 128 does not (72 - 92 bytes of scratch per lane and
      // 230 -> 315 us under the cap) and runs one workgroup per CU.
#define LAUNCH_BWD2(...)                                                                             \
  do {                                                                                               \
    rc = raise_lds(attn_bwd_dkv_dma2_kernel<__VA_ARGS__>, lds_dkv);                                  \
    if (rc) return rc;                                                                               \
    hipLaunchKernelGGL((attn_bwd_dq_dma2_kernel<__VA_ARGS__>), grid, block, lds_dq, stream, p);      \
    hipLaunchKernelGGL((attn_bwd_dkv_dma2_kernel<__VA_ARGS__>), grid, block, lds_dkv, stream, p);    \
  } while (0)
      if (a.d == 128) LAUNCH_BWD(128, 2);
      else if (a.d == 96) LAUNCH_BWD2(128, 2, 96);
      else LAUNCH_BWD2(128, 2, 80);
#undef LAUNCH_BWD
#undef LAUNCH_BWD2
    }
    return check_launch("attn_bwd_dma");
  }
  rc = attn_delta(HANAYO_BF16, a, stream);
  if (rc) return rc;
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
