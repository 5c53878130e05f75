// bf16 GEMM on the gfx950 matrix cores: v_mfma_f32_32x32x16_bf16, fp32
// accumulation, LDS-staged tiles, double-buffered LDS with register prefetch.
//
// Work split: a 256-thread workgroup (4 wavefronts, 2 x 2) owns a BM x BN tile
// of C; each wavefront owns (BM/2) x (BN/2) as a grid of 32 x 32 MFMA tiles.
// Operand tiles are copied to LDS in the orientation they have in memory (16-byte
// global loads, 16-byte LDS writes).  An operand whose contraction index is
// contiguous in memory is read back with one 16-byte LDS read per fragment; one
// whose contraction index is strided is read with the LDS transpose read
// (ds_read_b64_tr_b16), which hands every lane four consecutive contraction
// elements of its own row/column without a transposing pass.
//
// The MFMA is issued with the operands swapped (B fragment first), so a lane's
// accumulator registers hold 4 consecutive columns of one row of C and the
// epilogue moves 8-byte (bf16) or 16-byte (fp32) vectors.
#include <type_traits>

#include "device_util.h"
#include "epilogue.h"
#include "kernels.h"

namespace hanayo {
namespace k {

namespace {

typedef __attribute__((ext_vector_type(4))) short s16x4;

struct GemmDev {
  const bf16* A;
  const bf16* B;
  bf16* C;
  float* Cf;
  const bf16* bias;
  const bf16* aux;
  bf16* aux_out;
  int M, N, K;
  int lda, ldb, ldc;
  int k_per_split;  // multiple of BK
  int atomic;       // EPI_ACCUM_F32 with more than one K split
};

constexpr int kPadK = 8;   // elements; K-contiguous tiles: pitch = (BK + 8) * 2 bytes
constexpr int kPadT = 32;  // elements; transposed-read tiles: pitch = 64 bytes mod 256

// Tile of ROWS x COLS elements (COLS contiguous in memory), moved by 256 threads as
// 8-element vectors.  Vectors that start outside [row_lim) x [col_lim) read as zero.
template <int ROWS, int COLS>
struct TileMover {
  static constexpr int kVecPerRow = COLS / 8;
  static constexpr int kVecs = ROWS * kVecPerRow;
  static constexpr int kPerThread = kVecs / 256;
  static_assert(kVecs % 256 == 0, "tile must split evenly over 256 threads");

  template <bool EVEN>
  __device__ static void load(const bf16* __restrict__ g, int ld, int row0, int col0, int row_lim, int col_lim,
                              bf16x8 (&r)[kPerThread]) {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const int v = threadIdx.x + i * 256;
      const int row = row0 + v / kVecPerRow, col = col0 + (v % kVecPerRow) * 8;
      if constexpr (EVEN) {
        r[i] = *reinterpret_cast<const bf16x8*>(g + (size_t)row * ld + col);
      } else {
        bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
        r[i] = (row < row_lim && col < col_lim) ? *reinterpret_cast<const bf16x8*>(g + (size_t)row * ld + col) : z;
      }
    }
  }
  template <int PITCH>
  __device__ static void store(bf16* lds, const bf16x8 (&r)[kPerThread]) {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const int v = threadIdx.x + i * 256;
      *reinterpret_cast<bf16x8*>(lds + (v / kVecPerRow) * PITCH + (v % kVecPerRow) * 8) = r[i];
    }
  }
};

// Fragment for the 32-row (or 32-column) MFMA tile starting at `r0`, contraction
// step `kk` (16 elements), from a K-contiguous LDS tile [rows][PITCH].
template <int PITCH>
__device__ __forceinline__ bf16x8 frag_kcontig(const bf16* lds, int r0, int kk, int lane) {
  return *reinterpret_cast<const bf16x8*>(lds + (r0 + (lane & 31)) * PITCH + kk * 16 + 8 * (lane >> 5));
}

// Same fragment from a tile stored [k][PITCH] (rows/columns contiguous): two
// transpose reads, each returning 4 consecutive k for this lane's row.
template <int PITCH>
__device__ __forceinline__ bf16x8 frag_transposed(const bf16* lds, int r0, int kk, int lane) {
  const int krow = kk * 16 + 8 * (lane >> 5) + ((lane & 15) >> 2);
  const int col = r0 + 16 * ((lane >> 4) & 1) + (lane & 3) * 4;
  typedef __attribute__((address_space(3))) s16x4* lds_ptr;
  const bf16* p0 = lds + krow * PITCH + col;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p0));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p0 + 4 * PITCH));
  union {
    struct { s16x4 lo, hi; } s;
    bf16x8 v;
  } u;
  u.s.lo = lo;
  u.s.hi = hi;
  return u.v;
}

// EVEN: M, N and the K range are whole multiples of the tile, so no load or store is guarded.
template <int BM, int BN, int BK, bool A_T, bool B_T, int EPI, bool EVEN>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmDev p) {
  constexpr int WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32;
  constexpr int PA = A_T ? BM + kPadT : BK + kPadK;  // LDS pitch (elements) of the A tile
  constexpr int PB = B_T ? BN + kPadT : BK + kPadK;
  constexpr int A_ROWS = A_T ? BK : BM, A_COLS = A_T ? BM : BK;
  constexpr int B_ROWS = B_T ? BK : BN, B_COLS = B_T ? BN : BK;
  constexpr int A_ELEMS = A_ROWS * PA, B_ELEMS = B_ROWS * PB;
  using MoveA = TileMover<A_ROWS, A_COLS>;
  using MoveB = TileMover<B_ROWS, B_COLS>;

  extern __shared__ __attribute__((aligned(16))) char smem[];
  bf16* lds = reinterpret_cast<bf16*>(smem);  // [2][A_ELEMS + B_ELEMS]

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int k_begin = blockIdx.z * p.k_per_split;
  const int k_end = min(p.K, k_begin + p.k_per_split);
  const int nk = (k_end - k_begin + BK - 1) / BK;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  bf16x8 ra[MoveA::kPerThread], rb[MoveB::kPerThread];
  auto fetch = [&](int kt) {
    const int k0 = k_begin + kt * BK;
    if (A_T) MoveA::template load<EVEN>(p.A, p.lda, k0, m0, k_end, p.M, ra);
    else MoveA::template load<EVEN>(p.A, p.lda, m0, k0, p.M, k_end, ra);
    if (B_T) MoveB::template load<EVEN>(p.B, p.ldb, k0, n0, k_end, p.N, rb);
    else MoveB::template load<EVEN>(p.B, p.ldb, n0, k0, p.N, k_end, rb);
  };
  auto stage = [&](int buf) {
    bf16* a = lds + buf * (A_ELEMS + B_ELEMS);
    MoveA::template store<PA>(a, ra);
    MoveB::template store<PB>(a + A_ELEMS, rb);
  };

  if (nk > 0) {
    fetch(0);
    stage(0);
  }
  __syncthreads();
  // One K tile: prefetch the next tile into registers, run the MFMAs of this one from LDS,
  // park the prefetched tile in the other LDS buffer.  `more` is a compile-time flag so that the
  // last tile carries no branch inside the scheduled region.
  auto k_tile = [&](int kt, auto more) {
    constexpr bool kMore = decltype(more)::value;
    const bf16* a_lds = lds + (kt & 1) * (A_ELEMS + B_ELEMS);
    const bf16* b_lds = a_lds + A_ELEMS;
    if constexpr (kMore) fetch(kt + 1);
    // fragments of step kk+1 are requested from LDS before the MFMAs of step kk are issued
    bf16x8 fa[2][TM], fb[2][TN];
    auto read_frags = [&](int kk, int slot) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[slot][i] = A_T ? frag_transposed<PA>(a_lds, wm * WM + i * 32, kk, lane)
                          : frag_kcontig<PA>(a_lds, wm * WM + i * 32, kk, lane);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        fb[slot][j] = B_T ? frag_transposed<PB>(b_lds, wn * WN + j * 32, kk, lane)
                          : frag_kcontig<PB>(b_lds, wn * WN + j * 32, kk, lane);
    };
    read_frags(0, 0);
    __builtin_amdgcn_sched_barrier(0);  // step 0's own reads stay ahead of the interleaved region
    constexpr int kDsPerStep = (A_T ? 2 : 1) * TM + (B_T ? 2 : 1) * TN;  // LDS reads of one kk step
    constexpr int kMfmaPerStep = TM * TN;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      if (kk + 1 < BK / 16) read_frags(kk + 1, (kk + 1) & 1);
      else if constexpr (kMore) stage((kt + 1) & 1);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[kk & 1][j], fa[kk & 1][i], acc[i][j], 0, 0, 0);
      // Issue order inside the step: LDS traffic spread evenly between the MFMAs, so the
      // reads for the next step (or the writes of the next tile) complete under this step's math.
      if (kk + 1 < BK / 16) {
        constexpr int kRatio = kMfmaPerStep >= kDsPerStep ? kMfmaPerStep / kDsPerStep : 1;
        constexpr int kDsEach = kMfmaPerStep >= kDsPerStep ? 1 : (kDsPerStep + kMfmaPerStep - 1) / kMfmaPerStep;
#pragma unroll
        for (int g = 0; g < (kMfmaPerStep >= kDsPerStep ? kDsPerStep : kMfmaPerStep); ++g) {
          __builtin_amdgcn_sched_group_barrier(0x100, kDsEach, 0);  // DS read
          __builtin_amdgcn_sched_group_barrier(0x008, kRatio, 0);   // MFMA
        }
      } else if constexpr (kMore) {
        constexpr int kWrites = MoveA::kPerThread + MoveB::kPerThread;
        constexpr int kRatio = kMfmaPerStep >= kWrites ? kMfmaPerStep / kWrites : 1;
        constexpr int kWrEach = kMfmaPerStep >= kWrites ? 1 : (kWrites + kMfmaPerStep - 1) / kMfmaPerStep;
#pragma unroll
        for (int g = 0; g < (kMfmaPerStep >= kWrites ? kWrites : kMfmaPerStep); ++g) {
          __builtin_amdgcn_sched_group_barrier(0x200, kWrEach, 0);  // DS write
          __builtin_amdgcn_sched_group_barrier(0x008, kRatio, 0);   // MFMA
        }
      }
    }
    __syncthreads();
  };
  for (int kt = 0; kt + 1 < nk; ++kt) k_tile(kt, std::true_type{});
  if (nk > 0) k_tile(nk - 1, std::false_type{});

  // Epilogue.  Register group q of a tile holds columns n .. n+3 of row m with
  //   m = tile_m + lane % 32,  n = tile_n + 8 q + 4 (lane / 32).
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = m0 + wm * WM + i * 32 + (lane & 31);
    if (!EVEN && m >= p.M) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + wn * WN + j * 32 + 8 * q + 4 * (lane >> 5);
        if (!EVEN && n >= p.N) continue;
        const size_t at = (size_t)m * p.ldc + n;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * q + e];
        if constexpr (EPI == EPI_ACCUM_F32) {
          if (p.atomic) {
#pragma unroll
            for (int e = 0; e < 4; ++e) atomicAdd(p.Cf + at + e, v[e]);
          } else {
            f32x4 c = *reinterpret_cast<f32x4*>(p.Cf + at);
#pragma unroll
            for (int e = 0; e < 4; ++e) c[e] += v[e];
            *reinterpret_cast<f32x4*>(p.Cf + at) = c;
          }
        } else {
          if constexpr (EPI == EPI_BIAS || EPI == EPI_BIAS_GELU || EPI == EPI_BIAS_RES) {
            const bf16x4 b = *reinterpret_cast<const bf16x4*>(p.bias + n);
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] += (float)b[e];
          }
          if constexpr (EPI == EPI_BIAS_RES || EPI == EPI_ADD) {
            const bf16x4 x = *reinterpret_cast<const bf16x4*>(p.aux + at);
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] += (float)x[e];
          }
          if constexpr (EPI == EPI_MUL_DGELU) {
            const bf16x4 h = *reinterpret_cast<const bf16x4*>(p.aux + at);
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] *= gelu_grad_fast((float)h[e]);
          }
          if constexpr (EPI == EPI_BIAS_GELU) {
            bf16x4 h;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              h[e] = (bf16)v[e];
              v[e] = gelu_fast(v[e]);
            }
            *reinterpret_cast<bf16x4*>(p.aux_out + at) = h;
          }
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (bf16)v[e];
          *reinterpret_cast<bf16x4*>(p.C + at) = o;
        }
      }
    }
  }
}

template <int BM, int BN, int BK, bool A_T, bool B_T>
constexpr size_t lds_bytes() {
  constexpr int PA = A_T ? BM + kPadT : BK + kPadK;
  constexpr int PB = B_T ? BN + kPadT : BK + kPadK;
  return 2 * ((A_T ? BK : BM) * PA + (B_T ? BK : BN) * PB) * sizeof(bf16);
}

template <int BM, int BN, int BK, bool A_T, bool B_T, int EPI, bool EVEN>
int launch_even(const GemmDev& p, int splits, hipStream_t stream) {
  constexpr size_t lds = lds_bytes<BM, BN, BK, A_T, B_T>();
  auto kern = gemm_mfma_kernel<BM, BN, BK, A_T, B_T, EPI, EVEN>;
  if (lds > 64 * 1024) {
    static thread_local bool raised = false;
    if (!raised) {
      const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return set_error(HANAYO_EHIP, "gemm_mfma: cannot raise LDS limit: %s", hipGetErrorString(e));
      raised = true;
    }
  }
  const dim3 grid((p.N + BN - 1) / BN, (p.M + BM - 1) / BM, splits);
  hipLaunchKernelGGL(kern, grid, dim3(256), lds, stream, p);
  return check_launch("gemm_mfma");
}

template <int BM, int BN, int BK, bool A_T, bool B_T, int EPI>
int launch(const GemmDev& p, int splits, hipStream_t stream) {
  const bool even = p.M % BM == 0 && p.N % BN == 0 && p.K % BK == 0 && p.k_per_split % BK == 0;
  return even ? launch_even<BM, BN, BK, A_T, B_T, EPI, true>(p, splits, stream)
              : launch_even<BM, BN, BK, A_T, B_T, EPI, false>(p, splits, stream);
}

template <int BM, int BN, int BK>
int launch_layout(const GemmArgs& g, const GemmDev& p, int splits, hipStream_t stream) {
  if (!g.a_t && g.b_t) {
    switch (g.epi) {
      case EPI_NONE: return launch<BM, BN, BK, false, true, EPI_NONE>(p, splits, stream);
      case EPI_BIAS: return launch<BM, BN, BK, false, true, EPI_BIAS>(p, splits, stream);
      case EPI_BIAS_GELU: return launch<BM, BN, BK, false, true, EPI_BIAS_GELU>(p, splits, stream);
      case EPI_BIAS_RES: return launch<BM, BN, BK, false, true, EPI_BIAS_RES>(p, splits, stream);
      default: break;
    }
  } else if (!g.a_t && !g.b_t) {
    switch (g.epi) {
      case EPI_NONE: return launch<BM, BN, BK, false, false, EPI_NONE>(p, splits, stream);
      case EPI_MUL_DGELU: return launch<BM, BN, BK, false, false, EPI_MUL_DGELU>(p, splits, stream);
      case EPI_ADD: return launch<BM, BN, BK, false, false, EPI_ADD>(p, splits, stream);
      default: break;
    }
  } else if (g.a_t && g.b_t && g.epi == EPI_ACCUM_F32) {
    return launch<BM, BN, BK, true, true, EPI_ACCUM_F32>(p, splits, stream);
  }
  return set_error(HANAYO_EUNSUPPORTED, "gemm_mfma: layout/epilogue combination not built");
}

bool combo_built(const GemmArgs& g) {
  if (!g.a_t && g.b_t) return g.epi == EPI_NONE || g.epi == EPI_BIAS || g.epi == EPI_BIAS_GELU || g.epi == EPI_BIAS_RES;
  if (!g.a_t && !g.b_t) return g.epi == EPI_NONE || g.epi == EPI_MUL_DGELU || g.epi == EPI_ADD;
  return g.a_t && g.b_t && g.epi == EPI_ACCUM_F32;
}

}  // namespace

bool gemm_mfma_supported(const GemmArgs& g) {
  // 8-element vectors must never straddle a row end, and rows must stay 16-byte aligned
  return combo_built(g) && g.M % 8 == 0 && g.N % 8 == 0 && g.K % 8 == 0 && g.lda % 8 == 0 && g.ldb % 8 == 0 &&
         g.ldc % 4 == 0;
}

int gemm_mfma(const GemmArgs& g, hipStream_t stream) {
  if (!gemm_mfma_supported(g)) return set_error(HANAYO_EUNSUPPORTED, "gemm_mfma: shape not supported");
  GemmDev p;
  p.A = (const bf16*)g.A; p.B = (const bf16*)g.B; p.C = (bf16*)g.C; p.Cf = (float*)g.C;
  p.bias = (const bf16*)g.bias; p.aux = (const bf16*)g.aux; p.aux_out = (bf16*)g.aux_out;
  p.M = g.M; p.N = g.N; p.K = g.K; p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc;
  constexpr int BK = 64;
  const long tiles256 = (long)((g.M + 255) / 256) * ((g.N + 255) / 256);
  const long tiles128 = (long)((g.M + 127) / 128) * ((g.N + 127) / 128);
  const bool big = tiles256 >= 256;
  int splits = 1;
  if (g.epi == EPI_ACCUM_F32 && tiles128 < 64) {
    // A handful of output tiles with a long reduction: split K (fp32 atomics are slow, so
    // only when the machine would otherwise sit almost empty).
    const int ksteps = (g.K + BK - 1) / BK;
    splits = (int)((128 + tiles128 - 1) / tiles128);
    if (splits > ksteps) splits = ksteps;
    if (splits < 1) splits = 1;
  }
  const int ksteps = (g.K + BK - 1) / BK;
  p.k_per_split = ((ksteps + splits - 1) / splits) * BK;
  splits = (g.K + p.k_per_split - 1) / p.k_per_split;
  p.atomic = splits > 1;
  return big ? launch_layout<256, 256, BK>(g, p, splits, stream) : launch_layout<128, 128, BK>(g, p, splits, stream);
}

}  // namespace k
}  // namespace hanayo
