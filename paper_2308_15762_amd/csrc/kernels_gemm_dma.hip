// bf16 GEMM for shapes that are whole multiples of the tile: operand tiles go from
// global memory straight into LDS (global_load_lds_dwordx4, no VGPR staging and no
// LDS write instructions), through a ring of NSTAGE LDS buffers, so that loads
// for tile t+NSTAGE-1 are in flight while tile t is multiplied.  One workgroup
// barrier per K tile (32 elements; 64 in the two-stage form).
//
// LDS layouts are unpadded and XOR-swizzled in units of 16 bytes ("slots"); a
// direct load writes 64 consecutive slots per wavefront instruction, so the
// swizzle is applied by choosing which global vector each lane fetches:
//   * contraction-contiguous operand, tile [rows][32]: 4 slots per row,
//       slot' = slot ^ ((row >> 2) & 3)          (16-byte fragment reads of 16
//       consecutive rows then cover all 64 banks);
//     tile [rows][64] (two-stage form): 8 slots per row, slot' = slot ^ ((row >> 1) & 7)
//   * contraction-strided operand, tile [32 or 64][cols]: cols/8 slots per row,
//       slot' = slot ^ ((row & 3) << 2)          (the 4 rows x 4 slots one half
//       wavefront touches in a transpose read cover all 64 banks)
// MFMA and fragment orientation are those of the staged kernel (kernels_gemm_mfma.hip).
// The epilogue goes through LDS (the idle load ring) so that stores are whole rows; a
// launch may carry several problems of one layout (DmaGemmGroup); workgroups take their
// tiles in an XCD-aware order (xcd_tile).
#include <type_traits>

#include "device_util.h"
#include "epilogue.h"
#include "kernels.h"

namespace hanayo {
namespace k {

namespace {

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

struct DmaGemm {
  const bf16* A;
  const bf16* B;
  bf16* C;
  float* Cf;
  const bf16* bias;
  const bf16* aux;
  bf16* aux_out;
  int M, N, K;
  int lda, ldb, ldc;
  float* colsum;  // see GemmArgs; folded into the kernel (B_T only)
};

// One launch covers up to kMaxGroup independent problems of one layout and epilogue: workgroups
// first[i] .. first[i + 1] - 1 are the tiles of problem i.  Four weight-gradient GEMMs of a block,
// none of which fills the chip alone, share one grid this way.
constexpr int kMaxGroup = 4;
struct DmaGemmGroup {
  DmaGemm prob[kMaxGroup];
  int first[kMaxGroup + 1];
  int count;
};

constexpr int kBK = 32;

// One wavefront-wide 16-byte-per-lane load from global memory into LDS: lane L's
// vector lands at lds_byte_addr + 16 L.  `voff` is the lane's byte offset from `base`.
// M0 carries the LDS address; it is written and consumed inside the statement, and nothing
// else in these kernels lives in M0 (gfx950 LDS instructions do not use it).
__device__ __forceinline__ void dma16(const void* base, unsigned voff, unsigned lds_byte_addr) {
  asm volatile(
      "s_mov_b32 m0, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %0, %1"
      :
      : "v"(voff), "s"(base), "s"(lds_byte_addr)
      : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Waits until at most `tiles_in_flight` tiles (LOADS instructions each) are still outstanding.
template <int LOADS>
__device__ __forceinline__ void wait_tiles(int tiles_in_flight) {
  switch (tiles_in_flight) {
    case 0: wait_vmcnt<0>(); break;
    case 1: wait_vmcnt<LOADS>(); break;
    case 2: wait_vmcnt<2 * LOADS>(); break;
    case 3: wait_vmcnt<3 * LOADS>(); break;
    case 4: wait_vmcnt<(4 * LOADS > 63 ? 63 : 4 * LOADS)>(); break;
    case 5: wait_vmcnt<(5 * LOADS > 63 ? 63 : 5 * LOADS)>(); break;
    case 6: wait_vmcnt<(6 * LOADS > 63 ? 63 : 6 * LOADS)>(); break;
    default: wait_vmcnt<(7 * LOADS > 63 ? 63 : 7 * LOADS)>(); break;
  }
}

// Operand tile description.  T = contraction strided in memory (tile is [BK][EXT]); BK = 32 or 64.
template <int EXT, bool T, int NW, int BK>
struct Operand {
  static constexpr int kSlotsPerRow = T ? EXT / 8 : BK / 8;
  static constexpr int kRows = T ? BK : EXT;
  static constexpr int kBytes = kRows * kSlotsPerRow * 16;
  static constexpr int kInstr = kBytes / 1024;      // wavefront-wide loads per tile
  static constexpr int kPerWave = kInstr / NW;      // issued by each wavefront
  static constexpr int kRowsPerInstr = 64 / kSlotsPerRow == 0 ? 1 : 64 / kSlotsPerRow;
  static_assert(kInstr % NW == 0, "tile loads must divide evenly over the wavefronts");
  // row_base(q) is taken from the per-wavefront index i: valid when a wavefront's first
  // instruction starts at a multiple of 4 rows
  static_assert(!T || ((kPerWave * 64) / kSlotsPerRow) % 4 == 0, "wavefront's share must start on a 4-row boundary");

  // contraction-contiguous rows are 64 bytes (BK = 32: four rows per 256 bytes of banks, slot ^ (row / 4 mod 4)) or
  // 128 bytes (BK = 64: two rows, slot ^ (row / 2 mod 8)): 16 consecutive rows at one logical slot cover all banks
  __device__ static int swizzle(int row, int slot) {
    return T ? slot ^ ((row & 3) << 2) : (BK == 32 ? slot ^ ((row >> 2) & 3) : slot ^ ((row >> 1) & 7));
  }

  // Byte offset, from the first element an instruction covers, of the vector that lane `lane`
  // fetches.  `row_base` = the bits of the instruction's first tile row that the swizzle looks at: the
  // swizzle depends on the absolute row, and an instruction may start at a row that is not a multiple of
  // the swizzle's period (it covers 64 / slots-per-row rows).
  __device__ static unsigned lane_offset(int lane, int ld, int row_base) {
    const int row = lane / kSlotsPerRow, sp = lane % kSlotsPerRow;
    return (unsigned)((row * ld + swizzle(row_base + row, sp) * 8) * 2);
  }
  // row_base of instruction q: the bits of its first tile row that the swizzle looks at (a contraction-contiguous
  // tile's swizzle has period 16 rows; an instruction covers 16 rows of 64 bytes or 8 rows of 128 bytes)
  __device__ static constexpr int row_base(int q) { return T ? ((q * 64) / kSlotsPerRow) & 3 : ((q * 64) / kSlotsPerRow) & 15; }
  static_assert(T || ((kPerWave * 64) / kSlotsPerRow) % 16 == 0, "wavefront's share must start on a 16-row boundary");
};

template <int PITCH_SLOTS>
__device__ __forceinline__ bf16x8 frag_k(const char* lds, int r0, int kk, int lane) {
  const int row = r0 + (lane & 31), slot = 2 * kk + (lane >> 5);
  const int swz = PITCH_SLOTS == 4 ? (row >> 2) & 3 : (row >> 1) & 7;
  return *reinterpret_cast<const bf16x8*>(lds + (row * PITCH_SLOTS + (slot ^ swz)) * 16);
}

template <int SPR>
__device__ __forceinline__ bf16x8 frag_t(const char* lds, int c0, int kk, int lane) {
  const int krow = kk * 16 + 8 * (lane >> 5) + ((lane & 15) >> 2);
  const int col = c0 + 16 * ((lane >> 4) & 1) + (lane & 3) * 4;
  const int slot = (col >> 3) ^ ((krow & 3) << 2);
  const char* p = lds + (krow * SPR + slot) * 16 + (col & 7) * 2;
  union {
    struct { s16x4 lo, hi; } s;
    bf16x8 v;
  } u;
  u.s.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
  u.s.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 4 * SPR * 16));
  return u.v;
}

// MODE 0: fragments are read one MFMA step ahead (large wavefront tiles).
// MODE 1: fragments are read a whole K tile ahead (small wavefront tiles, where one MFMA step is
//         shorter than the LDS latency); a tile's LDS buffer is then free one iteration earlier,
//         so all NSTAGE buffers can be in flight.
// MODE 2: as 1, with twice the wavefronts: the first WGM*WGN take MFMA step 0 of every K tile, the
//         second WGM*WGN take step 1, and the two partial tiles are added through LDS at the end.
//         A SIMD then holds two wavefronts that fill each other's stalls, and twice as many
//         wavefronts issue LDS reads (the per-wavefront LDS request rate limits the 4-wavefront form).
template <int BM, int BN, int WGM, int WGN, int NSTAGE, int MODE, bool A_T, bool B_T, int EPI>
__global__ __launch_bounds__(WGM* WGN*(MODE == 2 ? 2 : 1) * 64) void gemm_dma_kernel(DmaGemmGroup grp) {
  int gi = 0;
#pragma unroll
  for (int j = 1; j < kMaxGroup; ++j)
    if (j < grp.count && (int)blockIdx.x >= grp.first[j]) gi = j;
  const DmaGemm p = grp.prob[gi];
  const int wg = (int)blockIdx.x - grp.first[gi];  // tile number within the problem
  constexpr bool FDEEP = MODE == 1 || MODE == 2;
  constexpr bool WIDE = NSTAGE == 2 || MODE == 3;  // 64-wide K tiles (MODE 3: in a ring of NSTAGE >= 2 stages)
  constexpr int NSP = WGM * WGN;                 // wavefronts that tile the output
  constexpr int NW = NSP * (MODE == 2 ? 2 : 1);  // wavefronts in the workgroup
  constexpr int WM = BM / WGM, WN = BN / WGN, TM = WM / 32, TN = WN / 32;
  // A ring of two stages holds 64-wide K tiles (the same bytes in flight as four stages of 32, half as many
  // barriers and waits per unit of work, whole 128-byte lines per row of a contraction-contiguous operand).
  constexpr int BK = WIDE ? 64 : 32;
  constexpr int KS = BK / 16;  // MFMA steps per K tile
  using OpA = Operand<BM, A_T, NW, BK>;
  using OpB = Operand<BN, B_T, NW, BK>;
  constexpr int STAGE_BYTES = OpA::kBytes + OpB::kBytes;
  constexpr int LOADS = OpA::kPerWave + OpB::kPerWave;  // per thread per tile
  static_assert((NSTAGE - 1) * LOADS <= 63, "vmcnt range");
  static_assert(NSTAGE >= 3 || (NSTAGE == 2 && MODE == 0), "two stages: the 64-wide pipeline of MODE 0 only");
  static_assert(MODE != 3 || NSTAGE >= 2, "the 64-wide pipeline needs at least two stages");

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  // LDS byte address of the ring (address-space-3 offset, what M0 takes)
  const unsigned lds0 = (unsigned)(unsigned long)((__attribute__((address_space(3))) char*)smem);

  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int khalf = wave / NSP;  // MODE 2: which MFMA step of a K tile this wavefront owns
  const int wm = (wave % NSP) / WGN, wn = (wave % NSP) % WGN;
  const int tiles_m = p.M / BM, tiles_n = p.N / BN;
  int tile_m, tile_n;
  xcd_tile(wg, tiles_m, tiles_n, tile_m, tile_n);
  tile_m = __builtin_amdgcn_readfirstlane(tile_m);
  tile_n = __builtin_amdgcn_readfirstlane(tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int nk = p.K / BK;

  // Direct loads of one K tile.  The wavefront's i-th instruction for an operand covers the 64
  // slots q = wave * kPerWave + i of the tile; which rows that is goes into the lane's byte
  // offset (one VGPR per instruction, constant over the K loop), so every instruction of a tile
  // shares one uniform base pointer that just advances by a K tile.
  unsigned voff_a[OpA::kPerWave], voff_b[OpB::kPerWave];
#pragma unroll
  for (int i = 0; i < OpA::kPerWave; ++i) {
    const int q = wave * OpA::kPerWave + i;
    const unsigned first = A_T ? (unsigned)((((q * 64) / OpA::kSlotsPerRow) * p.lda + ((q * 64) % OpA::kSlotsPerRow) * 8) * 2)
                               : (unsigned)((q * (64 / OpA::kSlotsPerRow) * p.lda) * 2);
    voff_a[i] = first + OpA::lane_offset(lane, p.lda, OpA::row_base(i));
  }
#pragma unroll
  for (int i = 0; i < OpB::kPerWave; ++i) {
    const int q = wave * OpB::kPerWave + i;
    const unsigned first = B_T ? (unsigned)((((q * 64) / OpB::kSlotsPerRow) * p.ldb + ((q * 64) % OpB::kSlotsPerRow) * 8) * 2)
                               : (unsigned)((q * (64 / OpB::kSlotsPerRow) * p.ldb) * 2);
    voff_b[i] = first + OpB::lane_offset(lane, p.ldb, OpB::row_base(i));
  }
  // uniform running state of the loader: next tile's base pointers and LDS buffer
  const bf16* a_next = A_T ? p.A + m0 : p.A + (size_t)m0 * p.lda;
  const bf16* b_next = B_T ? p.B + n0 : p.B + (size_t)n0 * p.ldb;
  const size_t a_step = A_T ? (size_t)BK * p.lda : (size_t)BK;
  const size_t b_step = B_T ? (size_t)BK * p.ldb : (size_t)BK;
  unsigned stage_next = 0;  // buffer index the next issued tile goes to
  const unsigned wave_lds_a = lds0 + wave * OpA::kPerWave * 1024;
  const unsigned wave_lds_b = lds0 + OpA::kBytes + wave * OpB::kPerWave * 1024;
  // the i-th of the LOADS direct loads of the next tile (i is a compile-time constant at every call)
  auto issue_part = [&](int i) {
    const unsigned st = stage_next * STAGE_BYTES;
    if (i < OpA::kPerWave) dma16(a_next, voff_a[i], wave_lds_a + st + i * 1024);
    else dma16(b_next, voff_b[i - OpA::kPerWave], wave_lds_b + st + (i - OpA::kPerWave) * 1024);
  };
  auto issue_done = [&]() {
    a_next += a_step;
    b_next += b_step;
    stage_next = stage_next + 1 == NSTAGE ? 0 : stage_next + 1;
  };
  auto issue = [&]() {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) issue_part(i);
    issue_done();
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // issue order of one step: the LDS reads go out one per MFMA at the start of the step, so the
  // last of them has a good part of the step to complete
  auto interleave = [&]() {
    constexpr int kDs = (A_T ? 2 : 1) * TM + (B_T ? 2 : 1) * TN;
    constexpr int kMfma = TM * TN;
    constexpr int kDsEach = kMfma >= kDs ? 1 : (kDs + kMfma - 1) / kMfma;
    constexpr int kGroups = kMfma >= kDs ? kDs : kMfma;
#pragma unroll
    for (int g = 0; g < kGroups; ++g) {
      __builtin_amdgcn_sched_group_barrier(0x100, kDsEach, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    }
    if (kMfma > kGroups) __builtin_amdgcn_sched_group_barrier(0x008, kMfma - kGroups, 0);
  };
  auto read_a = [&](int kt, int kk, bf16x8 (&f)[TM]) {
    const char* a_lds = smem + (kt % NSTAGE) * STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < TM; ++i)
      f[i] = A_T ? frag_t<OpA::kSlotsPerRow>(a_lds, wm * WM + i * 32, kk, lane)
                 : frag_k<OpA::kSlotsPerRow>(a_lds, wm * WM + i * 32, kk, lane);
  };
  auto read_b = [&](int kt, int kk, bf16x8 (&f)[TN]) {
    const char* b_lds = smem + (kt % NSTAGE) * STAGE_BYTES + OpA::kBytes;
#pragma unroll
    for (int j = 0; j < TN; ++j)
      f[j] = B_T ? frag_t<OpB::kSlotsPerRow>(b_lds, wn * WN + j * 32, kk, lane)
                 : frag_k<OpB::kSlotsPerRow>(b_lds, wn * WN + j * 32, kk, lane);
  };
  auto mfma_step = [&](const bf16x8 (&a)[TM], const bf16x8 (&b)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
  };

  // Column sums of B (bias gradient): the workgroup of tile row 0 sums every K tile of its tile column from
  // the B tiles that pass through LDS anyway (each thread adds 4 columns x (BK / kColRowGroups) rows per
  // tile).  One workgroup per column and a fixed order of additions: the sums are the same bits every run.
  constexpr int kColGroups = BN / 4, kColRowGroups = NW * 64 / kColGroups, kColRows = BK / kColRowGroups;
  float csum[4] = {0.f, 0.f, 0.f, 0.f};
  const bool sums_columns = B_T && p.colsum && tile_m == 0;
  auto colsum_tile = [&](int kt) {
    if constexpr (B_T) {
      if (sums_columns) {
        const char* b_lds = smem + (kt % NSTAGE) * STAGE_BYTES + OpA::kBytes;
        const int c = (threadIdx.x % kColGroups) * 4, rg = threadIdx.x / kColGroups;
#pragma unroll
        for (int r = 0; r < kColRows; ++r) {
          const int row = rg * kColRows + r;
          const int slot = (c >> 3) ^ ((row & 3) << 2);
          const bf16x4 v = *reinterpret_cast<const bf16x4*>(b_lds + (row * OpB::kSlotsPerRow + slot) * 16 + (c & 7) * 2);
#pragma unroll
          for (int e = 0; e < 4; ++e) csum[e] += (float)v[e];
        }
      }
    }
  };

  if constexpr (WIDE) {
    // NSTAGE 64-wide stages (two, or three where the tile leaves room: one more tile of look-ahead for launches
    // that have a single wavefront per SIMD and nothing else to cover a late load).  Per K tile (KS = 4 MFMA steps):
    //   steps 0 .. KS-2 of tile kt    | LDS reads: the following step of tile kt
    //   every fragment of tile kt is in registers; wait until tile kt+1 has landed; barrier (everyone is there)
    //   start the loads of tile kt+NSTAGE into the buffer tile kt occupied
    //   step KS-1 of tile kt          | LDS reads: step 0 of tile kt+1
#pragma unroll
    for (int t = 0; t < NSTAGE; ++t)
      if (t < nk) issue();
    bf16x8 fa[2][TM], fb[2][TN];
    wait_tiles<LOADS>(min(NSTAGE - 1, nk - 1));
    __syncthreads();
    colsum_tile(0);
    read_a(0, 0, fa[0]);
    read_b(0, 0, fb[0]);
    // A tile's direct loads go out one behind each MFMA: the first kFirst in the step after the barrier, the rest
    // (a 4-wavefront tile has more loads per wavefront than MFMAs per step) in step 0 of the next tile; `pending`
    // says that this rest is still to be issued.
    // (Only with three stages: with two, the rest would have less than a tile's time to land.)
    constexpr int kMf = TM * TN, kFirst = (LOADS < kMf || NSTAGE < 3) ? LOADS : kMf, kRest = LOADS - kFirst;
    constexpr int kPer = (kFirst + kMf - 1) / kMf;
    static_assert(kRest <= kMf, "at most two steps' worth of loads per tile");
    bool pending = false;
    auto steps_before_barrier = [&](int kt) {
      {  // step 0, one slot per MFMA: behind it, its share of step 1's fragment reads and of the pending loads
        const char* a_cur = smem + (kt % NSTAGE) * STAGE_BYTES;
        const char* b_cur = a_cur + OpA::kBytes;
        constexpr int kFr = (TM + TN + kMf - 1) / kMf;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            const int m = i * TN + j;
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[0][j], fa[0][i], acc[i][j], 0, 0, 0);
#pragma unroll
            for (int u = 0; u < kFr; ++u) {
              const int f = m * kFr + u;
              if (f < TM)
                fa[1][f] = A_T ? frag_t<OpA::kSlotsPerRow>(a_cur, wm * WM + f * 32, 1, lane)
                               : frag_k<OpA::kSlotsPerRow>(a_cur, wm * WM + f * 32, 1, lane);
              else if (f < TM + TN)
                fb[1][f - TM] = B_T ? frag_t<OpB::kSlotsPerRow>(b_cur, wn * WN + (f - TM) * 32, 1, lane)
                                    : frag_k<OpB::kSlotsPerRow>(b_cur, wn * WN + (f - TM) * 32, 1, lane);
            }
            if (m < kRest && pending) issue_part(kFirst + m);
            __builtin_amdgcn_sched_barrier(0);
          }
        if (kRest > 0 && pending) {
          issue_done();
          pending = false;
        }
      }
#pragma unroll
      for (int st = 1; st + 1 < KS; ++st) {
        read_a(kt, st + 1, fa[(st + 1) & 1]);
        read_b(kt, st + 1, fb[(st + 1) & 1]);
        mfma_step(fa[st & 1], fb[st & 1]);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
      }
      // the buffer of tile kt is overwritten right after the barrier: its last fragments must have arrived
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    };
    int kt = 0;
    // Steady state: tiles kt+2 .. kt+NSTAGE-1 may still be in flight at the barrier, and tile kt+NSTAGE is started
    // after it.  Every wavefront of the workgroup leaves the barrier in the same phase, so whatever stands between
    // the barrier and the next MFMA is time the matrix pipe idles on all four SIMDs at once.  The last step's
    // fragments are in registers: its MFMAs start at once, and behind each of them goes its share of the tile's
    // direct loads and of the first fragment reads of tile kt+1, one or two instructions, held there by
    // scheduling barriers.  (Left to the scheduler the loads, each with its M0 set-up, go out in runs of four
    // between two MFMAs; both wavefronts of a SIMD do that at the same moment and the pipe idles meanwhile.)
    for (; kt + NSTAGE < nk; ++kt) {
      steps_before_barrier(kt);
      wait_vmcnt<(NSTAGE - 2) * LOADS>();
      __syncthreads();
      __builtin_amdgcn_sched_barrier(0);
      constexpr int kFr = (TM + TN + kMf - 1) / kMf;
      const char* a_nx = smem + ((kt + 1) % NSTAGE) * STAGE_BYTES;
      const char* b_nx = a_nx + OpA::kBytes;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int m = i * TN + j;  // one slot per MFMA: its share of the fragment reads and of the direct loads
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[(KS - 1) & 1][j], fa[(KS - 1) & 1][i], acc[i][j], 0, 0, 0);
#pragma unroll
          for (int u = 0; u < kFr; ++u) {
            const int f = m * kFr + u;
            if (f < TM)
              fa[0][f] = A_T ? frag_t<OpA::kSlotsPerRow>(a_nx, wm * WM + f * 32, 0, lane)
                             : frag_k<OpA::kSlotsPerRow>(a_nx, wm * WM + f * 32, 0, lane);
            else if (f < TM + TN)
              fb[0][f - TM] = B_T ? frag_t<OpB::kSlotsPerRow>(b_nx, wn * WN + (f - TM) * 32, 0, lane)
                                  : frag_k<OpB::kSlotsPerRow>(b_nx, wn * WN + (f - TM) * 32, 0, lane);
          }
#pragma unroll
          for (int u = 0; u < kPer; ++u)
            if (m * kPer + u < kFirst) issue_part(m * kPer + u);
          __builtin_amdgcn_sched_barrier(0);
        }
      if (kRest > 0) pending = true;  // the rest goes out in step 0 of tile kt+1, which advances the loader's state
      else issue_done();
      colsum_tile(kt + 1);
    }
    // The last tiles: nothing left to start.
    for (; kt + 1 < nk; ++kt) {
      steps_before_barrier(kt);
      wait_tiles<LOADS>(min(NSTAGE - 2, nk - 2 - kt));
      __syncthreads();
      colsum_tile(kt + 1);
      __builtin_amdgcn_sched_barrier(0);
      read_a(kt + 1, 0, fa[0]);
      read_b(kt + 1, 0, fb[0]);
      mfma_step(fa[(KS - 1) & 1], fb[(KS - 1) & 1]);
      interleave();
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int st = 0; st + 1 < KS; ++st) {
      read_a(nk - 1, st + 1, fa[(st + 1) & 1]);
      read_b(nk - 1, st + 1, fb[(st + 1) & 1]);
      mfma_step(fa[st & 1], fb[st & 1]);
      interleave();
      __builtin_amdgcn_sched_barrier(0);
    }
    mfma_step(fa[(KS - 1) & 1], fb[(KS - 1) & 1]);
  } else if constexpr (!FDEEP) {
#pragma unroll
    for (int t = 0; t < NSTAGE - 1; ++t)
      if (t < nk) issue();
    bf16x8 fa[2][TM], fb[2][TN];
    // Tile 0 has landed once only tiles 1 .. NSTAGE-2 are outstanding.
    wait_tiles<LOADS>(min(NSTAGE - 2, nk - 1));
    __syncthreads();
    colsum_tile(0);
    read_a(0, 0, fa[0]);
    read_b(0, 0, fb[0]);
    // Steady state, per K tile (two MFMA steps of 16):
    //   step 0 of tile kt   | LDS reads: step 1 of tile kt
    //   wait until tile kt+1 has landed; barrier (also: everyone has finished tile kt-1)
    //   start the loads of tile kt+NSTAGE-1 into the buffer tile kt-1 occupied
    //   step 1 of tile kt   | LDS reads: step 0 of tile kt+1
    // so the barrier never drains the fragment pipeline.
    for (int kt = 0; kt + 1 < nk; ++kt) {
      read_a(kt, 1, fa[1]);
      read_b(kt, 1, fb[1]);
      mfma_step(fa[0], fb[0]);
      interleave();
      __builtin_amdgcn_sched_barrier(0);
      if (kt + NSTAGE - 1 < nk) {  // steady state: a fixed number of tiles stays in flight
        wait_vmcnt<(NSTAGE - 3) * LOADS>();
        __syncthreads();
        issue();
      } else {
        wait_tiles<LOADS>(min(NSTAGE - 3, nk - 2 - kt));
        __syncthreads();
      }
      colsum_tile(kt + 1);
      __builtin_amdgcn_sched_barrier(0);
      read_a(kt + 1, 0, fa[0]);
      read_b(kt + 1, 0, fb[0]);
      mfma_step(fa[1], fb[1]);
      interleave();
      __builtin_amdgcn_sched_barrier(0);
    }
    read_a(nk - 1, 1, fa[1]);
    read_b(nk - 1, 1, fb[1]);
    mfma_step(fa[0], fb[0]);
    interleave();
    __builtin_amdgcn_sched_barrier(0);
    mfma_step(fa[1], fb[1]);
  } else {
    // All NSTAGE buffers are filled up front.  In iteration kt the fragments of tile kt are already
    // in registers (read during iteration kt-1), so after the barrier its buffer takes tile kt+NSTAGE.
#pragma unroll
    for (int t = 0; t < NSTAGE; ++t)
      if (t < nk) issue();
    bf16x8 fa[2][2][TM], fb[2][2][TN];  // [tile parity][step]; MODE 2 uses step slot 0 only
    wait_tiles<LOADS>(min(NSTAGE - 1, nk - 1));
    __syncthreads();
    colsum_tile(0);
    if constexpr (MODE == 1) {
      read_a(0, 0, fa[0][0]);
      read_b(0, 0, fb[0][0]);
      read_a(0, 1, fa[0][1]);
      read_b(0, 1, fb[0][1]);
    } else {
      read_a(0, khalf, fa[0][0]);
      read_b(0, khalf, fb[0][0]);
    }
    auto tile_iter = [&](int kt, auto parity, auto more) {
      constexpr int P = decltype(parity)::value;
      if constexpr (decltype(more)::value) {
        // tile kt+1 has landed, for everyone after the barrier; tile kt's buffer is free then
        if (kt + NSTAGE < nk) {  // steady state
          wait_vmcnt<(NSTAGE - 2) * LOADS>();
          __syncthreads();
          issue();
        } else {
          wait_tiles<LOADS>(min(NSTAGE - 2, nk - 2 - kt));
          __syncthreads();
        }
        colsum_tile(kt + 1);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (MODE == 1) {
          read_a(kt + 1, 0, fa[P ^ 1][0]);
          read_b(kt + 1, 0, fb[P ^ 1][0]);
          mfma_step(fa[P][0], fb[P][0]);
          interleave();
          __builtin_amdgcn_sched_barrier(0);
          read_a(kt + 1, 1, fa[P ^ 1][1]);
          read_b(kt + 1, 1, fb[P ^ 1][1]);
          mfma_step(fa[P][1], fb[P][1]);
          interleave();
        } else {
          read_a(kt + 1, khalf, fa[P ^ 1][0]);
          read_b(kt + 1, khalf, fb[P ^ 1][0]);
          mfma_step(fa[P][0], fb[P][0]);
          interleave();
        }
        __builtin_amdgcn_sched_barrier(0);
      } else {
        mfma_step(fa[P][0], fb[P][0]);
        if constexpr (MODE == 1) mfma_step(fa[P][1], fb[P][1]);
      }
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    int kt = 0;
    for (; kt + 2 < nk; kt += 2) {
      tile_iter(kt, P0{}, std::true_type{});
      tile_iter(kt + 1, P1{}, std::true_type{});
    }
    if (kt + 1 < nk) {
      tile_iter(kt, P0{}, std::true_type{});
      tile_iter(kt + 1, P1{}, std::false_type{});
    } else {
      tile_iter(kt, P0{}, std::false_type{});
    }
  }

  if constexpr (MODE == 2) {
    // add the step-1 group's partial tile to the step-0 group's: through LDS, 16 KiB per pair
    __syncthreads();  // every wavefront is done with the load ring
    float* xch = reinterpret_cast<float*>(smem) + (size_t)(wave % NSP) * (TM * TN * 16 * 64);
    if (khalf == 1) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            f32x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * q + e];
            *reinterpret_cast<f32x4*>(xch + (((i * TN + j) * 4 + q) * 64 + lane) * 4) = v;
          }
    }
    __syncthreads();
    if (khalf == 0) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(xch + (((i * TN + j) * 4 + q) * 64 + lane) * 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[i][j][4 * q + e] += v[e];
          }
    }
  }

  if constexpr (B_T) {
    if (sums_columns) {  // combine the row groups through LDS (the ring is idle now); this workgroup alone owns the columns
      __syncthreads();
      float* red = reinterpret_cast<float*>(smem);
      const int c = (threadIdx.x % kColGroups) * 4, rg = threadIdx.x / kColGroups;
#pragma unroll
      for (int e = 0; e < 4; ++e) red[rg * BN + c + e] = csum[e];
      __syncthreads();
      if (threadIdx.x < BN) {
        float t = 0.f;
#pragma unroll
        for (int g = 0; g < kColRowGroups; ++g) t += red[g * BN + threadIdx.x];
        p.colsum[n0 + threadIdx.x] += t;
      }
    }
  }

  // Epilogue through LDS.  In registers a lane holds 4 consecutive columns of one row, and the 32
  // lanes of a half wavefront hold 32 different rows: stores (and the reads of the residual or
  // pre-activation operand) straight from that layout touch 16 bytes per row.  Instead, one band
  // of 32 rows per wavefront row (WGM * 32 rows x BN columns, fp32) at a time is parked in LDS and
  // taken out again with each thread owning 8 consecutive columns, so every global access of the
  // epilogue is a run of full rows: 16 bytes per lane, whole 128-byte lines.
  constexpr int EP = BN + 4;  // fp32 row pitch in LDS: +4 keeps the register-layout writes conflict-free
  float* stage = reinterpret_cast<float*>(smem);
  constexpr int kBandRows = WGM * 32, kVecPerRow = BN / 8, kVecs = kBandRows * kVecPerRow;
  static_assert((size_t)kBandRows * EP * 4 <= (size_t)NSTAGE * STAGE_BYTES, "epilogue band must fit the load ring");
  // GELU epilogues: Phi (forward) or GELU' (input gradient of FC2) comes from a table of kGeluN
  // intervals over [-8, 8) built next to the staging band with erff, read with linear interpolation
  // (error below 1e-5, far under bf16 rounding): 8 VALU operations and one LDS read per element
  // instead of an exponential, a reciprocal and a polynomial, which at one workgroup per CU nothing
  // else would overlap.
  constexpr bool kGelu = EPI == EPI_BIAS_GELU || EPI == EPI_MUL_DGELU;
  constexpr int kGeluN = 2048;
  constexpr int kStageBytes = ((WGM * 32 * EP * 4 + 15) / 16) * 16;
  static_assert(!kGelu || kStageBytes + kGeluN * 8 <= NSTAGE * STAGE_BYTES, "table does not fit behind the band");
  float2* gelu_tab = reinterpret_cast<float2*>(smem + kStageBytes);
  auto gelu_lookup = [&](float x) {
    const float t = fminf(fmaxf(fmaf(x, 128.f, 1024.f), 0.f), 2047.99f);
    const int k = (int)t;
    const float2 e = gelu_tab[k];
    return fmaf(t - (float)k, e.y, e.x);
  };
  // The operand an epilogue reads from global memory (residual, pre-activation, or the fp32 sums it
  // accumulates into) is fetched one band ahead into registers, so that its latency runs under the
  // staging of the band before instead of in front of every band's arithmetic.
  constexpr int VPT = kVecs / (NW * 64);  // 8-column vectors per thread per band
  static_assert(kVecs % (NW * 64) == 0, "band vectors divide among the threads");
  constexpr bool kReadsAux = EPI == EPI_BIAS_RES || EPI == EPI_ADD || EPI == EPI_MUL_DGELU;
  constexpr bool kReadsC = EPI == EPI_ACCUM_F32;
  bf16x8 pre_aux[2][kReadsAux ? VPT : 1];
  f32x4 pre_c[2][kReadsC ? VPT : 1][2];
  auto where = [&](int i, int u, int& br, int& c, size_t& at, int& n) {
    const int vi = threadIdx.x + u * NW * 64;
    br = vi / kVecPerRow;          // band row
    c = (vi % kVecPerRow) * 8;     // first column
    const int m = m0 + (br >> 5) * WM + i * 32 + (br & 31);
    n = n0 + c;
    at = (size_t)m * p.ldc + n;
  };
  auto prefetch = [&](int i, int buf) {
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
      int br, c, n;
      size_t at;
      where(i, u, br, c, at, n);
      if constexpr (kReadsAux) pre_aux[buf][u] = *reinterpret_cast<const bf16x8*>(p.aux + at);
      if constexpr (kReadsC) {
        pre_c[buf][u][0] = *reinterpret_cast<const f32x4*>(p.Cf + at);
        pre_c[buf][u][1] = *reinterpret_cast<const f32x4*>(p.Cf + at + 4);
      }
    }
  };
  if constexpr (kReadsAux || kReadsC) prefetch(0, 0);
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    __syncthreads();  // the ring (first band) or the previous band is no longer being read
    if constexpr (kGelu) {
      if (i == 0) {
        for (int k = threadIdx.x; k < kGeluN; k += NW * 64) {
          const float x0 = -8.f + (float)k * (1.f / 128.f), x1 = -8.f + (float)(k + 1) * (1.f / 128.f);
          float f0, f1;
          if constexpr (EPI == EPI_BIAS_GELU) {
            f0 = 0.5f * (1.0f + erff(x0 * 0.70710678118654752f));
            f1 = 0.5f * (1.0f + erff(x1 * 0.70710678118654752f));
          } else {
            f0 = gelu_grad_f(x0);
            f1 = gelu_grad_f(x1);
          }
          gelu_tab[k] = make_float2(f0, f1 - f0);
        }
      }
    }
    if (MODE != 2 || khalf == 0) {
      float* dst = stage + (wm * 32 + (lane & 31)) * EP + wn * WN + 4 * (lane >> 5);
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * q + e];
          *reinterpret_cast<f32x4*>(dst + j * 32 + 8 * q) = v;
        }
    }
    if constexpr (kReadsAux || kReadsC) {
      if (i + 1 < TM) prefetch(i + 1, (i + 1) & 1);
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
      int br, c, n;
      size_t at;
      where(i, u, br, c, at, n);
      float v[8];
      load8(stage + br * EP + c, v);
      if constexpr (EPI == EPI_ACCUM_F32) {
        float cur[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          cur[e] = pre_c[i & 1][u][0][e] + v[e];
          cur[4 + e] = pre_c[i & 1][u][1][e] + v[4 + e];
        }
        store8(p.Cf + at, cur);
      } else if constexpr (EPI == EPI_STORE_F32) {
        store8(p.Cf + at, v);
      } else {
        if constexpr (EPI == EPI_BIAS || EPI == EPI_BIAS_GELU || EPI == EPI_BIAS_RES) {
          float b[8];
          load8(p.bias + n, b);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += b[e];
        }
        if constexpr (EPI == EPI_BIAS_RES || EPI == EPI_ADD) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += (float)pre_aux[i & 1][u][e];
        }
        if constexpr (EPI == EPI_MUL_DGELU) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] *= gelu_lookup((float)pre_aux[i & 1][u][e]);
        }
        if constexpr (EPI == EPI_BIAS_GELU) {
          store8(p.aux_out + at, v);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] *= gelu_lookup(v[e]);
        }
        store8(p.C + at, v);
      }
    }
  }
}

template <int BM, int BN, int WGM, int WGN, int NSTAGE, int MODE, bool A_T, bool B_T, int EPI>
int launch(DmaGemmGroup& grp, hipStream_t stream) {
  constexpr int NW = WGM * WGN * (MODE == 2 ? 2 : 1);
  constexpr int BK = (NSTAGE == 2 || MODE == 3) ? 64 : 32;  // as in the kernel
  using OpA = Operand<BM, A_T, NW, BK>;
  using OpB = Operand<BN, B_T, NW, BK>;
  constexpr size_t lds = (size_t)NSTAGE * (OpA::kBytes + OpB::kBytes);
  auto kern = gemm_dma_kernel<BM, BN, WGM, WGN, NSTAGE, MODE, A_T, B_T, EPI>;
  static thread_local bool raised = false;
  if (lds > 64 * 1024 && !raised) {
    const hipError_t e =
        hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return set_error(HANAYO_EHIP, "gemm_dma: cannot raise LDS limit: %s", hipGetErrorString(e));
    raised = true;
  }
  long tiles = 0;
  for (int i = 0; i < grp.count; ++i) {
    grp.first[i] = (int)tiles;
    tiles += (long)(grp.prob[i].N / BN) * (grp.prob[i].M / BM);
  }
  for (int i = grp.count; i <= kMaxGroup; ++i) grp.first[i] = (int)tiles;
  if (tiles > 0x7fffffffL) return set_error(HANAYO_EUNSUPPORTED, "gemm_dma: too many tiles");
  hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(NW * 64), lds, stream, grp);
  return check_launch("gemm_dma");
}

template <int BM, int BN, int WGM, int WGN, int NSTAGE, int MODE>
int launch_layout(const GemmArgs& g, DmaGemmGroup& grp, hipStream_t stream) {
  if (!g.a_t && g.b_t) {
    switch (g.epi) {
      case EPI_NONE: return launch<BM, BN, WGM, WGN, NSTAGE, MODE, false, true, EPI_NONE>(grp, stream);
      case EPI_BIAS: return launch<BM, BN, WGM, WGN, NSTAGE, MODE, false, true, EPI_BIAS>(grp, stream);
      case EPI_BIAS_GELU: return launch<BM, BN, WGM, WGN, NSTAGE, MODE, false, true, EPI_BIAS_GELU>(grp, stream);
      case EPI_BIAS_RES: return launch<BM, BN, WGM, WGN, NSTAGE, MODE, false, true, EPI_BIAS_RES>(grp, stream);
      case EPI_STORE_F32: return launch<BM, BN, WGM, WGN, NSTAGE, MODE, false, true, EPI_STORE_F32>(grp, stream);
      default: break;
    }
  } else if (!g.a_t && !g.b_t) {
    switch (g.epi) {
      case EPI_NONE: return launch<BM, BN, WGM, WGN, NSTAGE, MODE, false, false, EPI_NONE>(grp, stream);
      case EPI_MUL_DGELU: return launch<BM, BN, WGM, WGN, NSTAGE, MODE, false, false, EPI_MUL_DGELU>(grp, stream);
      case EPI_ADD: return launch<BM, BN, WGM, WGN, NSTAGE, MODE, false, false, EPI_ADD>(grp, stream);
      default: break;
    }
  } else if (g.a_t && g.b_t && g.epi == EPI_ACCUM_F32) {
    return launch<BM, BN, WGM, WGN, NSTAGE, MODE, true, true, EPI_ACCUM_F32>(grp, stream);
  }
  return set_error(HANAYO_EUNSUPPORTED, "gemm_dma: layout/epilogue combination not built");
}

}  // namespace

// Tile configurations: 0 = 256 x 256, 1 = 128 x 128 with an 8-deep buffer ring, 2 = 256 x 128,
// 4 = 128 x 128 with a 4-deep ring (two workgroups fit a CU), 5 = as 4 with 8 wavefronts that split
// the MFMA steps of a K tile, 6 = 256 x 256 with 8 wavefronts (2 x 4, 128 x 64 each: two per SIMD
// that cover each other's stalls), 7, 8 and 9 = the tiles of 6, 2 and 4 with a ring of two 64-wide K tiles
// instead of four 32-wide ones (same bytes in flight, one barrier per 64 of K); 10 and 11 = the tiles of 2 and 4 with
// three 64-wide stages (one workgroup per CU: for launches whose single wavefront per SIMD has nothing else to cover
// a late load).  The others use 4 wavefronts.
void gemm_dma_tile(int config, int& bm, int& bn) {
  bm = (config == 1 || config == 4 || config == 5 || config == 9 || config == 11) ? 128 : 256;
  bn = (config == 0 || config == 6 || config == 7) ? 256 : 128;  // 2, 8 and 10: 256 x 128
}

bool gemm_dma_supported(const GemmArgs& g, int config) {
  const bool combo = (!g.a_t && g.b_t && (g.epi == EPI_NONE || g.epi == EPI_BIAS || g.epi == EPI_BIAS_GELU || g.epi == EPI_BIAS_RES ||
                                             g.epi == EPI_STORE_F32)) ||
                     (!g.a_t && !g.b_t && (g.epi == EPI_NONE || g.epi == EPI_MUL_DGELU || g.epi == EPI_ADD)) ||
                     (g.a_t && g.b_t && g.epi == EPI_ACCUM_F32);
  int bm, bn;
  gemm_dma_tile(config, bm, bn);
  // lane offsets are 32-bit byte offsets from the tile origin
  const int bk = config >= 7 ? 64 : kBK;
  const long span_a = (long)(g.a_t ? bk : bm) * g.lda * 2, span_b = (long)(g.b_t ? bk : bn) * g.ldb * 2;
  return combo && g.M % bm == 0 && g.N % bn == 0 && g.K % bk == 0 && g.K >= bk && g.lda % 8 == 0 && g.ldb % 8 == 0 &&
         g.ldc % 4 == 0 && span_a < (1L << 31) && span_b < (1L << 31);
}

// The problems of a group share layout and epilogue (those of gs[0]); each must pass gemm_dma_supported.
int gemm_dma_group(const GemmArgs* gs, int count, int config, hipStream_t stream) {
  if (count < 1 || count > kMaxGroup) return set_error(HANAYO_EINVAL, "gemm_dma: group of %d", count);
  DmaGemmGroup grp{};
  grp.count = count;
  for (int i = 0; i < count; ++i) {
    const GemmArgs& g = gs[i];
    if (!gemm_dma_supported(g, config) || g.a_t != gs[0].a_t || g.b_t != gs[0].b_t || g.epi != gs[0].epi)
      return set_error(HANAYO_EUNSUPPORTED, "gemm_dma: shape not supported");
    DmaGemm& p = grp.prob[i];
    p.A = (const bf16*)g.A; p.B = (const bf16*)g.B; p.C = (bf16*)g.C; p.Cf = (float*)g.C;
    p.bias = (const bf16*)g.bias; p.aux = (const bf16*)g.aux; p.aux_out = (bf16*)g.aux_out;
    p.M = g.M; p.N = g.N; p.K = g.K; p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc;
    p.colsum = g.b_t ? g.colsum : nullptr;
  }
  const GemmArgs& g = gs[0];
  switch (config) {
    case 0: return launch_layout<256, 256, 2, 2, 4, 0>(g, grp, stream);
    case 1: return launch_layout<128, 128, 2, 2, 8, 1>(g, grp, stream);  // 128 KiB LDS: one workgroup per CU
    case 4: return launch_layout<128, 128, 2, 2, 4, 1>(g, grp, stream);  // 64 KiB LDS: two per CU
    case 5: return launch_layout<128, 128, 2, 2, 4, 2>(g, grp, stream);
    case 6: return launch_layout<256, 256, 2, 4, 4, 0>(g, grp, stream);  // 8 wavefronts, 128 x 64 each
    case 7: return launch_layout<256, 256, 2, 4, 2, 0>(g, grp, stream);  // as 6 with two stages of 64-wide K tiles
    case 8: return launch_layout<256, 128, 2, 2, 2, 0>(g, grp, stream);  // as 2 with two stages of 64-wide K tiles
    case 9: return launch_layout<128, 128, 2, 2, 2, 0>(g, grp, stream);  // 128 x 128 likewise (two workgroups per CU)
    case 10: return launch_layout<256, 128, 2, 2, 3, 3>(g, grp, stream);  // as 8 with three stages (144 KiB): one more tile of look-ahead
    case 11: return launch_layout<128, 128, 2, 2, 3, 3>(g, grp, stream);  // 128 x 128, three 64-wide stages (96 KiB, one workgroup per CU)
    default: return launch_layout<256, 128, 2, 2, 4, 0>(g, grp, stream);
  }
}

int gemm_dma(const GemmArgs& g, int config, hipStream_t stream) { return gemm_dma_group(&g, 1, config, stream); }

}  // namespace k
}  // namespace hanayo
