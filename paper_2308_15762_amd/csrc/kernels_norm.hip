// LayerNorm forward / backward, column sums (bias gradients) and the partial-sum
// finaliser.  All of them stream [T][H]-shaped tensors once and are bound by HBM
// bandwidth: lanes read 8-element vectors so that a wavefront touches 1 KiB (bf16)
// of contiguous memory per load, row statistics are wavefront butterfly
// reductions (forward: one wavefront owns a whole row; backward: the wavefronts
// that share a row exchange two sums through LDS), and per-column sums live in
// registers across the rows a wavefront visits.
#include <atomic>

#include "device_util.h"
#include "kernels.h"

namespace hanayo {
namespace k {

namespace {

constexpr int kRowsPerBlock = 4;  // wavefronts per 256-thread block
constexpr int kLnBwdMaxBlocks = kLnPartialRows;  // workgroups of the LN backward = partial rows of gamma/beta sums it writes

// Eight consecutive elements in storage form: what a load that is still in flight occupies (for bf16 a
// quarter of the registers of eight floats).
template <typename T>
struct Raw8;
template <>
struct Raw8<bf16> {
  bf16x8 v;
  __device__ __forceinline__ void load(const bf16* p) { v = *reinterpret_cast<const bf16x8*>(p); }
  __device__ __forceinline__ float get(int j) const { return (float)v[j]; }
};
template <>
struct Raw8<float> {
  f32x4 v[2];
  __device__ __forceinline__ void load(const float* p) {
    v[0] = *reinterpret_cast<const f32x4*>(p);
    v[1] = *reinterpret_cast<const f32x4*>(p + 4);
  }
  __device__ __forceinline__ float get(int j) const { return v[j >> 2][j & 3]; }
};

// ------------------------------------------------------------------ LN forward
// NV = vectors of 8 per lane kept in registers (H <= 64 * 8 * NV).  FULL: H == 512 * NV exactly, so no lane's
// vector falls outside the row: the column guards vanish at compile time and a row's loads are one straight run
// of instructions (a guarded load sits in a branch of its own, and the waits the compiler places at the joins
// serialise the loads of a row).
template <typename T, int NV, bool FULL>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const T* __restrict__ x, const T* __restrict__ gamma,
                                                     const T* __restrict__ beta, T* __restrict__ out,
                                                     float2* __restrict__ stats, T* __restrict__ copy_out, int rows,
                                                     int H, float eps) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (row >= rows) return;
  const T* xr = x + (size_t)row * H;
  float v[NV][8];
  Raw8<T> g[NV], b[NV];  // fetched with the row (storage form), so that the last step waits for nothing
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = (i * 64 + lane) * 8;
    if (FULL || c < H) load8(xr + c, v[i]);
  }
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = (i * 64 + lane) * 8;
    if (FULL || c < H) {
      g[i].load(gamma + c);
      b[i].load(beta + c);
    }
  }
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = (i * 64 + lane) * 8;
    if (FULL || c < H) {
#pragma unroll
      for (int j = 0; j < 8; ++j) sum += v[i][j];
    }
  }
  const float mean = wave_sum(sum) / (float)H;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = (i * 64 + lane) * 8;
    if (FULL || c < H) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float dlt = v[i][j] - mean;
        sq += dlt * dlt;
      }
    }
  }
  const float rstd = rsqrtf(wave_sum(sq) / (float)H + eps);
  if (lane == 0) stats[row] = make_float2(mean, rstd);
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = (i * 64 + lane) * 8;
    if (FULL || c < H) {
      if (copy_out) store8(copy_out + (size_t)row * H + c, v[i]);
      float o[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) o[j] = (v[i][j] - mean) * rstd * g[i].get(j) + b[i].get(j);
      store8(out + (size_t)row * H + c, o);
    }
  }
}

// ------------------------------------------------------------------ LN backward
// A row is shared by RS wavefronts: lane l of part p owns vector p of the row's 512-element groups (8 columns
// from (p * 64 + l) * 8), so a lane keeps 8 columns of x, dout, gamma and of the two column sums whatever the
// width of the row, and the registers left over go to the NEXT row: every wavefront fetches its slice of the
// row after (storage form) before it reduces the current one, so loads, arithmetic and stores of neighbouring
// rows overlap.  (One wavefront per row holds the whole row and both column sums in registers: at 4096
// columns that is one wavefront per SIMD and nothing in flight while it computes.)  A workgroup of RS * RG
// wavefronts walks RG rows at a time.  The two row sums cross the RS parts through LDS (double-buffered slots:
// one barrier per row); the parts are added in a fixed order and every part computes the same totals.  The
// gamma / beta column sums stay in registers across the rows a wavefront walks; at the end the RG row groups
// are added in order through LDS and the workgroup writes one partial row [gamma sums | beta sums].
// FULL: H == 512 * RS, no column guard.
template <typename T, int RS, int RG, bool FULL>
__global__ __launch_bounds__(RS * RG * 64) void ln_bwd_kernel(const T* __restrict__ dout, const T* __restrict__ x,
                                                              const T* __restrict__ gamma, const float2* __restrict__ stats,
                                                              const T* __restrict__ addend, T* __restrict__ dz,
                                                              float* __restrict__ partial, int rows, int H) {
  extern __shared__ float red[];                 // [RG][2 * H] for the column sums; before that the row-sum exchange
  float2* xch = reinterpret_cast<float2*>(red);  // [2][RG][RS]
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int rg = wave / RS, part = wave % RS;
  const int col = (part * 64 + lane) * 8;
  const bool inside = FULL || col < H;
  float acc_g[8], acc_b[8], gm[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc_g[j] = acc_b[j] = gm[j] = 0.f;
  if (inside) load8(gamma + col, gm);
  Raw8<T> nx, ndy, nadd;
  float2 nst = make_float2(0.f, 0.f);
  auto fetch = [&](int row) {
    if (row < rows && inside) {
      nst = stats[row];
      const size_t at = (size_t)row * H + col;
      nx.load(x + at);
      ndy.load(dout + at);
      if (addend) nadd.load(addend + at);
    }
  };
  const int step = gridDim.x * RG;
  fetch(blockIdx.x * RG + rg);
  int it = 0;
  for (int first = blockIdx.x * RG; first < rows; first += step, ++it) {  // the same trip count for every wavefront
    const int row = first + rg;
    const bool valid = row < rows && inside;
    const float2 st = nst;
    float xh[8], dy[8];
    const Raw8<T> add = nadd;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      xh[j] = valid ? (nx.get(j) - st.x) * st.y : 0.f;
      dy[j] = valid ? ndy.get(j) : 0.f;
    }
    fetch(row + step);
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      acc_g[j] += dy[j] * xh[j];
      acc_b[j] += dy[j];
      const float dxh = dy[j] * gm[j];
      s1 += dxh;
      s2 += dxh * xh[j];
    }
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    if (RS > 1) {
      float2* slot = xch + ((it & 1) * RG + rg) * RS;
      if (lane == 0) slot[part] = make_float2(s1, s2);
      __syncthreads();
      s1 = s2 = 0.f;
#pragma unroll
      for (int p = 0; p < RS; ++p) {
        const float2 t = slot[p];
        s1 += t.x;
        s2 += t.y;
      }
    }
    if (valid) {
      const float c1 = s1 / (float)H, c2 = s2 / (float)H;
      float o[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        o[j] = (dy[j] * gm[j] - c1 - xh[j] * c2) * st.y;
        if (addend) o[j] += add.get(j);
      }
      store8(dz + (size_t)row * H + col, o);
    }
  }
  __syncthreads();  // the exchange slots are done with; the same memory now takes the column sums
  if (inside) {
    f32x4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      v[0][j] = acc_g[j];
      v[1][j] = acc_g[4 + j];
      v[2][j] = acc_b[j];
      v[3][j] = acc_b[4 + j];
    }
    float* mine = red + (size_t)rg * 2 * H + col;
    *reinterpret_cast<f32x4*>(mine) = v[0];
    *reinterpret_cast<f32x4*>(mine + 4) = v[1];
    *reinterpret_cast<f32x4*>(mine + H) = v[2];
    *reinterpret_cast<f32x4*>(mine + H + 4) = v[3];
  }
  __syncthreads();
  for (int c = threadIdx.x; c < 2 * H; c += RS * RG * 64) {
    float t = 0.f;
#pragma unroll
    for (int g = 0; g < RG; ++g) t += red[g * 2 * H + c];
    partial[(size_t)blockIdx.x * 2 * H + c] = t;
  }
}

// out[c] += sum_r partial[r][c] for c in [0, n), without atomics and in a fixed order: a workgroup owns 32
// columns; its 32 row groups each run down every 32nd partial row (32 lanes x 4 bytes = one 128-byte line per
// row; with 256 partial rows that is 8 loads per thread, all in flight at once), the group sums are added in
// order through LDS, and one thread per column adds the total to `out`.
// Columns >= split go to out1[c - split].  The same bits every run.
constexpr int kFinalizeCols = 32, kFinalizeGroups = 32;
__global__ __launch_bounds__(kFinalizeCols * kFinalizeGroups) void finalize_kernel(const float* __restrict__ partial, int rows, int ld, int n,
                                                       float* __restrict__ out0, float* __restrict__ out1, int split) {
  __shared__ float red[kFinalizeGroups][kFinalizeCols];
  const int cl = threadIdx.x % kFinalizeCols, rg = threadIdx.x / kFinalizeCols;
  const int c = blockIdx.x * kFinalizeCols + cl;
  float t = 0.f;
  if (c < n) {
#pragma unroll 8
    for (int r = rg; r < rows; r += kFinalizeGroups) t += partial[(size_t)r * ld + c];
  }
  red[rg][cl] = t;
  __syncthreads();
  if (rg == 0 && c < n) {
    float total = 0.f;
#pragma unroll
    for (int g = 0; g < kFinalizeGroups; ++g) total += red[g][cl];
    float* dst = c < split ? out0 + c : out1 + (c - split);
    *dst += total;
  }
}

// Several finaliser jobs in one launch (blockIdx.y = job): the gamma/beta sums of all the LayerNorms of a
// chunk's backward pass, whose partial rows wait in slots of their own until the pass is over.
struct FinalizeJobs {
  FinalizeJob job[kMaxFinalizeJobs];
};
__global__ __launch_bounds__(kFinalizeCols * kFinalizeGroups) void finalize_group_kernel(FinalizeJobs jobs) {
  const FinalizeJob j = jobs.job[blockIdx.y];
  if ((int)blockIdx.x * kFinalizeCols >= j.n) return;  // uniform over the workgroup: jobs may differ in width
  __shared__ float red[kFinalizeGroups][kFinalizeCols];
  const int cl = threadIdx.x % kFinalizeCols, rg = threadIdx.x / kFinalizeCols;
  const int c = blockIdx.x * kFinalizeCols + cl;
  float t = 0.f;
  if (c < j.n) {
#pragma unroll 8
    for (int r = rg; r < j.rows; r += kFinalizeGroups) t += j.partial[(size_t)r * j.ld + c];
  }
  red[rg][cl] = t;
  __syncthreads();
  if (rg == 0 && c < j.n) {
    float total = 0.f;
#pragma unroll
    for (int g = 0; g < kFinalizeGroups; ++g) total += red[g][cl];
    float* dst = c < j.split ? j.out0 + c : j.out1 + (c - j.split);
    *dst += total;
  }
}

// ------------------------------------------------------------------ column sums
// Block = 8 row groups x 32 lanes, each lane owning 8 consecutive columns.
template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(const T* __restrict__ in, int rows, int N,
                                                     float* __restrict__ partial) {
  __shared__ float red[8][256 + 8];
  const int cl = (threadIdx.x & 31) * 8;
  const int rg = threadIdx.x >> 5;
  const int c = blockIdx.x * 256 + cl;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (c < N) {
    for (int r = blockIdx.y * 8 + rg; r < rows; r += gridDim.y * 8) {
      float v[8];
      load8(in + (size_t)r * N + c, v);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] += v[j];
    }
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) red[rg][cl + j] = acc[j];
  __syncthreads();
  const int cc = blockIdx.x * 256 + threadIdx.x;
  if (cc < N) {
    float t = 0.f;
#pragma unroll
    for (int g = 0; g < 8; ++g) t += red[g][threadIdx.x];
    partial[(size_t)blockIdx.y * N + cc] = t;
  }
}

template <typename T>
int ln_forward_t(const void* x, const void* gamma, const void* beta, void* out, float2* stats, void* copy_out, int T_,
                 int H, float eps, hipStream_t stream) {
  const dim3 grid((T_ + kRowsPerBlock - 1) / kRowsPerBlock), block(256);
  const int nv = (H + 511) / 512;
#define LAUNCH(NV, FULL)                                                                                              \
  hipLaunchKernelGGL((ln_fwd_kernel<T, NV, FULL>), grid, block, 0, stream, (const T*)x, (const T*)gamma, (const T*)beta, \
                     (T*)out, stats, (T*)copy_out, T_, H, eps)
  if (H % 512 == 0) {  // every vector of every lane is inside the row
    switch (nv) {
      case 1: LAUNCH(1, true); break;
      case 2: LAUNCH(2, true); break;
      case 3: LAUNCH(3, true); break;
      case 4: LAUNCH(4, true); break;
      case 5: LAUNCH(5, true); break;
      case 6: LAUNCH(6, true); break;
      case 7: LAUNCH(7, true); break;
      default: LAUNCH(8, true); break;
    }
  } else if (nv <= 1) LAUNCH(1, false);
  else if (nv <= 2) LAUNCH(2, false);
  else if (nv <= 4) LAUNCH(4, false);
  else LAUNCH(8, false);
#undef LAUNCH
  return check_launch("ln_forward");
}

int launch_finalize(const float* partial, int rows, int ld, int n, float* out0, float* out1, int split, hipStream_t stream,
                    const char* what) {
  hipLaunchKernelGGL(finalize_kernel, dim3((n + kFinalizeCols - 1) / kFinalizeCols), dim3(kFinalizeCols * kFinalizeGroups), 0,
                     stream, partial, rows, ld, n, out0, out1, split);
  return check_launch(what);
}

template <typename T>
int ln_backward_t(const void* dout, const void* x, const void* gamma, const float2* stats, const void* addend, void* dz,
                  float* dgamma, float* dbeta, float* partial, int T_, int H, hipStream_t stream, FinalizeJob* later) {
  const int nv = (H + 511) / 512;  // wavefronts that share a row; 16 wavefronts (15 or 14 where nv does not divide 16)
  const int rg = 16 / nv;          // per workgroup walk rg rows at a time
  int blocks = (T_ + rg - 1) / rg;
  if (blocks > kLnBwdMaxBlocks) blocks = kLnBwdMaxBlocks;  // a workgroup then walks several groups of rows
  size_t lds = (size_t)rg * 2 * H * sizeof(float);         // at most 16 / nv * 2 * 512 nv * 4 = 64 KiB
  if (lds < 1024) lds = 1024;                              // the row-sum exchange slots
#define LAUNCH(RS, RG)                                                                                                \
  do {                                                                                                                \
    if (H == 512 * RS)                                                                                                \
      hipLaunchKernelGGL((ln_bwd_kernel<T, RS, RG, true>), dim3(blocks), dim3(RS * RG * 64), lds, stream, (const T*)dout, \
                         (const T*)x, (const T*)gamma, stats, (const T*)addend, (T*)dz, partial, T_, H);              \
    else                                                                                                              \
      hipLaunchKernelGGL((ln_bwd_kernel<T, RS, RG, false>), dim3(blocks), dim3(RS * RG * 64), lds, stream, (const T*)dout, \
                         (const T*)x, (const T*)gamma, stats, (const T*)addend, (T*)dz, partial, T_, H);              \
  } while (0)
  switch (nv) {
    case 1: LAUNCH(1, 16); break;
    case 2: LAUNCH(2, 8); break;
    case 3: LAUNCH(3, 5); break;
    case 4: LAUNCH(4, 4); break;
    case 5: LAUNCH(5, 3); break;
    case 6: LAUNCH(6, 2); break;
    case 7: LAUNCH(7, 2); break;
    default: LAUNCH(8, 2); break;
  }
#undef LAUNCH
  int rc = check_launch("ln_backward");
  if (rc) return rc;
  if (later) {  // the caller sums the partial rows later, with others (finalize_group)
    *later = FinalizeJob{partial, blocks, 2 * H, 2 * H, dgamma, dbeta, H};
    return HANAYO_OK;
  }
  return launch_finalize(partial, blocks, 2 * H, 2 * H, dgamma, dbeta, H, stream, "ln_backward finalize");
}

template <typename T>
int colsum_t(const void* in, int T_, int N, float* out, float* partial, hipStream_t stream) {
  int gy = (T_ + 31) / 32;
  if (gy > 64) gy = 64;
  if (gy < 1) gy = 1;
  const dim3 grid((N + 255) / 256, gy);
  hipLaunchKernelGGL((colsum_kernel<T>), grid, dim3(256), 0, stream, (const T*)in, T_, N, partial);
  int rc = check_launch("colsum");
  if (rc) return rc;
  return launch_finalize(partial, gy, N, N, out, out, N, stream, "colsum finalize");
}

}  // namespace

int check_launch(const char* what) {
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(HANAYO_EHIP, "%s: %s", what, hipGetErrorString(e));
  return HANAYO_OK;
}

int ln_forward(int dtype, const void* x, const void* gamma, const void* beta, void* out, float2* stats, void* copy_out,
               int T_, int H, float eps, hipStream_t stream) {
  if (T_ < 1 || H < 8 || H % 8 || H > 4096) return set_error(HANAYO_EUNSUPPORTED, "ln_forward: H=%d (need multiple of 8, <= 4096)", H);
  return dtype == HANAYO_BF16 ? ln_forward_t<bf16>(x, gamma, beta, out, stats, copy_out, T_, H, eps, stream)
                              : ln_forward_t<float>(x, gamma, beta, out, stats, copy_out, T_, H, eps, stream);
}

int ln_backward(int dtype, const void* dout, const void* x, const void* gamma, const float2* stats, const void* addend,
                void* dz, float* dgamma, float* dbeta, float* partial, int T_, int H, hipStream_t stream) {
  if (T_ < 1 || H < 8 || H % 8 || H > 4096) return set_error(HANAYO_EUNSUPPORTED, "ln_backward: H=%d (need multiple of 8, <= 4096)", H);
  return dtype == HANAYO_BF16
             ? ln_backward_t<bf16>(dout, x, gamma, stats, addend, dz, dgamma, dbeta, partial, T_, H, stream, nullptr)
             : ln_backward_t<float>(dout, x, gamma, stats, addend, dz, dgamma, dbeta, partial, T_, H, stream, nullptr);
}

int ln_backward_deferred(int dtype, const void* dout, const void* x, const void* gamma, const float2* stats,
                         const void* addend, void* dz, float* dgamma, float* dbeta, float* partial, int T_, int H,
                         hipStream_t stream, FinalizeJob* job) {
  if (T_ < 1 || H < 8 || H % 8 || H > 4096) return set_error(HANAYO_EUNSUPPORTED, "ln_backward: H=%d (need multiple of 8, <= 4096)", H);
  if (!job) return set_error(HANAYO_EINVAL, "ln_backward_deferred: no job to fill in");
  return dtype == HANAYO_BF16
             ? ln_backward_t<bf16>(dout, x, gamma, stats, addend, dz, dgamma, dbeta, partial, T_, H, stream, job)
             : ln_backward_t<float>(dout, x, gamma, stats, addend, dz, dgamma, dbeta, partial, T_, H, stream, job);
}

int finalize_group(const FinalizeJob* jobs, int count, hipStream_t stream) {
  for (int first = 0; first < count; first += kMaxFinalizeJobs) {
    const int n = count - first < kMaxFinalizeJobs ? count - first : kMaxFinalizeJobs;
    FinalizeJobs batch{};
    int widest = 0;
    for (int i = 0; i < n; ++i) {
      batch.job[i] = jobs[first + i];
      if (batch.job[i].n > widest) widest = batch.job[i].n;
    }
    if (widest < 1) continue;
    hipLaunchKernelGGL(finalize_group_kernel, dim3((widest + kFinalizeCols - 1) / kFinalizeCols, n),
                       dim3(kFinalizeCols * kFinalizeGroups), 0, stream, batch);
    const int rc = check_launch("finalize_group");
    if (rc) return rc;
  }
  return HANAYO_OK;
}

int colsum_add(int dtype, const void* in, int T_, int N, float* out, float* partial, hipStream_t stream) {
  if (T_ < 1 || N < 8 || N % 8) return set_error(HANAYO_EUNSUPPORTED, "colsum: N=%d (need multiple of 8)", N);
  return dtype == HANAYO_BF16 ? colsum_t<bf16>(in, T_, N, out, partial, stream)
                              : colsum_t<float>(in, T_, N, out, partial, stream);
}

namespace {
// Plain copy, 16 bytes per lane per step, grid-stride: the stash copy of a chunk's input, and the
// kernel of known traffic against which the HBM counters are scaled.
__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}
}  // namespace

int copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t stream, int max_workgroups) {
  if (bytes % 16 || ((uintptr_t)dst | (uintptr_t)src) % 16) return set_error(HANAYO_EINVAL, "copy: 16-byte granularity");
  const size_t n16 = bytes / 16;
  if (!n16) return HANAYO_OK;
  const size_t want = (n16 + 255) / 256;
  const size_t cap = max_workgroups > 0 ? (size_t)max_workgroups : (size_t)256 * 16;  // default: up to 16 workgroups per CU
  const unsigned blocks = (unsigned)(want < cap ? want : cap);
  hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, stream, (const uint4*)src, (uint4*)dst, n16);
  return check_launch("copy");
}

}  // namespace k
}  // namespace hanayo

// ---------------------------------------------------------------------------------------------
// LayerNorm backward for callers that cannot allocate and have no workspace to pass: the partial
// rows of the gamma/beta sums live in a fixed array of the library's own, one copy per GPU.
namespace {
constexpr int kStaticMaxHidden = 4096;
constexpr size_t kStaticScratchFloats = (size_t)hanayo::k::kLnBwdMaxBlocks * 2 * kStaticMaxHidden;  // 8 MiB
static __device__ __align__(256) float scratch[kStaticScratchFloats];

// Device address of `scratch` on each GPU: the array's name is only a host-side handle, so the
// address is looked up once per device (with that device current) and kept.
constexpr int kMaxDevices = 64;
std::atomic<float*> scratch_ptr[kMaxDevices];

int static_scratch(float** out) {
  int device = -1;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) return hanayo::set_error(HANAYO_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
  if (device < 0 || device >= kMaxDevices) return hanayo::set_error(HANAYO_EUNSUPPORTED, "device index %d", device);
  float* p = scratch_ptr[device].load(std::memory_order_acquire);
  if (!p) {
    void* sym = nullptr;
    e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !sym)
      return hanayo::set_error(HANAYO_EHIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    p = static_cast<float*>(sym);
    scratch_ptr[device].store(p, std::memory_order_release);  // two racing threads store the same address
  }
  *out = p;
  return HANAYO_OK;
}
}  // namespace

extern "C" int hanayo_op_layernorm_backward_static(int dtype, const void* dout, const void* x, const void* gamma,
                                                   const float* stats, const void* addend, void* dz, float* dgamma,
                                                   float* dbeta, int rows, int hidden, void* hip_stream) {
  if (dtype != HANAYO_FP32 && dtype != HANAYO_BF16)
    return hanayo::set_error(HANAYO_EINVAL, "dtype must be HANAYO_FP32 or HANAYO_BF16");
  if (!dout || !x || !gamma || !stats || !dz || !dgamma || !dbeta || rows < 1)
    return hanayo::set_error(HANAYO_EINVAL, "op_layernorm_backward_static: bad argument");
  if (hidden < 8 || hidden % 8 || hidden > kStaticMaxHidden)
    return hanayo::set_error(HANAYO_EINVAL, "op_layernorm_backward_static: hidden = %d, the fixed scratch array covers "
                             "multiples of 8 up to %d", hidden, kStaticMaxHidden);
  float* partial = nullptr;
  if (int rc = static_scratch(&partial)) return rc;
  // every partial row the finaliser reads is written by the backward kernel first: nothing to clear
  return hanayo::k::ln_backward(dtype, dout, x, gamma, reinterpret_cast<const float2*>(stats), addend, dz, dgamma, dbeta,
                                partial, rows, hidden, static_cast<hipStream_t>(hip_stream));
}
