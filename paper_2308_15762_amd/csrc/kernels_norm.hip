// LayerNorm forward / backward, column sums (bias gradients) and the partial-sum
// finaliser.  All of them stream [T][H]-shaped tensors once and are bound by HBM
// bandwidth: one wavefront owns a whole row, lanes read 8-element vectors so
// that a wavefront touches 1 KiB (bf16) of contiguous memory per load, row
// statistics are wavefront butterfly reductions, and per-column sums live in
// registers across the rows a wavefront visits.
#include <atomic>

#include "device_util.h"
#include "kernels.h"

namespace hanayo {
namespace k {

namespace {

constexpr int kRowsPerBlock = 4;  // wavefronts per 256-thread block
constexpr int kLnBwdMaxBlocks = 256;  // workgroups of the LN backward = partial rows of gamma/beta sums it writes

// ------------------------------------------------------------------ LN forward
// NV = vectors of 8 per lane kept in registers (H <= 64 * 8 * NV).
template <typename T, int NV>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const T* __restrict__ x, const T* __restrict__ gamma,
                                                     const T* __restrict__ beta, T* __restrict__ out,
                                                     float2* __restrict__ stats, T* __restrict__ copy_out, int rows,
                                                     int H, float eps) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (row >= rows) return;
  const T* xr = x + (size_t)row * H;
  float v[NV][8];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = (i * 64 + lane) * 8;
    if (c < H) {
      load8(xr + c, v[i]);
#pragma unroll
      for (int j = 0; j < 8; ++j) sum += v[i][j];
    }
  }
  const float mean = wave_sum(sum) / (float)H;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = (i * 64 + lane) * 8;
    if (c < H) {
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
    if (c < H) {
      if (copy_out) store8(copy_out + (size_t)row * H + c, v[i]);
      float g[8], b[8], o[8];
      load8(gamma + c, g);
      load8(beta + c, b);
#pragma unroll
      for (int j = 0; j < 8; ++j) o[j] = (v[i][j] - mean) * rstd * g[j] + b[j];
      store8(out + (size_t)row * H + c, o);
    }
  }
}

// ------------------------------------------------------------------ LN backward
// Workgroup = 8 wavefronts; each wavefront walks rows two at a time (both rows' loads are
// issued before either is reduced, which doubles the bytes in flight), its lanes keep the
// column sums of dout*xhat and dout for their columns in registers.  The eight wavefronts are
// combined through LDS (upper four into lower four, then the four into one partial row).
// U = rows in flight per wavefront (2 where the registers allow), WAVES = wavefronts per workgroup
// (8, or 4 for the widest rows whose register arrays need the larger per-wavefront budget).
template <typename T, int NV, int U, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void ln_bwd_kernel(const T* __restrict__ dout, const T* __restrict__ x,
                                                     const T* __restrict__ gamma, const float2* __restrict__ stats,
                                                     const T* __restrict__ addend, T* __restrict__ dz,
                                                     float* __restrict__ partial, int rows, int H) {
  extern __shared__ float red[];  // [4][H]
  constexpr int kBwdWaves = WAVES;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  float acc_g[NV][8], acc_b[NV][8], gm[NV][8];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = (i * 64 + lane) * 8;
#pragma unroll
    for (int j = 0; j < 8; ++j) acc_g[i][j] = acc_b[i][j] = gm[i][j] = 0.f;
    if (c < H) load8(gamma + c, gm[i]);
  }
  const int stride = gridDim.x * kBwdWaves;
  for (int row0 = blockIdx.x * kBwdWaves + wave; row0 < rows; row0 += U * stride) {
    const int row1 = row0 + stride;
    const bool has1 = U == 2 && row1 < rows;
    float xh[U][NV][8], dy[U][NV][8];
    bf16x8 add_raw[U][NV];    // residual addend in storage form, fetched with the other loads
    f32x4 add_f32[U][NV][2];  // (fp32 storage)
    float2 st[U];
    st[0] = stats[row0];
    if (U == 2) st[U - 1] = has1 ? stats[row1] : make_float2(0.f, 0.f);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t base = (size_t)(u ? row1 : row0) * H;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = (i * 64 + lane) * 8;
        if (c < H && (u == 0 || has1)) {
          load8(x + base + c, xh[u][i]);
          load8(dout + base + c, dy[u][i]);
          if (addend) {
            if constexpr (sizeof(T) == 2) {
              add_raw[u][i] = *reinterpret_cast<const bf16x8*>(addend + base + c);
            } else {
              add_f32[u][i][0] = *reinterpret_cast<const f32x4*>(addend + base + c);
              add_f32[u][i][1] = *reinterpret_cast<const f32x4*>(addend + base + c + 4);
            }
          }
        }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (u == 1 && !has1) break;
      const size_t base = (size_t)(u ? row1 : row0) * H;
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = (i * 64 + lane) * 8;
        if (c < H) {
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            xh[u][i][j] = (xh[u][i][j] - st[u].x) * st[u].y;
            acc_g[i][j] += dy[u][i][j] * xh[u][i][j];
            acc_b[i][j] += dy[u][i][j];
            const float dxh = dy[u][i][j] * gm[i][j];
            s1 += dxh;
            s2 += dxh * xh[u][i][j];
          }
        }
      }
      const float c1 = wave_sum(s1) / (float)H;
      const float c2 = wave_sum(s2) / (float)H;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = (i * 64 + lane) * 8;
        if (c < H) {
          float o[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) o[j] = (dy[u][i][j] * gm[i][j] - c1 - xh[u][i][j] * c2) * st[u].y;
          if (addend) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
              if constexpr (sizeof(T) == 2) o[j] += (float)add_raw[u][i][j];
              else o[j] += add_f32[u][i][j >> 2][j & 3];
            }
          }
          store8(dz + base + c, o);
        }
      }
    }
  }
  // combine: pass 0 = gamma sums, pass 1 = beta sums
  for (int pass = 0; pass < 2; ++pass) {
    if (WAVES == 8 && wave >= 4) {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = (i * 64 + lane) * 8;
        if (c < H) {
#pragma unroll
          for (int j = 0; j < 8; ++j) red[(wave - 4) * H + c + j] = pass == 0 ? acc_g[i][j] : acc_b[i][j];
        }
      }
    }
    if (WAVES == 8) __syncthreads();
    if (wave < 4) {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = (i * 64 + lane) * 8;
        if (c < H) {
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            float v = pass == 0 ? acc_g[i][j] : acc_b[i][j];
            if (WAVES == 8) v += red[wave * H + c + j];
            red[wave * H + c + j] = v;
          }
        }
      }
    }
    __syncthreads();
    for (int c = threadIdx.x; c < H; c += blockDim.x) {
      float t = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) t += red[w * H + c];
      partial[(size_t)blockIdx.x * 2 * H + pass * H + c] = t;
    }
    __syncthreads();
  }
}

// out[c] += sum_r partial[r][c] for c in [0, n), without atomics and in a fixed order: a workgroup owns 32
// columns; its 8 row groups each run down every 8th partial row (32 lanes x 4 bytes = one 128-byte line per
// row), the 8 group sums are added in order through LDS, and one thread per column adds the total to `out`.
// Columns >= split go to out1[c - split].  The same bits every run.
constexpr int kFinalizeCols = 32, kFinalizeGroups = 8;
__global__ __launch_bounds__(256) void finalize_kernel(const float* __restrict__ partial, int rows, int ld, int n,
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
#define LAUNCH(NV)                                                                                                 \
  hipLaunchKernelGGL((ln_fwd_kernel<T, NV>), grid, block, 0, stream, (const T*)x, (const T*)gamma, (const T*)beta, \
                     (T*)out, stats, (T*)copy_out, T_, H, eps)
  if (nv <= 1) LAUNCH(1);
  else if (nv <= 2) LAUNCH(2);
  else if (nv <= 4) LAUNCH(4);
  else LAUNCH(8);
#undef LAUNCH
  return check_launch("ln_forward");
}

template <typename T>
int ln_backward_t(const void* dout, const void* x, const void* gamma, const float2* stats, const void* addend, void* dz,
                  float* dgamma, float* dbeta, float* partial, int T_, int H, hipStream_t stream) {
  const int nv = (H + 511) / 512;
  const int waves = nv <= 4 ? 8 : 4;
  int blocks = (T_ + waves - 1) / waves;
  if (blocks > kLnBwdMaxBlocks) blocks = kLnBwdMaxBlocks;  // a wavefront then walks several rows
  const size_t lds = (size_t)4 * H * sizeof(float);
#define LAUNCH(NV, U, WAVES)                                                                                   \
  hipLaunchKernelGGL((ln_bwd_kernel<T, NV, U, WAVES>), dim3(blocks), dim3(WAVES * 64), lds, stream, (const T*)dout, \
                     (const T*)x, (const T*)gamma, stats, (const T*)addend, (T*)dz, partial, T_, H)
  if (nv <= 1) LAUNCH(1, 2, 8);
  else if (nv <= 2) LAUNCH(2, 2, 8);
  else if (nv <= 4) LAUNCH(4, 1, 8);
  else LAUNCH(8, 1, 4);
#undef LAUNCH
  int rc = check_launch("ln_backward");
  if (rc) return rc;
  hipLaunchKernelGGL(finalize_kernel, dim3((2 * H + kFinalizeCols - 1) / kFinalizeCols), dim3(256), 0, stream, partial, blocks,
                     2 * H, 2 * H, dgamma, dbeta, H);
  return check_launch("ln_backward finalize");
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
  hipLaunchKernelGGL(finalize_kernel, dim3((N + kFinalizeCols - 1) / kFinalizeCols), dim3(256), 0, stream, partial, gy, N, N,
                     out, out, N);
  return check_launch("colsum finalize");
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
             ? ln_backward_t<bf16>(dout, x, gamma, stats, addend, dz, dgamma, dbeta, partial, T_, H, stream)
             : ln_backward_t<float>(dout, x, gamma, stats, addend, dz, dgamma, dbeta, partial, T_, H, stream);
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
