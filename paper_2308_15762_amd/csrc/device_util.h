// Device-side helpers shared by the HIP kernels: storage types, 8-wide row
// access, wavefront (64-lane) reductions, GELU.
#pragma once

#include <hip/hip_runtime.h>

namespace hanayo {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kWave = 64;

// Eight consecutive elements <-> eight floats.
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
  const f32x4 a = *reinterpret_cast<const f32x4*>(p);
  const f32x4 b = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    v[i] = a[i];
    v[4 + i] = b[i];
  }
}
__device__ __forceinline__ void load8(const bf16* p, float (&v)[8]) {
  const bf16x8 a = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = (float)a[i];
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
  f32x4 a, b;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = v[i];
    b[i] = v[4 + i];
  }
  *reinterpret_cast<f32x4*>(p) = a;
  *reinterpret_cast<f32x4*>(p + 4) = b;
}
__device__ __forceinline__ void store8(bf16* p, const float (&v)[8]) {
  bf16x8 a;
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = (bf16)v[i];
  *reinterpret_cast<bf16x8*>(p) = a;
}

__device__ __forceinline__ float ld(const float* p) { return *p; }
__device__ __forceinline__ float ld(const bf16* p) { return (float)*p; }
__device__ __forceinline__ void st(float* p, float v) { *p = v; }
__device__ __forceinline__ void st(bf16* p, float v) { *p = (bf16)v; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

// Workgroup -> output tile, XCD-aware.  The dispatcher hands consecutive workgroup ids to the chip's
// 8 XCDs in turn, and each XCD has an L2 of its own, so workgroup w runs on XCD w % 8 as that XCD's
// (w / 8)-th.  Each XCD therefore gets one contiguous run of tile numbers, and tile numbers walk the
// tile grid in bands of kTileBand tile rows, column by column within a band: the workgroups resident
// on one XCD at a time then cover a compact patch of the output and share their operand panels in
// that L2 instead of each XCD fetching every panel.  Any bijection is correct; this one is fast.
constexpr int kXcds = 8, kTileBand = 8;
__device__ __forceinline__ void xcd_tile(int w, int tiles_m, int tiles_n, int& tm, int& tn) {
  const int total = tiles_m * tiles_n, per = total / kXcds, rem = total % kXcds;
  const int xcd = w % kXcds;
  const int t = xcd * per + (xcd < rem ? xcd : rem) + w / kXcds;
  const int band = t / (kTileBand * tiles_n), first = band * kTileBand;
  const int rows = tiles_m - first < kTileBand ? tiles_m - first : kTileBand;
  const int r = t - band * kTileBand * tiles_n;
  tm = first + r % rows;
  tn = r / rows;
}

// GELU(h) = h/2 (1 + erf(h / sqrt 2)) and its derivative Phi(h) + h phi(h).
__device__ __forceinline__ float gelu_f(float h) { return 0.5f * h * (1.0f + erff(h * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float h) {
  const float cdf = 0.5f * (1.0f + erff(h * 0.70710678118654752f));
  const float pdf = 0.39894228040143268f * __expf(-0.5f * h * h);
  return cdf + h * pdf;
}

// The same two functions from one exponential and a rational erfc approximation
// (Abramowitz & Stegun 7.1.26, absolute error of erf below 1.5e-7): used in the
// bf16 MFMA epilogues, where the result is rounded to bf16 anyway.
//   Phi(|h|) = 1 - 0.5 t (a1 + t (a2 + t (a3 + t (a4 + t a5)))) exp(-h^2 / 2),  t = 1 / (1 + p |h| / sqrt 2)
__device__ __forceinline__ void phi_fast(float h, float& cdf, float& pdf) {
  const float ah = fabsf(h);
  const float t = __frcp_rn(1.0f + 0.3275911f * 0.70710678118654752f * ah);
  const float e = exp2f(-0.72134752044448170f * h * h);  // exp(-h^2 / 2)
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  const float tail = 0.5f * poly * e;  // 1 - Phi(|h|)
  cdf = h >= 0.f ? 1.0f - tail : tail;
  pdf = 0.39894228040143268f * e;
}
__device__ __forceinline__ float gelu_fast(float h) {
  float cdf, pdf;
  phi_fast(h, cdf, pdf);
  return h * cdf;
}
__device__ __forceinline__ float gelu_grad_fast(float h) {
  float cdf, pdf;
  phi_fast(h, cdf, pdf);
  return cdf + h * pdf;
}

}  // namespace hanayo
