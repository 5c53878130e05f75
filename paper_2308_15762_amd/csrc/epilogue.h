// GEMM epilogues, shared by the ALU and the MFMA GEMM kernels.
#pragma once

#include "device_util.h"
#include "kernels.h"

namespace hanayo {
namespace k {

template <typename T>
struct EpiParams {
  T* C;
  float* Cf;  // EPI_ACCUM_F32 target
  const T* bias;
  const T* aux;
  T* aux_out;
  int ldc;
};

// One output element (m, n) with accumulator value `acc`.
template <typename T, int EPI>
__device__ __forceinline__ void epilogue_one(const EpiParams<T>& p, int m, int n, float acc) {
  const size_t at = (size_t)m * p.ldc + n;
  if constexpr (EPI == EPI_NONE) {
    st(p.C + at, acc);
  } else if constexpr (EPI == EPI_BIAS) {
    st(p.C + at, acc + ld(p.bias + n));
  } else if constexpr (EPI == EPI_BIAS_GELU) {
    const float h = acc + ld(p.bias + n);
    st(p.aux_out + at, h);
    st(p.C + at, gelu_f(h));
  } else if constexpr (EPI == EPI_BIAS_RES) {
    st(p.C + at, acc + ld(p.bias + n) + ld(p.aux + at));
  } else if constexpr (EPI == EPI_MUL_DGELU) {
    st(p.C + at, acc * gelu_grad_f(ld(p.aux + at)));
  } else if constexpr (EPI == EPI_ADD) {
    st(p.C + at, acc + ld(p.aux + at));
  } else if constexpr (EPI == EPI_STORE_F32) {
    p.Cf[at] = acc;
  } else {
    p.Cf[at] += acc;
  }
}

}  // namespace k
}  // namespace hanayo
