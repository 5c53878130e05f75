// The two ends of the model and the optimizer step: token + position embedding
// (stage 0), softmax cross-entropy over the vocabulary (after the last stage's
// head GEMM) and Adam.  All of them stream their tensors once or twice and are
// bound by HBM bandwidth; rows are read as 8-element vectors, one wavefront
// (embedding) or one workgroup (a vocabulary row) per row.
#include <cmath>

#include "device_util.h"
#include "kernels.h"

namespace hanayo {
namespace k {

namespace {

constexpr int kRowsPerBlock = 4;  // wavefronts per 256-thread block

// x[t][:] = wte[token[t]][:] + wpe[t mod s][:]; a token outside [0, vocab) contributes nothing.
template <typename T>
__global__ __launch_bounds__(256) void embed_fwd_kernel(const T* __restrict__ wte, const T* __restrict__ wpe,
                                                        const int32_t* __restrict__ tokens, T* __restrict__ x, int rows,
                                                        int s, int H, int vocab) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int tok = tokens[row];
  const bool known = tok >= 0 && tok < vocab;
  const T* te = wte + (size_t)(known ? tok : 0) * H;
  const T* pe = wpe + (size_t)(row % s) * H;
  for (int c = lane * 8; c < H; c += 64 * 8) {
    float a[8], b[8];
    load8(pe + c, b);
    if (known) {
      load8(te + c, a);
#pragma unroll
      for (int j = 0; j < 8; ++j) b[j] += a[j];
    }
    store8(x + (size_t)row * H + c, b);
  }
}

// d_wte[token[t]][:] += dx[t][:] without atomics and in a fixed order.  One workgroup per row t; the workgroup of
// the FIRST row that holds a token owns that token's table row for the launch: it lists, in ascending order, the
// rows that hold the same token (ballot + prefix counts, 256 rows at a time), its four wavefronts sum every fourth
// listed row each, and the four partial sums are added to the table row in
// wavefront order.  Workgroups of later occurrences leave at once.  NV = 8-element vectors per lane (H <= 512 NV).
// (the listed rows' loads: 8 in flight per wavefront, fewer for wide rows)
template <typename T, int NV>
__global__ __launch_bounds__(256) void embed_bwd_token_kernel(const int32_t* __restrict__ tokens, const T* __restrict__ dx,
                                                              float* __restrict__ d_wte, int rows, int H, int vocab) {
  __shared__ int list[256];
  __shared__ int cnt[4];
  extern __shared__ float part[];  // [3][H]: partial sums of wavefronts 1..3
  const int row = blockIdx.x;
  const int tok = tokens[row];
  if (tok < 0 || tok >= vocab) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int seen = 0;
  for (int t = threadIdx.x; t < row; t += 256) seen |= tokens[t] == tok;
  if (__syncthreads_or(seen)) return;  // an earlier row owns this token
  float acc[NV][8];
#pragma unroll
  for (int i = 0; i < NV; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;
  for (int base = row; base < rows; base += 256) {
    const int t = base + (int)threadIdx.x;
    const bool hit = t < rows && tokens[t] == tok;
    const unsigned long long mask = __ballot(hit);
    if (lane == 0) cnt[wave] = __popcll(mask);
    __syncthreads();
    int before = 0, n = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      if (w < wave) before += cnt[w];
      n += cnt[w];
    }
    if (hit) list[before + __popcll(mask & ((1ull << lane) - 1ull))] = t;
    __syncthreads();
    // wavefront w takes list entries w, w + 4, w + 8, ...; U of them in flight (fewer for wide rows: registers)
    constexpr int U = NV <= 2 ? 8 : NV <= 4 ? 4 : 2;
    for (int i0 = wave; i0 < n; i0 += 4 * U) {
      bf16x8 raw16[U][NV];
      f32x4 raw32[U][NV][2];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i = i0 + 4 * u;
        if (i < n) {
          const T* src = dx + (size_t)list[i] * H;
#pragma unroll
          for (int v = 0; v < NV; ++v) {
            const int c = (v * 64 + lane) * 8;
            if (c < H) {
              if constexpr (sizeof(T) == 2) {
                raw16[u][v] = *reinterpret_cast<const bf16x8*>(src + c);
              } else {
                raw32[u][v][0] = *reinterpret_cast<const f32x4*>(src + c);
                raw32[u][v][1] = *reinterpret_cast<const f32x4*>(src + c + 4);
              }
            }
          }
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (i0 + 4 * u < n) {
#pragma unroll
          for (int v = 0; v < NV; ++v) {
            if ((v * 64 + lane) * 8 < H) {
#pragma unroll
              for (int j = 0; j < 8; ++j) {
                if constexpr (sizeof(T) == 2) acc[v][j] += (float)raw16[u][v][j];
                else acc[v][j] += raw32[u][v][j >> 2][j & 3];
              }
            }
          }
        }
      }
    }
    __syncthreads();  // the list is rebuilt in the next round
  }
  // wavefronts 1..3 hand their sums to wavefront 0, which adds them in order and updates the table row
  if (wave > 0) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int c = (v * 64 + lane) * 8;
      if (c < H) store8(part + (size_t)(wave - 1) * H + c, acc[v]);
    }
  }
  __syncthreads();
  if (wave == 0) {
    float* out = d_wte + (size_t)tok * H;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int c = (v * 64 + lane) * 8;
      if (c < H) {
        float cur[8];
        load8(out + c, cur);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          float add[8];
          if (w == 0) {
#pragma unroll
            for (int j = 0; j < 8; ++j) add[j] = acc[v][j];
          } else {
            load8(part + (size_t)(w - 1) * H + c, add);
          }
#pragma unroll
          for (int j = 0; j < 8; ++j) cur[j] += add[j];
        }
        store8(out + c, cur);
      }
    }
  }
}

// d_wpe[i][:] += sum over the b sequences of dx[n][i][:], in sequence order.
template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_pos_kernel(const T* __restrict__ dx, float* __restrict__ d_wpe, int b,
                                                            int s, int H) {
  const int vecs = H / 8;
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long)s * vecs) return;
  const int i = (int)(idx / vecs), c = (int)(idx % vecs) * 8;
  float acc[8];
  load8(d_wpe + (size_t)i * H + c, acc);
  for (int n = 0; n < b; ++n) {
    float v[8];
    load8(dx + ((size_t)n * s + i) * H + c, v);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] += v[j];
  }
  store8(d_wpe + (size_t)i * H + c, acc);
}

// count[0] = number of labels inside [0, vocab).  One workgroup; integer counting, so exact in any order.
__global__ __launch_bounds__(256) void count_labels_kernel(const int32_t* __restrict__ labels, int rows, int vocab,
                                                           float* __restrict__ count) {
  __shared__ int total;
  if (threadIdx.x == 0) total = 0;
  __syncthreads();
  int mine = 0;
  for (int t = threadIdx.x; t < rows; t += 256) mine += (labels[t] >= 0 && labels[t] < vocab) ? 1 : 0;
  atomicAdd(&total, mine);
  __syncthreads();
  if (threadIdx.x == 0) count[0] = (float)total;
}

// One workgroup per row of logits [rows][V]: the row's log-sum-exp by an online max / sum pass, then a
// second pass (the row is still in cache) that overwrites the logits with the gradient of
// loss_scale * mean negative log-likelihood:  (softmax - onehot(label)) * loss_scale / count.
// nll[row] = lse - logit[label]; a row whose label is outside [0, V) gets nll 0 and a zero gradient.
template <typename T>
__global__ __launch_bounds__(256) void xent_kernel(T* __restrict__ logits, const int32_t* __restrict__ labels,
                                                   const float* __restrict__ count, float loss_scale,
                                                   float* __restrict__ nll, int V) {
  __shared__ float red_m[4], red_s[4];
  const int row = blockIdx.x;
  T* lr = logits + (size_t)row * V;
  const int label = labels[row];
  const int vecs = V / 8;
  if (label < 0 || label >= V) {
    const float zero[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int i = threadIdx.x; i < vecs; i += 256) store8(lr + i * 8, zero);
    if (threadIdx.x == 0) nll[row] = 0.f;
    return;
  }
  float m = -INFINITY, sum = 0.f;
  for (int i = threadIdx.x; i < vecs; i += 256) {
    float v[8];
    load8(lr + i * 8, v);
    float vm = v[0];
#pragma unroll
    for (int j = 1; j < 8; ++j) vm = fmaxf(vm, v[j]);
    const float mn = fmaxf(m, vm);
    float add = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) add += __expf(v[j] - mn);
    sum = sum * __expf(m - mn) + add;  // m = -inf the first time: exp(-inf) = 0
    m = mn;
  }
  // lanes that saw no vector hold (-inf, 0) and drop out of the sums below
  const float wm = wave_max(m);
  sum = wave_sum(m == -INFINITY ? 0.f : sum * __expf(m - wm));
  if ((threadIdx.x & 63) == 0) red_m[threadIdx.x >> 6] = wm, red_s[threadIdx.x >> 6] = sum;
  __syncthreads();
  float gm = red_m[0];
#pragma unroll
  for (int w = 1; w < 4; ++w) gm = fmaxf(gm, red_m[w]);
  float gs = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w) gs += red_m[w] == -INFINITY ? 0.f : red_s[w] * __expf(red_m[w] - gm);
  const float lse = gm + __logf(gs);
  const float n = count[0];
  const float scale = n > 0.f ? loss_scale / n : 0.f;
  for (int i = threadIdx.x; i < vecs; i += 256) {
    float v[8], g[8];
    load8(lr + i * 8, v);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bool hit = i * 8 + j == label;
      if (hit) nll[row] = lse - v[j];
      g[j] = (__expf(v[j] - lse) - (hit ? 1.f : 0.f)) * scale;
    }
    store8(lr + i * 8, g);
  }
}

// The same for bf16 rows of at most 1024 * 8 * NV columns: the workgroup's 1024 lanes hold the whole row
// in registers, so the logits are read from memory once.
template <int NV>
__global__ __launch_bounds__(1024) void xent_row_kernel(bf16* __restrict__ logits, const int32_t* __restrict__ labels,
                                                        const float* __restrict__ count, float loss_scale,
                                                        float* __restrict__ nll, int V) {
  __shared__ float red_m[16], red_s[16];
  const int row = blockIdx.x;
  bf16* lr = logits + (size_t)row * V;
  const int label = labels[row];
  const int vecs = V / 8;
  if (label < 0 || label >= V) {
    const float zero[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int i = threadIdx.x; i < vecs; i += 1024) store8(lr + i * 8, zero);
    if (threadIdx.x == 0) nll[row] = 0.f;
    return;
  }
  bf16x8 v[NV];
  float m = -INFINITY;
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int i = k * 1024 + threadIdx.x;
    if (i < vecs) {
      v[k] = *reinterpret_cast<const bf16x8*>(lr + i * 8);
#pragma unroll
      for (int j = 0; j < 8; ++j) m = fmaxf(m, (float)v[k][j]);
    }
  }
  m = wave_max(m);
  if ((threadIdx.x & 63) == 0) red_m[threadIdx.x >> 6] = m;
  __syncthreads();
  float gm = red_m[0];
#pragma unroll
  for (int w = 1; w < 16; ++w) gm = fmaxf(gm, red_m[w]);
  float sum = 0.f;
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    if (k * 1024 + (int)threadIdx.x < vecs) {
#pragma unroll
      for (int j = 0; j < 8; ++j) sum += __expf((float)v[k][j] - gm);
    }
  }
  sum = wave_sum(sum);
  if ((threadIdx.x & 63) == 0) red_s[threadIdx.x >> 6] = sum;
  __syncthreads();
  float gs = 0.f;
#pragma unroll
  for (int w = 0; w < 16; ++w) gs += red_s[w];
  const float lse = gm + __logf(gs);
  const float n = count[0];
  const float scale = n > 0.f ? loss_scale / n : 0.f;
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int i = k * 1024 + threadIdx.x;
    if (i < vecs) {
      float g[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float x = (float)v[k][j];
        const bool hit = i * 8 + j == label;
        if (hit) nll[row] = lse - x;
        g[j] = (__expf(x - lse) - (hit ? 1.f : 0.f)) * scale;
      }
      store8(lr + i * 8, g);
    }
  }
}

// loss[0] = sum(nll) / count (0 if nothing was counted).  One workgroup, fixed summation order.
__global__ __launch_bounds__(256) void loss_finish_kernel(const float* __restrict__ nll, const float* __restrict__ count,
                                                          int rows, float* __restrict__ loss) {
  __shared__ float part[256];
  float mine = 0.f;
  for (int t = threadIdx.x; t < rows; t += 256) mine += nll[t];
  part[threadIdx.x] = mine;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) loss[0] = count[0] > 0.f ? part[0] / count[0] : 0.f;
}

// out[i] = sum over the slices of parts[s][i], 8 elements per thread.
template <typename T>
__global__ __launch_bounds__(256) void sum_slices_kernel(const float* __restrict__ parts, int slices, size_t count,
                                                         T* __restrict__ out) {
  const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i >= count) return;
  float acc[8];
  load8(parts + i, acc);
  for (int s = 1; s < slices; ++s) {
    float v[8];
    load8(parts + (size_t)s * count + i, v);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] += v[j];
  }
  store8(out + i, acc);
}

// Adam with bias correction and decoupled weight decay on 4-element vectors.  The moments and, for
// bf16 parameters, the fp32 master copy are updated in place; the stored parameter is the rounded
// master.  Weight decay applies to the vectors for which decays() says so: everything, or only the
// four matrices of a packed transformer block.
struct AdamDev {
  void* params;
  float* master;  // nullptr: the parameters are their own master (fp32 storage)
  float* grads;
  float* m;
  float* v;
  size_t count;
  float lr, beta1, beta2, eps, weight_decay;
  float corr1, corr2;  // 1 / (1 - beta^t)
  int zero_grads;
  // decay mask: block_elems == 0 -> every element; else only positions (i mod block_elems) inside one of
  // the four [lo, hi) ranges
  size_t block_elems;
  size_t lo[4], hi[4];
};

template <typename T>
__global__ __launch_bounds__(256) void adam_kernel(AdamDev a) {
  const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= a.count) return;
  bool decay = true;
  if (a.block_elems) {
    const size_t pos = i % a.block_elems;
    decay = false;
#pragma unroll
    for (int r = 0; r < 4; ++r) decay = decay || (pos >= a.lo[r] && pos < a.hi[r]);
  }
  const float wd = decay ? a.weight_decay : 0.f;
  const f32x4 g = *reinterpret_cast<const f32x4*>(a.grads + i);
  f32x4 m = *reinterpret_cast<const f32x4*>(a.m + i);
  f32x4 v = *reinterpret_cast<const f32x4*>(a.v + i);
  f32x4 p;
  if (a.master) {
    p = *reinterpret_cast<const f32x4*>(a.master + i);
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) p[e] = ld(static_cast<const T*>(a.params) + i + e);
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    m[e] = a.beta1 * m[e] + (1.f - a.beta1) * g[e];
    v[e] = a.beta2 * v[e] + (1.f - a.beta2) * g[e] * g[e];
    const float mhat = m[e] * a.corr1, vhat = v[e] * a.corr2;
    p[e] = p[e] - a.lr * (mhat / (sqrtf(vhat) + a.eps) + wd * p[e]);
  }
  *reinterpret_cast<f32x4*>(a.m + i) = m;
  *reinterpret_cast<f32x4*>(a.v + i) = v;
  if (a.master) *reinterpret_cast<f32x4*>(a.master + i) = p;
  if constexpr (sizeof(T) == 2) {
    bf16x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (bf16)p[e];
    *reinterpret_cast<bf16x4*>(static_cast<bf16*>(a.params) + i) = o;
  } else {
    *reinterpret_cast<f32x4*>(static_cast<float*>(a.params) + i) = p;
  }
  if (a.zero_grads) *reinterpret_cast<f32x4*>(a.grads + i) = f32x4{0.f, 0.f, 0.f, 0.f};
}

}  // namespace

int embed_forward(int dtype, const void* wte, const void* wpe, const int32_t* tokens, void* x, int b, int s, int H,
                  int vocab, hipStream_t stream) {
  if (b < 1 || s < 1 || H < 8 || H % 8 || vocab < 1) return set_error(HANAYO_EINVAL, "embed_forward: bad shape");
  const int rows = b * s;
  const dim3 grid((rows + kRowsPerBlock - 1) / kRowsPerBlock);
  if (dtype == HANAYO_BF16)
    hipLaunchKernelGGL(embed_fwd_kernel<bf16>, grid, dim3(256), 0, stream, (const bf16*)wte, (const bf16*)wpe, tokens,
                       (bf16*)x, rows, s, H, vocab);
  else
    hipLaunchKernelGGL(embed_fwd_kernel<float>, grid, dim3(256), 0, stream, (const float*)wte, (const float*)wpe, tokens,
                       (float*)x, rows, s, H, vocab);
  return check_launch("embed_forward");
}

namespace {
template <typename T>
int embed_backward_t(const int32_t* tokens, const void* dx, float* d_wte, float* d_wpe, int b, int s, int H, int vocab,
                     hipStream_t stream) {
  const int rows = b * s;
  const size_t lds = (size_t)3 * H * sizeof(float);
  const int nv = (H + 511) / 512;
#define LAUNCH(NV)                                                                                              \
  hipLaunchKernelGGL((embed_bwd_token_kernel<T, NV>), dim3(rows), dim3(256), lds, stream, tokens, (const T*)dx, d_wte, \
                     rows, H, vocab)
  if (nv <= 1) LAUNCH(1);
  else if (nv <= 2) LAUNCH(2);
  else if (nv <= 4) LAUNCH(4);
  else LAUNCH(8);
#undef LAUNCH
  int rc = check_launch("embed_backward (tokens)");
  if (rc) return rc;
  const dim3 pgrid((unsigned)(((long)s * (H / 8) + 255) / 256));
  hipLaunchKernelGGL(embed_bwd_pos_kernel<T>, pgrid, dim3(256), 0, stream, (const T*)dx, d_wpe, b, s, H);
  return check_launch("embed_backward (positions)");
}
}  // namespace

int embed_backward(int dtype, const int32_t* tokens, const void* dx, float* d_wte, float* d_wpe, int b, int s, int H,
                   int vocab, hipStream_t stream) {
  if (b < 1 || s < 1 || H < 8 || H % 8 || H > 4096 || vocab < 1) return set_error(HANAYO_EINVAL, "embed_backward: bad shape");
  return dtype == HANAYO_BF16 ? embed_backward_t<bf16>(tokens, dx, d_wte, d_wpe, b, s, H, vocab, stream)
                              : embed_backward_t<float>(tokens, dx, d_wte, d_wpe, b, s, H, vocab, stream);
}

int count_labels(const int32_t* labels, int rows, int vocab, float* count, hipStream_t stream) {
  if (rows < 1 || vocab < 1) return set_error(HANAYO_EINVAL, "count_labels: bad shape");
  hipLaunchKernelGGL(count_labels_kernel, dim3(1), dim3(256), 0, stream, labels, rows, vocab, count);
  return check_launch("count_labels");
}

int softmax_xent(int dtype, void* logits, const int32_t* labels, const float* count, float loss_scale, float* nll,
                 int rows, int V, hipStream_t stream) {
  if (rows < 1 || V < 8 || V % 8) return set_error(HANAYO_EINVAL, "softmax_xent: bad shape");
  if (dtype == HANAYO_BF16 && V > 2048 && V <= 1024 * 8 * 8) {
    const int nv = (V / 8 + 1023) / 1024;
    auto kern = nv <= 2 ? xent_row_kernel<2> : nv <= 4 ? xent_row_kernel<4> : nv <= 6 ? xent_row_kernel<6> : xent_row_kernel<8>;
    hipLaunchKernelGGL(kern, dim3(rows), dim3(1024), 0, stream, (bf16*)logits, labels, count, loss_scale, nll, V);
  } else if (dtype == HANAYO_BF16)
    hipLaunchKernelGGL(xent_kernel<bf16>, dim3(rows), dim3(256), 0, stream, (bf16*)logits, labels, count, loss_scale, nll, V);
  else
    hipLaunchKernelGGL(xent_kernel<float>, dim3(rows), dim3(256), 0, stream, (float*)logits, labels, count, loss_scale, nll, V);
  return check_launch("softmax_xent");
}

int loss_finish(const float* nll, const float* count, int rows, float* loss, hipStream_t stream) {
  if (rows < 1) return set_error(HANAYO_EINVAL, "loss_finish: bad shape");
  hipLaunchKernelGGL(loss_finish_kernel, dim3(1), dim3(256), 0, stream, nll, count, rows, loss);
  return check_launch("loss_finish");
}

int sum_slices(int dtype, const float* parts, int slices, size_t count, void* out, hipStream_t stream) {
  if (slices < 1 || count == 0 || count % 8) return set_error(HANAYO_EINVAL, "sum_slices: bad shape");
  const size_t blocks = (count / 8 + 255) / 256;
  if (blocks > 0x7fffffffu) return set_error(HANAYO_EUNSUPPORTED, "sum_slices: too many elements");
  if (dtype == HANAYO_BF16)
    hipLaunchKernelGGL(sum_slices_kernel<bf16>, dim3((unsigned)blocks), dim3(256), 0, stream, parts, slices, count, (bf16*)out);
  else
    hipLaunchKernelGGL(sum_slices_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, stream, parts, slices, count, (float*)out);
  return check_launch("sum_slices");
}

int adam(int dtype, const AdamArgs& g, hipStream_t stream) {
  if (!g.params || !g.grads || !g.m || !g.v) return set_error(HANAYO_EINVAL, "adam: NULL argument");
  if (g.count == 0 || g.count % 4) return set_error(HANAYO_EINVAL, "adam: element count %zu is not a positive multiple of 4", g.count);
  if (dtype == HANAYO_BF16 && !g.master) return set_error(HANAYO_EINVAL, "adam: bf16 parameters need an fp32 master copy");
  if (g.step < 1 || !(g.beta1 >= 0.f && g.beta1 < 1.f) || !(g.beta2 >= 0.f && g.beta2 < 1.f))
    return set_error(HANAYO_EINVAL, "adam: step %d beta1 %g beta2 %g", g.step, g.beta1, g.beta2);
  AdamDev a{};
  a.params = g.params; a.master = dtype == HANAYO_BF16 ? g.master : nullptr; a.grads = g.grads; a.m = g.m; a.v = g.v;
  a.count = g.count;
  a.lr = g.lr; a.beta1 = g.beta1; a.beta2 = g.beta2; a.eps = g.eps; a.weight_decay = g.weight_decay;
  a.corr1 = (float)(1.0 / (1.0 - std::pow((double)g.beta1, g.step)));
  a.corr2 = (float)(1.0 / (1.0 - std::pow((double)g.beta2, g.step)));
  a.zero_grads = g.zero_grads;
  a.block_elems = g.block_elems;
  for (int r = 0; r < 4; ++r) a.lo[r] = g.lo[r], a.hi[r] = g.hi[r];
  const size_t vec = g.count / 4, blocks = (vec + 255) / 256;
  if (blocks > 0x7fffffffu) return set_error(HANAYO_EUNSUPPORTED, "adam: too many elements");
  if (dtype == HANAYO_BF16) hipLaunchKernelGGL(adam_kernel<bf16>, dim3((unsigned)blocks), dim3(256), 0, stream, a);
  else hipLaunchKernelGGL(adam_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, stream, a);
  return check_launch("adam");
}

}  // namespace k
}  // namespace hanayo
