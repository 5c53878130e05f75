// Descriptor validation, packed-parameter layout, stash-entry and workspace
// layouts, error strings.
#include <cstdarg>
#include <cstdio>

#include "internal.h"

namespace hanayo {

namespace {
thread_local char g_err[512] = "";
}

int set_error(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int make_shape(const hanayo_chunk_desc* d, Shape& sh) {
  if (!d) return set_error(HANAYO_EINVAL, "descriptor is NULL");
  if (d->n_blocks < 1 || d->hidden < 1 || d->heads < 1 || d->ffn < 1 || d->seq < 1 || d->mb < 1)
    return set_error(HANAYO_EINVAL, "descriptor: sizes must be >= 1");
  if (d->hidden % d->heads) return set_error(HANAYO_EINVAL, "descriptor: hidden %d not divisible by heads %d", d->hidden, d->heads);
  if (d->norm != HANAYO_PRE_LN && d->norm != HANAYO_POST_LN) return set_error(HANAYO_EINVAL, "descriptor: norm");
  if (d->mask != HANAYO_MASK_NONE && d->mask != HANAYO_MASK_CAUSAL) return set_error(HANAYO_EINVAL, "descriptor: mask");
  if (d->dtype != HANAYO_FP32 && d->dtype != HANAYO_BF16) return set_error(HANAYO_EINVAL, "descriptor: dtype");
  if (!(d->ln_eps > 0.f)) return set_error(HANAYO_EINVAL, "descriptor: ln_eps must be > 0");
  if (d->hidden % 8 || d->ffn % 8) return set_error(HANAYO_EUNSUPPORTED, "descriptor: hidden and ffn must be multiples of 8");
  if (d->hidden > 4096) return set_error(HANAYO_EUNSUPPORTED, "descriptor: hidden > 4096");
  const int hd = d->hidden / d->heads;
  if (hd % 8 || hd > 128) return set_error(HANAYO_EUNSUPPORTED, "descriptor: head dim %d (need multiple of 8, <= 128)", hd);
  if ((long)d->seq * d->mb > (1 << 24)) return set_error(HANAYO_EUNSUPPORTED, "descriptor: too many tokens");
  sh.nb = d->n_blocks;
  sh.H = d->hidden;
  sh.heads = d->heads;
  sh.d = hd;
  sh.F = d->ffn;
  sh.s = d->seq;
  sh.b = d->mb;
  sh.T = d->seq * d->mb;
  sh.norm = d->norm;
  sh.mask = d->mask;
  sh.dtype = d->dtype;
  sh.eps = d->ln_eps;
  sh.esz = d->dtype == HANAYO_BF16 ? 2 : 4;
  return HANAYO_OK;
}

ParamOffsets param_offsets(const Shape& sh) {
  const size_t H = sh.H, F = sh.F;
  const size_t cnt[HANAYO_N_PARAMS] = {H, H, H * 3 * H, 3 * H, H * H, H, H, H, H * F, F, F * H, H};
  ParamOffsets po;
  size_t at = 0;
  for (int i = 0; i < HANAYO_N_PARAMS; ++i) {
    po.off[i] = at;
    po.cnt[i] = cnt[i];
    at += cnt[i];
  }
  po.block_elems = at;  // every count is a multiple of 8, so 16-byte vectors stay aligned
  return po;
}

StashLayout stash_layout(const Shape& sh) {
  StashLayout L;
  size_t at = 0;
  const size_t th = align_up((size_t)sh.T * sh.H * sh.esz, 256);
  const size_t tf = align_up((size_t)sh.T * sh.F * sh.esz, 256);
  auto take = [&](size_t bytes) {
    const size_t o = at;
    at += bytes;
    return o;
  };
  L.x = take(th);
  L.ln_a = take(th);
  L.qkv = take(3 * th);
  L.ctx = take(th);
  L.x1 = take(th);
  L.ln_b = take(th);
  L.hpre = take(tf);
  L.act = take(tf);
  L.stats1 = take(align_up((size_t)sh.T * 8, 256));
  L.stats2 = take(align_up((size_t)sh.T * 8, 256));
  L.lse = take(align_up((size_t)sh.b * sh.heads * sh.s * 4, 256));
  L.block_bytes = at;
  return L;
}

WorkLayout work_layout(const Shape& sh) {
  WorkLayout L;
  size_t at = 0;
  const size_t th = align_up((size_t)sh.T * sh.H * sh.esz, 256);
  const size_t tf = align_up((size_t)sh.T * sh.F * sh.esz, 256);
  auto take = [&](size_t bytes) {
    const size_t o = at;
    at += bytes;
    return o;
  };
  L.d_act = take(tf);
  L.d_h0 = take(th);
  L.d_h1 = take(th);
  L.d_h2 = take(th);
  L.d_h3 = take(th);
  L.d_qkv = take(3 * th);
  L.d_ping = take(th);
  L.d_pong = take(th);
  L.delta = take(align_up((size_t)sh.b * sh.heads * sh.s * 4, 256));
  L.partial = take(align_up((size_t)kMaxPartialRows * 2 * sh.H * 4, 256));
  L.ln_slot_bytes = align_up((size_t)kLnPartialRows * 2 * sh.H * 4, 256);
  L.ln_partial = take(2 * (size_t)sh.nb * L.ln_slot_bytes);
  L.bytes = at;
  return L;
}

}  // namespace hanayo

using namespace hanayo;

extern "C" {

const char* hanayo_strerror(int code) {
  switch (code) {
    case HANAYO_OK: return "ok";
    case HANAYO_EINVAL: return "invalid argument";
    case HANAYO_EBUFSIZE: return "output buffer too small";
    case HANAYO_ESTATE: return "task list not executable";
    case HANAYO_EUNSUPPORTED: return "unsupported shape or device";
    case HANAYO_EHIP: return "HIP runtime error";
    default: return "unknown error";
  }
}

const char* hanayo_last_error(void) { return g_err; }

int hanayo_param_span(const hanayo_chunk_desc* d, int block, int param, size_t* elem_offset, size_t* elem_count) {
  Shape sh;
  int rc = make_shape(d, sh);
  if (rc) return rc;
  if (block < 0 || block >= sh.nb || param < 0 || param >= HANAYO_N_PARAMS || !elem_offset || !elem_count)
    return set_error(HANAYO_EINVAL, "param_span: bad block or param");
  const ParamOffsets po = param_offsets(sh);
  *elem_offset = (size_t)block * po.block_elems + po.off[param];
  *elem_count = po.cnt[param];
  return HANAYO_OK;
}

size_t hanayo_weight_bytes(const hanayo_chunk_desc* d) {
  Shape sh;
  if (make_shape(d, sh)) return 0;
  return align_up(param_offsets(sh).block_elems * sh.nb * sh.esz, 256);
}
size_t hanayo_grad_bytes(const hanayo_chunk_desc* d) {
  Shape sh;
  if (make_shape(d, sh)) return 0;
  return align_up(param_offsets(sh).block_elems * sh.nb * 4, 256);
}
size_t hanayo_stash_bytes(const hanayo_chunk_desc* d) {
  Shape sh;
  if (make_shape(d, sh)) return 0;
  return stash_layout(sh).block_bytes * sh.nb;
}
size_t hanayo_workspace_bytes(const hanayo_chunk_desc* d) {
  Shape sh;
  if (make_shape(d, sh)) return 0;
  return work_layout(sh).bytes;
}
size_t hanayo_act_bytes(const hanayo_chunk_desc* d) {
  Shape sh;
  if (make_shape(d, sh)) return 0;
  return align_up((size_t)sh.T * sh.H * sh.esz, 256);
}

}  // extern "C"
