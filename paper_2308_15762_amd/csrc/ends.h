// Host-side entry points of the model's ends and the optimizer step, shared by
// ends.cpp (the C entry points) and the executor.
#pragma once

#include <hip/hip_runtime.h>

#include "internal.h"

namespace hanayo {

int device_ok();  // HANAYO_OK on gfx950
int check_ends(const Shape& sh, const hanayo_ends_desc* e);
size_t head_workspace_bytes(const Shape& sh, int vocab);
int embed_forward(const Shape& sh, const hanayo_ends_desc* e, const void* wte, const void* wpe, const int32_t* tokens,
                  void* x, hipStream_t st);
int embed_backward(const Shape& sh, const hanayo_ends_desc* e, const int32_t* tokens, const void* dx, float* d_wte,
                   float* d_wpe, hipStream_t st);
// Loss of one micro-batch and, right away, the gradients of loss_scale * loss: dy (w.r.t. the last
// stage's output y), d_head and d_lnf (added to).
int head_loss(const Shape& sh, const hanayo_ends_desc* e, const void* lnf, const void* head, const void* y,
              const int32_t* labels, float loss_scale, float* loss, void* dy, float* d_lnf, float* d_head,
              void* workspace, hipStream_t st);
int chunk_adam_step(const hanayo_adam* o, const Shape& sh, void* weights, float* master, float* grads, float* m,
                    float* v, hipStream_t st);

}  // namespace hanayo
