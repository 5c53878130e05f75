/*
 * hanayo.h -- C ABI of the per-rank hot path of a Hanayo wave pipeline on one
 * MI355X (gfx950).
 *
 * The paper's runtime section describes a scheduler that emits, per worker, an
 * ordered "action list" whose compute actions carry the local module rank, and
 * an interpreter on each worker that executes the list.  This library is that
 * pair for ONE worker: it generates the worker's ordered forward/backward task
 * list for a (P devices, W waves, M micro-batches) wave pipeline, sizes the
 * activation stash from the list, and executes the list with hand-written HIP
 * kernels, stage boundaries being buffers in HBM instead of sends to peers.
 *
 * Conventions for every function
 *   - returns HANAYO_OK (0) or a negative error code; never throws or aborts;
 *     hanayo_last_error() gives a thread-local detail string
 *   - "host" / "device" on a pointer says where the memory lives
 *   - the library allocates no device memory: all device buffers belong to the
 *     caller, must be 256-byte aligned, and must stay alive until the stream
 *     has passed the work enqueued by the call
 *   - device work is enqueued on the given HIP stream (a hipStream_t passed as
 *     void*, NULL = default stream) and the call returns without synchronising
 */
#ifndef HANAYO_H
#define HANAYO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  HANAYO_OK = 0,
  HANAYO_EINVAL = -1,       /* bad argument (range, shape, NULL, misalignment) */
  HANAYO_EBUFSIZE = -2,     /* caller's output buffer too small; needed size reported */
  HANAYO_ESTATE = -3,       /* list not executable: B before its F, repeated task, stash overflow */
  HANAYO_EUNSUPPORTED = -4, /* shape or device outside what the kernels cover (not gfx950, ...) */
  HANAYO_EHIP = -5          /* a HIP runtime call or kernel launch failed */
};

const char* hanayo_strerror(int code); /* static string */
const char* hanayo_last_error(void);   /* thread-local, valid until the next call on this thread */

/* ------------------------------------------------------------------------- *
 * Wave schedule (Table 1: W = S / 2P; sections on wave-like pipelines and the
 * theoretical analysis).  S = 2*W*P stages; stage s sits on device
 *   rank(s) = s mod P           if floor(s / P) is even
 *           = P - 1 - (s mod P) if floor(s / P) is odd
 * so a micro-batch runs down the devices and back W times and the two stages
 * at every turn share a device.  "chunk" = floor(s / P) is the local module
 * rank of the stage on its device (0 .. 2W-1).
 * ------------------------------------------------------------------------- */

enum { HANAYO_F = 0, HANAYO_B = 1 };

typedef struct hanayo_task {
  uint8_t kind;   /* HANAYO_F or HANAYO_B */
  uint8_t chunk;  /* local chunk 0 .. 2W-1 */
  uint16_t rsvd;  /* 0 */
  uint32_t mb;    /* micro-batch 0 .. M-1 */
  uint32_t stage; /* global stage 0 .. 2WP-1 */
} hanayo_task;    /* 12 bytes, no padding */

int hanayo_stage_rank(int P, int W, int stage, int* rank /* host out */);
int hanayo_rank_stage(int P, int W, int rank, int chunk, int* stage /* host out */);

/*
 * Ordered task list of one rank.  The paper draws the order only in figures;
 * the order produced is the deterministic greedy list schedule of the whole
 * P-rank pipeline under the cost model of the theoretical analysis (forward 1,
 * backward 2, transfer 0): a free rank starts a ready task, backward before
 * forward, lowest micro-batch first; the forward of micro-batch m >= P on
 * stage 0 waits for the forward of micro-batch m-P on the last stage.
 *
 * out: host, caller-owned, capacity `cap` records.  *n (host, required)
 * always receives the needed count 4*W*M, also on HANAYO_EBUFSIZE (out may be
 * NULL with cap 0 to query).  Pure and thread-safe.
 * HANAYO_EINVAL: P, W or M < 1, rank outside [0, P), 2W > 255, n NULL.
 */
int hanayo_schedule(int P, int W, int M, int rank, hanayo_task* out, size_t cap, size_t* n);

/*
 * The other schedulers (runtime section: "scheduling algorithms for existing mainstream pipeline schemes" next
 * to Hanayo's, all emitting the same kind of per-worker list; background section for what each scheme does).
 *   HANAYO_SCHEME_HANAYO        hanayo_schedule(P, W, M, rank)
 *   HANAYO_SCHEME_CHIMERA_WAVE  Chimera after the swap of the section on transforming it into wave-like
 *                               pipelines (mirrored blocks exchanged, replicas become data parallelism, order
 *                               of computation unchanged): the one-wave list; W must be 1
 *   HANAYO_SCHEME_GPIPE         one stage per device; every forward pass of the iteration, then every backward
 *   HANAYO_SCHEME_1F1B          DAPPLE's one-forward-one-backward: P-1-rank forward passes, then forward and
 *                               backward alternate, then the remaining backward passes (at most P - rank
 *                               activations alive on device `rank`)
 * Placements.  The two wave schemes use the placement above (2W chunks per device).  GPipe and 1F1B use the
 * straight placement: S = P stages, stage s on device s, one chunk per device; in Table 1's notation that is
 * W = S / 2P = 1/2, and it is written W = 0 in this interface: pass W = 0 to hanayo_schedule_scheme and to
 * hanayo_stage_rank, hanayo_rank_stage, hanayo_stash_plan, hanayo_stash_arena_bytes*, hanayo_executor_plan,
 * hanayo_executor_run, hanayo_pipeline_run and hanayo_replay when they handle such a list (2*M records per
 * rank, chunk 0, stage = rank).  Same calling convention and error codes as hanayo_schedule; HANAYO_EINVAL
 * for a W that does not fit the scheme.
 */
enum { HANAYO_SCHEME_HANAYO = 0, HANAYO_SCHEME_CHIMERA_WAVE = 1, HANAYO_SCHEME_GPIPE = 2, HANAYO_SCHEME_1F1B = 3 };
int hanayo_schedule_scheme(int scheme, int P, int W, int M, int rank, hanayo_task* out, size_t cap, size_t* n);

/*
 * Bubble model (theoretical-analysis section; host only).  t_f / t_b: a device's whole forward / backward
 * time for one micro-batch (the paper's T_F and T_B: all its stages added), t_c: one transfer (T_C).
 *   wave schemes (M must equal P, the case the paper's equation covers):
 *     *ratio         = ( T_B/W + (1 + 2W + 2/P + (P-2)/3) T_C )
 *                      / ( P/(P-1) T_F + (1/(2W) + P/(P-1)) T_B + ((P-2)/2 + 4W) T_C )       as printed;
 *                      (2P-2)/(3PW+P-1) at T_B = 2 T_F, T_C = 0
 *     *idle          = (P-1) times the numerator: the idle time per device that the summed bubble zones give
 *     *ratio_of_idle = idle / (idle + M (T_F + T_B)): the same bubble over the iteration time that follows
 *                      from it (the printed denominator counts only half of the idle term)
 *   GPipe, 1F1B (any M): idle = (P-1)(T_F + T_B + 2 T_C): the fill before the last device starts and the
 *     drain after its last backward; ratio = ratio_of_idle = idle / (idle + M (T_F + T_B)).  Exact for GPipe
 *     while the other transfers hide behind compute (receives posted one task ahead, T_C <= T_F); for 1F1B
 *     exact at T_C = 0; a lower bound otherwise (hanayo_replay_actions simulates those cases).
 * Outputs may be NULL.  HANAYO_EINVAL: bad scheme / W combination, M != P for a wave scheme, negative times.
 */
int hanayo_bubble_model(int scheme, int P, int W, int M, double t_f, double t_b, double t_c, double* ratio,
                        double* idle, double* ratio_of_idle);

/*
 * Activation-stash accounting of a list (M_a of Table 1 counted per chunk):
 * an entry lives from the F task of (mb, chunk) to its B task.
 *   peak_total  host out, may be NULL: peak number of live entries
 *   per_chunk   host out [2W], may be NULL: peak live entries of each chunk
 *   slot        host out [n], may be NULL: for an F task the smallest slot id
 *               of its chunk that is free at that point, for a B task the id
 *               its F took; always < per_chunk[chunk]
 * HANAYO_ESTATE: a B whose (mb, chunk) is not live, an F of a live one, or
 * entries left live at the end.  HANAYO_EINVAL: chunk >= 2W, bad kind.
 */
int hanayo_stash_plan(const hanayo_task* list /* host */, size_t n, int W, int* peak_total, int* per_chunk,
                      int32_t* slot);

/* ------------------------------------------------------------------------- *
 * Chunk = n_blocks transformer blocks (the paper's T_F / 2W and T_B / 2W unit
 * of work; the evaluation section gives the model families by layer, head and
 * hidden counts only, so the block is the standard one):
 *   pre-LN   x1 = x + Attn(LN1(x)),  y = x1 + MLP(LN2(x1))
 *   post-LN  x1 = LN1(x + Attn(x)),  y = LN2(x1 + MLP(x1))
 *   Attn(u) = softmax(Q K^T / sqrt(d) with masked keys removed) V Wo + bo
 *   MLP(v)  = GELU_erf(v W1 + b1) W2 + b2,   LN with biased variance and eps
 * ------------------------------------------------------------------------- */

enum { HANAYO_PRE_LN = 0, HANAYO_POST_LN = 1 };
enum { HANAYO_MASK_NONE = 0, HANAYO_MASK_CAUSAL = 1 };
enum { HANAYO_FP32 = 0, HANAYO_BF16 = 1 }; /* storage type; accumulation is always fp32 */

typedef struct hanayo_chunk_desc {
  int n_blocks;
  int hidden; /* H; multiple of 8, at most 4096 (the fast bf16 kernels want multiples of 128) */
  int heads;  /* H / heads: multiple of 8, at most 128 (64 and 128 take the fastest attention kernels) */
  int ffn;    /* F; multiple of 8 */
  int seq;    /* s; any length >= 1; seq * mb at most 2^24 */
  int mb;     /* sequences per micro-batch b; tokens T = b * s */
  int norm;   /* HANAYO_PRE_LN / HANAYO_POST_LN */
  int mask;   /* HANAYO_MASK_NONE / HANAYO_MASK_CAUSAL; key padding comes from valid_len */
  int dtype;  /* HANAYO_FP32 / HANAYO_BF16 */
  float ln_eps;
} hanayo_chunk_desc;

/*
 * Parameter layout.  Weights are one packed array of the storage type, grads
 * one packed fp32 array with the same element offsets.  Per block, in order
 * (ids for hanayo_param_span):
 *   0 ln1_gamma[H] 1 ln1_beta[H] 2 Wqkv[H][3H] 3 bqkv[3H] 4 Wo[H][H] 5 bo[H]
 *   6 ln2_gamma[H] 7 ln2_beta[H] 8 W1[H][F]    9 b1[F]   10 W2[F][H] 11 b2[H]
 * Matrices are row-major [in][out] (y = x W + b); Wqkv columns are [Q | K | V]
 * and head j owns columns j*d .. (j+1)*d-1 of each third.
 */
enum { HANAYO_N_PARAMS = 12 };
int hanayo_param_span(const hanayo_chunk_desc* d, int block, int param, size_t* elem_offset, size_t* elem_count);

size_t hanayo_weight_bytes(const hanayo_chunk_desc* d);    /* 0 on a bad descriptor */
size_t hanayo_grad_bytes(const hanayo_chunk_desc* d);      /* fp32 */
size_t hanayo_stash_bytes(const hanayo_chunk_desc* d);     /* one (micro-batch, chunk) entry, multiple of 256 */
size_t hanayo_workspace_bytes(const hanayo_chunk_desc* d); /* scratch shared by forward and backward */
size_t hanayo_act_bytes(const hanayo_chunk_desc* d);       /* one [b][s][H] boundary tensor */

/*
 * Forward of one micro-batch through one chunk.
 *   weights      device, packed parameters (read)
 *   x            device [b][s][H] storage type (read)
 *   valid_len    device int32 [b] or NULL: keys j >= valid_len[n] of sequence n are
 *                masked for every query row; each must be in [1, s]
 *   y            device [b][s][H] (fully overwritten; may not alias x)
 *   stash_entry  device, hanayo_stash_bytes(): written here, read-only in backward;
 *                holds a copy of x, so x may be reused once the call's work is done
 *   workspace    device, hanayo_workspace_bytes(); contents undefined afterwards
 */
int hanayo_chunk_forward(const hanayo_chunk_desc* d, const void* weights, const void* x, const int32_t* valid_len,
                         void* y, void* stash_entry, void* workspace, void* hip_stream);

/*
 * Backward of one micro-batch through one chunk.
 *   grads        device fp32, packed like weights; every parameter gradient is ADDED
 *                (caller zeroes at the start of an iteration: the flush boundary
 *                of synchronous pipeline training)
 *   dy           device [b][s][H] storage type, gradient of the loss w.r.t. y (read)
 *   stash_entry  what the matching forward wrote (read)
 *   dx           device [b][s][H] (fully overwritten; may not alias dy)
 */
int hanayo_chunk_backward(const hanayo_chunk_desc* d, const void* weights, float* grads, const void* dy,
                          const int32_t* valid_len, const void* stash_entry, void* dx, void* workspace,
                          void* hip_stream);

/* ------------------------------------------------------------------------- *
 * The two ends of the model and the optimizer step.  The paper trains GPT-style
 * and BERT-style language models with synchronous pipeline parallelism (its
 * background section: one flush and one parameter update per iteration, from
 * the gradients summed over the micro-batches) and prints none of these pieces,
 * so they are the standard ones:
 *   embedding  x[n][i][:] = wte[token[n][i]][:] + wpe[i][:]     (in front of stage 0)
 *   head       logits = LN_f(y) head^T, head a [V][H] table (LN_f optional);
 *              loss = mean over the labelled positions of -log softmax(logits)[label]
 *   Adam       with bias correction and decoupled weight decay
 * In a wave placement stage 0 and the last stage share rank 0, so a head tied to
 * the token table (head == wte, d_head == d_wte) needs no exchange between ranks.
 * Tables are row-major in the storage type, gradients fp32 and ADDED to.
 * ------------------------------------------------------------------------- */
typedef struct hanayo_ends_desc {
  int vocab;    /* V; multiple of 8 (multiples of 128 take the fast bf16 GEMM kernels) */
  int max_pos;  /* rows of the position table wpe, >= seq */
  int final_ln; /* 1: LayerNorm (gamma[H] then beta[H], the chunk's ln_eps) in front of the head */
} hanayo_ends_desc;

/*
 * tokens  device int32 [b][s]; a token outside [0, V) contributes no table row
 *         (forward) and receives no gradient (backward)
 * x       device [b][s][H], fully overwritten
 * d_wte   device fp32 [V][H]: rows of equal tokens are added in a fixed order, without atomics (H <= 4096)
 * d_wpe   device fp32 [max_pos][H]
 */
int hanayo_embed_forward(const hanayo_chunk_desc* d, const hanayo_ends_desc* e, const void* wte, const void* wpe,
                         const int32_t* tokens, void* x, void* hip_stream);
int hanayo_embed_backward(const hanayo_chunk_desc* d, const hanayo_ends_desc* e, const int32_t* tokens, const void* dx,
                          float* d_wte, float* d_wpe, void* hip_stream);

/*
 * Loss of one micro-batch and, in the same call, the gradients of loss_scale * loss (loss_scale = 1 / M
 * makes the iteration's loss the mean over its micro-batches).
 *   lnf, d_lnf  device [2][H] (gamma, beta) and fp32 [2][H]; read only with final_ln
 *   head        device [V][H];  d_head fp32 [V][H]
 *   y           device [b][s][H], output of the last stage (read)
 *   labels      device int32 [b][s]; a label outside [0, V) (e.g. -1) marks a position that does not count
 *   loss        device float [1], written: the mean over the counted positions, 0 if there is none
 *   dy          device [b][s][H], fully overwritten; may not alias y
 *   workspace   device, hanayo_head_workspace_bytes(); holds the [b*s][V] logits
 */
size_t hanayo_head_workspace_bytes(const hanayo_chunk_desc* d, const hanayo_ends_desc* e); /* 0 on a bad descriptor */
int hanayo_head_loss(const hanayo_chunk_desc* d, const hanayo_ends_desc* e, const void* lnf, const void* head,
                     const void* y, const int32_t* labels, float loss_scale, float* loss, void* dy, float* d_lnf,
                     float* d_head, void* workspace, void* hip_stream);

/*
 * One Adam update (Kingma & Ba, Algorithm 1; decay as in Loshchilov & Hutter, Algorithm 2), in place:
 *   m = beta1 m + (1 - beta1) g;   v = beta2 v + (1 - beta2) g^2
 *   p = p - lr ( (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps) + weight_decay p )
 * params is the storage type; for bf16 storage `master` (fp32, same element count) is the copy that is
 * updated and params receives its rounding; for fp32 storage master is ignored (may be NULL).  grads, m, v
 * are fp32.  zero_grads = 1 clears the gradients in the same pass (the next iteration starts from zero).
 * count: multiple of 4.  hanayo_chunk_adam_step updates a chunk's packed parameters and applies the decay
 * to its four matrices only (not to biases and LayerNorm parameters).
 */
typedef struct hanayo_adam {
  float lr, beta1, beta2, eps, weight_decay;
  int step;       /* 1 for the first update */
  int zero_grads;
} hanayo_adam;
int hanayo_adam_step(const hanayo_adam* o, int dtype, void* params, float* master, float* grads, float* m, float* v,
                     size_t count, void* hip_stream);
int hanayo_chunk_adam_step(const hanayo_adam* o, const hanayo_chunk_desc* d, void* weights, float* master, float* grads,
                           float* m, float* v, void* hip_stream);

/* ------------------------------------------------------------------------- *
 * Per-rank task executor (the worker-side interpreter of the runtime section,
 * compute actions only).  Runs `list` in order (on one stream unless lanes
 * are asked for, see below).  All chunks of
 * the rank share one descriptor.  Tables are host arrays of device pointers
 * indexed [mb * 2W + chunk].
 *
 * Forward input of (mb, chunk): if the previous stage is on this rank (the
 * local turn-around) it is act_out[mb][chunk-1], else act_in[mb][chunk], a
 * buffer the caller filled ("received" activation, or the data for stage 0).
 * Forward output goes to act_out[mb][chunk] ("sent" activation).
 * Backward input of (mb, chunk): if the next stage is on this rank it is
 * grad_out[mb][chunk+1], else grad_in[mb][chunk] ("received" gradient, or the
 * loss gradient for the last stage).  Backward output goes to
 * grad_out[mb][chunk].  act_in / grad_in entries that are never read may be NULL.
 *
 * The stash arena is carved by the plan of `list`: chunk c owns
 * per_chunk[c] entries starting after those of the chunks before it.
 * ------------------------------------------------------------------------- */
typedef struct hanayo_exec_args {
  const hanayo_chunk_desc* desc;
  int P, W, M, rank;                /* W = 0: straight placement (GPipe / 1F1B lists), one chunk: read "1" for "2W" below */
  const void* const* weights;      /* host [2W] -> device */
  float* const* grads;             /* host [2W] -> device fp32 */
  const void* const* act_in;       /* host [M*2W] -> device */
  const void* const* grad_in;      /* host [M*2W] -> device */
  void* const* act_out;            /* host [M*2W] -> device */
  void* const* grad_out;           /* host [M*2W] -> device */
  const int32_t* const* valid_len; /* host [M] -> device int32 [b], or NULL */
  void* stash_arena;               /* device */
  size_t stash_arena_bytes;        /* >= hanayo_stash_arena_bytes() */
  void* workspace;                 /* device, lanes * hanayo_workspace_bytes() */
  void* hip_stream;
  int lanes;                       /* 0 or 1: everything on hip_stream; 2..4: see below */
  int stash_mode;                  /* HANAYO_STASH_FULL or HANAYO_STASH_INPUT, see below */
  void* recompute_scratch;         /* device; HANAYO_STASH_INPUT only: max(lanes, 1) * hanayo_recompute_scratch_bytes() */
  const struct hanayo_ends_args* ends; /* NULL, or the model's ends on rank 0 (see below) */
} hanayo_exec_args;

/*
 * The model's ends in the executor.  With args->ends set, rank 0 (which holds stage 0 and the last stage in
 * every wave placement; other ranks ignore the field) builds the input of stage 0 of micro-batch m from
 * tokens[m] instead of reading act_in, and right after the forward task of the last stage computes loss[m]
 * and the gradients of loss_scale * loss: the head's and final LayerNorm's are added to d_head / d_lnf, the
 * one w.r.t. the stage's output goes to loss_grad[m], which that stage's backward task reads instead of
 * grad_in.  The backward task of stage 0 is followed by the embedding's backward into d_wte / d_wpe.
 * head may be wte and d_head d_wte (tied weights).  With lanes, the tasks that add to these gradients wait
 * for one another in list order.
 */
typedef struct hanayo_ends_args {
  hanayo_ends_desc desc;
  const void* wte;  float* d_wte;        /* device [V][H] */
  const void* wpe;  float* d_wpe;        /* device [max_pos][H] */
  const void* head; float* d_head;       /* device [V][H] */
  const void* lnf;  float* d_lnf;        /* device [2][H]; NULL without final_ln */
  const int32_t* const* tokens;          /* host [M] -> device int32 [b][s] */
  const int32_t* const* labels;          /* host [M] -> device int32 [b][s] */
  float* loss;                           /* device float [M], written */
  void* const* loss_grad;                /* host [M] -> device [b][s][H], written then read */
  float loss_scale;
  void* workspace;                       /* device, max(lanes, 1) * hanayo_ends_workspace_bytes() */
} hanayo_ends_args;
size_t hanayo_ends_workspace_bytes(const hanayo_chunk_desc* d, const hanayo_ends_desc* e); /* 0 on a bad descriptor */

/*
 * Stash modes.  HANAYO_STASH_FULL (0): a stash entry holds every tensor the forward pass materialises
 * (hanayo_stash_bytes() per entry); backward recomputes only the attention probabilities.
 * HANAYO_STASH_INPUT (1): an entry holds the chunk's input only (hanayo_act_bytes() rounded up to 256 per
 * entry, arena size from hanayo_stash_arena_bytes_input()); a backward task first runs the chunk's forward
 * again from that input into a scratch entry (one per lane, recompute_scratch) and then the backward.
 * Same results (the recomputed forward is the same kernels on the same data); about one forward more per
 * backward in time, two orders of magnitude less stash.
 */
enum { HANAYO_STASH_FULL = 0, HANAYO_STASH_INPUT = 1 };
size_t hanayo_stash_arena_bytes_input(const hanayo_task* list, size_t n, int W, const hanayo_chunk_desc* d);
size_t hanayo_recompute_scratch_bytes(const hanayo_chunk_desc* d);

/* Arena size the executor needs for `list`; 0 on error. */
size_t hanayo_stash_arena_bytes(const hanayo_task* list, size_t n, int W, const hanayo_chunk_desc* d);

/*
 * HANAYO_ESTATE if the list is not exactly the rank's 4*W*M tasks, each once,
 * every B after its F and after the task it depends on locally; nothing is
 * enqueued in that case.  *peak_seen (host, may be NULL) receives the largest
 * number of stash entries that were live at once.
 */
int hanayo_executor_run(const hanayo_task* list, size_t n, const hanayo_exec_args* args, int* peak_seen);

/*
 * Lanes.  With args->lanes > 1 the executor spreads the list over that many HIP
 * streams (lane 0 is hip_stream, the others belong to the library: default
 * priority, created once per device and kept), so that tasks which do not
 * depend on each other overlap on the GPU.  A task waits, through events, for
 * the tasks hanayo_executor_plan lists for it; tasks of one lane run in list
 * order; the side lanes start after the work hip_stream already holds and
 * hip_stream ends after all of them, so the caller sees one ordered stream.
 * Results equal those of one lane (a chunk's gradient accumulations keep their
 * list order).  Calls with lanes > 1 on one device are serialised on the host.
 *
 * The lanes are chosen by list scheduling with the schedule's own costs (forward 1, backward 2).
 *
 * hanayo_executor_plan reports that plan without touching the GPU:
 *   lane  host [n]     lane of each task
 *   d, e  NULL, or the descriptors of a run with args->ends set: the plan then has the dependencies [4]
 *         below and counts the head's work (from the shapes) into the forward task of the last stage
 *   deps  host [n][5]  indices of earlier tasks that task i waits for, -1 = none:
 *         [0] the local stage producing its input, [1] (B) its own forward,
 *         [2] (F) the backward that last read the stash entry it overwrites,
 *         [3] (B) the previous backward of the same chunk,
 *         [4] (with ends, on rank 0: forward of the last stage, backward of stage 0) the previous task
 *             that added to the gradients of the embedding tables and the head.
 * Same list checks and error codes as hanayo_executor_run.
 */
int hanayo_executor_plan(const hanayo_task* list, size_t n, int P, int W, int M, int rank, int lanes,
                         const hanayo_chunk_desc* d, const hanayo_ends_desc* e, int32_t* lane, int32_t* deps);


/* ------------------------------------------------------------------------- *
 * Action lists (runtime section of the paper): the scheduler's output at the
 * granularity the workers interpret, i.e. compute actions carrying the local
 * module (chunk) index plus send / receive actions carrying the target rank.
 * Rank r's action list is its task list with, around every task, the
 * communication it needs: a receive immediately in front of a compute whose
 * input is produced on another rank, a send immediately behind a compute whose
 * output is consumed on another rank.  The turns of the wave (two consecutive
 * stages on one rank) have no communication actions.  For a communication
 * action `stage`, `chunk` and `mb` are those of the local compute it serves and
 * `peer` is the other rank (always a neighbour); for a compute action `peer` is
 * the rank itself.  Same calling convention as hanayo_schedule (*n receives the
 * count, HANAYO_EBUFSIZE if cap is too small).
 * ------------------------------------------------------------------------- */
enum { HANAYO_SEND_ACT = 2, HANAYO_RECV_ACT = 3, HANAYO_SEND_GRAD = 4, HANAYO_RECV_GRAD = 5 };

typedef struct hanayo_action {
  uint8_t kind;   /* HANAYO_F, HANAYO_B or one of the four above */
  uint8_t chunk;
  uint16_t peer;
  uint32_t mb;
  uint32_t stage;
} hanayo_action;  /* 12 bytes, no padding */

int hanayo_actions(int P, int W, int M, int rank, hanayo_action* out, size_t cap, size_t* n);
/* The same for any task list of rank `rank` (a list of hanayo_schedule_scheme; W = 0 for the straight
   placement): the list with its receive and send actions put around the tasks.  HANAYO_ESTATE if a record is
   not a task of that rank. */
int hanayo_actions_of(const hanayo_task* tasks /* host */, size_t count, int P, int W, int rank, hanayo_action* out,
                      size_t cap, size_t* n);

/*
 * Host only: the P interpreters simulated.  Sends are asynchronous (no time on the sender); a transfer starts
 * once the message has been sent AND its receive has been posted, and takes t_c; a rank waits at a receive until
 * the message has arrived.  prefetch = 0: a receive is posted when the interpreter reaches it.  prefetch = 1 (the
 * paper's look-ahead): before starting a compute action the interpreter posts the receive that feeds the
 * following compute action.  cost[r][i] (may be NULL: forward t_f, backward t_b) = duration of action i of rank r
 * if it is a compute action (entries of communication actions are ignored).
 * *makespan = time the last rank finishes; idle[r], waited[r] (may be NULL) = makespan minus rank r's compute
 * time, and the time rank r spent blocked in receives.  HANAYO_ESTATE if the compute actions of a list are not
 * its rank's task set in a valid order, a communication action does not belong to the compute next to it, or
 * the lists deadlock.
 */
int hanayo_replay_actions(const hanayo_action* const* lists, const size_t* counts, int P, int W, int M, double t_f,
                          double t_b, double t_c, int prefetch, const float* const* cost, double* makespan,
                          double* idle, double* waited);

/* ------------------------------------------------------------------------- *
 * The whole pipeline on one device.  Synchronous pipeline training computes
 * what the model computes without a pipeline (the premise of the paper's
 * comparison of schedules); hanayo_pipeline_run executes ALL P ranks' lists
 * with true dataflow, so that this can be checked end to end, and measures the
 * tasks; hanayo_replay turns measured task durations into the makespan and idle
 * time the schedule would have on P devices (the paper's bubble analysis with
 * measured T_F and T_B and T_C = 0).
 *
 * Tables are host arrays of device pointers.  S = 2*W*P stages; stage s belongs
 * to rank hanayo_stage_rank(P, W, s).
 *   weights, grads   [S]     per stage (grads are ADDED to, fp32)
 *   x, dy            [M]     stage-0 input / gradient w.r.t. the last stage's output, per micro-batch (read)
 *   act, grad        [M*S]   index mb*S + stage: output activation of the stage (written; act[mb][S-1] is
 *                            the model output) and gradient w.r.t. the stage's input (written; grad[mb][0] is dL/dx)
 *   stash_arena      [P]     one arena per rank, stash_arena_bytes[r] >= hanayo_stash_arena_bytes(lists[r], ...)
 *   workspace                hanayo_workspace_bytes()
 * Everything goes to hip_stream, in a dataflow merge of the lists: the ranks are polled in turn and a rank's
 * head task runs once the task that produces its input has run.
 * lists[r] / counts[r]: rank r's list.  HANAYO_ESTATE if a list is not its rank's task set in an order that
 * respects the rank-local dependencies, or if the lists deadlock against each other; nothing is enqueued then.
 * peak_seen (host [P], may be NULL): stash peak of each rank.
 * task_ms (host [P] -> host float [counts[r]], may be NULL): if given, every task is bracketed by HIP events,
 * the call waits for the stream to drain and writes each task's duration in milliseconds.
 * ------------------------------------------------------------------------- */
typedef struct hanayo_pipeline_args {
  const hanayo_chunk_desc* desc;
  int P, W, M;
  const void* const* weights;
  float* const* grads;
  const void* const* x;
  const void* const* dy;
  void* const* act;
  void* const* grad;
  const int32_t* const* valid_len; /* host [M] -> device int32 [b], or NULL */
  void* const* stash_arena;
  const size_t* stash_arena_bytes;
  void* workspace;
  void* hip_stream;
  const struct hanayo_ends_args* ends; /* NULL, or the model's ends as in hanayo_exec_args (one lane); then x and
                                          dy are not read and may be NULL.  hanayo_pipeline_run only. */
} hanayo_pipeline_args;

int hanayo_pipeline_run(const hanayo_task* const* lists, const size_t* counts, const hanayo_pipeline_args* args,
                        int* peak_seen, float* const* task_ms);

/*
 * Host only.  Every rank runs its list strictly in order; a task starts when its rank is free and the task that
 * produces its input has finished; transfers take no time.  cost[r][i] = duration of task i of rank r in any
 * unit (NULL: forward 1, backward 2, the paper's model).  *makespan = time the last rank finishes;
 * idle[r] (may be NULL) = makespan minus rank r's summed durations.  HANAYO_ESTATE on lists that are not the
 * ranks' task sets or that deadlock.
 */
int hanayo_replay(const hanayo_task* const* lists, const size_t* counts, int P, int W, int M, const float* const* cost,
                  double* makespan, double* idle);

/*
 * The whole pipeline on one device from ACTION lists, with the communication carried out: every rank has
 * receive buffers of its own, and a send / receive pair is one device copy from the producer's output buffer
 * into the consumer's receive buffer (the emulated link).  Tables as for hanayo_pipeline_run, plus
 *   act_recv  [M*S]  index mb*S + stage: where rank(stage+1) receives the output of (mb, stage);
 *                    used only where stage+1 lives on another rank (may be NULL elsewhere)
 *   grad_recv [M*S]  index mb*S + stage: where rank(stage-1) receives the input gradient of (mb, stage);
 *                    used only where stage-1 lives on another rank
 *   async = 0        a transfer runs on hip_stream at the position of its receive action: a blocking receive,
 *                    nothing overlaps it
 *   async = 1        a transfer runs on a stream of the library's own (default priority, created once per
 *                    device) as soon as the message has been sent and its receive posted; receives are posted
 *                    with the paper's look-ahead (before a compute is enqueued, the receive of the following
 *                    compute is posted); only the consuming compute waits for the arrival
 *   link_workgroups  workgroups of the copy kernel (0 = as many as the size allows): a few workgroups move
 *                    data at a small, fixed fraction of the memory bandwidth, which stands in for a slow link
 * action_ms (host [P] -> host float [counts[r]], may be NULL): durations of the compute actions and, stored at
 * the receive action, of the transfers; send actions get 0; the call then waits for the stream to drain.
 * Results equal those of hanayo_pipeline_run.  Same list checks as hanayo_replay_actions; nothing is enqueued
 * if they fail.
 */
typedef struct hanayo_link_args {
  void* const* act_recv;
  void* const* grad_recv;
  int async;
  int link_workgroups;
} hanayo_link_args;

int hanayo_pipeline_run_actions(const hanayo_action* const* lists, const size_t* counts, const hanayo_pipeline_args* args,
                                const hanayo_link_args* link, int* peak_seen, float* const* action_ms);

/* ------------------------------------------------------------------------- *
 * Single kernels of the chunk path, exported so that each can be checked and
 * timed on its own (per-kernel parity tests and roofline measurements).  Same
 * conventions as above; `dtype` is HANAYO_FP32 / HANAYO_BF16.
 * ------------------------------------------------------------------------- */

enum {
  HANAYO_EPI_NONE = 0,      /* C = acc */
  HANAYO_EPI_BIAS = 1,      /* C = acc + bias[n] */
  HANAYO_EPI_BIAS_GELU = 2, /* aux_out = acc + bias[n]; C = GELU(aux_out) */
  HANAYO_EPI_BIAS_RES = 3,  /* C = acc + bias[n] + aux[m][n] */
  HANAYO_EPI_MUL_DGELU = 4, /* C = acc * GELU'(aux[m][n]) */
  HANAYO_EPI_ADD = 5,       /* C = acc + aux[m][n] */
  HANAYO_EPI_ACCUM_F32 = 6  /* C is fp32 and is accumulated into: C += acc */
};

/*
 * C[M][N] = A[M][K] B[K][N] with fp32 accumulation, then the epilogue.
 *   a_t = 0: A stored [M][lda], K contiguous;  1: stored [K][lda], M contiguous
 *   b_t = 0: B stored [N][ldb], K contiguous;  1: stored [K][ldb], N contiguous
 * C, aux, aux_out are row-major with leading dimension ldc; bias has N entries.
 * The forward linears use (a_t, b_t) = (0, 1), the input gradients (0, 0), the
 * weight gradients (1, 1) with HANAYO_EPI_ACCUM_F32.
 * colsum (device fp32 [N], may be NULL; needs b_t = 1 and ldb = N): colsum[n] += sum over k of B[k][n],
 * the bias gradient that belongs to a weight-gradient GEMM; the tiled bf16 MFMA kernels fold it into the
 * GEMM (the workgroups of the first tile row sum the B tiles they load anyway), the others run a
 * column-sum pass using colsum_scratch (device, at least 64 * N floats).  No atomics either way: the
 * sums are added in a fixed order and repeat bit for bit.
 */
int hanayo_op_gemm(int dtype, const void* A, const void* B, void* C, int M, int N, int K, int lda, int ldb, int ldc,
                   int a_t, int b_t, int epilogue, const void* bias, const void* aux, void* aux_out, float* colsum,
                   float* colsum_scratch, void* hip_stream);

/*
 * Up to 4 independent GEMMs of one layout and epilogue (arguments as for
 * hanayo_op_gemm) that go out as ONE launch where the tiled bf16 kernels take
 * every problem, else one after the other.  chunk_backward sends a block's four
 * weight-gradient GEMMs this way: none of them fills the chip alone.  The
 * problems must not write the same memory.
 */
typedef struct hanayo_gemm_problem {
  const void* A;
  const void* B;
  void* C;
  const void* bias;
  const void* aux;
  void* aux_out;
  int M, N, K;
  int lda, ldb, ldc;
  float* colsum;
  float* colsum_scratch;
} hanayo_gemm_problem;
int hanayo_op_gemm_group(int dtype, int a_t, int b_t, int epilogue, const hanayo_gemm_problem* problems, int count,
                         void* hip_stream);

/*
 * dst[0..bytes) = src[0..bytes), device to device, by a plain copy kernel
 * (16-byte granularity: bytes and both pointers multiples of 16; the ranges
 * must not overlap).  The post-LN chunk forward stashes its input with it; its
 * HBM traffic is exactly `bytes` read plus `bytes` written, which makes it the
 * kernel the hardware traffic counters are scaled against.
 */
int hanayo_op_copy(void* dst, const void* src, size_t bytes, void* hip_stream);

/* Tuning knob for measurements: which bf16 MFMA GEMM kernel hanayo_op_gemm and the chunk calls use.
   -1 (default) = chosen from the shape by a fitted cost model; 0 / 1 / 2 / 4 / 5 / 6 = direct-to-LDS
   kernel with 256x256 / 128x128 (8-deep load ring) / 256x128 / 128x128 (4-deep ring, two workgroups per
   CU) / 128x128 (8 wavefronts that split a K tile's MFMA steps) / 256x256 (8 wavefronts) tiles wherever
   the shape is a whole number of tiles; 7 / 8 / 9 = 256x256 (8 wavefronts) / 256x128 / 128x128 with two stages
   of 64-wide K tiles instead of four of 32 (K a multiple of 64); 10 / 11 = 256x128 / 128x128 with three such
   stages; 3 = register-staged kernel only.
   HANAYO_EINVAL outside -1..11.
   The setting belongs to the calling thread: it changes what this thread's later hanayo_op_gemm*, hanayo_chunk_*
   and executor calls dispatch, and nothing for other threads. */
int hanayo_op_gemm_config(int config);

/* out = LN(x) over the last dimension; stats[t] = (mean, rstd) as two floats;
   copy_out (may be NULL) receives a copy of x. */
int hanayo_op_layernorm_forward(int dtype, const void* x, const void* gamma, const void* beta, void* out,
                                float* stats, void* copy_out, int rows, int hidden, float eps, void* hip_stream);
/* dz = dLN(dout) (+ addend if not NULL); dgamma, dbeta (fp32, [hidden]) are added to.
   scratch: device, at least 1024 * hidden floats. */
int hanayo_op_layernorm_backward(int dtype, const void* dout, const void* x, const void* gamma, const float* stats,
                                 const void* addend, void* dz, float* dgamma, float* dbeta, float* scratch, int rows,
                                 int hidden, void* hip_stream);
/* For callers that cannot allocate device memory or have no workspace to hand over (code under HIP graph
   capture, tight serving loops, harnesses that forbid hipMalloc): hanayo_op_layernorm_backward without the
   scratch argument.  The partial gamma/beta sums go to a fixed 8 MiB device array inside the library (one
   copy per GPU, held until the process ends); the call allocates nothing and uses the same kernels, so the
   results are those of hanayo_op_layernorm_backward.  hidden: multiple of 8, at most 4096, HANAYO_EINVAL
   beyond that.  All calls on one GPU share the array: calls that may overlap on one GPU (different streams
   or threads) race on it and must be ordered by the caller. */
int hanayo_op_layernorm_backward_static(int dtype, const void* dout, const void* x, const void* gamma,
                                        const float* stats, const void* addend, void* dz, float* dgamma, float* dbeta,
                                        int rows, int hidden, void* hip_stream);
/* out[n] (fp32) += sum over rows of in[row][n].  scratch: at least 64 * n floats. */
int hanayo_op_colsum_add(int dtype, const void* in, int rows, int n, float* out, float* scratch, void* hip_stream);

/* qkv [b*s][3H] (Q | K | V), ctx [b*s][H], lse [b][heads][s] fp32 (log-sum-exp of the
   scaled, masked scores).  Backward reads qkv, ctx, lse, dctx and writes all of
   dqkv [b*s][3H]; delta is scratch [b][heads][s] fp32. */
int hanayo_op_attention_forward(int dtype, const void* qkv, const int32_t* valid_len, void* ctx, float* lse, int b,
                                int s, int heads, int head_dim, int causal, void* hip_stream);
int hanayo_op_attention_backward(int dtype, const void* qkv, const int32_t* valid_len, const void* ctx,
                                 const float* lse, const void* dctx, void* dqkv, float* delta, int b, int s,
                                 int heads, int head_dim, int causal, void* hip_stream);

/* Library / device facts for reports: writes a NUL-terminated description. */
int hanayo_device_info(char* buf /* host */, size_t cap);

#ifdef __cplusplus
}
#endif
#endif /* HANAYO_H */
