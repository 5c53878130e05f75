"""Device-side plumbing for callers of the binding: moves seeded host arrays into
torch device tensors, owns the buffers one chunk or one rank needs, and calls
the library.  No arithmetic of the method happens here."""

import numpy as np
import torch

from . import hanayo as hn
from . import synth


def dev(a, dtype):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.bfloat16() if dtype == "bf16" else t


def host(t):
    return t.float().cpu().numpy()


def dev_bytes(n):
    return torch.empty(int(n), dtype=torch.uint8, device="cuda")


class GpuChunk:
    """One chunk's device state: packed weights, fp32 grads, workspace."""

    def __init__(self, wl, params):
        self.wl = wl
        self.desc = hn.desc_for(wl)
        self.params = params
        self.weights = dev(hn.pack_params(self.desc, params), wl.dtype)
        assert self.weights.numel() * self.weights.element_size() <= hn.hanayo_weight_bytes(self.desc)
        self.grads = torch.zeros(hn.hanayo_grad_bytes(self.desc) // 4, dtype=torch.float32, device="cuda")
        self.work = dev_bytes(hn.hanayo_workspace_bytes(self.desc))

    def new_stash(self):
        return dev_bytes(hn.hanayo_stash_bytes(self.desc))

    def forward(self, x, valid_len=None, stash=None):
        wl = self.wl
        xd = dev(x, wl.dtype)
        y = torch.empty_like(xd)
        stash = self.new_stash() if stash is None else stash
        vl = None if valid_len is None else torch.from_numpy(np.asarray(valid_len, dtype=np.int32)).cuda()
        hn.hanayo_chunk_forward(self.desc, self.weights, xd, vl, y, stash, self.work)
        torch.cuda.synchronize()
        return host(y), (stash, vl)

    def backward(self, dy, stash):
        wl = self.wl
        st, vl = stash
        dyd = dev(dy, wl.dtype)
        dx = torch.empty_like(dyd)
        hn.hanayo_chunk_backward(self.desc, self.weights, self.grads, dyd, vl, st, dx, self.work)
        torch.cuda.synchronize()
        return host(dx)

    def grad_dicts(self):
        return hn.unpack_params(self.desc, self.grads.cpu().numpy(), self.params)


class _EndsState:
    """Device state of the model's ends (tables, their gradients, tokens, labels, losses, workspace), set
    as attributes on the GpuRank / GpuPipeline that owns it."""

    @staticmethod
    def init(o, wl, desc, lanes, like, tied):
        M = wl.M
        o.ends_params = p = synth.ends_params(wl)
        o.ends_desc = e = hn.EndsDesc(wl.vocab, wl.seq, int(p["lnf"] is not None))
        f32 = lambda shape: torch.zeros(shape, dtype=torch.float32, device="cuda")
        o.wte, o.wpe = dev(p["wte"], wl.dtype), dev(p["wpe"], wl.dtype)
        o.d_wte, o.d_wpe = f32(p["wte"].shape), f32(p["wpe"].shape)
        o.tied = tied
        if tied:
            o.head, o.d_head = o.wte, o.d_wte
        else:
            o.head_host = synth.untied_head(wl)
            o.head, o.d_head = dev(o.head_host, wl.dtype), f32(p["wte"].shape)
        o.lnf = dev(np.concatenate(p["lnf"]), wl.dtype) if p["lnf"] is not None else None
        o.d_lnf = f32(2 * wl.hidden) if p["lnf"] is not None else None
        o.tokens = [torch.from_numpy(synth.token_ids(wl, m)).cuda() for m in range(M)]
        o.labels = [torch.from_numpy(synth.labels(wl, m)).cuda() for m in range(M)]
        o.loss = torch.full((M,), -1.0, dtype=torch.float32, device="cuda")
        o.loss_grad = [torch.empty_like(like) for _ in range(M)]
        o.ends_work = dev_bytes(max(lanes, 1) * hn.hanayo_ends_workspace_bytes(desc, e))
        o.ends = hn.make_ends_args(e, o.wte, o.d_wte, o.wpe, o.d_wpe, o.head, o.d_head, o.lnf, o.d_lnf, o.tokens,
                                   o.labels, o.loss, o.loss_grad, 1.0 / M, o.ends_work)

    @staticmethod
    def tensors(o):
        """[(name, parameter tensor, fp32 gradient tensor)] of the embedding tables, head and final LayerNorm."""
        out = [("wte", o.wte, o.d_wte), ("wpe", o.wpe, o.d_wpe)]
        if not o.tied:
            out.append(("head", o.head, o.d_head))
        if o.lnf is not None:
            out.append(("lnf", o.lnf, o.d_lnf))
        return out


class GpuRank:
    """Device state of one rank of a workload: per-chunk weights/grads, boundary
    tables, stash arena, workspace; runs a task list through hanayo_executor_run."""

    def __init__(self, wl, rank=0, tasks=None, unique_outputs=True, lanes=1, stash_mode=0, ends=False, tied=True):
        """ends: rank 0 embeds tokens in front of stage 0 and ends the last stage in the loss (tied: the
        head is the token table itself)."""
        self.wl, self.rank, self.lanes, self.stash_mode = wl, rank, lanes, stash_mode
        self.desc = hn.desc_for(wl)
        P, W, M = wl.P, wl.W, wl.M
        self.nchunk = hn.chunks_per_rank(W)        # W = 0: the straight placement of a GPipe / 1F1B list
        assert W > 0 or tasks is not None, "a straight placement has no wave schedule: pass the scheme's list"
        self.tasks = hn.hanayo_schedule(P, W, M, rank) if tasks is None else tasks
        self.params = [synth.chunk_params(wl, c) for c in range(self.nchunk)]
        self.weights = [dev(hn.pack_params(self.desc, p), wl.dtype) for p in self.params]
        self.grads = [torch.zeros(hn.hanayo_grad_bytes(self.desc) // 4, dtype=torch.float32, device="cuda")
                      for _ in range(self.nchunk)]
        self.work = dev_bytes(lanes * hn.hanayo_workspace_bytes(self.desc))
        self.scratch = None
        if stash_mode == hn.STASH_INPUT:
            self.arena_bytes = hn.hanayo_stash_arena_bytes_input(self.tasks, W, self.desc)
            self.scratch = dev_bytes(max(lanes, 1) * hn.hanayo_recompute_scratch_bytes(self.desc))
        else:
            self.arena_bytes = hn.hanayo_stash_arena_bytes(self.tasks, W, self.desc)
        self.arena = dev_bytes(self.arena_bytes)
        S = self.nchunk * P
        n = M * self.nchunk
        self.act_in, self.grad_in = [None] * n, [None] * n
        self.act_out, self.grad_out = [None] * n, [None] * n
        tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
        shape = (wl.mb, wl.seq, wl.hidden)
        for m in range(M):
            for c in range(self.nchunk):
                stage = hn.hanayo_rank_stage(P, W, rank, c)
                i = m * self.nchunk + c
                if not (stage > 0 and hn.hanayo_stage_rank(P, W, stage - 1) == rank):
                    self.act_in[i] = dev(synth.forward_input(wl, m, c), wl.dtype)
                if not (stage < S - 1 and hn.hanayo_stage_rank(P, W, stage + 1) == rank):
                    self.grad_in[i] = dev(synth.upstream_grad(wl, m, c), wl.dtype)
                self.act_out[i] = torch.empty(shape, dtype=tdt, device="cuda")
                self.grad_out[i] = torch.empty(shape, dtype=tdt, device="cuda")
        self.valid_len = None
        if wl.valid_len_range is not None:
            self.valid_len = [torch.from_numpy(synth.valid_lengths(wl, m)).cuda() for m in range(M)]
        self.ends = None
        if ends and rank == 0:
            self._init_ends(tied)
        self.opt = None

    def _init_ends(self, tied):
        _EndsState.init(self, self.wl, self.desc, self.lanes, self.act_out[0], tied)
        # with ends the executor must not read the synthetic stage-0 inputs and last-stage gradients
        for m in range(self.wl.M):
            self.act_in[m * self.nchunk] = None
            self.grad_in[m * self.nchunk + self.nchunk - 1] = None

    def ends_tensors(self):
        return _EndsState.tensors(self)

    def zero_grads(self):
        for g in self.grads:
            g.zero_()
        if self.ends is not None:
            for _, _, g in self.ends_tensors():
                g.zero_()

    def run(self, tasks=None, stream=None):
        wl = self.wl
        return hn.hanayo_executor_run(self.tasks if tasks is None else tasks, self.desc, wl.P, wl.W, wl.M, self.rank,
                                      self.weights, self.grads, self.act_in, self.grad_in, self.act_out,
                                      self.grad_out, self.valid_len, self.arena, self.arena_bytes, self.work, stream, self.lanes,
                                      self.stash_mode, self.scratch, self.ends)

    def grad_dicts(self, chunk):
        return hn.unpack_params(self.desc, self.grads[chunk].cpu().numpy(), self.params[chunk])

    # ---- the parameter update at the flush

    def init_optimizer(self):
        """Adam state for every parameter of the rank: fp32 moments, and fp32 master copies for bf16 storage."""
        bf16 = self.wl.dtype == "bf16"
        groups = [("chunk", w, g) for w, g in zip(self.weights, self.grads)]
        if self.ends is not None:
            groups += [(n, w.view(-1), g.view(-1)) for n, w, g in self.ends_tensors()]
        self.opt = [dict(kind=k, w=w, g=g, master=w.float() if bf16 else None, m=torch.zeros_like(g),
                         v=torch.zeros_like(g)) for k, w, g in groups]
        self.opt_step = 0

    def adam_step(self, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, zero_grads=True, stream=None):
        """One update of everything the rank owns, to be called after run(): the flush of the iteration.
        Decay goes to the chunks' matrices and the tables, not to biases and LayerNorm parameters."""
        self.opt_step += 1
        dt = hn.BF16 if self.wl.dtype == "bf16" else hn.FP32
        for o in self.opt:
            wd = 0.0 if o["kind"] == "lnf" else weight_decay
            adam = hn.Adam(lr, beta1, beta2, eps, wd, self.opt_step, int(zero_grads))
            if o["kind"] == "chunk":
                hn.hanayo_chunk_adam_step(adam, self.desc, o["w"], o["master"], o["g"], o["m"], o["v"], stream)
            else:
                hn.hanayo_adam_step(adam, dt, o["w"], o["master"], o["g"], o["m"], o["v"], o["g"].numel(), stream)


class GpuPipeline:
    """Device state of ALL ranks of a workload on one GPU: per-stage weights/grads, model inputs and loss
    gradients per micro-batch, every stage-boundary buffer, one stash arena per rank; runs the P task
    lists with true dataflow through hanayo_pipeline_run."""

    def __init__(self, wl, ends=False, lists=None):
        """ends: the model starts from token ids and ends in the loss (tied head), see GpuRank.
        lists: the P task lists (default: the wave schedule's; required for a straight placement, wl.W = 0)."""
        self.wl = wl
        self.desc = hn.desc_for(wl)
        P, W, M = wl.P, wl.W, wl.M
        self.S = S = hn.chunks_per_rank(W) * P
        self.lists = [hn.hanayo_schedule(P, W, M, r) for r in range(P)] if lists is None else lists
        self.params = [synth.stage_params(wl, s) for s in range(S)]
        self.weights = [dev(hn.pack_params(self.desc, p), wl.dtype) for p in self.params]
        self.grads = [torch.zeros(hn.hanayo_grad_bytes(self.desc) // 4, dtype=torch.float32, device="cuda")
                      for _ in range(S)]
        self.work = dev_bytes(hn.hanayo_workspace_bytes(self.desc))
        self.arenas = [dev_bytes(hn.hanayo_stash_arena_bytes(t, W, self.desc)) for t in self.lists]
        tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
        shape = (wl.mb, wl.seq, wl.hidden)
        self.x = [dev(synth.model_input(wl, m), wl.dtype) for m in range(M)]
        self.dy = [dev(synth.loss_grad(wl, m), wl.dtype) for m in range(M)]
        self.act = [torch.empty(shape, dtype=tdt, device="cuda") for _ in range(M * S)]
        self.grad = [torch.empty(shape, dtype=tdt, device="cuda") for _ in range(M * S)]
        self.valid_len = None
        if wl.valid_len_range is not None:
            self.valid_len = [torch.from_numpy(synth.valid_lengths(wl, m)).cuda() for m in range(M)]
        self.ends = None
        if ends:
            _EndsState.init(self, wl, self.desc, 1, self.act[0], True)
            self.x = self.dy = None

    def zero_grads(self):
        for g in self.grads:
            g.zero_()
        if self.ends is not None:
            for _, _, g in _EndsState.tensors(self):
                g.zero_()

    def run(self, lists=None, timing=False, stream=None):
        wl = self.wl
        return hn.hanayo_pipeline_run(self.lists if lists is None else lists, self.desc, wl.P, wl.W, wl.M,
                                      self.weights, self.grads, self.x, self.dy, self.act, self.grad, self.valid_len,
                                      self.arenas, self.work, stream, timing, self.ends)

    def grad_dicts(self, stage):
        return hn.unpack_params(self.desc, self.grads[stage].cpu().numpy(), self.params[stage])

    def enable_links(self):
        """Action lists and per-rank receive buffers for every stage boundary that crosses ranks."""
        wl, S = self.wl, self.S
        self.actions = [hn.hanayo_actions(wl.P, wl.W, wl.M, r) for r in range(wl.P)]
        rank = [hn.hanayo_stage_rank(wl.P, wl.W, s) for s in range(S)]
        like = self.act[0]
        self.act_recv = [None] * (wl.M * S)
        self.grad_recv = [None] * (wl.M * S)
        for m in range(wl.M):
            for s in range(S):
                if s < S - 1 and rank[s + 1] != rank[s]:
                    self.act_recv[m * S + s] = torch.empty_like(like)
                if s > 0 and rank[s - 1] != rank[s]:
                    self.grad_recv[m * S + s] = torch.empty_like(like)

    def run_actions(self, async_copies=True, link_workgroups=0, timing=False, lists=None, stream=None):
        wl = self.wl
        return hn.hanayo_pipeline_run_actions(self.actions if lists is None else lists, self.desc, wl.P, wl.W, wl.M,
                                              self.weights, self.grads, self.x, self.dy, self.act, self.grad,
                                              self.valid_len, self.arenas, self.work, self.act_recv, self.grad_recv,
                                              async_copies, link_workgroups, stream, timing, self.ends)
