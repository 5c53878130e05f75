"""Oracle for the whole pipeline on one device.  TEST INFRASTRUCTURE ONLY.

Synchronous pipeline training computes exactly what the same model computes
without a pipeline (the paper's premise for comparing schedules: they differ in
time and memory, never in the result).  Two functions say that in code:

`monolithic` is the definition: every micro-batch goes forward through stages
0 .. S-1 in order, then backward from the loss gradient through S-1 .. 0;
parameter gradients are summed over the micro-batches.  No schedule is involved.

`run_pipeline` executes all P ranks' task lists the way P workers would: each
rank takes its own list strictly in order and a task starts as soon as the task
that produces its input has finished (the forward of the stage before, the
backward of the stage after, or, for the last stage's backward, its own
forward).  Stage boundaries are the dictionaries `act` and `grad`.

Both are built from the block oracle's chunk_forward / chunk_backward.  With
`ends` (dict(wte, wpe, head (None = tied to wte), lnf, tokens(m), labels(m),
loss_scale), see oracle/ends.py) the model starts from token ids and ends in
the loss: xs and dys are not used, and both functions also return the
micro-batch losses and the gradients of the tables, head and final LayerNorm.
"""

import numpy as np

from . import block as OB
from . import ends as OE
from . import schedule as OS


class _Ends:
    """Gradient accumulators of the model's ends, shared by the two functions below."""

    def __init__(self, ends):
        self.e = ends
        self.tied = ends["head"] is None
        self.head = ends["wte"] if self.tied else ends["head"]
        z = lambda a: np.zeros_like(a, dtype=np.float64)
        self.g = {"wte": z(ends["wte"]), "wpe": z(ends["wpe"]), "head": None if self.tied else z(self.head),
                  "lnf": None if ends["lnf"] is None else [z(ends["lnf"][0]), z(ends["lnf"][1])]}
        self.loss = {}

    def embed(self, m):
        return OE.embed_forward(self.e["wte"], self.e["wpe"], self.e["tokens"](m))

    def head_loss(self, m, y, eps):
        self.loss[m], dy, d_head, d_lnf = OE.head_loss(np.asarray(y, dtype=np.float64), self.e["labels"](m), self.head,
                                                      self.e["lnf"], eps, self.e["loss_scale"])
        self.g["wte" if self.tied else "head"] += d_head
        if d_lnf is not None:
            self.g["lnf"][0] += d_lnf[0]
            self.g["lnf"][1] += d_lnf[1]
        return dy

    def embed_backward(self, m, dx):
        a, b = OE.embed_backward(self.e["tokens"](m), np.asarray(dx, dtype=np.float64), self.e["wte"].shape[0],
                                 self.e["wpe"].shape[0])
        self.g["wte"] += a
        self.g["wpe"] += b


def monolithic(cfg, stage_params, xs, dys, valid_len=None, dtype=None, ends=None, M=None):
    """stage_params[s]: list of block dicts of stage s.  xs[m], dys[m]: input and loss gradient of
    micro-batch m (ignored with ends; then M gives the number of micro-batches).
    valid_len(m) -> key-padding lengths or None.
    Returns (ys, dxs, grads): model outputs, input gradients, grads[s] = list of per-block dicts;
    with ends (ys, dxs, grads, losses {m: value}, ends_grads)."""
    kw = {} if dtype is None else {"dtype": dtype}
    S = len(stage_params)
    grads = [None] * S
    ys, dxs = [], []
    en = _Ends(ends) if ends is not None else None
    for m in range(len(xs) if en is None else M):
        vl = valid_len(m) if valid_len is not None else None
        a = xs[m] if en is None else en.embed(m)
        stashes = []
        for s in range(S):
            a, st = OB.chunk_forward(stage_params[s], a, cfg, vl, **kw)
            stashes.append(st)
        ys.append(a)
        g = dys[m] if en is None else en.head_loss(m, a, cfg.eps)
        for s in range(S - 1, -1, -1):
            g, grads[s] = OB.chunk_backward(cfg, stashes[s], g, grads[s])
        dxs.append(g)
        if en is not None:
            en.embed_backward(m, g)
    if en is not None:
        return ys, dxs, grads, en.loss, en.g
    return ys, dxs, grads


def run_pipeline(lists, P, W, M, cfg, stage_params, xs, dys, valid_len=None, dtype=None, rank_order=None, ends=None):
    """lists[r]: rank r's ordered tasks (kind, mb, chunk, stage).  rank_order: the order in which the
    ranks are polled for a runnable head task (any order gives the same result; default 0 .. P-1).
    Returns dict(ys, dxs, grads, peak): as `monolithic`, plus the largest number of live stash
    entries per rank (with ends also losses and ends_grads; the head's forward and backward follow the
    forward task of the last stage, the embedding's backward the backward task of stage 0).
    Raises AssertionError on a list that deadlocks or runs a task twice."""
    kw = {} if dtype is None else {"dtype": dtype}
    S = OS.n_stages(P, W)          # W = 0: straight placement (GPipe / 1F1B lists)
    en = _Ends(ends) if ends is not None else None
    loss_grad = {}
    assert len(lists) == P and len(stage_params) == S and (en is not None or (len(xs) == M and len(dys) == M))
    order = list(range(P)) if rank_order is None else list(rank_order)
    act, grad, stash = {}, {}, {}
    grads = [None] * S
    head = [0] * P
    live = [0] * P
    peak = [0] * P
    progressed = True
    while progressed:
        progressed = False
        for r in order:
            while head[r] < len(lists[r]):
                kind, mb, chunk, stage = lists[r][head[r]]
                assert OS.stage_rank(P, W, stage) == r and chunk == stage // P
                vl = valid_len(mb) if valid_len is not None else None
                if kind == OS.F:
                    if stage > 0 and (mb, stage - 1) not in act:
                        break
                    assert (mb, stage) not in act, "forward repeated"
                    if stage == 0:
                        x = xs[mb] if en is None else en.embed(mb)
                    else:
                        x = act[(mb, stage - 1)]
                    act[(mb, stage)], stash[(mb, stage)] = OB.chunk_forward(stage_params[stage], x, cfg, vl, **kw)
                    if en is not None and stage == S - 1:
                        loss_grad[mb] = en.head_loss(mb, act[(mb, stage)], cfg.eps)
                    live[r] += 1
                    peak[r] = max(peak[r], live[r])
                else:
                    if stage < S - 1 and (mb, stage + 1) not in grad:
                        break
                    if (mb, stage) not in stash:
                        assert (mb, stage) not in grad, "backward repeated"
                        break
                    if stage == S - 1:
                        dy = dys[mb] if en is None else loss_grad.pop(mb)
                    else:
                        dy = grad[(mb, stage + 1)]
                    grad[(mb, stage)], grads[stage] = OB.chunk_backward(cfg, stash.pop((mb, stage)), dy, grads[stage])
                    if en is not None and stage == 0:
                        en.embed_backward(mb, grad[(mb, stage)])
                    live[r] -= 1
                head[r] += 1
                progressed = True
    assert all(head[r] == len(lists[r]) for r in range(P)), "deadlock"
    assert len(act) == M * S and len(grad) == M * S, "task missing"
    out = {"ys": [act[(m, S - 1)] for m in range(M)], "dxs": [grad[(m, 0)] for m in range(M)],
           "grads": grads, "peak": peak}
    if en is not None:
        out["losses"], out["ends_grads"] = en.loss, en.g
    return out
