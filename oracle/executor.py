"""Oracle for the per-rank task executor.  TEST INFRASTRUCTURE ONLY.

Walks one rank's ordered task list (the worker-side interpreter of the paper's
runtime section, compute actions only) with the block oracle.  Boundary data
follow the single-rank reading of a pipeline: the forward input of (mb, chunk)
is the output of the rank's previous chunk when the previous stage lives on the
same rank (the local turn-around), otherwise a given "received" tensor; the
backward input is the input-gradient of the rank's next chunk when the next
stage is local, otherwise a given "received" gradient.

With `ends` the rank that holds stage 0 builds that stage's input from token ids
(embedding) and the rank that holds the last stage turns that stage's output
into a loss and the gradient the backward pass starts from (head); in a wave
placement both are rank 0.  The head's forward and backward both happen right
after the last stage's forward task: the loss gradient needs nothing from
another rank.
"""

import numpy as np

from . import block as OB
from . import ends as OE
from . import schedule as OS


def run_rank(tasks, P, W, rank, cfg, chunk_params, act_in, grad_in, valid_len=None, dtype=None, ends=None):
    """tasks: list of (kind, mb, chunk, stage).  chunk_params[c]: list of block dicts.
    act_in(mb, chunk), grad_in(mb, chunk), valid_len(mb): callables returning arrays.
    ends: None or dict(wte, wpe, head (None = tied to wte), lnf ((gamma, beta) or None), tokens(mb),
    labels(mb), loss_scale); then act_in / grad_in are not asked for stage 0 / the last stage.
    Returns dict(act_out, grad_out, grads, peak) and with ends also loss {mb: value} and
    ends_grads dict(wte, wpe, head (None if tied: its gradient is inside wte), lnf)."""
    S = OS.n_stages(P, W)          # W = 0: the straight placement of a GPipe / 1F1B list (one chunk per rank)
    kw = {} if dtype is None else {"dtype": dtype}
    act_out, grad_out, stash = {}, {}, {}
    grads = [None] * OS.chunks_per_rank(W)
    peak = 0
    loss, loss_grad, eg = {}, {}, None
    if ends is not None:
        tied = ends["head"] is None
        head = ends["wte"] if tied else ends["head"]
        eg = {"wte": np.zeros_like(ends["wte"], dtype=np.float64), "wpe": np.zeros_like(ends["wpe"], dtype=np.float64),
              "head": None if tied else np.zeros_like(head, dtype=np.float64),
              "lnf": None if ends["lnf"] is None else [np.zeros_like(ends["lnf"][0], dtype=np.float64),
                                                       np.zeros_like(ends["lnf"][1], dtype=np.float64)]}
    for (kind, mb, chunk, stage) in tasks:
        assert OS.rank_stage(P, W, rank, chunk) == stage
        vl = valid_len(mb) if valid_len is not None else None
        if kind == OS.F:
            local = stage > 0 and OS.stage_rank(P, W, stage - 1) == rank
            if ends is not None and stage == 0:
                x = OE.embed_forward(ends["wte"], ends["wpe"], ends["tokens"](mb))
            else:
                x = act_out[(mb, chunk - 1)] if local else act_in(mb, chunk)
            y, st = OB.chunk_forward(chunk_params[chunk], x, cfg, vl, **kw)
            act_out[(mb, chunk)] = y
            if ends is not None and stage == S - 1:
                loss[mb], loss_grad[mb], d_head, d_lnf = OE.head_loss(
                    np.asarray(y, dtype=np.float64), ends["labels"](mb), head, ends["lnf"], cfg.eps, ends["loss_scale"])
                eg["wte" if tied else "head"] += d_head
                if d_lnf is not None:
                    eg["lnf"][0] += d_lnf[0]
                    eg["lnf"][1] += d_lnf[1]
            stash[(mb, chunk)] = st
            peak = max(peak, len(stash))
        else:
            local = stage < S - 1 and OS.stage_rank(P, W, stage + 1) == rank
            if ends is not None and stage == S - 1:
                dy = loss_grad.pop(mb)
            else:
                dy = grad_out[(mb, chunk + 1)] if local else grad_in(mb, chunk)
            dx, g = OB.chunk_backward(cfg, stash.pop((mb, chunk)), dy)
            grad_out[(mb, chunk)] = dx
            if ends is not None and stage == 0:
                d_wte, d_wpe = OE.embed_backward(ends["tokens"](mb), np.asarray(dx, dtype=np.float64),
                                                 ends["wte"].shape[0], ends["wpe"].shape[0])
                eg["wte"] += d_wte
                eg["wpe"] += d_wpe
            if grads[chunk] is None:
                grads[chunk] = g
            else:
                grads[chunk] = [{k: a[k] + b[k] for k in a} for a, b in zip(grads[chunk], g)]
    out = {"act_out": act_out, "grad_out": grad_out, "grads": grads, "peak": peak}
    if ends is not None:
        out["loss"], out["ends_grads"] = loss, eg
    return out
