"""Oracle for the per-rank task executor.  TEST INFRASTRUCTURE ONLY.

Walks one rank's ordered task list (the worker-side interpreter of the paper's
runtime section, compute actions only) with the block oracle.  Boundary data
follow the single-rank reading of a pipeline: the forward input of (mb, chunk)
is the output of the rank's previous chunk when the previous stage lives on the
same rank (the local turn-around), otherwise a given "received" tensor; the
backward input is the input-gradient of the rank's next chunk when the next
stage is local, otherwise a given "received" gradient.
"""

from . import block as OB
from . import schedule as OS


def run_rank(tasks, P, W, rank, cfg, chunk_params, act_in, grad_in, valid_len=None, dtype=None):
    """tasks: list of (kind, mb, chunk, stage).  chunk_params[c]: list of block dicts.
    act_in(mb, chunk), grad_in(mb, chunk), valid_len(mb): callables returning arrays.
    Returns dict(act_out, grad_out, grads, peak)."""
    S = 2 * W * P
    kw = {} if dtype is None else {"dtype": dtype}
    act_out, grad_out, stash = {}, {}, {}
    grads = [None] * (2 * W)
    peak = 0
    for (kind, mb, chunk, stage) in tasks:
        assert OS.rank_stage(P, W, rank, chunk) == stage
        vl = valid_len(mb) if valid_len is not None else None
        if kind == OS.F:
            local = stage > 0 and OS.stage_rank(P, W, stage - 1) == rank
            x = act_out[(mb, chunk - 1)] if local else act_in(mb, chunk)
            y, st = OB.chunk_forward(chunk_params[chunk], x, cfg, vl, **kw)
            act_out[(mb, chunk)] = y
            stash[(mb, chunk)] = st
            peak = max(peak, len(stash))
        else:
            local = stage < S - 1 and OS.stage_rank(P, W, stage + 1) == rank
            dy = grad_out[(mb, chunk + 1)] if local else grad_in(mb, chunk)
            dx, g = OB.chunk_backward(cfg, stash.pop((mb, chunk)), dy)
            grad_out[(mb, chunk)] = dx
            if grads[chunk] is None:
                grads[chunk] = g
            else:
                grads[chunk] = [{k: a[k] + b[k] for k in a} for a, b in zip(grads[chunk], g)]
    return {"act_out": act_out, "grad_out": grad_out, "grads": grads, "peak": peak}
