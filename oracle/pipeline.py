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

Both are built from the block oracle's chunk_forward / chunk_backward.
"""

from . import block as OB
from . import schedule as OS


def monolithic(cfg, stage_params, xs, dys, valid_len=None, dtype=None):
    """stage_params[s]: list of block dicts of stage s.  xs[m], dys[m]: input and loss gradient of
    micro-batch m.  valid_len(m) -> key-padding lengths or None.
    Returns (ys, dxs, grads): model outputs, input gradients, grads[s] = list of per-block dicts."""
    kw = {} if dtype is None else {"dtype": dtype}
    S = len(stage_params)
    grads = [None] * S
    ys, dxs = [], []
    for m in range(len(xs)):
        vl = valid_len(m) if valid_len is not None else None
        a = xs[m]
        stashes = []
        for s in range(S):
            a, st = OB.chunk_forward(stage_params[s], a, cfg, vl, **kw)
            stashes.append(st)
        ys.append(a)
        g = dys[m]
        for s in range(S - 1, -1, -1):
            g, grads[s] = OB.chunk_backward(cfg, stashes[s], g, grads[s])
        dxs.append(g)
    return ys, dxs, grads


def run_pipeline(lists, P, W, M, cfg, stage_params, xs, dys, valid_len=None, dtype=None, rank_order=None):
    """lists[r]: rank r's ordered tasks (kind, mb, chunk, stage).  rank_order: the order in which the
    ranks are polled for a runnable head task (any order gives the same result; default 0 .. P-1).
    Returns dict(ys, dxs, grads, peak): as `monolithic`, plus the largest number of live stash
    entries per rank.  Raises AssertionError on a list that deadlocks or runs a task twice."""
    kw = {} if dtype is None else {"dtype": dtype}
    S = 2 * W * P
    assert len(lists) == P and len(stage_params) == S and len(xs) == M and len(dys) == M
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
                    x = xs[mb] if stage == 0 else act[(mb, stage - 1)]
                    act[(mb, stage)], stash[(mb, stage)] = OB.chunk_forward(stage_params[stage], x, cfg, vl, **kw)
                    live[r] += 1
                    peak[r] = max(peak[r], live[r])
                else:
                    if stage < S - 1 and (mb, stage + 1) not in grad:
                        break
                    if (mb, stage) not in stash:
                        assert (mb, stage) not in grad, "backward repeated"
                        break
                    dy = dys[mb] if stage == S - 1 else grad[(mb, stage + 1)]
                    grad[(mb, stage)], grads[stage] = OB.chunk_backward(cfg, stash.pop((mb, stage)), dy, grads[stage])
                    live[r] -= 1
                head[r] += 1
                progressed = True
    assert all(head[r] == len(lists[r]) for r in range(P)), "deadlock"
    assert len(act) == M * S and len(grad) == M * S, "task missing"
    return {"ys": [act[(m, S - 1)] for m in range(M)], "dxs": [grad[(m, 0)] for m in range(M)],
            "grads": grads, "peak": peak}
