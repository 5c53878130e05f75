"""Brute-force replay of a full set of per-rank task lists.  TEST INFRASTRUCTURE ONLY.

Independent of schedule.py: it knows only the dependency rules of synchronous
pipeline training (forward of a stage needs the forward of the stage before,
the last stage's backward needs its own forward, every other backward needs
the backward of the stage after) and the cost model F = 1, B = 2, transfer = 0
of the paper's theoretical analysis.  Each rank executes ITS list strictly in
order, blocking until the head task's dependency has finished.

`replay` validates any lists (from the oracle, from the HIP library's host
code, or hand-written).  `greedy_audit` additionally re-derives, at every
decision the lists imply, the complete ready set from the per-task dependency
rules and checks the choice against "backward first, then lowest micro-batch",
the injection gate and work conservation.
"""

F, B = 0, 1


def _placement(P, W, stage):
    lap, pos = divmod(stage, P)
    return pos if lap % 2 == 0 else P - 1 - pos


def _n_stages(P, W):
    """W waves: 2*W*P stages.  W = 0 stands for the straight placement of GPipe and 1F1B (one stage per
    device, half a wave in Table 1's W = S / 2P), where stage s sits on device s."""
    return 2 * W * P if W else P


def replay(lists, P, W, M, cost_f=1, cost_b=2, cost=None):
    """Execute the lists; return dict(makespan, idle, start, finish, peak).

    cost (optional): callable (kind, mb, stage) -> duration of that task, instead of the
    uniform cost_f / cost_b (used to replay measured task times).

    Raises AssertionError on: wrong rank for a stage, a task missing or
    repeated, chunk field inconsistent with the stage, deadlock.
    """
    S = _n_stages(P, W)
    assert len(lists) == P
    seen = set()
    for r, lst in enumerate(lists):
        assert len(lst) == 2 * (S // P) * M, "rank %d: list length" % r
        for (kind, mb, chunk, stage) in lst:
            assert kind in (F, B) and 0 <= mb < M and 0 <= stage < S
            assert _placement(P, W, stage) == r, "task on the wrong rank"
            assert chunk == stage // P, "chunk field"
            assert (kind, mb, stage) not in seen, "task repeated"
            seen.add((kind, mb, stage))
    assert len(seen) == 2 * M * S, "task missing"

    finish = {}
    start = {}
    head = [0] * P
    free_at = [0] * P
    progressed = True
    while progressed:
        progressed = False
        for r in range(P):
            while head[r] < len(lists[r]):
                kind, mb, chunk, stage = lists[r][head[r]]
                if kind == F:
                    dep = None if stage == 0 else (F, mb, stage - 1)
                else:
                    dep = (F, mb, stage) if stage == S - 1 else (B, mb, stage + 1)
                if dep is not None and dep not in finish:
                    break
                if kind == B:
                    assert (F, mb, stage) in finish, "backward before its forward"
                ready_at = 0 if dep is None else finish[dep]
                t0 = max(free_at[r], ready_at)
                t1 = t0 + (cost(kind, mb, stage) if cost is not None else (cost_f if kind == F else cost_b))
                start[(kind, mb, stage)] = t0
                finish[(kind, mb, stage)] = t1
                free_at[r] = t1
                head[r] += 1
                progressed = True
    assert all(head[r] == len(lists[r]) for r in range(P)), "deadlock"
    makespan = max(free_at)
    busy = [sum(cost(k, m, s) if cost is not None else (cost_f if k == F else cost_b) for (k, m, _, s) in lst)
            for lst in lists]

    peak = []
    for lst in lists:
        live = 0
        top = 0
        for (kind, _, _, _) in lst:
            live += 1 if kind == F else -1
            top = max(top, live)
        peak.append(top)
    return {
        "makespan": makespan,
        "idle": [makespan - b for b in busy],
        "start": start,
        "finish": finish,
        "peak": peak,
    }


def greedy_audit(lists, P, W, M):
    """Check that the lists are what the stated greedy rules produce.

    Uses the replay's start/finish times.  For every task X started on rank r
    at time t: enumerate ALL 2*M*S tasks, keep those on rank r, not started
    before t, whose dependency finished at or before t and (for a first-stage
    forward) whose gates are open; X must be the minimum of that set under
    (backward first, micro-batch).  Also the rank must not have been idle just
    before t while something was ready (work conservation): the rank's previous
    task must end at t, or nothing was ready at any earlier event time.
    """
    S = 2 * W * P
    rep = replay(lists, P, W, M)
    start, finish = rep["start"], rep["finish"]
    event_times = sorted(set(finish.values()) | {0})

    def ready_set(r, t):
        out = []
        for kind in (F, B):
            for mb in range(M):
                for stage in range(S):
                    if _placement(P, W, stage) != r:
                        continue
                    if start[(kind, mb, stage)] < t:
                        continue
                    if kind == F:
                        if stage > 0:
                            ok = finish[(F, mb, stage - 1)] <= t
                        else:
                            ok = True
                            if mb >= P:
                                ok = ok and finish[(F, mb - P, S - 1)] <= t
                            if mb >= 1:
                                # both live on rank 0, one start per instant
                                ok = ok and start[(F, mb - 1, 0)] < t
                    else:
                        if stage == S - 1:
                            ok = finish[(F, mb, stage)] <= t
                        else:
                            ok = finish[(B, mb, stage + 1)] <= t
                    if ok:
                        out.append((0 if kind == B else 1, mb, kind, stage))
        return sorted(out)

    for r in range(P):
        prev_end = 0
        for (kind, mb, chunk, stage) in lists[r]:
            t = start[(kind, mb, stage)]
            rs = ready_set(r, t)
            assert rs, "started a task that is not ready"
            assert rs[0][1:] == (mb, kind, stage), (
                "rank %d t=%d chose %s but rules pick %s" % (r, t, (kind, mb, stage), rs[0]))
            if t > prev_end:
                for te in event_times:
                    if prev_end <= te < t:
                        assert not ready_set(r, te), "rank idled while a task was ready"
            prev_end = finish[(kind, mb, stage)]
    return rep
