"""Oracle for the wave schedule of one pipeline rank.  TEST INFRASTRUCTURE ONLY.

What the paper fixes (Table 1 and the section on transforming Chimera into
wave-like pipelines):

  * S = 2*W*P stages live on P devices, 2W per device (W = S / 2P).
  * A micro-batch walks down the devices 0..P-1, turns round, walks back
    P-1..0, and does so W times ("V" shapes); the two stages at each turn sit
    on the same device, so that hand-off is local.
  * Backward costs twice forward (figure captions, theoretical analysis with
    T_B = 2 T_F and T_C = 0).
  * Activations are consumed by the backward pass as soon as they exist
    (memory evaluation), and M_a is the same as for other synchronous schemes.

The order of tasks on a rank is drawn only in figures, so the order produced
here is a stated reading: a deterministic, work-conserving list schedule

  R1  integer clock; every rank that is free at time t starts one ready task
  R2  ready = on this rank, not started, predecessor finished at or before t
  R3  any ready backward beats any ready forward
  R4  ties: smallest micro-batch index
  R5  F(m, 0) for m >= P waits until F(m-P, S-1) has finished (at most P
      micro-batches in their forward phase, so the stash stays bounded)
  R6  F(m, 0) waits until F(m-1, 0) has started
  R7  a rank with nothing ready idles until the next finish event

with costs F = 1, B = 2, transfers = 0.

Because F(m,s) needs F(m,s-1), B(m,S-1) needs F(m,S-1) and B(m,s) needs
B(m,s+1), each micro-batch is one linear chain F0..F(S-1), B(S-1)..B0: the
ready set of a rank is the set of micro-batches whose next chain element lives
on that rank and whose previous element has finished.
"""

from collections import namedtuple

F, B = 0, 1
COST = {F: 1, B: 2}

Task = namedtuple("Task", "kind mb chunk stage")


def n_stages(P, W):
    """W waves: 2*W*P stages.  W = 0 denotes the straight placement of the comparison schemes (GPipe, 1F1B):
    one stage per device, S = P, half a wave in Table 1's W = S / 2P; stage_rank / rank_stage then reduce to
    stage s on device s."""
    return 2 * W * P if W else P


def chunks_per_rank(W):
    return 2 * W if W else 1


def stage_rank(P, W, stage):
    """Device that holds a stage: even passes run 0..P-1, odd passes P-1..0."""
    if not (0 <= stage < n_stages(P, W)):
        raise ValueError("stage out of range")
    c, r = divmod(stage, P)
    return r if c % 2 == 0 else P - 1 - r


def rank_stage(P, W, rank, chunk):
    """Global stage of a rank's local chunk (chunk = stage // P)."""
    if not (0 <= rank < P and 0 <= chunk < chunks_per_rank(W)):
        raise ValueError("rank/chunk out of range")
    return chunk * P + (rank if chunk % 2 == 0 else P - 1 - rank)


def _check(P, W, M):
    if P < 1 or W < 1 or M < 1:
        raise ValueError("P, W, M must be >= 1")


def simulate(P, W, M):
    """Run the whole pipeline under R1-R7.

    Returns a dict with
      lists[r]   ordered list of Task for rank r (its start order)
      starts[r]  start time of each of those tasks
      makespan   finish time of the last task
      idle[r]    makespan - busy time of rank r
    """
    _check(P, W, M)
    S = n_stages(P, W)
    chain = [(F, s) for s in range(S)] + [(B, s) for s in range(S - 1, -1, -1)]
    nxt = [0] * M                 # index into chain of the next task of micro-batch m
    prev_finish = [0] * M         # finish time of the chain element before it
    started_f0 = [False] * M
    finish_last_f = [None] * M    # finish time of F(m, S-1)
    free_at = [0] * P
    lists = [[] for _ in range(P)]
    starts = [[] for _ in range(P)]
    running = []                  # finish times of tasks in flight
    remaining = M * len(chain)
    t = 0
    while remaining:
        for r in range(P):
            if free_at[r] > t:
                continue
            best = None
            for m in range(M):
                if nxt[m] >= len(chain):
                    continue
                kind, s = chain[nxt[m]]
                if stage_rank(P, W, s) != r or prev_finish[m] > t:
                    continue
                if kind == F and s == 0:
                    if m >= P and (finish_last_f[m - P] is None or finish_last_f[m - P] > t):
                        continue                        # R5
                    if m >= 1 and not started_f0[m - 1]:
                        continue                        # R6
                key = (0 if kind == B else 1, m)        # R3 then R4
                if best is None or key < best[0]:
                    best = (key, m, kind, s)
            if best is None:
                continue                                # R7
            _, m, kind, s = best
            end = t + COST[kind]
            lists[r].append(Task(kind, m, s // P, s))
            starts[r].append(t)
            free_at[r] = end
            prev_finish[m] = end
            nxt[m] += 1
            if kind == F and s == 0:
                started_f0[m] = True
            if kind == F and s == S - 1:
                finish_last_f[m] = end
            running.append(end)
            remaining -= 1
        later = [e for e in running if e > t]
        if not later:
            if remaining:
                raise RuntimeError("schedule deadlocked")
            break
        running = later
        t = min(later)
    makespan = max(free_at)
    busy = [sum(COST[k.kind] for k in lists[r]) for r in range(P)]
    return {
        "lists": lists,
        "starts": starts,
        "makespan": makespan,
        "idle": [makespan - b for b in busy],
    }


def schedule(P, W, M, rank):
    """Ordered F/B task list of one rank: 4*W*M records (kind, mb, chunk, stage)."""
    _check(P, W, M)
    if not (0 <= rank < P):
        raise ValueError("rank out of range")
    return simulate(P, W, M)["lists"][rank]


def stash_plan(tasks, W):
    """Activation-stash accounting of one rank's list.

    An entry is alive from the F task of (mb, chunk) to its B task.  Returns
    (peak_total, per_chunk_peak[2W], slot[len(tasks)]) where slot[i] is, for an
    F task, the smallest slot id of its chunk that is free at that point, for
    a B task the id its F took.  Raises on a B without a live F or a second F
    of a live (mb, chunk).
    """
    nchunk = chunks_per_rank(W)
    live = {}
    used = [set() for _ in range(nchunk)]
    per_chunk = [0] * nchunk
    peak = 0
    slot = []
    for tk in tasks:
        key = (tk.mb, tk.chunk)
        if tk.kind == F:
            if key in live:
                raise ValueError("forward of a live entry")
            sid = 0
            while sid in used[tk.chunk]:
                sid += 1
            used[tk.chunk].add(sid)
            live[key] = sid
            per_chunk[tk.chunk] = max(per_chunk[tk.chunk], len(used[tk.chunk]))
            peak = max(peak, len(live))
        else:
            if key not in live:
                raise ValueError("backward without a live forward")
            sid = live.pop(key)
            used[tk.chunk].remove(sid)
        slot.append(sid)
    if live:
        raise ValueError("entries still live at the end of the list")
    return peak, per_chunk, slot


def bubble_ratio_printed(P, W):
    """Simplified ratio the theoretical analysis prints for T_B = 2 T_F, T_C = 0."""
    return (2 * P - 2) / (3 * P * W + P - 1)


def bubble_idle_numerator(P, W, t_f_stage=1):
    """Idle time per rank implied by the numerator of the bubble equation at
    T_C = 0: (P-1) * T_B / W with T_B = 2 T_F and T_F = 2W chunk-forwards,
    i.e. 4 (P-1) in units of one chunk forward."""
    T_F = 2 * W * t_f_stage
    T_B = 2 * T_F
    return (P - 1) * T_B / W
