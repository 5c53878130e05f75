"""Oracle for the comparison schedules and the bubble model.  TEST INFRASTRUCTURE ONLY.

The paper's background section describes the synchronous schemes Hanayo is
measured against, and its runtime section says the scheduler ships "scheduling
algorithms for existing mainstream pipeline schemes" that emit the same kind
of per-worker list.  This module writes those schemes out as their definitions:

  GPipe         one stage per device (S = P).  Every device runs the forward
                passes of all micro-batches, then the backward passes of all
                micro-batches (background section: the devices pipeline the
                forward computation and, after all forward computations, the
                backward computation; every activation is kept until then).
  1F1B (DAPPLE) the same placement; device r runs P-1-r forward passes, then
                alternates one forward / one backward, then drains the
                remaining backward passes (background section: the backward is
                computed earlier so that activations are released as early as
                possible; memory does not drop on the first device and drops
                most on the last).
  Chimera       two pipelines of depth D over the same D devices in opposite
                directions, every device holding one stage of each (background
                section), run by the same greedy rules as the wave schedule.
  Chimera-wave  the section on transforming Chimera: swapping the blocks of one
                direction on the lower half of the devices with the blocks of
                the other direction at the mirrored positions turns a depth-2P
                Chimera into two identical one-wave pipelines on P devices
                each, the order of computation unchanged.  `chimera_wave`
                performs that fold; the claim pinned in the tests is that it
                yields exactly the W = 1 wave schedule.

Placements.  The wave schemes use oracle.schedule's placement (2W chunks per
device).  GPipe and 1F1B use the straight placement: stage s on device s, one
chunk per device; in Table 1's notation W = S / 2P = 1/2, written W = 0 here.

Bubble model: the equation of the theoretical-analysis section, as printed, and
the closed forms the straight schemes' own definitions give.
"""

from . import schedule as OS

F, B = OS.F, OS.B
Task = OS.Task

SCHEMES = ("hanayo", "chimera_wave", "gpipe", "1f1b")


# ------------------------------------------------------------------ straight placement: GPipe, 1F1B

def gpipe(P, M, rank):
    """All forwards, then all backwards, both in micro-batch order."""
    _check(P, M, rank)
    return [Task(F, m, 0, rank) for m in range(M)] + [Task(B, m, 0, rank) for m in range(M)]


def one_f_one_b(P, M, rank):
    """Warm-up of P-1-rank forwards, then (forward, backward) pairs, then the remaining backwards."""
    _check(P, M, rank)
    warm = min(P - 1 - rank, M)
    out = [Task(F, m, 0, rank) for m in range(warm)]
    for i in range(M - warm):
        out.append(Task(F, warm + i, 0, rank))
        out.append(Task(B, i, 0, rank))
    out += [Task(B, m, 0, rank) for m in range(M - warm, M)]
    return out


def _check(P, M, rank):
    if P < 1 or M < 1 or not (0 <= rank < P):
        raise ValueError("bad P, M or rank")


# ------------------------------------------------------------------ Chimera and its fold into a wave

def chimera(D, N_half, cost_f=1, cost_b=2):
    """Bidirectional pipeline of depth D (even) on D devices: N_half micro-batches run "down" (stage s on
    device s) and N_half run "up" (stage s on device D-1-s).  Greedy list schedule with the rules of the
    wave oracle: a free device starts a ready task, backward before forward, lowest micro-batch index
    (within its direction) first; a device never has two ready tasks of equal index because an index's
    down and up tasks sit on mirrored devices.  At most D/2 micro-batches per direction are in their
    forward phase (the basic unit of Chimera schedules D/2 per direction).

    Returns dict(lists[device] = [(direction, kind, mb, stage, start)], makespan)."""
    if D < 2 or D % 2 or N_half < 1:
        raise ValueError("D must be even and >= 2")
    half = D // 2
    chain = [(F, s) for s in range(D)] + [(B, s) for s in range(D - 1, -1, -1)]
    dev = lambda direction, s: s if direction == 0 else D - 1 - s
    nxt = {(d, m): 0 for d in (0, 1) for m in range(N_half)}
    prev_finish = {k: 0 for k in nxt}
    last_f_finish = {}
    started_f0 = set()
    free_at = [0] * D
    lists = [[] for _ in range(D)]
    running = []
    remaining = len(nxt) * len(chain)
    t = 0
    while remaining:
        for r in range(D):
            if free_at[r] > t:
                continue
            best = None
            for (d, m), i in nxt.items():
                if i >= len(chain):
                    continue
                kind, s = chain[i]
                if dev(d, s) != r or prev_finish[(d, m)] > t:
                    continue
                if kind == F and s == 0:
                    if m >= half and last_f_finish.get((d, m - half), t + 1) > t:
                        continue
                    if m >= 1 and (d, m - 1) not in started_f0:
                        continue
                key = (0 if kind == B else 1, m)
                if best is None or key < best[0]:
                    best = (key, d, m, kind, s)
            if best is None:
                continue
            _, d, m, kind, s = best
            end = t + (cost_f if kind == F else cost_b)
            lists[r].append((d, kind, m, s, t))
            free_at[r] = end
            prev_finish[(d, m)] = end
            nxt[(d, m)] += 1
            if kind == F and s == 0:
                started_f0.add((d, m))
            if kind == F and s == D - 1:
                last_f_finish[(d, m)] = end
            running.append(end)
            remaining -= 1
        later = [e for e in running if e > t]
        if not later:
            if remaining:
                raise RuntimeError("chimera schedule deadlocked")
            break
        running = later
        t = min(later)
    return {"lists": lists, "makespan": max(free_at)}


def chimera_wave(P, M, rank):
    """One rank's list of the Chimera-wave schedule on P devices: the "down" direction of a depth-2P
    Chimera with M micro-batches per direction, after the swap of the transformation section: device
    `rank` keeps its own down-blocks (stage = rank, local chunk 0) and takes over the down-blocks of the
    mirrored device 2P-1-rank (stage 2P-1-rank, local chunk 1) in the time slots that device's mirrored
    up-blocks held.  Order = start time in the Chimera schedule."""
    _check(P, M, rank)
    sim = chimera(2 * P, M)
    mine = [(t, kind, m, s) for (d, kind, m, s, t) in sim["lists"][rank] if d == 0]
    mine += [(t, kind, m, s) for (d, kind, m, s, t) in sim["lists"][2 * P - 1 - rank] if d == 0]
    mine.sort()
    for a, b in zip(mine, mine[1:]):
        assert a[0] + OS.COST[a[1]] <= b[0], "folded blocks overlap in time"
    return [Task(kind, m, s // P, s) for (t, kind, m, s) in mine]


# ------------------------------------------------------------------ one entry for every scheme

def scheme_list(scheme, P, W, M, rank):
    """Ordered task list of one rank under a scheme.  W: waves (hanayo), 1 (chimera_wave), 0 (gpipe, 1f1b)."""
    if scheme == "hanayo":
        return OS.schedule(P, W, M, rank)
    if scheme == "chimera_wave":
        if W != 1:
            raise ValueError("Chimera-wave has one wave")
        return chimera_wave(P, M, rank)
    if W != 0:
        raise ValueError("straight placement is written W = 0")
    if scheme == "gpipe":
        return gpipe(P, M, rank)
    if scheme == "1f1b":
        return one_f_one_b(P, M, rank)
    raise ValueError("unknown scheme")


# ------------------------------------------------------------------ bubble model

def hanayo_bubble_equation(P, W, t_f, t_b, t_c):
    """The bubble ratio printed at the end of the theoretical-analysis section (sum of the four bubble
    zones over the iteration time), T_F / T_B = a device's whole forward / backward time per micro-batch,
    T_C = one transfer, for B = P micro-batches."""
    num = t_b / W + (1 + 2 * W + 2.0 / P + (P - 2) / 3.0) * t_c
    den = P / (P - 1.0) * t_f + (1.0 / (2 * W) + P / (P - 1.0)) * t_b + ((P - 2) / 2.0 + 4 * W) * t_c
    return num / den


def straight_bubble(P, M, t_f, t_b, t_c):
    """GPipe and 1F1B on a straight pipeline: the first micro-batch reaches the last device after P-1
    forward stages and transfers, the last gradient leaves it P-1 backward stages and transfers before
    the end, and a device computes for M (T_F + T_B): idle (P-1)(T_F + T_B + 2 T_C) per device.  Exact
    for GPipe while the remaining transfers hide behind compute (receives posted ahead, T_C <= T_F); for
    1F1B exact at T_C = 0 (its steady state waits on round trips); a lower bound otherwise."""
    idle = (P - 1) * (t_f + t_b + 2 * t_c)
    return idle / (M * (t_f + t_b) + idle)


def bubble_model(scheme, P, W, M, t_f, t_b, t_c):
    if scheme in ("gpipe", "1f1b"):
        return straight_bubble(P, M, t_f, t_b, t_c)
    if scheme == "chimera_wave":
        W = 1
    if M != P:
        raise ValueError("the paper's equation is for B = P micro-batches")
    return hanayo_bubble_equation(P, W, t_f, t_b, t_c)
