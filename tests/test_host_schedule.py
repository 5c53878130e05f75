"""Host logic of the library against the schedule oracle: task lists and stash plans are
bit-exact for every rank; stored lists guard both against drift; error paths."""

import os

import numpy as np
import pytest

from oracle import replay, schedule as S
from paper_2308_15762_amd import hanayo as hn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GRID = [(2, 1, 4), (4, 2, 8), (4, 1, 16), (16, 2, 32), (8, 4, 64),          # the BASELINE configurations
        (1, 1, 1), (1, 2, 3), (2, 1, 1), (3, 2, 5), (5, 3, 2), (4, 2, 3), (6, 3, 7), (7, 1, 20), (2, 5, 9)]


def as_tuples(tasks):
    return [(int(t["kind"]), int(t["mb"]), int(t["chunk"]), int(t["stage"])) for t in tasks]


@pytest.mark.parametrize("P,W,M", GRID)
def test_lists_and_plans_bit_exact(P, W, M):
    sim = S.simulate(P, W, M)
    lists = []
    for r in range(P):
        t = hn.hanayo_schedule(P, W, M, r)
        assert (t["rsvd"] == 0).all()
        got = as_tuples(t)
        assert got == [tuple(x) for x in sim["lists"][r]]
        lists.append(got)
        peak, per_chunk, slot = hn.hanayo_stash_plan(t, W)
        o_peak, o_per_chunk, o_slot = S.stash_plan(sim["lists"][r], W)
        assert (peak, list(per_chunk), list(slot)) == (o_peak, o_per_chunk, o_slot)
    # the library's lists also pass the brute-force replay on their own
    rep = replay.replay(lists, P, W, M)
    assert rep["makespan"] == sim["makespan"]


def test_lists_bit_exact_on_a_seeded_sweep():
    """60 seeded (P, W, M) triples beyond the fixed grid: every rank's list and stash plan equal the oracle's."""
    rng = np.random.default_rng(20230815)
    seen = set()
    while len(seen) < 60:
        P, W, M = int(rng.integers(1, 9)), int(rng.integers(1, 5)), int(rng.integers(1, 25))
        if (P, W, M) in seen:
            continue
        seen.add((P, W, M))
        sim = S.simulate(P, W, M)
        for r in range(P):
            t = hn.hanayo_schedule(P, W, M, r)
            assert as_tuples(t) == [tuple(x) for x in sim["lists"][r]], (P, W, M, r)
            peak, per_chunk, slot = hn.hanayo_stash_plan(t, W)
            o_peak, o_per_chunk, o_slot = S.stash_plan(sim["lists"][r], W)
            assert (peak, list(per_chunk), list(slot)) == (o_peak, o_per_chunk, o_slot), (P, W, M, r)


def test_placement_helpers_agree():
    for (P, W) in [(1, 1), (2, 1), (4, 2), (8, 4), (16, 2), (5, 3)]:
        for s in range(2 * W * P):
            r = hn.hanayo_stage_rank(P, W, s)
            assert r == S.stage_rank(P, W, s)
            assert hn.hanayo_rank_stage(P, W, r, s // P) == s
    for bad in [(2, 1, 4), (2, 1, -1)]:
        with pytest.raises(hn.HanayoError):
            hn.hanayo_stage_rank(*bad)


def test_stored_lists():
    path = os.path.join(ROOT, "tests", "golden", "schedule_rank_lists.txt")
    n = 0
    for line in open(path):
        if line.startswith("#"):
            continue
        head, toks = line.split(":")
        P, W, M, r = (int(v) for v in head.split())
        want = toks.split()
        lib = ["%s%d.%d" % ("FB"[int(t["kind"])], t["mb"], t["chunk"]) for t in hn.hanayo_schedule(P, W, M, r)]
        ora = ["%s%d.%d" % ("FB"[t.kind], t.mb, t.chunk) for t in S.schedule(P, W, M, r)]
        assert lib == want and ora == want
        n += 1
    assert n >= 40


def test_stash_plan_errors():
    t = hn.hanayo_schedule(2, 1, 2, 0)
    b_idx = int(np.argmax(t["kind"] == hn.B))
    bad = t.copy()
    bad[[0, b_idx]] = bad[[b_idx, 0]]
    with pytest.raises(hn.HanayoError) as ei:
        hn.hanayo_stash_plan(bad, 1)
    assert ei.value.code == hn.ESTATE
    with pytest.raises(hn.HanayoError) as ei:
        hn.hanayo_stash_plan(np.concatenate([t, t[:1]]), 1)
    assert ei.value.code == hn.ESTATE
    wrong_chunk = t.copy()
    wrong_chunk["chunk"][0] = 7
    with pytest.raises(hn.HanayoError) as ei:
        hn.hanayo_stash_plan(wrong_chunk, 1)
    assert ei.value.code == hn.EINVAL
    peak, per_chunk, slot = hn.hanayo_stash_plan(t[:0], 1)
    assert peak == 0 and list(per_chunk) == [0, 0]


def test_arena_size_follows_the_plan():
    d = hn.make_desc(1, 256, 4, 1024, 128, 2, hn.PRE_LN, hn.MASK_CAUSAL, hn.FP32)
    t = hn.hanayo_schedule(4, 2, 8, 0)
    _, per_chunk, _ = hn.hanayo_stash_plan(t, 2)
    assert hn.hanayo_stash_arena_bytes(t, 2, d) == int(per_chunk.sum()) * hn.hanayo_stash_bytes(d)


# ---------------------------------------------------------------- executor lane plan

def _accesses(P, W, rank, tasks, slot, lane, ends=False):
    """Read and write sets of every task over the buffers the executor touches.  With ends, rank 0's
    forward of stage 0 / of the last stage and backward of stage 0 also touch the lane's ends workspace,
    the loss-gradient buffer of the micro-batch and the (possibly shared) table gradients."""
    S_ = 2 * W * P
    ends = ends and rank == 0
    out = []
    for i, t in enumerate(tasks):
        kind, m, c, stage = (int(t[k]) for k in ("kind", "mb", "chunk", "stage"))
        reads, writes = set(), set()
        if kind == 0:
            if stage > 0 and S.stage_rank(P, W, stage - 1) == rank:
                reads.add(("act", m, c - 1))
            writes.add(("act", m, c))
            writes.add(("stash", c, int(slot[i])))
            if ends and stage in (0, S_ - 1):
                writes.add(("ends workspace", int(lane[i])))
            if ends and stage == S_ - 1:
                writes.add(("loss grad", m))
                writes.add(("table grads",))
        else:
            reads.add(("stash", c, int(slot[i])))
            if stage < S_ - 1 and S.stage_rank(P, W, stage + 1) == rank:
                reads.add(("grad", m, c + 1))
            writes.add(("grad", m, c))
            writes.add(("weight grads", c))          # read-modify-write
            writes.add(("workspace", int(lane[i])))
            if ends and stage == S_ - 1:
                reads.add(("loss grad", m))
            if ends and stage == 0:
                writes.add(("table grads",))
        out.append((reads, writes))
    return out


@pytest.mark.parametrize("ends", [False, True])
@pytest.mark.parametrize("lanes", [1, 2, 3, 4])
@pytest.mark.parametrize("P,W,M", [(2, 1, 4), (4, 2, 8), (4, 1, 16), (8, 4, 12), (3, 2, 5), (1, 2, 3), (5, 3, 2)])
def test_lane_plan_orders_every_conflict(P, W, M, lanes, ends):
    """Any two tasks that touch one buffer, at least one of them writing, are ordered by the plan's
    event waits together with the in-order execution of each lane."""
    for rank in range(P):
        tasks = hn.hanayo_schedule(P, W, M, rank)
        n = len(tasks)
        desc = hn.make_desc(2, 256, 4, 1024, 128, 2, hn.PRE_LN, hn.MASK_CAUSAL, hn.BF16)
        lane, deps = hn.hanayo_executor_plan(tasks, P, W, M, rank, lanes, desc, hn.EndsDesc(4096, 128, 1) if ends else None)
        assert lane.min() >= 0 and lane.max() < lanes
        assert ends and rank == 0 or (deps[:, 4] == -1).all()
        _, _, slot = S.stash_plan(S.schedule(P, W, M, rank), W)
        acc = _accesses(P, W, rank, tasks, slot, lane, ends)
        before = [0] * n           # bit j set: task j is known to finish before task i starts
        last_on_lane = {}
        for i in range(n):
            preds = [int(j) for j in deps[i] if j >= 0]
            assert all(j < i for j in preds)
            if int(lane[i]) in last_on_lane:
                preds.append(last_on_lane[int(lane[i])])
            last_on_lane[int(lane[i])] = i
            for j in preds:
                before[i] |= before[j] | (1 << j)
        for i in range(n):
            ri, wi = acc[i]
            for j in range(i):
                rj, wj = acc[j]
                if (wj & (ri | wi)) or (rj & wi):
                    assert before[i] >> j & 1, "tasks %d and %d share %s unordered" % (j, i, (wj & (ri | wi)) | (rj & wi))
        if lanes > 1 and P >= 2 and M >= 4:
            assert len(set(lane.tolist())) > 1   # the plan does use more than one lane


def test_lane_plan_rejects_bad_arguments():
    tasks = hn.hanayo_schedule(2, 1, 4, 0)
    for lanes in (0, 5):
        with pytest.raises(hn.HanayoError) as e:
            hn.hanayo_executor_plan(tasks, 2, 1, 4, 0, lanes)
        assert e.value.code == hn.EINVAL
    with pytest.raises(hn.HanayoError) as e:
        hn.hanayo_executor_plan(tasks[::-1].copy(), 2, 1, 4, 0, 2)
    assert e.value.code == hn.ESTATE
