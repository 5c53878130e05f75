"""Host logic of the whole-pipeline entry points (CPU only): hanayo_replay against the brute-force
replay of the oracle, with the paper's unit costs and with arbitrary per-task durations; error paths."""

import numpy as np
import pytest

from oracle import replay as R
from oracle import schedule as S
from paper_2308_15762_amd import hanayo as hn

GRID = [(2, 1, 4), (4, 2, 8), (4, 1, 16), (8, 4, 12), (3, 2, 5), (1, 2, 3), (5, 3, 2), (16, 2, 32)]


def lib_lists(P, W, M):
    return [hn.hanayo_schedule(P, W, M, r) for r in range(P)]


def as_tuples(t):
    return [(int(x["kind"]), int(x["mb"]), int(x["chunk"]), int(x["stage"])) for x in t]


@pytest.mark.parametrize("P,W,M", GRID)
def test_replay_unit_costs(P, W, M):
    lists = lib_lists(P, W, M)
    makespan, idle = hn.hanayo_replay(lists, P, W, M)
    ref = R.replay([as_tuples(t) for t in lists], P, W, M)
    assert makespan == ref["makespan"] == S.simulate(P, W, M)["makespan"]
    assert list(idle) == ref["idle"]


@pytest.mark.parametrize("P,W,M", GRID[:6])
def test_replay_measured_costs(P, W, M):
    """Arbitrary positive durations per task (as measured times would be): same makespan and idle as
    the oracle's replay fed the same durations."""
    rng = np.random.default_rng(P * 1000 + W * 100 + M)
    lists = lib_lists(P, W, M)
    cost = [rng.uniform(0.1, 3.0, size=t.size).astype(np.float32) for t in lists]
    table = {}
    for t, c in zip(lists, cost):
        for x, v in zip(as_tuples(t), c):
            table[(x[0], x[1], x[3])] = float(v)
    makespan, idle = hn.hanayo_replay(lists, P, W, M, cost)
    ref = R.replay([as_tuples(t) for t in lists], P, W, M, cost=lambda k, m, s: table[(k, m, s)])
    assert abs(makespan - ref["makespan"]) <= 1e-9 * ref["makespan"]
    assert np.allclose(idle, ref["idle"], rtol=0, atol=1e-6 * ref["makespan"])


def deadlocking_lists():
    """P = 2, W = 1, M = 4: each list is its rank's task set in a locally valid order, but rank 0 wants
    micro-batch 0 back from rank 1 before it sends micro-batch 1, and rank 1 wants micro-batch 1 first."""
    P, W, M = 2, 1, 4
    lists = lib_lists(P, W, M)
    t0 = list(as_tuples(lists[0]))
    i, j = t0.index((0, 1, 0, 0)), t0.index((0, 0, 1, 3))          # F of mb 1 stage 0; F of mb 0 stage 3
    assert i < j
    t0[i], t0[j] = t0[j], t0[i]
    t1 = list(as_tuples(lists[1]))
    first = [x for x in t1 if x[0] == 0 and x[1] == 1]               # forwards of micro-batch 1 ...
    rest = [x for x in t1 if not (x[0] == 0 and x[1] == 1)]
    t1 = first + rest                                                 # ... before everything else
    out = []
    for t in (t0, t1):
        a = np.zeros(len(t), dtype=hn.TASK_DTYPE)
        for k, (kind, mb, chunk, stage) in enumerate(t):
            a[k] = (kind, chunk, 0, mb, stage)
        out.append(a)
    return P, W, M, out


def test_replay_rejects_deadlock_and_bad_lists():
    P, W, M, bad = deadlocking_lists()
    with pytest.raises(AssertionError):
        R.replay([as_tuples(t) for t in bad], P, W, M)
    with pytest.raises(hn.HanayoError) as e:
        hn.hanayo_replay(bad, P, W, M)
    assert e.value.code == hn.ESTATE
    good = lib_lists(P, W, M)
    with pytest.raises(hn.HanayoError) as e:
        hn.hanayo_replay([good[1], good[0]], P, W, M)                 # lists on the wrong ranks
    assert e.value.code == hn.ESTATE
    with pytest.raises(hn.HanayoError) as e:
        hn.hanayo_replay(good, P, W, M, [np.full(t.size, -1.0, np.float32) for t in good])
    assert e.value.code == hn.EINVAL
    with pytest.raises(hn.HanayoError) as e:
        hn.hanayo_replay(good, 0, W, M)
    assert e.value.code == hn.EINVAL


def test_paper_bubble_equation_reduces_to_its_simplified_form():
    """The bubble-ratio equation of the theoretical analysis section, as typed into the bubble report: with
    T_B = 2 T_F and T_C = 0 it is (2P - 2) / (3PW + P - 1) exactly; it falls with W; communication time raises it."""
    from fractions import Fraction
    from paper_2308_15762_amd import bubble
    for P in (2, 3, 4, 8, 16):
        for W in (1, 2, 4):
            got = bubble.paper_ratio(P, W, 1.0, 2.0, 0.0)
            assert abs(got - float(Fraction(2 * P - 2, 3 * P * W + P - 1))) < 1e-12
            assert abs(got - bubble.printed_ratio(P, W)) < 1e-12
            assert bubble.paper_ratio(P, W, 1.0, 2.0, 0.05) > got
        assert bubble.paper_ratio(P, 1, 1.0, 2.0, 0.0) > bubble.paper_ratio(P, 2, 1.0, 2.0, 0.0) > bubble.paper_ratio(P, 4, 1.0, 2.0, 0.0)
    # a value worked by hand from the equation: P = 4, W = 2, T_F = 1, T_B = 2, T_C = 0.1
    num = 2.0 / 2 + (1 + 4 + 0.5 + 2.0 / 3.0) * 0.1
    den = 4.0 / 3.0 * 1.0 + (0.25 + 4.0 / 3.0) * 2.0 + (1.0 + 8.0) * 0.1
    assert abs(bubble.paper_ratio(4, 2, 1.0, 2.0, 0.1) - num / den) < 1e-12
