"""Pins for the schedule oracle: placement facts the paper states, a brute-force
replay with an independent ready-set audit, the bubble analysis, and the values
of the stated reading (R1-R7) on worked cases."""

import pytest

from oracle import replay, schedule as S

CONFIG_PWM = [(2, 1, 4), (4, 2, 8), (4, 1, 16), (16, 2, 32), (8, 4, 64)]


def tup(lists):
    return [[tuple(t) for t in l] for l in lists]


def fmt(lst):
    return " ".join("%s%d.%d" % ("FB"[t.kind], t.mb, t.chunk) for t in lst)


# --- placement (Table 1: W = S / 2P; wave-like pipelines change direction) ---

@pytest.mark.parametrize("P,W", [(1, 1), (2, 1), (3, 2), (4, 2), (8, 4), (16, 2)])
def test_placement_is_a_wave(P, W):
    stages = 2 * W * P
    ranks = [S.stage_rank(P, W, s) for s in range(stages)]
    expect = (list(range(P)) + list(range(P - 1, -1, -1))) * W
    assert ranks == expect
    for r in range(P):
        assert ranks.count(r) == 2 * W                      # 2W stages per device
    for k in range(1, 2 * W):
        assert ranks[k * P - 1] == ranks[k * P]             # turn-around is local
    assert ranks[0] == 0 and ranks[-1] == 0
    for r in range(P):
        for c in range(2 * W):
            s = S.rank_stage(P, W, r, c)
            assert S.stage_rank(P, W, s) == r and s // P == c


# --- brute force -------------------------------------------------------------

@pytest.mark.parametrize("P,W,M", CONFIG_PWM + [(3, 2, 5), (4, 1, 6), (5, 1, 10), (1, 2, 3), (4, 2, 3), (6, 3, 7)])
def test_replay_agrees_with_generator_clock(P, W, M):
    sim = S.simulate(P, W, M)
    rep = replay.replay(tup(sim["lists"]), P, W, M)
    assert rep["makespan"] == sim["makespan"]
    assert rep["idle"] == sim["idle"]
    for r in range(P):
        for tk, t0 in zip(sim["lists"][r], sim["starts"][r]):
            assert rep["start"][(tk.kind, tk.mb, tk.stage)] == t0
        assert len(sim["lists"][r]) == 4 * W * M
        assert S.stash_plan(sim["lists"][r], W)[0] == rep["peak"][r]
        assert rep["peak"][r] <= 2 * W * P                  # same M_a as other schemes


@pytest.mark.parametrize("P", [1, 2, 3])
@pytest.mark.parametrize("W", [1, 2])
@pytest.mark.parametrize("M", [1, 2, 3, 5])
def test_every_decision_is_the_rule_minimum(P, W, M):
    sim = S.simulate(P, W, M)
    replay.greedy_audit(tup(sim["lists"]), P, W, M)


def test_audit_catches_a_planted_swap():
    lists = tup(S.simulate(3, 1, 3)["lists"])
    l0 = lists[0]
    i = next(i for i in range(len(l0) - 1) if l0[i][0] == 1 and l0[i + 1][0] == 0)
    l0[i], l0[i + 1] = l0[i + 1], l0[i]                     # run an F before a ready B
    with pytest.raises(AssertionError):
        replay.greedy_audit(lists, 3, 1, 3)


def test_replay_catches_missing_and_misplaced_tasks():
    lists = tup(S.simulate(2, 1, 2)["lists"])
    bad = [list(l) for l in lists]
    bad[0][0] = bad[0][1]
    with pytest.raises(AssertionError):
        replay.replay(bad, 2, 1, 2)
    bad = [list(l) for l in lists]
    bad[0], bad[1] = bad[1], bad[0]
    with pytest.raises(AssertionError):
        replay.replay(bad, 2, 1, 2)


# --- the paper's bubble analysis (T_B = 2 T_F, T_C = 0) -----------------------

@pytest.mark.parametrize("P", [2, 3, 4, 6, 8, 16])
def test_idle_equals_bubble_numerator_one_wave(P):
    sim = S.simulate(P, 1, P)
    assert sim["idle"] == [4 * (P - 1)] * P
    assert S.bubble_idle_numerator(P, 1) == 4 * (P - 1)


@pytest.mark.parametrize("P,W", [(2, 2), (2, 3), (2, 4), (3, 2), (3, 3), (3, 4)])
def test_idle_equals_bubble_numerator_small_P(P, W):
    assert S.simulate(P, W, P)["idle"] == [4 * (P - 1)] * P


@pytest.mark.parametrize("P,W", [(4, 2), (4, 4), (6, 2), (8, 2), (8, 4), (16, 2)])
def test_idle_close_to_bubble_numerator(P, W):
    idle = S.simulate(P, W, P)["idle"]
    for v in idle:
        assert 4 * (P - 1) <= v <= 1.1 * 4 * (P - 1)


@pytest.mark.parametrize("P", [4, 8])
def test_bubble_ratio_falls_with_waves_and_tracks_printed_formula(P):
    prev = None
    for W in (1, 2, 3, 4):
        sim = S.simulate(P, W, P)
        ratio = sim["idle"][0] / sim["makespan"]
        if prev is not None:
            assert ratio < prev
        if W >= 2:
            assert abs(ratio - S.bubble_ratio_printed(P, W)) < 0.02
        prev = ratio


def test_zone_a_warmup_idle_on_rank0():
    # Zone A bubble is T_F / 2W each; rank 0 waits for the wave to come back
    # through P-1 peers' chunk forwards before its second chunk can start.
    for (P, W, M) in [(4, 1, 4), (4, 2, 8), (8, 4, 64), (16, 2, 32)]:
        sim = S.simulate(P, W, M)
        lst, st = sim["lists"][0], sim["starts"][0]
        gaps = 0
        t = 0
        for tk, t0 in zip(lst, st):
            if tk.kind == S.B:
                break
            gaps += t0 - t
            t = t0 + 1
        assert gaps == P - 1


# --- values of the stated reading ---------------------------------------------

def test_worked_example_P2_W1_M4():
    sim = S.simulate(2, 1, 4)
    assert fmt(sim["lists"][0]) == ("F0.0 F1.0 F0.1 B0.1 F1.1 B1.1 F2.0 B0.0 F3.0 B1.0 "
                                    "F2.1 B2.1 F3.1 B3.1 B2.0 B3.0")
    assert fmt(sim["lists"][1]) == ("F0.0 F0.1 F1.0 F1.1 B0.1 B0.0 B1.1 B1.0 F2.0 F2.1 "
                                    "F3.0 F3.1 B2.1 B2.0 B3.1 B3.0")


def test_worked_example_P4_W1_M4():
    sim = S.simulate(4, 1, 4)
    want = [
        "F0.0 F1.0 F2.0 F3.0 F0.1 B0.1 F1.1 B1.1 F2.1 B2.1 F3.1 B3.1 B0.0 B1.0 B2.0 B3.0",
        "F0.0 F1.0 F2.0 F3.0 F0.1 F1.1 B0.1 F2.1 B1.1 F3.1 B2.1 B3.1 B0.0 B1.0 B2.0 B3.0",
        "F0.0 F1.0 F2.0 F0.1 F3.0 F1.1 F2.1 F3.1 B0.1 B1.1 B0.0 B2.1 B1.0 B3.1 B2.0 B3.0",
        "F0.0 F0.1 F1.0 F1.1 F2.0 F2.1 F3.0 F3.1 B0.1 B0.0 B1.1 B1.0 B2.1 B2.0 B3.1 B3.0",
    ]
    assert [fmt(l) for l in sim["lists"]] == want
    assert sim["makespan"] == 36


MAKESPAN_M_EQ_P = {(2, 1): 16, (2, 2): 28, (2, 4): 52, (3, 1): 26, (3, 2): 44, (4, 1): 36, (4, 2): 61,
                   (4, 4): 109, (6, 1): 56, (8, 1): 76, (8, 2): 126, (8, 4): 222, (16, 1): 156, (16, 2): 258}


def test_makespans_at_M_equal_P():
    for (P, W), want in MAKESPAN_M_EQ_P.items():
        assert S.simulate(P, W, P)["makespan"] == want


def test_config_values():
    want = {
        (2, 1, 4): (29, 5, [3, 4], [3, 1]),
        (4, 2, 8): (115, 19, [16, 14, 16, 16], [8, 4, 4, 1]),
        (4, 1, 16): (123, 27, [8, 7, 8, 8], [8, 1]),
        (16, 2, 32): (514, 130, [64, 64, 61, 58, 56, 56, 58, 59, 61, 62] + [64] * 6, [32, 16, 16, 1]),
        (8, 4, 64): (1681, 145, [64, 63, 63, 62, 63, 64, 64, 64], [16, 8, 8, 8, 8, 8, 8, 1]),
    }
    for (P, W, M), (mk, idle, peaks, per_chunk0) in want.items():
        sim = S.simulate(P, W, M)
        assert sim["makespan"] == mk and sim["idle"][0] == idle
        assert [S.stash_plan(l, W)[0] for l in sim["lists"]] == peaks
        assert S.stash_plan(sim["lists"][0], W)[1] == per_chunk0
    assert S.simulate(1, 2, 3)["makespan"] == 36            # P = 1: no idle at all
    assert S.simulate(1, 2, 3)["idle"] == [0]


@pytest.mark.parametrize("P,W,M", CONFIG_PWM + [(3, 2, 5), (5, 1, 10), (4, 2, 3)])
def test_order_invariants(P, W, M):
    sim = S.simulate(P, W, M)
    for r in range(P):
        for c in range(2 * W):
            for kind in (S.F, S.B):
                mbs = [t.mb for t in sim["lists"][r] if t.chunk == c and t.kind == kind]
                assert mbs == list(range(M))
    head = sim["lists"][0][:min(P, M)]
    assert [(t.kind, t.mb, t.chunk) for t in head] == [(S.F, m, 0) for m in range(min(P, M))]


# --- stash planning ------------------------------------------------------------

def test_stash_plan_slots_are_disjoint_while_live():
    for (P, W, M) in [(4, 2, 8), (3, 2, 5), (8, 4, 64)]:
        for lst in S.simulate(P, W, M)["lists"]:
            peak, per_chunk, slot = S.stash_plan(lst, W)
            live = {}
            for tk, sid in zip(lst, slot):
                assert 0 <= sid < per_chunk[tk.chunk]
                if tk.kind == S.F:
                    assert (tk.chunk, sid) not in live.values()
                    live[(tk.mb, tk.chunk)] = (tk.chunk, sid)
                else:
                    assert live.pop((tk.mb, tk.chunk)) == (tk.chunk, sid)
            assert not live and peak <= sum(per_chunk)


def test_stash_plan_rejects_bad_lists():
    lst = S.schedule(2, 1, 2, 0)
    b_first = [t for t in lst if t.kind == S.B][:1] + lst
    with pytest.raises(ValueError):
        S.stash_plan(b_first, 1)
    with pytest.raises(ValueError):
        S.stash_plan(lst + [lst[0]], 1)


def test_bad_arguments():
    for args in [(0, 1, 1, 0), (2, 0, 1, 0), (2, 1, 0, 0), (2, 1, 1, 2), (2, 1, 1, -1)]:
        with pytest.raises(ValueError):
            S.schedule(*args)
