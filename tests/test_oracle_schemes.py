"""Pins of the oracle's comparison schedules (GPipe, 1F1B, Chimera, Chimera-wave) and of the bubble model
against what the paper and the schemes' own definitions fix.  CPU only."""

import itertools

import pytest

from oracle import replay as OR
from oracle import schedule as OS
from oracle import schemes as SC

F, B = OS.F, OS.B


def lists_of(scheme, P, W, M):
    return [[tuple(t) for t in SC.scheme_list(scheme, P, W, M, r)] for r in range(P)]


STRAIGHT = [(1, 1), (1, 3), (2, 2), (2, 5), (3, 3), (4, 4), (4, 8), (4, 2), (8, 8), (8, 20), (16, 16), (5, 3)]


@pytest.mark.parametrize("scheme", ["gpipe", "1f1b"])
@pytest.mark.parametrize("P,M", STRAIGHT)
def test_straight_schemes_replay_and_idle(scheme, P, M):
    """The brute-force replay accepts the lists (every task once, on its device, dependencies met, no
    deadlock), and with the paper's costs (forward 1, backward 2, transfers 0) every device idles exactly
    (P-1)(T_F + T_B): the three bubble parts the background section lists for GPipe, which 1F1B keeps."""
    rep = OR.replay(lists_of(scheme, P, 0, M), P, 0, M)
    assert rep["makespan"] == 3 * M + 3 * (P - 1)
    assert rep["idle"] == [3 * (P - 1)] * P


@pytest.mark.parametrize("P,M", STRAIGHT)
def test_stash_peaks_of_the_straight_schemes(P, M):
    """GPipe keeps every micro-batch's activation until the backward phase: peak M on every device.
    1F1B: P - rank in flight (capped by M): no drop on the first device, the largest on the last."""
    g = OR.replay(lists_of("gpipe", P, 0, M), P, 0, M)
    assert g["peak"] == [M] * P
    d = OR.replay(lists_of("1f1b", P, 0, M), P, 0, M)
    assert d["peak"] == [min(P - r, M) for r in range(P)]
    for r in range(P):
        assert OS.stash_plan(SC.scheme_list("1f1b", P, 0, M, r), 1)[0] == min(P - r, M)


def test_worked_1f1b_lists():
    """P = 4, M = 4, the example the background section walks through (four micro-batches on four devices)."""
    name = lambda lst: " ".join("%s%d" % ("FB"[k], m) for (k, m, _, _) in lst)
    L = lists_of("1f1b", 4, 0, 4)
    assert name(L[0]) == "F0 F1 F2 F3 B0 B1 B2 B3"
    assert name(L[1]) == "F0 F1 F2 B0 F3 B1 B2 B3"
    assert name(L[2]) == "F0 F1 B0 F2 B1 F3 B2 B3"
    assert name(L[3]) == "F0 B0 F1 B1 F2 B2 F3 B3"
    G = lists_of("gpipe", 4, 0, 4)
    assert all(name(l) == "F0 F1 F2 F3 B0 B1 B2 B3" for l in G)
    assert all(s == r and c == 0 for r, l in enumerate(L) for (_, _, c, s) in l)


def test_1f1b_is_the_greedy_early_backward_schedule_under_a_memory_cap():
    """An independent construction: simulate the straight pipeline with 'backward first, lowest
    micro-batch, at most P - rank activations alive on a device'; the start orders are the 1F1B lists."""
    for P, M in [(2, 2), (3, 5), (4, 4), (4, 9), (6, 6), (8, 12)]:
        done, finish, free_at = set(), {}, [0] * P
        lists = [[] for _ in range(P)]
        nextf, nextb, live = [0] * P, [0] * P, [0] * P
        t, left = 0, 2 * P * M
        while left:
            for r in range(P):
                if free_at[r] > t:
                    continue
                m = nextb[r]
                b_ready = m < M and (finish.get((F, m, r), 1 << 60) <= t) and (
                    r == P - 1 or finish.get((B, m, r + 1), 1 << 60) <= t)
                m2 = nextf[r]
                f_ready = m2 < M and live[r] < P - r and (r == 0 or finish.get((F, m2, r - 1), 1 << 60) <= t)
                if b_ready:
                    lists[r].append((B, m, 0, r)); finish[(B, m, r)] = t + 2; free_at[r] = t + 2
                    nextb[r] += 1; live[r] -= 1; left -= 1
                elif f_ready:
                    lists[r].append((F, m2, 0, r)); finish[(F, m2, r)] = t + 1; free_at[r] = t + 1
                    nextf[r] += 1; live[r] += 1; left -= 1
            t = min(v for v in finish.values() if v > t) if any(v > t for v in finish.values()) else t + 1
        assert lists == lists_of("1f1b", P, 0, M), (P, M)


@pytest.mark.parametrize("D", [2, 4, 6, 8, 12])
def test_chimera_basic_unit_matches_its_published_bubble_count(D):
    """Li & Hoefler's Chimera (the scheme the background section describes) with equal forward and backward
    costs and one basic unit (N = D micro-batches, D/2 per direction) finishes in 2N + D - 2 slots: D - 2
    bubbles per device.  Also: the schedule is mirror-symmetric (device r's blocks are device D-1-r's with
    the directions exchanged, at the same times), which is what the swap of the transformation relies on."""
    sim = SC.chimera(D, D // 2, 1, 1)
    assert sim["makespan"] == 2 * D + D - 2
    sim = SC.chimera(D, D // 2)     # the paper's costs
    for r in range(D):
        mirrored = sorted((t, 1 - d, k, m, s) for (d, k, m, s, t) in sim["lists"][D - 1 - r])
        assert sorted((t, d, k, m, s) for (d, k, m, s, t) in sim["lists"][r]) == mirrored


@pytest.mark.parametrize("P,M", [(1, 1), (2, 2), (2, 4), (3, 3), (4, 4), (4, 8), (4, 6), (5, 7), (8, 8), (8, 24), (16, 16)])
def test_chimera_wave_is_the_one_wave_schedule(P, M):
    """The transformation section's claim: folding Chimera gives wave pipelines with the order of
    computation unchanged.  The folded lists are exactly the W = 1 lists of the wave oracle, and they
    replay to Chimera's own makespan."""
    folded = lists_of("chimera_wave", P, 1, M)
    assert folded == [[tuple(t) for t in OS.schedule(P, 1, M, r)] for r in range(P)]
    assert OR.replay(folded, P, 1, M)["makespan"] == SC.chimera(2 * P, M)["makespan"]


def test_scheme_arguments():
    with pytest.raises(ValueError):
        SC.scheme_list("gpipe", 4, 1, 4, 0)
    with pytest.raises(ValueError):
        SC.scheme_list("chimera_wave", 4, 2, 4, 0)
    with pytest.raises(ValueError):
        SC.scheme_list("nonesuch", 4, 0, 4, 0)
    with pytest.raises(ValueError):
        SC.gpipe(4, 4, 4)


# ------------------------------------------------------------------ bubble model

@pytest.mark.parametrize("P,W", list(itertools.product([2, 4, 8, 16, 32], [1, 2, 4, 8])))
def test_bubble_equation_reduces_to_the_printed_simplification(P, W):
    """At T_B = 2 T_F and T_C = 0 the equation is (2P-2)/(3PW+P-1), as the paper states."""
    got = SC.hanayo_bubble_equation(P, W, 1.0, 2.0, 0.0)
    assert abs(got - (2 * P - 2) / (3 * P * W + P - 1)) < 1e-12
    assert abs(got - OS.bubble_ratio_printed(P, W)) < 1e-12


def test_bubble_equation_behaviour():
    """Falls with W at T_C = 0 ("decreases with an increasing number of waves"); grows with T_C; the
    communication terms grow with W (the ratio tends to 2 T_C / 4 T_C = 1/2), so with T_C > 0 there is a
    wave count beyond which more waves stop paying."""
    for P in (4, 8, 16):
        r = [SC.hanayo_bubble_equation(P, W, 1.0, 2.0, 0.0) for W in (1, 2, 4, 8)]
        assert all(a > b for a, b in zip(r, r[1:]))
        assert SC.hanayo_bubble_equation(P, 2, 1.0, 2.0, 0.1) > SC.hanayo_bubble_equation(P, 2, 1.0, 2.0, 0.0)
    link = [SC.hanayo_bubble_equation(8, W, 1.0, 2.0, 0.05) for W in (1, 2, 4, 8, 16, 32, 64, 128)]
    assert 0 < link.index(min(link)) < len(link) - 1
    assert abs(SC.hanayo_bubble_equation(8, 1 << 20, 1.0, 2.0, 0.05) - 0.5) < 1e-3
    # one value worked by hand: P = 4, W = 2, T_F = 3, T_B = 5, T_C = 0.5
    num = 5 / 2 + (1 + 4 + 0.5 + 2 / 3) * 0.5
    den = 4 / 3 * 3 + (0.25 + 4 / 3) * 5 + (1 + 8) * 0.5
    assert abs(SC.hanayo_bubble_equation(4, 2, 3.0, 5.0, 0.5) - num / den) < 1e-12


@pytest.mark.parametrize("P,M", [(2, 2), (4, 4), (4, 8), (8, 8), (8, 32), (16, 16)])
def test_straight_bubble_equals_the_replayed_schedules(P, M):
    """The closed form for GPipe / 1F1B against the replay of their lists (T_C = 0): same ratio."""
    for scheme in ("gpipe", "1f1b"):
        rep = OR.replay(lists_of(scheme, P, 0, M), P, 0, M)
        ratio = rep["idle"][0] / rep["makespan"]
        assert abs(SC.bubble_model(scheme, P, 0, M, 1.0, 2.0, 0.0) - ratio) < 1e-12
    # at B = P the familiar (P-1)/(2P-1)
    assert abs(SC.bubble_model("gpipe", P, 0, P, 1.0, 2.0, 0.0) - (P - 1) / (2 * P - 1)) < 1e-12


def test_scheme_ranking_of_the_bubble_figure():
    """The ordering the paper's bubble figure and evaluation report: GPipe = 1F1B > Chimera-wave (= one
    wave) > two waves > four waves, at every device count."""
    for P in (4, 8, 16, 32):
        g = SC.bubble_model("gpipe", P, 0, P, 1.0, 2.0, 0.0)
        c = SC.bubble_model("chimera_wave", P, 1, P, 1.0, 2.0, 0.0)
        h2 = SC.bubble_model("hanayo", P, 2, P, 1.0, 2.0, 0.0)
        h4 = SC.bubble_model("hanayo", P, 4, P, 1.0, 2.0, 0.0)
        assert g > c > h2 > h4
