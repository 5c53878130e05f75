"""Pins for the action-list oracle (CPU only): structure of the lists, matching of sends and receives,
and the interpreter simulation against closed forms and against the task-level replay."""

import pytest

from oracle import actions as A
from oracle import replay as R
from oracle import schedule as S

GRID = [(2, 1, 4), (4, 2, 8), (4, 1, 16), (3, 2, 5), (1, 2, 3), (5, 3, 2), (8, 4, 12)]


def all_lists(P, W, M):
    return [A.actions(P, W, M, r) for r in range(P)]


@pytest.mark.parametrize("P,W,M", GRID)
def test_structure_and_matching(P, W, M):
    lists = all_lists(P, W, M)
    n_stage = 2 * W * P
    # compute actions, in order, are the rank's task list
    for r, lst in enumerate(lists):
        comp = [(k, m, c, s) for (k, m, c, s, _) in lst if k in A.COMPUTE]
        assert comp == [tuple(t) for t in S.schedule(P, W, M, r)]
        # a receive sits immediately before the compute it feeds, a send immediately after its producer
        for i, a in enumerate(lst):
            if a[0] in A.RECVS:
                nxt = lst[i + 1]
                assert nxt[0] == (A.F if a[0] == A.RECV_ACT else A.B) and nxt[1:4] == a[1:4]
            if a[0] in A.SENDS:
                prv = lst[i - 1]
                assert prv[0] == (A.F if a[0] == A.SEND_ACT else A.B) and prv[1:4] == a[1:4]
            if a[0] not in A.COMPUTE:
                assert a[4] != r and abs(a[4] - r) == 1           # neighbours only
    # one message per micro-batch, direction and stage boundary that crosses ranks: the wave has
    # 2W - 1 local turns among its S - 1 boundaries
    crossing = (n_stage - 1) - (2 * W - 1) if P > 1 else 0
    assert A.check_matching(lists, P, W, M) == 2 * M * crossing


def test_single_rank_has_no_communication():
    assert all(a[0] in A.COMPUTE for a in A.actions(1, 2, 3, 0))


@pytest.mark.parametrize("prefetch", [False, True])
def test_one_micro_batch_closed_form(prefetch):
    """P = 2, W = 1, M = 1: one chain through 4 stages and back, 4 messages, nothing to overlap with:
    makespan = 4 T_F + 4 T_B + 4 T_C."""
    lists = all_lists(2, 1, 1)
    for tc in (0.0, 0.25, 3.0):
        rep = A.replay(lists, 2, 1, 1, 1.0, 2.0, tc, prefetch)
        assert rep["makespan"] == pytest.approx(12.0 + 4 * tc)


@pytest.mark.parametrize("P,W,M", GRID)
def test_zero_transfer_time_is_the_task_level_replay(P, W, M):
    lists = all_lists(P, W, M)
    want = R.replay([[a[:4] for a in lst if a[0] in A.COMPUTE] for lst in lists], P, W, M)
    for prefetch in (False, True):
        rep = A.replay(lists, P, W, M, 1, 2, 0.0, prefetch)
        assert rep["makespan"] == want["makespan"] and rep["idle"] == want["idle"]


@pytest.mark.parametrize("P,W,M", [(2, 1, 4), (4, 2, 8), (4, 1, 16), (3, 2, 5)])
def test_prefetch_never_hurts_and_cost_grows_with_transfer_time(P, W, M):
    lists = all_lists(P, W, M)
    last = None
    for tc in (0.0, 0.1, 0.5, 1.0):
        plain = A.replay(lists, P, W, M, 1, 2, tc, False)["makespan"]
        pre = A.replay(lists, P, W, M, 1, 2, tc, True)["makespan"]
        assert pre <= plain + 1e-12
        if last is not None:
            assert plain >= last[0] - 1e-12 and pre >= last[1] - 1e-12
        last = (plain, pre)
    # with M > 1 there is compute to hide transfers behind: prefetch strictly helps at T_C = 0.5
    assert A.replay(lists, P, W, M, 1, 2, 0.5, True)["makespan"] < A.replay(lists, P, W, M, 1, 2, 0.5, False)["makespan"]


def test_two_micro_batches_by_hand():
    """P = 2, W = 1, M = 2, T_F = 1, T_B = 2, T_C = 0.5.  Rank 0: F0.0 S F1.0 S R F0.3 B0.3 S R F1.3 B1.3 S R B0.0 R B1.0.
    Without prefetch the receive for stage 3 of micro-batch 0 is posted at t = 2 (after F1.0); the message
    left rank 1 at t = 3.5 and lands at 4.0."""
    lists = all_lists(2, 1, 2)
    kinds0 = [a[0] for a in lists[0]]
    assert kinds0 == [A.F, A.SEND_ACT, A.F, A.SEND_ACT, A.RECV_ACT, A.F, A.B, A.SEND_GRAD, A.RECV_ACT, A.F, A.B,
                      A.SEND_GRAD, A.RECV_GRAD, A.B, A.RECV_GRAD, A.B]
    rep = A.replay(lists, 2, 1, 2, 1.0, 2.0, 0.5, False)
    # rank 1: recv (1.5) F0.1 F0.2 -> 3.5 send; recv (posted 3.5, sent 2.0 -> 4.0) F1.1 F1.2 -> 6.0 send
    # rank 0: recv 4.0, F0.3 5.0, B0.3 7.0 send; recv (posted 7.0, sent 6.0) 7.5, F1.3 8.5, B1.3 10.5 send
    # rank 1: recv grad (posted 6.0, sent 7.0) 7.5, B0.2 9.5, B0.1 11.5 send; recv (posted 11.5, sent 10.5) 12.0, B1.2 14, B1.1 16 send
    # rank 0: recv (posted 10.5, sent 11.5) 12.0, B0.0 14.0; recv (posted 14, sent 16) 16.5, B1.0 18.5
    assert rep["makespan"] == pytest.approx(18.5)
