"""Oracle for the action lists at the paper's granularity.  TEST INFRASTRUCTURE ONLY.

The paper's runtime section: the scheduler emits, per worker, a list of
instructions finer than "forward pass / backward pass": compute actions carrying
the local module index, and send / receive actions carrying the target rank; a
worker's interpreter executes its list, and before a slice of computation it
looks ahead to the next receive instruction and launches that receive first
(prefetch), with asynchronous communication.

Reading used here (the paper prints no list):
* rank r's action list is its task list with, around every compute task, the
  communication that task needs: a RECV immediately before a compute whose
  input is produced on another rank, a SEND immediately after a compute whose
  output is consumed on another rank.  Boundaries between two stages of the same
  rank (the turns of the wave) have no actions.
* SENDs are asynchronous (they cost the sender no time); a transfer starts when
  the message has been sent AND the receive has been posted, and takes t_c.
* without prefetch a receive is posted when the interpreter reaches it and the
  rank waits there for the arrival; with prefetch the interpreter, before it
  starts a compute action, looks ahead and posts the receive that feeds the
  following compute action (if there is one), and only waits for the arrival
  when it reaches that receive in the list.
"""

from . import schedule as OS

F, B, SEND_ACT, RECV_ACT, SEND_GRAD, RECV_GRAD = range(6)
COMPUTE = (F, B)
SENDS = (SEND_ACT, SEND_GRAD)
RECVS = (RECV_ACT, RECV_GRAD)


def actions(P, W, M, rank):
    """[(kind, mb, chunk, stage, peer)] for one rank; peer = own rank for compute actions.
    `stage` of a communication action is the stage of the local compute it serves."""
    return actions_from_tasks(OS.schedule(P, W, M, rank), P, W, rank)


def actions_from_tasks(tasks, P, W, rank):
    """The action list of any scheme's task list (W = 0: straight placement), same reading."""
    S = OS.n_stages(P, W)
    out = []
    for t in tasks:
        kind, mb, chunk, stage = t
        if kind == OS.F:
            src = OS.stage_rank(P, W, stage - 1) if stage > 0 else rank
            dst = OS.stage_rank(P, W, stage + 1) if stage < S - 1 else rank
            if src != rank:
                out.append((RECV_ACT, mb, chunk, stage, src))
            out.append((F, mb, chunk, stage, rank))
            if dst != rank:
                out.append((SEND_ACT, mb, chunk, stage, dst))
        else:
            src = OS.stage_rank(P, W, stage + 1) if stage < S - 1 else rank
            dst = OS.stage_rank(P, W, stage - 1) if stage > 0 else rank
            if src != rank:
                out.append((RECV_GRAD, mb, chunk, stage, src))
            out.append((B, mb, chunk, stage, rank))
            if dst != rank:
                out.append((SEND_GRAD, mb, chunk, stage, dst))
    return out


def message_of(action):
    """Identity of the message a communication action moves: (type, mb, producing stage)."""
    kind, mb, _, stage, _ = action
    if kind == SEND_ACT:
        return ("act", mb, stage)
    if kind == RECV_ACT:
        return ("act", mb, stage - 1)
    if kind == SEND_GRAD:
        return ("grad", mb, stage)
    if kind == RECV_GRAD:
        return ("grad", mb, stage + 1)
    raise ValueError(kind)


def check_matching(lists, P, W, M):
    """Every message is sent once and received once, by the right pair of ranks, and the messages of one
    type between one ordered pair of ranks are received in the order they are sent (so that tag-less
    point-to-point calls would pair up)."""
    sent, received = {}, {}
    for r, lst in enumerate(lists):
        for a in lst:
            if a[0] in SENDS:
                assert message_of(a) not in sent
                sent[message_of(a)] = (r, a[4])
            elif a[0] in RECVS:
                assert message_of(a) not in received
                received[message_of(a)] = (a[4], r)
            else:
                assert a[4] == r
    assert sent == received
    for r in range(P):
        for q in range(P):
            for typ, sk, rk in (("act", SEND_ACT, RECV_ACT), ("grad", SEND_GRAD, RECV_GRAD)):
                out = [message_of(a) for a in lists[r] if a[0] == sk and a[4] == q]
                inn = [message_of(a) for a in lists[q] if a[0] == rk and a[4] == r]
                assert out == inn, (typ, r, q)
    return len(sent)


def replay(lists, P, W, M, t_f=1.0, t_b=2.0, t_c=0.0, prefetch=False):
    """Event simulation of the P interpreters.  Returns dict(makespan, idle, waited): `waited[r]` = time
    rank r spent blocked in receives.  Raises AssertionError on deadlock."""
    S = OS.n_stages(P, W)
    done = {}       # (kind, mb, stage) of compute actions -> finish time
    sent = {}       # message -> time the send was executed
    posted = {}     # message -> time the receive was posted
    arrived = {}    # message -> arrival time
    head = [0] * P
    now = [0.0] * P
    busy = [0.0] * P
    waited = [0.0] * P

    def try_arrive(msg):
        if msg in sent and msg in posted and msg not in arrived:
            arrived[msg] = max(sent[msg], posted[msg]) + t_c

    progressed = True
    while progressed:
        progressed = False
        for r in range(P):
            while head[r] < len(lists[r]):
                a = lists[r][head[r]]
                kind, mb, _, stage, _ = a
                if kind in COMPUTE:
                    # local dependencies (remote ones were satisfied by the receive in front of this action)
                    if kind == F and stage > 0 and OS.stage_rank(P, W, stage - 1) == r and (F, mb, stage - 1) not in done:
                        break
                    if kind == B:
                        if (F, mb, stage) not in done:
                            break
                        if stage < S - 1 and OS.stage_rank(P, W, stage + 1) == r and (B, mb, stage + 1) not in done:
                            break
                    if prefetch:
                        # look ahead: the next receive, if it sits between this compute and the next one
                        for nxt in lists[r][head[r] + 1:]:
                            if nxt[0] in COMPUTE:
                                break
                            if nxt[0] in RECVS:
                                m2 = message_of(nxt)
                                if m2 not in posted:
                                    posted[m2] = now[r]
                                    try_arrive(m2)
                                break
                    # local producers may have finished later than this rank's clock
                    ready = now[r]
                    if kind == F and stage > 0 and OS.stage_rank(P, W, stage - 1) == r:
                        ready = max(ready, done[(F, mb, stage - 1)])
                    if kind == B:
                        ready = max(ready, done[(F, mb, stage)])
                        if stage < S - 1 and OS.stage_rank(P, W, stage + 1) == r:
                            ready = max(ready, done[(B, mb, stage + 1)])
                    c = t_f if kind == F else t_b
                    now[r] = ready + c
                    busy[r] += c
                    done[(kind, mb, stage)] = now[r]
                elif kind in SENDS:
                    msg = message_of(a)
                    sent[msg] = now[r]
                    try_arrive(msg)
                else:
                    msg = message_of(a)
                    if msg not in posted:
                        posted[msg] = now[r]
                        try_arrive(msg)
                    if msg not in arrived:
                        break           # the peer has not sent yet
                    if arrived[msg] > now[r]:
                        waited[r] += arrived[msg] - now[r]
                        now[r] = arrived[msg]
                head[r] += 1
                progressed = True
    assert all(head[r] == len(lists[r]) for r in range(P)), "deadlock"
    makespan = max(now)
    return {"makespan": makespan, "idle": [makespan - b for b in busy], "waited": waited}
