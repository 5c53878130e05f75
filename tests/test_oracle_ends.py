"""Pins for the oracle of the model's two ends and the optimizer step (CPU only).

Nothing here re-types the oracle's formulas: the embedding is pinned by a case worked by hand and by
finite differences; the head by closed forms (zero table -> log V, a dominant logit -> 0), by torch's
cross_entropy / layer_norm / autograd in float64 (library routines) and by finite differences; Adam by
the closed form of its first step and by torch.optim.AdamW / Adam over several steps; the rank walk
with ends by finite differences of the iteration's loss through embedding, chunks and head, with tied
and untied tables."""

import math

import numpy as np
import pytest
import torch

from oracle import block as OB
from oracle import ends as OE
from oracle import executor as OX
from oracle import schedule as OS


def test_embedding_worked_by_hand():
    wte = np.array([[1.0, 2.0], [10.0, 20.0], [100.0, 200.0]])
    wpe = np.array([[0.5, 0.25], [0.125, 0.0625], [7.0, 7.0]])
    tokens = np.array([[2, 0], [1, 1]])
    x = OE.embed_forward(wte, wpe, tokens)
    assert np.array_equal(x, np.array([[[100.5, 200.25], [1.125, 2.0625]], [[10.5, 20.25], [10.125, 20.0625]]]))
    dx = np.array([[[1.0, 2.0], [3.0, 4.0]], [[5.0, 6.0], [7.0, 8.0]]])
    d_wte, d_wpe = OE.embed_backward(tokens, dx, 3, 3)
    assert np.array_equal(d_wte, np.array([[3.0, 4.0], [12.0, 14.0], [1.0, 2.0]]))      # token 1 twice: rows add
    assert np.array_equal(d_wpe, np.array([[6.0, 8.0], [10.0, 12.0], [0.0, 0.0]]))      # position 2 unused


def test_embedding_backward_by_finite_differences():
    rng = np.random.default_rng(0)
    V, H, b, s = 5, 3, 2, 4
    wte, wpe = rng.normal(size=(V, H)), rng.normal(size=(6, H))
    tokens = rng.integers(0, V, size=(b, s))
    dx = rng.normal(size=(b, s, H))
    d_wte, d_wpe = OE.embed_backward(tokens, dx, V, 6)
    f = lambda: float((OE.embed_forward(wte, wpe, tokens) * dx).sum())
    for tab, grad in ((wte, d_wte), (wpe, d_wpe)):
        for idx in np.ndindex(tab.shape):
            keep = tab[idx]
            tab[idx] = keep + 1e-6
            up = f()
            tab[idx] = keep - 1e-6
            dn = f()
            tab[idx] = keep
            assert abs((up - dn) / 2e-6 - grad[idx]) < 1e-8


def test_loss_closed_forms():
    rng = np.random.default_rng(1)
    b, s, H, V = 2, 3, 4, 7
    y = rng.normal(size=(b, s, H))
    labels = rng.integers(0, V, size=(b, s))
    loss, dy, d_head, _ = OE.head_loss(y, labels, np.zeros((V, H)))
    assert abs(loss - math.log(V)) < 1e-14                         # all logits equal
    assert np.array_equal(dy, np.zeros_like(dy))
    # one dominant logit at the label: loss -> 0, gradient -> 0
    head = np.zeros((V, H))
    head[3, 0] = 100.0
    yy = np.zeros((1, 1, H))
    yy[0, 0, 0] = 1.0
    loss, dy, d_head, _ = OE.head_loss(yy, np.array([[3]]), head)
    assert 0.0 <= loss < 1e-40 and np.abs(d_head).max() < 1e-40
    # ignored positions: no labelled position at all -> zero loss and gradients
    loss, dy, d_head, _ = OE.head_loss(y, -np.ones((b, s), dtype=int), rng.normal(size=(V, H)))
    assert loss == 0.0 and not dy.any() and not d_head.any()


@pytest.mark.parametrize("final_ln", [False, True])
def test_head_against_torch(final_ln):
    rng = np.random.default_rng(2)
    b, s, H, V = 2, 5, 6, 11
    y = rng.normal(size=(b, s, H))
    head = rng.normal(size=(V, H))
    g, be = 1.0 + 0.3 * rng.normal(size=H), 0.3 * rng.normal(size=H)
    labels = rng.integers(0, V, size=(b, s))
    labels[0, 1] = -1
    labels[1, 4] = -1
    scale = 0.25
    loss, dy, d_head, d_lnf = OE.head_loss(y, labels, head, (g, be) if final_ln else None, 1e-5, scale)
    ty = torch.tensor(y, requires_grad=True)
    th = torch.tensor(head, requires_grad=True)
    tg, tb = torch.tensor(g, requires_grad=True), torch.tensor(be, requires_grad=True)
    hn = torch.nn.functional.layer_norm(ty, (H,), tg, tb, 1e-5) if final_ln else ty
    tl = torch.nn.functional.cross_entropy((hn @ th.T).reshape(-1, V), torch.tensor(labels).reshape(-1), ignore_index=-1)
    (tl * scale).backward()
    assert abs(loss - tl.item()) < 1e-12
    assert np.abs(dy - ty.grad.numpy()).max() < 1e-12
    assert np.abs(d_head - th.grad.numpy()).max() < 1e-12
    if final_ln:
        assert np.abs(d_lnf[0] - tg.grad.numpy()).max() < 1e-12 and np.abs(d_lnf[1] - tb.grad.numpy()).max() < 1e-12
    else:
        assert d_lnf is None


def test_head_by_finite_differences():
    rng = np.random.default_rng(3)
    b, s, H, V = 1, 3, 4, 6
    y, head = rng.normal(size=(b, s, H)), rng.normal(size=(V, H))
    g, be = 1.0 + 0.3 * rng.normal(size=H), 0.3 * rng.normal(size=H)
    labels = np.array([[2, -1, 5]])
    loss, dy, d_head, (dg, db) = OE.head_loss(y, labels, head, (g, be), 1e-5, 3.0)
    f = lambda: 3.0 * OE.head_loss(y, labels, head, (g, be), 1e-5)[0]
    for tab, grad in ((y, dy), (head, d_head), (g, dg), (be, db)):
        for idx in np.ndindex(tab.shape):
            keep = tab[idx]
            tab[idx] = keep + 1e-6
            up = f()
            tab[idx] = keep - 1e-6
            dn = f()
            tab[idx] = keep
            assert abs((up - dn) / 2e-6 - grad[idx]) < 1e-7


def test_adam_first_step_closed_form():
    rng = np.random.default_rng(4)
    p, g = rng.normal(size=50), rng.normal(size=50)
    lr, wd = 1e-2, 0.1
    # from m = v = 0 the bias-corrected moments of step 1 are g and g^2
    q, m, v = OE.adam_step(p, g, np.zeros(50), np.zeros(50), 1, lr, 0.9, 0.999, 1e-8, wd)
    assert np.abs(q - (p - lr * g / (np.abs(g) + 1e-8) - lr * wd * p)).max() < 1e-15
    assert np.allclose(m, 0.1 * g, rtol=1e-14) and np.allclose(v, 0.001 * g * g, rtol=1e-12)


@pytest.mark.parametrize("wd", [0.0, 0.05])
def test_adam_against_torch(wd):
    rng = np.random.default_rng(5)
    p = rng.normal(size=(7, 3))
    tp = torch.tensor(p.copy(), requires_grad=True)
    opt = (torch.optim.AdamW([tp], lr=3e-3, betas=(0.8, 0.95), eps=1e-6, weight_decay=wd) if wd
           else torch.optim.Adam([tp], lr=3e-3, betas=(0.8, 0.95), eps=1e-6))
    m, v = np.zeros_like(p), np.zeros_like(p)
    for t in range(1, 7):
        g = rng.normal(size=p.shape)
        p, m, v = OE.adam_step(p, g, m, v, t, 3e-3, 0.8, 0.95, 1e-6, wd)
        tp.grad = torch.tensor(g)
        opt.step()
        assert np.abs(p - tp.detach().numpy()).max() < 1e-14, t


def tiny_model(P, W, M, tied, final_ln, norm="pre", seed=0, H=8, V=13, s=4, b=2):
    rng = np.random.default_rng(seed)
    cfg = OB.BlockCfg(H, 2, 2 * H, norm=norm, causal=(norm == "pre"))

    def block():
        q = {"wqkv": rng.normal(0, 0.3, (H, 3 * H)), "bqkv": rng.normal(0, 0.3, 3 * H),
             "wo": rng.normal(0, 0.3, (H, H)), "bo": rng.normal(0, 0.3, H),
             "w1": rng.normal(0, 0.3, (H, 2 * H)), "b1": rng.normal(0, 0.3, 2 * H),
             "w2": rng.normal(0, 0.3, (2 * H, H)), "b2": rng.normal(0, 0.3, H)}
        for k in ("ln1_g", "ln2_g"):
            q[k] = 1.0 + 0.2 * rng.normal(size=H)
        for k in ("ln1_b", "ln2_b"):
            q[k] = 0.2 * rng.normal(size=H)
        return q

    params = [[block()] for _ in range(2 * W)]
    tokens = [rng.integers(0, V, size=(b, s)) for _ in range(M)]
    labels = [rng.integers(-1, V, size=(b, s)) for _ in range(M)]
    ends = {"wte": rng.normal(0, 0.5, (V, H)), "wpe": rng.normal(0, 0.5, (s + 1, H)),
            "head": None if tied else rng.normal(0, 0.5, (V, H)),
            "lnf": (1.0 + 0.2 * rng.normal(size=H), 0.2 * rng.normal(size=H)) if final_ln else None,
            "tokens": lambda m: tokens[m], "labels": lambda m: labels[m], "loss_scale": 1.0 / M}
    return cfg, params, ends


@pytest.mark.parametrize("tied,final_ln,norm", [(True, True, "pre"), (False, False, "post")])
def test_rank_walk_with_ends_by_finite_differences(tied, final_ln, norm):
    """P = 1: rank 0 holds every stage, so its walk is the whole model.  The iteration's loss is the mean
    of the micro-batch losses; its gradient w.r.t. every kind of parameter (tables, chunk weights, final
    LayerNorm) must match central differences, which fails if the embedding or the head is attached to
    the wrong stage, a tied table misses one of its two contributions, or the loss scale is dropped."""
    P, W, M = 1, 1, 3
    cfg, params, ends = tiny_model(P, W, M, tied, final_ln, norm)
    tasks = OS.schedule(P, W, M, 0)
    run = lambda: OX.run_rank(tasks, P, W, 0, cfg, params, None, None, ends=ends)
    out = run()
    total = lambda: sum(run()["loss"].values()) / M
    rng = np.random.default_rng(9)
    eg = out["ends_grads"]
    assert (eg["head"] is None) == tied
    checks = [(ends["wte"], eg["wte"]), (ends["wpe"], eg["wpe"]),
              (params[0][0]["wqkv"], out["grads"][0][0]["wqkv"]), (params[1][0]["w2"], out["grads"][1][0]["w2"]),
              (params[1][0]["ln2_g"], out["grads"][1][0]["ln2_g"])]
    if not tied:
        checks.append((ends["head"], eg["head"]))
    if final_ln:
        checks += [(ends["lnf"][0], eg["lnf"][0]), (ends["lnf"][1], eg["lnf"][1])]
    for tab, grad in checks:
        for _ in range(6):
            idx = tuple(int(rng.integers(0, n)) for n in tab.shape)
            keep = tab[idx]
            tab[idx] = keep + 1e-6
            up = total()
            tab[idx] = keep - 1e-6
            dn = total()
            tab[idx] = keep
            assert abs((up - dn) / 2e-6 - grad[idx]) < 2e-7 * max(1.0, abs(grad[idx])), (tab.shape, idx)
    assert not eg["wpe"][-1].any()                                   # the position past the sequence is never used


def test_rank_walk_with_ends_on_rank_0_of_a_wave():
    """P = 2, W = 1: rank 0 holds stage 0 and stage 3.  Its walk with ends needs no act_in for stage 0
    and no grad_in for stage 3, and the loss gradient it starts the backward from is the head's."""
    P, W, M = 2, 1, 2
    cfg, params, ends = tiny_model(P, W, M, True, True)
    rng = np.random.default_rng(11)
    recv_act = {m: rng.normal(size=(2, 4, 8)) for m in range(M)}
    recv_grad = {m: rng.normal(size=(2, 4, 8)) for m in range(M)}

    def act_in(m, c):
        assert c == 1
        return recv_act[m]

    def grad_in(m, c):
        assert c == 0
        return recv_grad[m]

    out = OX.run_rank(OS.schedule(P, W, M, 0), P, W, 0, cfg, params, act_in, grad_in, ends=ends)
    for m in range(M):
        y = out["act_out"][(m, 1)]
        loss, dy, _, _ = OE.head_loss(y, ends["labels"](m), ends["wte"], ends["lnf"], cfg.eps, 1.0 / M)
        assert out["loss"][m] == loss
        want, _ = OB.chunk_backward(cfg, OB.chunk_forward(params[1], recv_act[m], cfg)[1], dy)
        assert np.array_equal(out["grad_out"][(m, 1)], want)
