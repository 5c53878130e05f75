"""Pins for the whole-pipeline oracle (CPU only).

`monolithic` is the definition of what any synchronous pipeline schedule must compute; it is
pinned by finite differences of the scalar L = sum_m <y_m, dy_m> through ALL stages (a wrong stage
order, a dropped stage or a gradient routed to the wrong stage fails it) and by the two-stage case
written out with the block oracle directly.  `run_pipeline` is pinned against `monolithic`:
bit-identical results for every (P, W, M) tried, whatever order the ranks are polled in, with the
stash peaks of the plan; lists that violate a dependency deadlock."""

import numpy as np
import pytest

from oracle import block as OB
from oracle import pipeline as OP
from oracle import schedule as OS


def tiny(P, W, M, norm="pre", causal=True, padded=False, H=8, heads=2, s=4, b=2, nb=1, seed=0):
    rng = np.random.default_rng(seed)
    S = 2 * W * P
    cfg = OB.BlockCfg(H, heads, 2 * H, norm=norm, causal=causal)
    F = 2 * H

    def block():
        p = {"wqkv": rng.normal(0, 0.3, (H, 3 * H)), "bqkv": rng.normal(0, 0.3, 3 * H),
             "wo": rng.normal(0, 0.3, (H, H)), "bo": rng.normal(0, 0.3, H),
             "w1": rng.normal(0, 0.3, (H, F)), "b1": rng.normal(0, 0.3, F),
             "w2": rng.normal(0, 0.3, (F, H)), "b2": rng.normal(0, 0.3, H)}
        for k in ("ln1_g", "ln2_g"):
            p[k] = 1.0 + 0.2 * rng.normal(size=H)
        for k in ("ln1_b", "ln2_b"):
            p[k] = 0.2 * rng.normal(size=H)
        return p

    params = [[block() for _ in range(nb)] for _ in range(S)]
    xs = [rng.normal(size=(b, s, H)) for _ in range(M)]
    dys = [rng.normal(size=(b, s, H)) for _ in range(M)]
    lens = [rng.integers(max(1, s // 2), s + 1, size=b) for _ in range(M)] if padded else None
    vl = (lambda m: lens[m]) if padded else None
    return cfg, params, xs, dys, vl


def loss(cfg, params, xs, dys, vl):
    ys, _, _ = OP.monolithic(cfg, params, xs, dys, vl)
    return sum(float((y * dy).sum()) for y, dy in zip(ys, dys))


@pytest.mark.parametrize("norm,causal,padded", [("pre", True, False), ("post", False, True)])
def test_monolithic_by_finite_differences(norm, causal, padded):
    cfg, params, xs, dys, vl = tiny(2, 1, 2, norm, causal, padded)        # S = 4 stages
    _, dxs, grads = OP.monolithic(cfg, params, xs, dys, vl)
    eps = 1e-6
    rng = np.random.default_rng(5)
    # input gradient of micro-batch 1: every entry
    for idx in np.ndindex(xs[1].shape):
        keep = xs[1][idx]
        xs[1][idx] = keep + eps
        up = loss(cfg, params, xs, dys, vl)
        xs[1][idx] = keep - eps
        dn = loss(cfg, params, xs, dys, vl)
        xs[1][idx] = keep
        assert abs((up - dn) / (2 * eps) - dxs[1][idx]) <= 1e-6 * max(1.0, abs(dxs[1][idx]))
    # parameters: three random entries of every tensor of every stage (summed over both micro-batches)
    for s in range(len(params)):
        for name, w in params[s][0].items():
            for _ in range(3):
                idx = tuple(int(rng.integers(0, n)) for n in w.shape)
                keep = w[idx]
                w[idx] = keep + eps
                up = loss(cfg, params, xs, dys, vl)
                w[idx] = keep - eps
                dn = loss(cfg, params, xs, dys, vl)
                w[idx] = keep
                want = grads[s][0][name][idx]
                assert abs((up - dn) / (2 * eps) - want) <= 2e-6 * max(1.0, abs(want)), (s, name, idx)


def test_monolithic_two_stages_written_out():
    cfg, params, xs, dys, vl = tiny(1, 1, 1)                               # S = 2
    ys, dxs, grads = OP.monolithic(cfg, params, xs, dys, vl)
    a, st0 = OB.chunk_forward(params[0], xs[0], cfg)
    y, st1 = OB.chunk_forward(params[1], a, cfg)
    g1, gr1 = OB.chunk_backward(cfg, st1, dys[0])
    g0, gr0 = OB.chunk_backward(cfg, st0, g1)
    assert np.array_equal(ys[0], y) and np.array_equal(dxs[0], g0)
    for got, want in ((grads[0], gr0), (grads[1], gr1)):
        for k in want[0]:
            assert np.array_equal(got[0][k], want[0][k])


def same(a, b):
    assert len(a["ys"]) == len(b[0])
    for x, y in zip(a["ys"], b[0]):
        assert np.array_equal(x, y)
    for x, y in zip(a["dxs"], b[1]):
        assert np.array_equal(x, y)
    for gs, hs in zip(a["grads"], b[2]):
        for g, h in zip(gs, hs):
            for k in h:
                assert np.array_equal(g[k], h[k]), k


@pytest.mark.parametrize("P,W,M", [(2, 1, 4), (1, 2, 3), (3, 2, 5), (4, 1, 4), (2, 2, 1), (4, 2, 8)])
def test_pipeline_equals_monolithic(P, W, M):
    """Every parameter's B tasks come in ascending micro-batch order on their rank, which is the order
    `monolithic` sums in: the results are bit-identical, not just close."""
    cfg, params, xs, dys, vl = tiny(P, W, M, nb=1, s=3, b=1, seed=P * 100 + W * 10 + M)
    sim = OS.simulate(P, W, M)
    ref = OP.monolithic(cfg, params, xs, dys, vl)
    out = OP.run_pipeline(sim["lists"], P, W, M, cfg, params, xs, dys, vl)
    same(out, ref)
    assert out["peak"] == [OS.stash_plan(sim["lists"][r], W)[0] for r in range(P)]
    # polling the ranks in another order changes the interleaving, not the result
    out2 = OP.run_pipeline(sim["lists"], P, W, M, cfg, params, xs, dys, vl, rank_order=list(range(P))[::-1])
    same(out2, ref)


def test_pipeline_with_padding_and_post_ln():
    P, W, M = 2, 2, 3
    cfg, params, xs, dys, vl = tiny(P, W, M, "post", False, True, nb=2, seed=9)
    sim = OS.simulate(P, W, M)
    same(OP.run_pipeline(sim["lists"], P, W, M, cfg, params, xs, dys, vl), OP.monolithic(cfg, params, xs, dys, vl))


def test_bad_lists_deadlock_or_are_caught():
    P, W, M = 2, 1, 2
    cfg, params, xs, dys, vl = tiny(P, W, M, s=2, b=1)
    lists = [list(l) for l in OS.simulate(P, W, M)["lists"]]
    # a backward moved in front of its own forward
    bad = [list(l) for l in lists]
    i = next(k for k, t in enumerate(bad[1]) if t[0] == OS.B)
    bad[1].insert(0, bad[1].pop(i))
    with pytest.raises(AssertionError):
        OP.run_pipeline(bad, P, W, M, cfg, params, xs, dys, vl)
    # a task dropped
    bad = [list(l) for l in lists]
    bad[0].pop()
    with pytest.raises(AssertionError):
        OP.run_pipeline(bad, P, W, M, cfg, params, xs, dys, vl)
    # a task on the wrong rank
    bad = [list(l) for l in lists]
    bad[0][0], bad[1][0] = bad[1][0], bad[0][0]
    with pytest.raises(AssertionError):
        OP.run_pipeline(bad, P, W, M, cfg, params, xs, dys, vl)


# ------------------------------------------------------------------ with the model's ends

def tiny_ends(M, tied, final_ln, H=8, V=11, s=4, b=2, seed=3):
    rng = np.random.default_rng(seed)
    tokens = [rng.integers(0, V, size=(b, s)) for _ in range(M)]
    labels = [rng.integers(-1, V, size=(b, s)) for _ in range(M)]
    return {"wte": rng.normal(0, 0.5, (V, H)), "wpe": rng.normal(0, 0.5, (s, H)),
            "head": None if tied else rng.normal(0, 0.5, (V, H)),
            "lnf": (1.0 + 0.2 * rng.normal(size=H), 0.2 * rng.normal(size=H)) if final_ln else None,
            "tokens": lambda m: tokens[m], "labels": lambda m: labels[m], "loss_scale": 1.0 / M}


@pytest.mark.parametrize("tied,final_ln", [(True, True), (False, False)])
def test_monolithic_with_ends_by_finite_differences(tied, final_ln):
    """The mean of the micro-batch losses of the whole model (embedding, 4 stages, head) against central
    differences, for table entries (a tied table collects two contributions), a chunk weight of the first
    and of the last stage, and the final LayerNorm."""
    M = 2
    cfg, params, _, _, _ = tiny(2, 1, M)
    ends = tiny_ends(M, tied, final_ln)
    _, _, grads, losses, eg = OP.monolithic(cfg, params, None, None, ends=ends, M=M)
    total = lambda: sum(OP.monolithic(cfg, params, None, None, ends=ends, M=M)[3].values()) / M
    assert abs(total() - sum(losses.values()) / M) == 0.0
    rng = np.random.default_rng(8)
    checks = [(ends["wte"], eg["wte"]), (ends["wpe"], eg["wpe"]), (params[0][0]["w1"], grads[0][0]["w1"]),
              (params[3][0]["wo"], grads[3][0]["wo"])]
    if not tied:
        checks.append((ends["head"], eg["head"]))
    if final_ln:
        checks += [(ends["lnf"][0], eg["lnf"][0]), (ends["lnf"][1], eg["lnf"][1])]
    for tab, grad in checks:
        for _ in range(5):
            idx = tuple(int(rng.integers(0, n)) for n in tab.shape)
            keep = tab[idx]
            tab[idx] = keep + 1e-6
            up = total()
            tab[idx] = keep - 1e-6
            dn = total()
            tab[idx] = keep
            assert abs((up - dn) / 2e-6 - grad[idx]) <= 2e-7 * max(1.0, abs(grad[idx])), (tab.shape, idx)


@pytest.mark.parametrize("P,W,M", [(2, 1, 4), (3, 2, 5), (1, 1, 2)])
def test_pipeline_with_ends_equals_monolithic(P, W, M):
    cfg, params, _, _, _ = tiny(P, W, M, nb=1, s=4, b=2, seed=P * 100 + W * 10 + M)
    ends = tiny_ends(M, True, True)
    sim = OS.simulate(P, W, M)
    ys, dxs, grads, losses, eg = OP.monolithic(cfg, params, None, None, ends=ends, M=M)
    out = OP.run_pipeline(sim["lists"], P, W, M, cfg, params, None, None, ends=ends)
    same(out, (ys, dxs, grads))
    assert out["losses"] == losses
    # the head's contributions to the tied table arrive in another order than the embedding's: equal up to rounding
    assert np.allclose(out["ends_grads"]["wte"], eg["wte"], rtol=1e-12, atol=1e-15)
    assert np.array_equal(out["ends_grads"]["wpe"], eg["wpe"])
    assert np.array_equal(out["ends_grads"]["lnf"][0], eg["lnf"][0])


def test_rounding_error_grows_like_the_square_root_of_the_depth():
    """Where the whole-pipeline GPU tests get their tolerance from.  A tensor that has passed through d blocks
    whose stored outputs are rounded to bf16 carries d independent roundings of relative size 2^-9; through the
    residual stream they add in quadrature.  Emulated in the oracle (every block's output rounded to bf16, against
    the same model unrounded, float64): the normalised error at depth 32 is sqrt(8) times the error at depth 4
    within a factor 1.6, far from the factor 8 of errors that add up linearly, and stays below the stated bf16
    tolerance scaled by sqrt(depth / 4), the rule of tests/test_gpu_pipeline.py."""
    import numpy as np
    from oracle import block as OB
    from paper_2308_15762_amd import synth
    wl = synth.WORKLOADS["gpt_1024_bf16"].scaled(hidden=64, heads=2, ffn=256, seq=32, mb=2, n_blocks=1)
    cfg = OB.BlockCfg(wl.hidden, wl.heads, wl.ffn, norm=wl.norm, causal=wl.causal)
    x = synth.model_input(wl, 0)
    exact, rounded = np.asarray(x, dtype=np.float64), np.asarray(x, dtype=np.float64)
    err = {}
    for depth in range(1, 33):
        params = synth.stage_params(wl, depth - 1)
        exact, _ = OB.chunk_forward(params, exact, cfg)
        rounded, _ = OB.chunk_forward(params, rounded, cfg)
        rounded = synth.bf16_round(rounded.astype(np.float32)).astype(np.float64)
        err[depth] = float(np.abs(rounded - exact).max() / np.abs(exact).max())
    growth = err[32] / err[4]
    assert 8 ** 0.5 / 1.6 <= growth <= 8 ** 0.5 * 1.6, growth
    for depth in (4, 8, 16, 32):
        assert err[depth] <= 2e-2 * (depth / 4.0) ** 0.5
