"""Pins for the block oracle: finite differences, an autograd build of the same
block from torch's library layers, invariants and closed-form special cases."""

import numpy as np
import pytest
import torch
import torch.nn.functional as TF

from oracle import block as O
from paper_2308_15762_amd import synth

CASES = [
    # norm, causal, padded, H, heads, s, b, nb
    ("pre", True, False, 16, 2, 6, 2, 1),
    ("pre", True, False, 8, 1, 5, 2, 2),
    ("post", False, True, 16, 4, 6, 3, 1),
    ("post", False, True, 12, 2, 4, 2, 2),
    ("pre", False, True, 8, 2, 5, 2, 1),
    ("post", True, False, 8, 2, 4, 2, 1),
]


def make(norm, causal, padded, H, heads, s, b, nb, seed=0, scale=0.3):
    rng = np.random.default_rng(seed)
    cfg = O.BlockCfg(H, heads, 4 * H, norm=norm, causal=causal)
    params = []
    for _ in range(nb):
        p = {}
        for name, shape in (("wqkv", (H, 3 * H)), ("bqkv", (3 * H,)), ("wo", (H, H)), ("bo", (H,)),
                            ("w1", (H, 4 * H)), ("b1", (4 * H,)), ("w2", (4 * H, H)), ("b2", (H,))):
            p[name] = rng.normal(0, scale, size=shape)
        for name in ("ln1_g", "ln2_g"):
            p[name] = 1.0 + 0.2 * rng.normal(size=H)
        for name in ("ln1_b", "ln2_b"):
            p[name] = 0.2 * rng.normal(size=H)
        params.append(p)
    x = rng.normal(size=(b, s, H))
    dy = rng.normal(size=(b, s, H))
    vl = rng.integers(max(1, s // 2), s + 1, size=b) if padded else None
    return cfg, params, x, dy, vl


def loss(params, x, cfg, vl, dy):
    y, _ = O.chunk_forward(params, x, cfg, vl)
    return float((y * dy).sum())


@pytest.mark.parametrize("case", CASES)
def test_finite_differences(case):
    cfg, params, x, dy, vl = make(*case)
    y, stash = O.chunk_forward(params, x, cfg, vl)
    dx, grads = O.chunk_backward(cfg, stash, dy)
    eps = 1e-5
    rng = np.random.default_rng(1)
    num = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        xp, xm = x.copy(), x.copy()
        xp[i] += eps
        xm[i] -= eps
        num[i] = (loss(params, xp, cfg, vl, dy) - loss(params, xm, cfg, vl, dy)) / (2 * eps)
    assert np.abs(num - dx).max() <= 1e-6 * max(1.0, np.abs(dx).max())
    for bi, p in enumerate(params):
        for name in O.PARAM_NAMES:
            flat = p[name].reshape(-1)
            for j in rng.choice(flat.size, size=min(4, flat.size), replace=False):
                keep = flat[j]
                flat[j] = keep + eps
                lp = loss(params, x, cfg, vl, dy)
                flat[j] = keep - eps
                lm = loss(params, x, cfg, vl, dy)
                flat[j] = keep
                want = (lp - lm) / (2 * eps)
                got = grads[bi][name].reshape(-1)[j]
                assert abs(want - got) <= 1e-6 * max(1.0, abs(want)), (bi, name, j)


def torch_chunk(params, x, cfg, vl):
    """Same block from torch library layers; gradients come from autograd."""
    H, h = cfg.hidden, cfg.heads
    d = H // h
    b, s, _ = x.shape
    allow = torch.ones(b, 1, s, s, dtype=torch.bool)
    if cfg.causal:
        allow &= torch.ones(s, s).tril().bool()[None, None]
    if vl is not None:
        allow &= (torch.arange(s)[None, :] < torch.as_tensor(vl)[:, None])[:, None, None, :]

    def attn(u, p):
        qkv = TF.linear(u, p["wqkv"].T, p["bqkv"])
        q, k, v = (t.reshape(b, s, h, d).transpose(1, 2) for t in qkv.split(H, dim=-1))
        c = TF.scaled_dot_product_attention(q, k, v, attn_mask=allow)
        return TF.linear(c.transpose(1, 2).reshape(b, s, H), p["wo"].T, p["bo"])

    def mlp(v, p):
        return TF.linear(TF.gelu(TF.linear(v, p["w1"].T, p["b1"])), p["w2"].T, p["b2"])

    y = x
    for p in params:
        if cfg.norm == "pre":
            x1 = y + attn(TF.layer_norm(y, (H,), p["ln1_g"], p["ln1_b"], cfg.eps), p)
            y = x1 + mlp(TF.layer_norm(x1, (H,), p["ln2_g"], p["ln2_b"], cfg.eps), p)
        else:
            x1 = TF.layer_norm(y + attn(y, p), (H,), p["ln1_g"], p["ln1_b"], cfg.eps)
            y = TF.layer_norm(x1 + mlp(x1, p), (H,), p["ln2_g"], p["ln2_b"], cfg.eps)
    return y


@pytest.mark.parametrize("case", CASES + [("pre", True, False, 64, 4, 33, 2, 2), ("post", False, True, 64, 4, 40, 3, 2)])
def test_against_torch_autograd(case):
    cfg, params, x, dy, vl = make(*case, seed=3)
    y, stash = O.chunk_forward(params, x, cfg, vl)
    dx, grads = O.chunk_backward(cfg, stash, dy)
    tp = [{k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()} for p in params]
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    ty = torch_chunk(tp, tx, cfg, vl)
    ty.backward(torch.tensor(dy, dtype=torch.float64))
    tol = lambda ref: 1e-9 * max(1.0, np.abs(ref).max())
    assert np.abs(ty.detach().numpy() - y).max() <= tol(y)
    assert np.abs(tx.grad.numpy() - dx).max() <= tol(dx)
    for bi in range(len(params)):
        for name in O.PARAM_NAMES:
            ref = tp[bi][name].grad.numpy()
            assert np.abs(ref - grads[bi][name]).max() <= tol(ref), (bi, name)


def test_fp32_instance_agrees_with_fp64():
    cfg, params, x, dy, vl = make("pre", True, False, 64, 4, 32, 2, 2, seed=5, scale=0.05)
    y64, st64 = O.chunk_forward(params, x, cfg, vl)
    dx64, g64 = O.chunk_backward(cfg, st64, dy)
    y32, st32 = O.chunk_forward(params, x, cfg, vl, dtype=np.float32)
    dx32, g32 = O.chunk_backward(cfg, st32, dy)
    assert y32.dtype == np.float32 and dx32.dtype == np.float32
    nerr = lambda a, r: np.abs(a - r).max() / np.abs(r).max()
    assert nerr(y32, y64) < 1e-5 and nerr(dx32, dx64) < 1e-5
    for name in O.PARAM_NAMES:
        assert nerr(g32[0][name], g64[0][name]) < 1e-5


# --- invariants ---------------------------------------------------------------

def test_softmax_rows_sum_to_one_and_masks_are_exact_zero():
    cfg, params, x, dy, vl = make("pre", True, True, 16, 2, 7, 3, 1, seed=2)
    _, (_, caches) = O.chunk_forward(params, x, cfg, vl)
    prob = caches[0][1][4]
    assert np.allclose(prob.sum(-1), 1.0, atol=1e-12)
    s = x.shape[1]
    for n in range(x.shape[0]):
        for i in range(s):
            for j in range(s):
                if j > i or j >= vl[n]:
                    assert (prob[n, :, i, j] == 0).all()
                else:
                    assert (prob[n, :, i, j] > 0).all()


def test_layer_norm_statistics_and_backward_sums():
    rng = np.random.default_rng(0)
    z = rng.normal(2.0, 3.0, size=(5, 32))
    out, cache = O.ln_fwd(z, np.ones(32), np.zeros(32), 1e-5)
    assert np.allclose(out.mean(-1), 0, atol=1e-12)
    var = z.var(-1)
    assert np.allclose(out.var(-1), var / (var + 1e-5), rtol=1e-12)
    dout = rng.normal(size=z.shape)
    g = rng.normal(size=32)
    dz, dg, db = O.ln_bwd(dout, g, cache)
    assert np.allclose(dz.sum(-1), 0, atol=1e-12)
    assert np.allclose(db, dout.sum(0))


def test_gelu_values():
    # closed-form points of 0.5 h (1 + erf(h / sqrt 2)) and its derivative
    assert O.gelu(np.array([0.0]))[0] == 0.0
    assert np.isclose(O.gelu(np.array([1.0]))[0], 0.841344746068543)       # Phi(1)
    assert np.isclose(O.gelu(np.array([-1.0]))[0], -0.158655253931457)
    assert np.isclose(O.gelu_grad(np.array([0.0]))[0], 0.5)
    h = np.linspace(-4, 4, 41)
    num = (O.gelu(h + 1e-6) - O.gelu(h - 1e-6)) / 2e-6
    assert np.allclose(num, O.gelu_grad(h), atol=1e-8)


def test_causal_outputs_ignore_later_positions():
    cfg, params, x, dy, _ = make("pre", True, False, 16, 2, 8, 2, 2, seed=4)
    y, _ = O.chunk_forward(params, x, cfg)
    x2 = x.copy()
    x2[:, 5:] += 1.0
    y2, _ = O.chunk_forward(params, x2, cfg)
    assert np.array_equal(y[:, :5], y2[:, :5]) and not np.allclose(y[:, 5:], y2[:, 5:])


def test_padded_keys_do_not_reach_valid_rows():
    cfg, params, x, dy, _ = make("post", False, True, 16, 2, 8, 2, 2, seed=4)
    vl = np.array([5, 8])
    y, _ = O.chunk_forward(params, x, cfg, vl)
    x2 = x.copy()
    x2[0, 5:] -= 2.0
    y2, _ = O.chunk_forward(params, x2, cfg, vl)
    assert np.allclose(y[0, :5], y2[0, :5], atol=1e-13) and np.array_equal(y[1], y2[1])


def test_bias_grads_are_column_sums_and_grads_accumulate():
    cfg, params, x, dy, _ = make("pre", True, False, 16, 2, 6, 2, 1, seed=6)
    _, stash = O.chunk_forward(params, x, cfg)
    _, g = O.chunk_backward(cfg, stash, dy)
    assert np.allclose(g[0]["b2"], dy.reshape(-1, 16).sum(0))
    rng = np.random.default_rng(9)
    x_b, dy_b = rng.normal(size=x.shape), rng.normal(size=x.shape)
    _, stash_b = O.chunk_forward(params, x_b, cfg)
    _, g_b = O.chunk_backward(cfg, stash_b, dy_b)
    acc = [{k: np.zeros_like(v) for k, v in g[0].items()}]
    O.chunk_backward(cfg, stash, dy, acc)
    O.chunk_backward(cfg, stash_b, dy_b, acc)
    for k in O.PARAM_NAMES:
        assert np.allclose(acc[0][k], g[0][k] + g_b[0][k], rtol=1e-13, atol=1e-13)


# --- closed forms ---------------------------------------------------------------

def test_single_position_attention_is_the_value_path():
    cfg, params, x, dy, _ = make("pre", True, False, 16, 4, 1, 3, 1, seed=7)
    p = params[0]
    u = np.random.default_rng(0).normal(size=(3, 1, 16))
    out, _ = O.attn_fwd(u, p, cfg, None)
    want = (u @ p["wqkv"][:, 32:] + p["bqkv"][32:]) @ p["wo"] + p["bo"]
    assert np.allclose(out, want, atol=1e-13)


def test_zero_output_projections_make_pre_ln_block_the_identity():
    cfg, params, x, dy, _ = make("pre", True, False, 16, 2, 6, 2, 2, seed=8)
    for p in params:
        for k in ("wo", "bo", "w2", "b2"):
            p[k][...] = 0
    y, stash = O.chunk_forward(params, x, cfg)
    dx, _ = O.chunk_backward(cfg, stash, dy)
    assert np.array_equal(y, x) and np.array_equal(dx, dy)


def test_uniform_attention_when_scores_are_constant():
    # Wq = 0, bq = 0: every allowed key gets the same probability 1/count
    cfg, params, x, dy, _ = make("post", False, True, 8, 2, 6, 2, 1, seed=10)
    p = params[0]
    p["wqkv"][:, :8] = 0
    p["bqkv"][:8] = 0
    vl = np.array([3, 6])
    _, cache = O.attn_fwd(x, p, cfg, vl)
    prob = cache[4]
    assert np.allclose(prob[0, :, :, :3], 1 / 3) and np.allclose(prob[1], 1 / 6)


def test_two_block_chunk_equals_two_chained_chunks():
    cfg, params, x, dy, vl = make("post", False, True, 16, 2, 6, 2, 2, seed=11)
    y, stash = O.chunk_forward(params, x, cfg, vl)
    dx, g = O.chunk_backward(cfg, stash, dy)
    y1, s1 = O.chunk_forward(params[:1], x, cfg, vl)
    y2, s2 = O.chunk_forward(params[1:], y1, cfg, vl)
    d2, g2 = O.chunk_backward(cfg, s2, dy)
    d1, g1 = O.chunk_backward(cfg, s1, d2)
    assert np.array_equal(y, y2) and np.array_equal(dx, d1)
    assert all(np.array_equal(g[0][k], g1[0][k]) and np.array_equal(g[1][k], g2[0][k]) for k in O.PARAM_NAMES)


def test_synth_bf16_rounding_matches_torch():
    a = np.random.default_rng(0).normal(size=4096).astype(np.float32)
    a[:4] = [1.00390625, 1.01171875, -1.00390625, 3.0e-39]
    want = torch.tensor(a).bfloat16().float().numpy()
    assert np.array_equal(synth.bf16_round(a), want)
    assert np.array_equal(synth.from_bf16_bits(synth.to_bf16_bits(want)), want)
