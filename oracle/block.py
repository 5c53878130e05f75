"""Oracle for the transformer-block chunk forward / backward.  TEST INFRASTRUCTURE ONLY.

The paper treats a pipeline stage as a black box of transformer layers
(evaluation section: "BERT-style" and "GPT-style" stacks given by layer, head
and hidden counts), so the block below is the textbook one, written out as its
definition with numpy (matmul and scipy's erf are the only library steps):

  LN(z)     = (z - mean) / sqrt(var + eps) * gamma + beta      (biased var, over H)
  Attn(u)   = concat_heads( softmax(Q K^T / sqrt(d), masked) V ) Wo + bo,
              [Q|K|V] = u Wqkv + bqkv
  MLP(v)    = GELU(v W1 + b1) W2 + b2,  GELU(h) = h/2 (1 + erf(h / sqrt 2))
  pre-LN    x1 = x + Attn(LN1(x));      y = x1 + MLP(LN2(x1))
  post-LN   x1 = LN1(x + Attn(x));      y = LN2(x1 + MLP(x1))

Masks: causal excludes key j > query i; key padding excludes keys j >= valid
length of that sequence for every query row.  Excluded scores get probability
exactly 0.  A chunk is n_blocks blocks composed, nothing else.

Arrays: x is [b, s, H]; matrices are [in, out] (y = x W + b); Wqkv columns are
[Q | K | V], head j owning columns j*d .. (j+1)*d-1 of each third.  All
arithmetic runs in `dtype` (float64 unless asked otherwise).
"""

import math

import numpy as np
from scipy.special import erf

PARAM_NAMES = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo",
               "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


class BlockCfg:
    def __init__(self, hidden, heads, ffn, norm="pre", causal=True, eps=1e-5):
        assert hidden % heads == 0 and norm in ("pre", "post")
        self.hidden, self.heads, self.ffn = hidden, heads, ffn
        self.norm, self.causal, self.eps = norm, causal, eps


# ----------------------------------------------------------------- pieces

def ln_fwd(z, g, b, eps):
    mu = z.mean(axis=-1, keepdims=True)
    var = ((z - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    zhat = (z - mu) * rstd
    return zhat * g + b, (zhat, rstd)


def ln_bwd(dout, g, cache):
    zhat, rstd = cache
    dzhat = dout * g
    dz = (dzhat - dzhat.mean(axis=-1, keepdims=True)
          - zhat * (dzhat * zhat).mean(axis=-1, keepdims=True)) * rstd
    dg = (dout * zhat).reshape(-1, zhat.shape[-1]).sum(axis=0)
    db = dout.reshape(-1, zhat.shape[-1]).sum(axis=0)
    return dz, dg, db


def gelu(h):
    return 0.5 * h * (1.0 + erf(h / math.sqrt(2.0)))


def gelu_grad(h):
    cdf = 0.5 * (1.0 + erf(h / math.sqrt(2.0)))
    pdf = np.exp(-0.5 * h * h) / math.sqrt(2.0 * math.pi)
    return cdf + h * pdf


def _allowed(s, causal, valid_len, b):
    """Boolean [b, 1, s_query, s_key]: True where the key takes part."""
    ok = np.ones((b, 1, s, s), dtype=bool)
    if causal:
        ok &= np.tril(np.ones((s, s), dtype=bool))[None, None]
    if valid_len is not None:
        keys = np.arange(s)[None, :] < np.asarray(valid_len)[:, None]      # [b, s_key]
        ok &= keys[:, None, None, :]
    return ok


def attn_fwd(u, p, cfg, valid_len):
    b, s, H = u.shape
    h, d = cfg.heads, H // cfg.heads
    qkv = u @ p["wqkv"] + p["bqkv"]
    q, k, v = (qkv[..., i * H:(i + 1) * H].reshape(b, s, h, d).transpose(0, 2, 1, 3)
               for i in range(3))                                          # [b, h, s, d]
    scores = (q @ k.transpose(0, 1, 3, 2)) / math.sqrt(d)
    ok = _allowed(s, cfg.causal, valid_len, b)
    masked = np.where(ok, scores, -np.inf)
    e = np.exp(masked - masked.max(axis=-1, keepdims=True))
    e = np.where(ok, e, 0.0)
    prob = e / e.sum(axis=-1, keepdims=True)
    ctx = (prob @ v).transpose(0, 2, 1, 3).reshape(b, s, H)
    out = ctx @ p["wo"] + p["bo"]
    return out, (u, q, k, v, prob, ctx)


def attn_bwd(dout, p, cfg, cache):
    u, q, k, v, prob, ctx = cache
    b, s, H = u.shape
    h, d = cfg.heads, H // cfg.heads
    g = {}
    g["wo"] = ctx.reshape(-1, H).T @ dout.reshape(-1, H)
    g["bo"] = dout.reshape(-1, H).sum(axis=0)
    dctx = (dout @ p["wo"].T).reshape(b, s, h, d).transpose(0, 2, 1, 3)
    dv = prob.transpose(0, 1, 3, 2) @ dctx
    dprob = dctx @ v.transpose(0, 1, 3, 2)
    dscore = prob * (dprob - (dprob * prob).sum(axis=-1, keepdims=True))
    dq = (dscore @ k) / math.sqrt(d)
    dk = (dscore.transpose(0, 1, 3, 2) @ q) / math.sqrt(d)
    dqkv = np.concatenate([t.transpose(0, 2, 1, 3).reshape(b, s, H) for t in (dq, dk, dv)], axis=-1)
    g["wqkv"] = u.reshape(-1, H).T @ dqkv.reshape(-1, 3 * H)
    g["bqkv"] = dqkv.reshape(-1, 3 * H).sum(axis=0)
    du = dqkv @ p["wqkv"].T
    return du, g


def mlp_fwd(v, p):
    hpre = v @ p["w1"] + p["b1"]
    act = gelu(hpre)
    return act @ p["w2"] + p["b2"], (v, hpre, act)


def mlp_bwd(dout, p, cache):
    v, hpre, act = cache
    H, Fd = p["w1"].shape
    g = {}
    g["w2"] = act.reshape(-1, Fd).T @ dout.reshape(-1, H)
    g["b2"] = dout.reshape(-1, H).sum(axis=0)
    dh = (dout @ p["w2"].T) * gelu_grad(hpre)
    g["w1"] = v.reshape(-1, H).T @ dh.reshape(-1, Fd)
    g["b1"] = dh.reshape(-1, Fd).sum(axis=0)
    return dh @ p["w1"].T, g


# ----------------------------------------------------------------- block / chunk

def block_forward(p, x, cfg, valid_len=None):
    if cfg.norm == "pre":
        u, c_ln1 = ln_fwd(x, p["ln1_g"], p["ln1_b"], cfg.eps)
        a, c_att = attn_fwd(u, p, cfg, valid_len)
        x1 = x + a
        v, c_ln2 = ln_fwd(x1, p["ln2_g"], p["ln2_b"], cfg.eps)
        f, c_mlp = mlp_fwd(v, p)
        y = x1 + f
    else:
        a, c_att = attn_fwd(x, p, cfg, valid_len)
        x1, c_ln1 = ln_fwd(x + a, p["ln1_g"], p["ln1_b"], cfg.eps)
        f, c_mlp = mlp_fwd(x1, p)
        y, c_ln2 = ln_fwd(x1 + f, p["ln2_g"], p["ln2_b"], cfg.eps)
    return y, (c_ln1, c_att, c_ln2, c_mlp)


def block_backward(p, cfg, cache, dy):
    """Returns dx and a dict of parameter gradients of <y, dy>."""
    c_ln1, c_att, c_ln2, c_mlp = cache
    g = {}
    if cfg.norm == "pre":
        dv, gm = mlp_bwd(dy, p, c_mlp)
        dx1_branch, g["ln2_g"], g["ln2_b"] = ln_bwd(dv, p["ln2_g"], c_ln2)
        dx1 = dy + dx1_branch
        du, ga = attn_bwd(dx1, p, cfg, c_att)
        dx_branch, g["ln1_g"], g["ln1_b"] = ln_bwd(du, p["ln1_g"], c_ln1)
        dx = dx1 + dx_branch
    else:
        df, g["ln2_g"], g["ln2_b"] = ln_bwd(dy, p["ln2_g"], c_ln2)
        dx1_branch, gm = mlp_bwd(df, p, c_mlp)
        dx1 = df + dx1_branch
        da, g["ln1_g"], g["ln1_b"] = ln_bwd(dx1, p["ln1_g"], c_ln1)
        dx_branch, ga = attn_bwd(da, p, cfg, c_att)
        dx = da + dx_branch
    g.update(gm)
    g.update(ga)
    return dx, g


def _cast(params, dtype):
    return [{k: np.asarray(v, dtype=dtype) for k, v in blk.items()} for blk in params]


def chunk_forward(params, x, cfg, valid_len=None, dtype=np.float64):
    """params: list (one dict per block).  Returns (y, stash)."""
    params = _cast(params, dtype)
    caches = []
    y = np.asarray(x, dtype=dtype)
    for p in params:
        y, c = block_forward(p, y, cfg, valid_len)
        caches.append(c)
    return y, (params, caches)


def chunk_backward(cfg, stash, dy, grads=None):
    """Returns (dx, grads); `grads` (list of dicts) is accumulated into if given."""
    params, caches = stash
    dx = np.asarray(dy, dtype=params[0]["wqkv"].dtype)
    new = [None] * len(params)
    for i in range(len(params) - 1, -1, -1):
        dx, new[i] = block_backward(params[i], cfg, caches[i], dx)
    if grads is None:
        return dx, new
    for acc, g in zip(grads, new):
        for k in g:
            acc[k] = acc[k] + g[k]
    return dx, grads

