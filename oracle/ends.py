"""Oracle for the two ends of the model and the optimizer step.  TEST INFRASTRUCTURE ONLY.

The paper trains GPT-style and BERT-style language models with synchronous
pipeline parallelism: stage 0 starts from token ids, the last stage ends in a
loss, and the parameters are updated once per iteration, at the flush, from the
gradients summed over the micro-batches (background section on synchronous
pipelines).  It prints none of these pieces, so they are the textbook ones,
written out as their definitions:

  embedding   x[n, i, :] = wte[token[n, i], :] + wpe[i, :]
              (learned token and position tables, as in GPT-2 and BERT)
  head        hn = LN_f(y) (optional final LayerNorm), logits = hn head^T with
              head a [V, H] table (the token table itself when weights are tied)
  loss        mean over the labelled positions (label >= 0) of
              -log softmax(logits)[label]; positions with a negative label do
              not count
  gradient    of loss_scale * loss (loss_scale = 1 / M makes the iteration's
              loss the mean over its micro-batches)
  Adam        Kingma & Ba, Algorithm 1, with bias correction, plus the decoupled
              weight decay of Loshchilov & Hutter (Algorithm 2):
              m = b1 m + (1 - b1) g;  v = b2 v + (1 - b2) g^2
              p = p - lr * ( (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps) + wd * p )

All arithmetic in float64 unless the arrays passed in say otherwise.
"""

import numpy as np

from . import block as OB


def embed_forward(wte, wpe, tokens):
    """tokens: int [b, s].  Returns x [b, s, H]."""
    tokens = np.asarray(tokens)
    s = tokens.shape[1]
    return wte[tokens] + wpe[:s][None, :, :]


def embed_backward(tokens, dx, vocab, max_pos):
    """Returns (d_wte [V, H], d_wpe [max_pos, H]) of <x, dx>."""
    tokens = np.asarray(tokens)
    b, s = tokens.shape
    H = dx.shape[-1]
    d_wte = np.zeros((vocab, H), dtype=dx.dtype)
    for n in range(b):
        for i in range(s):
            d_wte[tokens[n, i]] += dx[n, i]
    d_wpe = np.zeros((max_pos, H), dtype=dx.dtype)
    d_wpe[:s] = dx.sum(axis=0)
    return d_wte, d_wpe


def head_loss(y, labels, head, lnf=None, eps=1e-5, loss_scale=1.0):
    """y [b, s, H], labels int [b, s] (negative = not counted), head [V, H],
    lnf = (gamma, beta) or None.
    Returns (loss, dy, d_head, d_lnf) with d_lnf = (dgamma, dbeta) or None; the gradients are those
    of loss_scale * loss.  With no labelled position the loss and all gradients are 0."""
    labels = np.asarray(labels)
    b, s, H = y.shape
    if lnf is not None:
        hn, cache = OB.ln_fwd(y, lnf[0], lnf[1], eps)
    else:
        hn = y
    logits = hn @ head.T                                           # [b, s, V]
    top = logits.max(axis=-1, keepdims=True)
    lse = top[..., 0] + np.log(np.exp(logits - top).sum(axis=-1))
    counted = labels >= 0
    n = int(counted.sum())
    if n == 0:
        zero = np.zeros_like(y)
        return 0.0, zero, np.zeros_like(head), (None if lnf is None else (np.zeros(H), np.zeros(H)))
    safe = np.where(counted, labels, 0)
    picked = np.take_along_axis(logits, safe[..., None], axis=-1)[..., 0]
    loss = float(((lse - picked) * counted).sum() / n)
    prob = np.exp(logits - lse[..., None])
    onehot = np.zeros_like(prob)
    np.put_along_axis(onehot, safe[..., None], 1.0, axis=-1)
    dlogits = (prob - onehot) * counted[..., None] * (loss_scale / n)
    d_head = dlogits.reshape(-1, dlogits.shape[-1]).T @ hn.reshape(-1, H)
    dhn = dlogits @ head
    if lnf is None:
        return loss, dhn, d_head, None
    dy, dg, db = OB.ln_bwd(dhn, lnf[0], cache)
    return loss, dy, d_head, (dg, db)


def adam_step(p, g, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0):
    """One update, step count t >= 1.  Returns (p, m, v), new arrays."""
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    p = p - lr * (mhat / (np.sqrt(vhat) + eps) + weight_decay * p)
    return p, m, v
