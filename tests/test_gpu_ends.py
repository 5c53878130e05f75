"""GPU parity of the model's ends (embedding, head + loss) and the Adam step against the oracle,
through the C ABI, on seeded inputs: tiny fp32 shapes, bf16 shapes that span several GEMM tiles with a
ragged vocabulary, and the benchmark workload's head at its full size."""

import numpy as np
import pytest
import torch

from oracle import ends as OE
from paper_2308_15762_amd import hanayo as hn
from paper_2308_15762_amd import synth
from helpers import TOL, dev, dev_bytes, host, nerr

pytestmark = pytest.mark.gpu


def small(dtype, hidden, seq, mb, vocab, norm="pre"):
    base = synth.WORKLOADS["tiny_gpt_fp32" if dtype == "fp32" else "gpt_1024_bf16"]
    return base.scaled(hidden=hidden, heads=hidden // 64, ffn=4 * hidden, seq=seq, mb=mb, vocab=vocab, norm=norm,
                       causal=(norm == "pre"), n_blocks=1)


def ends_desc(wl, final_ln=None):
    return hn.EndsDesc(wl.vocab, wl.seq, int(wl.norm == "pre") if final_ln is None else int(final_ln))


CASES = [("fp32", 256, 37, 3, 512), ("fp32", 64, 5, 1, 8), ("bf16", 256, 100, 3, 1000), ("bf16", 1024, 128, 4, 2048)]


@pytest.mark.parametrize("dtype,hidden,seq,mb,vocab", CASES)
def test_embedding(dtype, hidden, seq, mb, vocab):
    wl = small(dtype, hidden, seq, mb, vocab)
    d, e = hn.desc_for(wl), ends_desc(wl)
    p = synth.ends_params(wl)
    tok = synth.token_ids(wl, 0)
    tok[0, 0] = tok[0, 1]                                              # at least one repeated token
    wte, wpe, tokd = dev(p["wte"], dtype), dev(p["wpe"], dtype), torch.from_numpy(tok).cuda()
    x = torch.empty((mb, seq, hidden), dtype=wte.dtype, device="cuda")
    hn.hanayo_embed_forward(d, e, wte, wpe, tokd, x)
    want = OE.embed_forward(p["wte"].astype(np.float64), p["wpe"].astype(np.float64), tok)
    assert nerr(host(x), want) <= (2.0 ** -23 if dtype == "fp32" else 2.0 ** -8)   # one rounding of the sum
    dx = synth.upstream_grad(wl, 0, 0)
    d_wte = torch.zeros((vocab, hidden), dtype=torch.float32, device="cuda")
    d_wpe = torch.zeros((seq, hidden), dtype=torch.float32, device="cuda")
    for _ in range(2):                                                  # gradients are added to
        hn.hanayo_embed_backward(d, e, tokd, dev(dx, dtype), d_wte, d_wpe)
    w_wte, w_wpe = OE.embed_backward(tok, dx.astype(np.float64), vocab, seq)
    assert nerr(host(d_wte), 2 * w_wte) <= 1e-6 and nerr(host(d_wpe), 2 * w_wpe) <= 1e-6


def test_embedding_ignores_tokens_outside_the_vocabulary():
    wl = small("fp32", 64, 6, 2, 16)
    d, e = hn.desc_for(wl), ends_desc(wl)
    p = synth.ends_params(wl)
    tok = synth.token_ids(wl, 0)
    tok[0, 2], tok[1, 5] = -3, 16
    wte, wpe, tokd = dev(p["wte"], "fp32"), dev(p["wpe"], "fp32"), torch.from_numpy(tok).cuda()
    x = torch.empty((2, 6, 64), dtype=torch.float32, device="cuda")
    hn.hanayo_embed_forward(d, e, wte, wpe, tokd, x)
    got = host(x)
    assert np.array_equal(got[0, 2], p["wpe"][2]) and np.array_equal(got[1, 5], p["wpe"][5])
    d_wte = torch.zeros((16, 64), dtype=torch.float32, device="cuda")
    d_wpe = torch.zeros((6, 64), dtype=torch.float32, device="cuda")
    dx = synth.upstream_grad(wl, 0, 0)
    hn.hanayo_embed_backward(d, e, tokd, dev(dx, "fp32"), d_wte, d_wpe)
    keep = (tok >= 0) & (tok < 16)
    w_wte, _ = OE.embed_backward(np.where(keep, tok, 0), dx.astype(np.float64) * keep[..., None], 16, 6)
    assert nerr(host(d_wte), w_wte) <= 1e-6


def run_head(wl, final_ln, labels, y, p, head, loss_scale):
    d, e = hn.desc_for(wl), ends_desc(wl, final_ln)
    dtype, H = wl.dtype, wl.hidden
    lnf = dev(np.concatenate(p["lnf"]), dtype) if final_ln else None
    d_lnf = torch.zeros(2 * H, dtype=torch.float32, device="cuda") if final_ln else None
    headd = dev(head, dtype)
    d_head = torch.zeros(head.shape, dtype=torch.float32, device="cuda")
    yd = dev(y, dtype)
    dy = torch.empty_like(yd)
    loss = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
    work = dev_bytes(hn.hanayo_head_workspace_bytes(d, e))
    hn.hanayo_head_loss(d, e, lnf, headd, yd, torch.from_numpy(labels).cuda(), loss_scale, loss, dy, d_lnf, d_head, work)
    torch.cuda.synchronize()
    return float(loss.item()), host(dy), host(d_head), (None if d_lnf is None else host(d_lnf))


def check_head(wl, final_ln, labels, loss_scale=0.125, y_scale=1.0):
    p = synth.ends_params(wl, ln_random=True)
    if final_ln and p["lnf"] is None:
        p["lnf"] = (np.ones(wl.hidden, np.float32), np.zeros(wl.hidden, np.float32))
    head = synth.untied_head(wl)
    y = synth.forward_input(wl, 0, 0) * np.float32(y_scale)
    loss, dy, d_head, d_lnf = run_head(wl, final_ln, labels, y, p, head, loss_scale)
    f = lambda a: a.astype(np.float64)
    w_loss, w_dy, w_dhead, w_dlnf = OE.head_loss(f(y), labels, f(head), (f(p["lnf"][0]), f(p["lnf"][1])) if final_ln else None,
                                                 1e-5, loss_scale)
    tol = TOL[wl.dtype]
    assert abs(loss - w_loss) <= tol * max(abs(w_loss), 1e-30), (loss, w_loss)
    assert nerr(dy, w_dy) <= tol and nerr(d_head, w_dhead) <= tol
    if final_ln:
        assert nerr(d_lnf[:wl.hidden], w_dlnf[0]) <= tol and nerr(d_lnf[wl.hidden:], w_dlnf[1]) <= tol
    return loss


@pytest.mark.parametrize("dtype,hidden,seq,mb,vocab", CASES)
@pytest.mark.parametrize("final_ln", [False, True])
def test_head_and_loss(dtype, hidden, seq, mb, vocab, final_ln):
    wl = small(dtype, hidden, seq, mb, vocab)
    labels = synth.labels(wl, 0)
    labels[0, 0] = vocab - 1                                            # the last column of the last tile
    check_head(wl, final_ln, labels)


def test_head_with_peaked_logits():
    """Activations scaled so that the logits spread over tens of units: the log-sum-exp must not overflow."""
    wl = small("fp32", 256, 16, 2, 512)
    check_head(wl, False, synth.labels(wl, 0), y_scale=100.0)


def test_head_with_no_counted_position():
    wl = small("bf16", 256, 16, 2, 512)
    p = synth.ends_params(wl)
    labels = np.full((2, 16), -1, dtype=np.int32)
    loss, dy, d_head, d_lnf = run_head(wl, True, labels, synth.forward_input(wl, 0, 0), p, p["wte"], 1.0)
    assert loss == 0.0 and not dy.any() and not d_head.any() and not d_lnf.any()


def test_masked_lm_labels_post_ln():
    wl = synth.WORKLOADS["bert_1024_bf16"].scaled(hidden=256, heads=4, ffn=1024, seq=64, mb=4, vocab=1024,
                                                   valid_len_range=(32, 64))
    labels = synth.labels(wl, 0)
    assert (labels >= 0).sum() > 0 and (labels < 0).sum() > labels.size // 2
    check_head(wl, False, labels)


def test_head_at_the_benchmark_size():
    """gpt_1024_bf16: 4096 tokens against the 50304-row table (tied head: the token table itself)."""
    wl = synth.WORKLOADS["gpt_1024_bf16"]
    p = synth.ends_params(wl)
    labels = synth.labels(wl, 0)
    y = synth.forward_input(wl, 0, 0)
    loss, dy, d_head, d_lnf = run_head(wl, True, labels, y, p, p["wte"], 1.0 / wl.M)
    f = lambda a: a.astype(np.float64)
    w_loss, w_dy, w_dhead, w_dlnf = OE.head_loss(f(y), labels, f(p["wte"]), (f(p["lnf"][0]), f(p["lnf"][1])), 1e-5, 1.0 / wl.M)
    tol = TOL["bf16"]
    assert abs(loss - w_loss) <= tol * w_loss
    assert nerr(dy, w_dy) <= tol and nerr(d_head, w_dhead) <= tol
    assert nerr(d_lnf[:wl.hidden], w_dlnf[0]) <= tol and nerr(d_lnf[wl.hidden:], w_dlnf[1]) <= tol


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_adam_steps(dtype):
    rng = synth.rng_for(77, 1)
    n = 4 * 1000 + 4                                                    # several workgroups and a ragged last one
    p0 = synth._finish(rng.normal(0, 0.02, size=n), dtype)
    params = dev(p0, dtype)
    master = torch.from_numpy(p0.copy()).cuda() if dtype == "bf16" else None
    m = torch.zeros(n, dtype=torch.float32, device="cuda")
    v = torch.zeros(n, dtype=torch.float32, device="cuda")
    wp, wm, wv = p0.astype(np.float64), np.zeros(n), np.zeros(n)
    for t in range(1, 5):
        g = rng.normal(0, 1e-3, size=n).astype(np.float32)
        grads = torch.from_numpy(g.copy()).cuda()
        adam = hn.Adam(2.0 ** -10, 0.875, 0.9375, 1e-8, 0.125, t, int(t % 2 == 0))                # exact in fp32
        hn.hanayo_adam_step(adam, hn.BF16 if dtype == "bf16" else hn.FP32, params, master, grads, m, v, n)
        wp, wm, wv = OE.adam_step(wp, g.astype(np.float64), wm, wv, t, 2.0 ** -10, 0.875, 0.9375, 1e-8, 0.125)
        got = host(master) if dtype == "bf16" else host(params)
        assert nerr(got, wp) <= 1e-6 and nerr(host(m), wm) <= 1e-6 and nerr(host(v), wv) <= 1e-6, t
        if dtype == "bf16":                                              # the stored parameter is the rounded master
            assert np.array_equal(host(params), synth.bf16_round(host(master)))
        assert (not host(grads).any()) == (t % 2 == 0)


def test_chunk_adam_decays_matrices_only():
    wl = synth.WORKLOADS["tiny_gpt_fp32"].scaled(n_blocks=2)
    d = hn.desc_for(wl)
    params = synth.chunk_params(wl, 0, ln_random=True)
    flat = hn.pack_params(d, params)
    rng = synth.rng_for(78, 1)
    g = rng.normal(0, 1e-3, size=flat.size).astype(np.float32)
    weights, grads = dev(flat, "fp32"), torch.from_numpy(g.copy()).cuda()
    m, v = torch.zeros_like(grads), torch.zeros_like(grads)
    hn.hanayo_chunk_adam_step(hn.Adam(2.0 ** -7, 0.875, 0.9375, 1e-8, 0.5, 1, 0), d, weights, None, grads, m, v)
    got = hn.unpack_params(d, host(weights), params)
    gd = hn.unpack_params(d, g, params)
    for blk in range(2):
        for name in hn.PARAM_NAMES:
            wd = 0.5 if name in ("wqkv", "wo", "w1", "w2") else 0.0
            z = np.zeros_like(params[blk][name], dtype=np.float64)
            want, _, _ = OE.adam_step(params[blk][name].astype(np.float64), gd[blk][name].astype(np.float64), z, z, 1,
                                      2.0 ** -7, 0.875, 0.9375, 1e-8, wd)
            assert nerr(got[blk][name], want) <= 1e-6, (blk, name)


def test_bad_arguments_are_rejected():
    wl = small("fp32", 64, 8, 1, 16)
    d = hn.desc_for(wl)
    buf = dev_bytes(1 << 16)
    for bad in (hn.EndsDesc(12, 8, 0), hn.EndsDesc(16, 4, 0), hn.EndsDesc(16, 8, 2)):
        with pytest.raises(hn.HanayoError):
            hn.hanayo_embed_forward(d, bad, buf, buf, buf, buf)
    with pytest.raises(hn.HanayoError):
        hn.hanayo_adam_step(hn.Adam(1e-3, 0.9, 0.999, 1e-8, 0.0, 0, 0), hn.FP32, buf, None, buf, buf, buf, 16)      # step 0
    with pytest.raises(hn.HanayoError):
        hn.hanayo_adam_step(hn.Adam(1e-3, 0.9, 0.999, 1e-8, 0.0, 1, 0), hn.BF16, buf, None, buf, buf, buf, 16)      # no master
    with pytest.raises(hn.HanayoError):
        hn.hanayo_adam_step(hn.Adam(1e-3, 0.9, 0.999, 1e-8, 0.0, 1, 0), hn.FP32, buf, None, buf, buf, buf, 18)      # count % 4
