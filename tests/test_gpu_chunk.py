"""GPU parity: hanayo_chunk_forward / hanayo_chunk_backward against the fp64 oracle,
element by element on the same seeded inputs.  Tolerances (normalised max error):
1e-4 for fp32 storage, 2e-2 for bf16 storage with fp32 accumulation."""

import numpy as np
import pytest

from oracle import block as OB
from paper_2308_15762_amd import synth
from helpers import TOL, GpuChunk, compare_grads, perr, oracle_cfg

pytestmark = pytest.mark.gpu

W = synth.WORKLOADS

CASES = {
    # the smallest BASELINE configuration at its full size
    "tiny_gpt_fp32": W["tiny_gpt_fp32"],
    # reduced copies of the others: several tiles plus ragged tails in T, H, F and seq
    "gpt_bf16_small": W["gpt_1024_bf16"].scaled(hidden=256, heads=4, ffn=1024, seq=192, mb=2),
    "gpt_bf16_ragged": W["gpt_1024_bf16"].scaled(hidden=192, heads=3, ffn=328, seq=100, mb=3, n_blocks=2),
    "bert_bf16_small": W["bert_1024_bf16"].scaled(hidden=256, heads=4, ffn=1024, seq=160, mb=3, n_blocks=2,
                                                  valid_len_range=(70, 160)),
    "bert_fp32_small": W["bert_1024_bf16"].scaled(dtype="fp32", hidden=128, heads=2, ffn=512, seq=96, mb=2,
                                                  n_blocks=2, valid_len_range=(40, 96)),
    "gpt_bf16_d128": W["gpt_4096_bf16"].scaled(hidden=512, heads=4, ffn=2048, seq=256, mb=1, n_blocks=1),
    "gpt_bf16_d80": W["gpt_2560_wave4_bf16"].scaled(hidden=320, heads=4, ffn=1280, seq=128, mb=2),
    "gpt_fp32_ragged": W["tiny_gpt_fp32"].scaled(hidden=72, heads=3, ffn=200, seq=37, mb=2, n_blocks=2),
}


@pytest.mark.parametrize("name", list(CASES))
def test_chunk_forward_backward_matches_oracle(name):
    wl = CASES[name]
    tol = TOL[wl.dtype]
    params = synth.chunk_params(wl, 0, ln_random=True)
    x = synth.forward_input(wl, 0, 0)
    dy = synth.upstream_grad(wl, 0, 0)
    vl = synth.valid_lengths(wl, 0)
    cfg = oracle_cfg(wl)
    y_ref, stash_ref = OB.chunk_forward(params, x, cfg, vl)
    dx_ref, g_ref = OB.chunk_backward(cfg, stash_ref, dy)

    gpu = GpuChunk(wl, params)
    y, stash = gpu.forward(x, vl)
    assert np.isfinite(y).all()
    assert perr(y, y_ref) <= tol, "y: %.3g" % perr(y, y_ref)
    dx = gpu.backward(dy, stash)
    assert np.isfinite(dx).all()
    assert perr(dx, dx_ref) <= tol, "dx: %.3g" % perr(dx, dx_ref)
    compare_grads(gpu.grad_dicts(), g_ref, tol, name)


def test_grads_accumulate_across_micro_batches():
    wl = CASES["gpt_bf16_small"]
    params = synth.chunk_params(wl, 1)
    cfg = oracle_cfg(wl)
    gpu = GpuChunk(wl, params)
    acc = None
    for m in range(3):
        x, dy = synth.forward_input(wl, m, 1), synth.upstream_grad(wl, m, 1)
        _, st_ref = OB.chunk_forward(params, x, cfg)
        _, g = OB.chunk_backward(cfg, st_ref, dy)
        acc = g if acc is None else [{k: a[k] + b[k] for k in a} for a, b in zip(acc, g)]
        _, st = gpu.forward(x)
        gpu.backward(dy, st)
    compare_grads(gpu.grad_dicts(), acc, TOL["bf16"], "accumulate")


def test_forward_does_not_modify_inputs_and_stash_survives_other_forwards():
    wl = CASES["bert_bf16_small"]
    params = synth.chunk_params(wl, 0)
    cfg = oracle_cfg(wl)
    gpu = GpuChunk(wl, params)
    x0, x1 = synth.forward_input(wl, 0, 0), synth.forward_input(wl, 1, 0)
    vl0, vl1 = synth.valid_lengths(wl, 0), synth.valid_lengths(wl, 1)
    dy0 = synth.upstream_grad(wl, 0, 0)
    _, st0 = gpu.forward(x0, vl0)
    gpu.forward(x1, vl1)                      # another micro-batch in flight
    dx = gpu.backward(dy0, st0)
    _, st_ref = OB.chunk_forward(params, x0, cfg, vl0)
    dx_ref, _ = OB.chunk_backward(cfg, st_ref, dy0)
    assert perr(dx, dx_ref) <= TOL["bf16"]
