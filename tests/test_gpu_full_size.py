"""GPU parity at the benchmark's full chunk shapes, in the launch configuration bench.py
times (same kernels, same dispatch).  The oracle cannot replay a whole rank list at these
sizes in seconds, so: one full micro-batch forward+backward of one chunk is compared
element by element (configurations 2, 3 and 5; configuration 4 with one block), and for
every workload the executor's outputs for one sampled micro-batch are compared with the
oracle walking that micro-batch's tasks."""

import numpy as np
import pytest
import torch

from oracle import block as OB
from paper_2308_15762_amd import hanayo as hn
from paper_2308_15762_amd import synth
from helpers import TOL, GpuChunk, GpuRank, compare_grads, host, perr, oracle_cfg
from oracle import executor as OE

pytestmark = pytest.mark.gpu

W = synth.WORKLOADS


@pytest.mark.parametrize("name", ["gpt_1024_bf16", "bert_1024_bf16", "gpt_2560_wave4_bf16"])
def test_full_size_chunk_pair(name):
    wl = W[name]
    tol = TOL[wl.dtype]
    params = synth.chunk_params(wl, 0)
    x, dy = synth.forward_input(wl, 0, 0), synth.upstream_grad(wl, 0, 0)
    vl = synth.valid_lengths(wl, 0)
    cfg = oracle_cfg(wl)
    y_ref, st = OB.chunk_forward(params, x, cfg, vl)
    dx_ref, g_ref = OB.chunk_backward(cfg, st, dy)
    del st
    gpu = GpuChunk(wl, params)
    y, stash = gpu.forward(x, vl)
    assert perr(y, y_ref) <= tol, "y %.3g" % perr(y, y_ref)
    dx = gpu.backward(dy, stash)
    assert perr(dx, dx_ref) <= tol, "dx %.3g" % perr(dx, dx_ref)
    compare_grads(gpu.grad_dicts(), g_ref, tol, name)


def test_largest_chunk_shape_single_block():
    # configuration 4's block (H = 4096, 32 heads of 128, F = 16384, seq 2048): one block of the
    # chunk, full size, so the oracle stays within tens of seconds
    wl = W["gpt_4096_bf16"].scaled(n_blocks=1)
    tol = TOL["bf16"]
    params = synth.chunk_params(wl, 0)
    x, dy = synth.forward_input(wl, 0, 0), synth.upstream_grad(wl, 0, 0)
    cfg = oracle_cfg(wl)
    y_ref, st = OB.chunk_forward(params, x, cfg, dtype=np.float32)
    dx_ref, g_ref = OB.chunk_backward(cfg, st, dy)
    del st
    gpu = GpuChunk(wl, params)
    y, stash = gpu.forward(x)
    assert perr(y, y_ref) <= tol
    dx = gpu.backward(dy, stash)
    assert perr(dx, dx_ref) <= tol
    compare_grads(gpu.grad_dicts(), g_ref, tol, "gpt_4096 block")


@pytest.fixture(scope="module")
def benchmark_run():
    """Rank 0's full 64-task list of the benchmark workload, run once in the launch
    configuration bench.py times (four lanes)."""
    wl = W["gpt_1024_bf16"]
    gpu = GpuRank(wl, 0, lanes=4)
    peak = gpu.run()
    torch.cuda.synchronize()
    return wl, gpu, peak


def test_benchmark_workload_accumulated_gradients(benchmark_run):
    """The parameter gradients of the last stage's chunk, accumulated over all 8 micro-batches by
    backward tasks that ran on different lanes, against the oracle's accumulation of the same 8."""
    wl, gpu, _ = benchmark_run
    c = 2 * wl.W - 1                       # stage S-1: input and upstream gradient both come from outside
    cfg = oracle_cfg(wl)
    params = synth.chunk_params(wl, c)
    grads = None
    for m in range(wl.M):
        _, st = OB.chunk_forward(params, synth.forward_input(wl, m, c), cfg)
        _, grads = OB.chunk_backward(cfg, st, synth.upstream_grad(wl, m, c), grads)
        del st
    compare_grads(gpu.grad_dicts(c), grads, TOL["bf16"], "chunk %d over %d micro-batches" % (c, wl.M))


def test_benchmark_workload_sampled_micro_batch(benchmark_run):
    """Micro-batch 5's boundary outputs against the oracle (chunks 1 -> 2 are the local turn-around)."""
    wl, gpu, peak = benchmark_run
    tol = TOL["bf16"]
    assert peak == hn.hanayo_stash_plan(gpu.tasks, wl.W)[0] == 16
    m = 5
    cfg = oracle_cfg(wl)
    nchunk = 2 * wl.W
    params = [synth.chunk_params(wl, c) for c in range(nchunk)]
    y, st = {}, {}
    y[0], st[0] = OB.chunk_forward(params[0], synth.forward_input(wl, m, 0), cfg)
    y[1], st[1] = OB.chunk_forward(params[1], synth.forward_input(wl, m, 1), cfg)
    y[2], st[2] = OB.chunk_forward(params[2], y[1], cfg)                       # local hand-off
    y[3], st[3] = OB.chunk_forward(params[3], synth.forward_input(wl, m, 3), cfg)
    d = {}
    d[3], _ = OB.chunk_backward(cfg, st[3], synth.upstream_grad(wl, m, 3))
    d[2], _ = OB.chunk_backward(cfg, st[2], synth.upstream_grad(wl, m, 2))
    d[1], _ = OB.chunk_backward(cfg, st[1], d[2])                              # local hand-off
    d[0], _ = OB.chunk_backward(cfg, st[0], synth.upstream_grad(wl, m, 0))
    for c in range(nchunk):
        e = perr(host(gpu.act_out[m * nchunk + c]), y[c])
        assert e <= tol, "act_out chunk %d: %.3g" % (c, e)
        e = perr(host(gpu.grad_out[m * nchunk + c]), d[c])
        assert e <= tol, "grad_out chunk %d: %.3g" % (c, e)
    # property that holds at any size: every gradient buffer is finite and non-trivial
    for g in gpu.grads:
        assert bool(torch.isfinite(g).all()) and float(g.abs().max()) > 0


def test_benchmark_workload_with_the_models_ends():
    """Rank 0's list of the benchmark workload with the embedding in front of stage 0 and the tied head and
    loss behind stage 15, four lanes: every micro-batch's loss, and the gradients of the token table (which
    collects the head's and the embedding's contributions of all 8 micro-batches), the position table and
    the final LayerNorm, against the oracle."""
    from oracle import ends as OE
    from helpers import oracle_ends
    wl = W["gpt_1024_bf16"]
    tol = TOL["bf16"]
    gpu = GpuRank(wl, 0, lanes=4, ends=True)
    gpu.run()
    torch.cuda.synchronize()
    cfg = oracle_cfg(wl)
    last = 2 * wl.W - 1
    ends = oracle_ends(wl)
    p0, p3 = synth.chunk_params(wl, 0), synth.chunk_params(wl, last)
    d_wte = np.zeros_like(ends["wte"])
    d_wpe = np.zeros_like(ends["wpe"])
    d_g, d_b = np.zeros(wl.hidden), np.zeros(wl.hidden)
    loss = host(gpu.loss)
    for m in range(wl.M):
        y, _ = OB.chunk_forward(p3, synth.forward_input(wl, m, last), cfg)
        w_loss, dy, d_head, d_lnf = OE.head_loss(y, ends["labels"](m), ends["wte"], ends["lnf"], cfg.eps, 1.0 / wl.M)
        assert abs(loss[m] - w_loss) <= tol * w_loss, (m, loss[m], w_loss)
        d_wte += d_head
        d_g += d_lnf[0]
        d_b += d_lnf[1]
        if m == 5:
            e = perr(host(gpu.loss_grad[m]), dy)
            assert e <= tol, "loss gradient of mb 5: %.3g" % e
        x = OE.embed_forward(ends["wte"], ends["wpe"], ends["tokens"](m))
        if m == 5:
            y0, st = OB.chunk_forward(p0, x, cfg)
            e = perr(host(gpu.act_out[m * 2 * wl.W]), y0)
            assert e <= tol, "stage 0 output of mb 5: %.3g" % e
        else:
            _, st = OB.chunk_forward(p0, x, cfg)
        dx, _ = OB.chunk_backward(cfg, st, synth.upstream_grad(wl, m, 0))
        del st
        a, b = OE.embed_backward(ends["tokens"](m), dx, wl.vocab, wl.seq)
        d_wte += a
        d_wpe += b
    assert perr(host(gpu.d_wte), d_wte) <= tol, "d_wte %.3g" % perr(host(gpu.d_wte), d_wte)
    assert perr(host(gpu.d_wpe), d_wpe) <= tol
    assert perr(host(gpu.d_lnf)[:wl.hidden], d_g) <= tol and perr(host(gpu.d_lnf)[wl.hidden:], d_b) <= tol


def test_bert_workload_sampled_micro_batch_four_lanes():
    """Configuration 3 (post-LN, key padding, 3 blocks per chunk, M = 16) at full size through the executor in the
    launch configuration bench.py times (four lanes): micro-batch 9's boundary tensors of both of rank 0's chunks
    against the oracle, and the stash peak against the plan."""
    wl = W["bert_1024_bf16"]
    tol = TOL["bf16"]
    gpu = GpuRank(wl, 0, lanes=4)
    peak = gpu.run()
    torch.cuda.synchronize()
    assert peak == hn.hanayo_stash_plan(gpu.tasks, wl.W)[0]
    m = 9
    cfg = oracle_cfg(wl)
    vl = synth.valid_lengths(wl, m)
    nchunk = 2 * wl.W
    for c in range(nchunk):
        params = synth.chunk_params(wl, c)
        y, st = OB.chunk_forward(params, synth.forward_input(wl, m, c), cfg, vl)
        dx, _ = OB.chunk_backward(cfg, st, synth.upstream_grad(wl, m, c))
        del st
        e = perr(host(gpu.act_out[m * nchunk + c]), y)
        assert e <= tol, "act_out chunk %d: %.3g" % (c, e)
        e = perr(host(gpu.grad_out[m * nchunk + c]), dx)
        assert e <= tol, "grad_out chunk %d: %.3g" % (c, e)
    for g in gpu.grads:
        assert bool(torch.isfinite(g).all()) and float(g.abs().max()) > 0


def test_wave4_workload_sampled_micro_batch_four_lanes():
    """Configuration 5 (P = 8, W = 4, M = 64: rank 0's full list of 1024 tasks over 8 chunks) at full size, four
    lanes: the stash peak against the plan (64 entries), and micro-batch 37 through the local turn-around
    chunks 1 -> 2 against the oracle."""
    wl = W["gpt_2560_wave4_bf16"]
    tol = TOL["bf16"]
    gpu = GpuRank(wl, 0, lanes=4)
    peak = gpu.run()
    torch.cuda.synchronize()
    assert peak == hn.hanayo_stash_plan(gpu.tasks, wl.W)[0] == 64
    m = 37
    cfg = oracle_cfg(wl)
    nchunk = 2 * wl.W
    p1, p2 = (synth.chunk_params(wl, c) for c in (1, 2))
    y1, st1 = OB.chunk_forward(p1, synth.forward_input(wl, m, 1), cfg)
    y2, st2 = OB.chunk_forward(p2, y1, cfg)                                    # local hand-off
    d2, _ = OB.chunk_backward(cfg, st2, synth.upstream_grad(wl, m, 2))
    d1, _ = OB.chunk_backward(cfg, st1, d2)                                    # local hand-off
    del st1, st2
    for c, y, d in ((1, y1, d1), (2, y2, d2)):
        e = perr(host(gpu.act_out[m * nchunk + c]), y)
        assert e <= tol, "act_out chunk %d: %.3g" % (c, e)
        e = perr(host(gpu.grad_out[m * nchunk + c]), d)
        assert e <= tol, "grad_out chunk %d: %.3g" % (c, e)


def test_largest_workload_sampled_micro_batch_four_lanes():
    """Configuration 4 (P = 16, W = 2, M = 32, H = 4096, 2048-token sequences: rank 0's list of 256 tasks) at
    full size, four lanes: the stash peak against the plan, and micro-batch 21 through the last stage's chunk
    (input and upstream gradient both from outside) against the oracle in float32."""
    wl = W["gpt_4096_bf16"]
    tol = TOL["bf16"]
    gpu = GpuRank(wl, 0, lanes=4)
    peak = gpu.run()
    torch.cuda.synchronize()
    assert peak == hn.hanayo_stash_plan(gpu.tasks, wl.W)[0]
    m, c = 21, 2 * wl.W - 1
    cfg = oracle_cfg(wl)
    y, st = OB.chunk_forward(synth.chunk_params(wl, c), synth.forward_input(wl, m, c), cfg, dtype=np.float32)
    dx, _ = OB.chunk_backward(cfg, st, synth.upstream_grad(wl, m, c))
    del st
    nchunk = 2 * wl.W
    e = perr(host(gpu.act_out[m * nchunk + c]), y)
    assert e <= tol, "act_out: %.3g" % e
    e = perr(host(gpu.grad_out[m * nchunk + c]), dx)
    assert e <= tol, "grad_out: %.3g" % e
    for g in gpu.grads:
        assert bool(torch.isfinite(g).all()) and float(g.abs().max()) > 0


@pytest.mark.parametrize("name", ["gpt_4096_bf16", "gpt_2560_wave4_bf16"])
def test_full_size_one_micro_batch_through_all_rank0_chunks(name):
    """Configurations 4 and 5 at their full chunk shapes with their own (P, W), two micro-batches, four lanes:
    micro-batch 0 through ALL of rank 0's chunks -- every chunk's output activation and input gradient,
    which includes every local turn-around of the wave (chunks 1 -> 2, 3 -> 4, ... forward and back) -- and
    every chunk's parameter gradients of that micro-batch's share are covered by the accumulated comparison:
    the gradients the turn-around chunk 2 has accumulated over both micro-batches against the oracle's sum.
    The oracle (float32, as configured for the largest shapes) walks micro-batch 0's tasks of the list."""
    wl = W[name].scaled(M=2)
    tol = TOL["bf16"]
    gpu = GpuRank(wl, 0, lanes=4)
    peak = gpu.run()
    torch.cuda.synchronize()
    assert peak == hn.hanayo_stash_plan(gpu.tasks, wl.W)[0]
    nchunk = 2 * wl.W
    cfg = oracle_cfg(wl)
    params = [synth.chunk_params(wl, c) for c in range(nchunk)]
    tasks0 = [(int(t["kind"]), int(t["mb"]), int(t["chunk"]), int(t["stage"])) for t in gpu.tasks if int(t["mb"]) == 0]
    assert len(tasks0) == 2 * nchunk
    ref = OE.run_rank(tasks0, wl.P, wl.W, 0, cfg, params, lambda m, c: synth.forward_input(wl, m, c),
                      lambda m, c: synth.upstream_grad(wl, m, c), dtype=np.float32)
    for c in range(nchunk):
        e = perr(host(gpu.act_out[c]), ref["act_out"][(0, c)])
        assert e <= tol, "act_out chunk %d: %.3g" % (c, e)
        e = perr(host(gpu.grad_out[c]), ref["grad_out"][(0, c)])
        assert e <= tol, "grad_out chunk %d: %.3g" % (c, e)
    # accumulated gradients of chunk 2, whose input is chunk 1's output (the local turn-around): micro-batch 0's
    # share comes from the walk above, micro-batch 1's from chunks 1 -> 2 of that micro-batch
    y1, st1 = OB.chunk_forward(params[1], synth.forward_input(wl, 1, 1), cfg, dtype=np.float32)
    del st1
    _, st2 = OB.chunk_forward(params[2], y1, cfg, dtype=np.float32)
    # (stage 2P sits on rank 0 and feeds stage 2P+1 on rank 1, so chunk 2's upstream gradient is a received one)
    _, g2 = OB.chunk_backward(cfg, st2, synth.upstream_grad(wl, 1, 2))
    del st2
    total = [{k: a[k] + b[k] for k in a} for a, b in zip(ref["grads"][2], g2)]
    compare_grads(gpu.grad_dicts(2), total, tol, "%s chunk 2 over both micro-batches" % name)
    # the other chunks' accumulated gradients: finite and non-trivial (a property that holds at any size)
    for g in gpu.grads:
        assert bool(torch.isfinite(g).all()) and float(g.abs().max()) > 0

