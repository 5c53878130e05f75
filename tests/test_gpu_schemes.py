"""GPU parity of the comparison schemes through the same executor: a GPipe and a 1F1B list (straight
placement, W = 0) through hanayo_executor_run against the oracle's walk of the oracle's own list, and all
P ranks' lists through hanayo_pipeline_run against the oracle's model without a pipeline.  Synchronous
schemes differ in time and memory only: results equal the non-pipelined model, stash peaks follow the
scheme (GPipe M everywhere, 1F1B P - rank)."""

import numpy as np
import pytest
import torch

from oracle import pipeline as OP
from oracle import schemes as SC
from paper_2308_15762_amd import hanayo as hn
from paper_2308_15762_amd import synth
from paper_2308_15762_amd.runner import GpuPipeline
from helpers import TOL, GpuRank, compare_grads, elem_err, host, perr, oracle_cfg, oracle_rank

pytestmark = pytest.mark.gpu

W = synth.WORKLOADS
SCHEME_ID = {"gpipe": hn.SCHEME_GPIPE, "1f1b": hn.SCHEME_1F1B, "chimera_wave": hn.SCHEME_CHIMERA_WAVE}

RANK_CASES = {
    # reduced GPT-like chunk (bf16, d = 64) on a straight 4-device pipeline, 6 micro-batches
    "gpt_small": W["gpt_1024_bf16"].scaled(hidden=128, heads=2, ffn=512, seq=128, mb=1, P=4, W=0, M=6),
    # the tiny fp32 configuration's chunk on 3 devices
    "tiny_fp32": W["tiny_gpt_fp32"].scaled(P=3, W=0, M=5),
    # BERT-like: post-LN, key padding, 2 blocks per stage
    "bert_small": W["bert_1024_bf16"].scaled(hidden=128, heads=2, ffn=512, seq=96, mb=2, n_blocks=2, P=4, W=0, M=5,
                                             valid_len_range=(48, 96)),
}


@pytest.mark.parametrize("lanes", [1, 3])
@pytest.mark.parametrize("scheme", ["gpipe", "1f1b"])
@pytest.mark.parametrize("name,rank", [("gpt_small", 0), ("gpt_small", 2), ("gpt_small", 3), ("tiny_fp32", 1),
                                       ("bert_small", 0)])
def test_straight_scheme_rank_list_matches_oracle(name, rank, scheme, lanes):
    wl = RANK_CASES[name]
    tol = TOL[wl.dtype]
    tasks = hn.hanayo_schedule_scheme(SCHEME_ID[scheme], wl.P, 0, wl.M, rank)
    want = [tuple(t) for t in SC.scheme_list(scheme, wl.P, 0, wl.M, rank)]
    assert [(int(t["kind"]), int(t["mb"]), int(t["chunk"]), int(t["stage"])) for t in tasks] == want
    gpu = GpuRank(wl, rank, tasks=tasks, lanes=lanes)
    peak = gpu.run()
    torch.cuda.synchronize()
    assert peak == hn.hanayo_stash_plan(tasks, 0)[0] == (wl.M if scheme == "gpipe" else min(wl.P - rank, wl.M))
    ref = oracle_rank(wl, rank, tasks)
    assert ref["peak"] == peak
    for (m, c), y in ref["act_out"].items():
        e = perr(host(gpu.act_out[m]), y)
        assert c == 0 and e <= tol, "act_out mb %d: %.3g" % (m, e)
    for (m, c), dx in ref["grad_out"].items():
        e = perr(host(gpu.grad_out[m]), dx)
        assert e <= tol, "grad_out mb %d: %.3g" % (m, e)
        if wl.dtype == "fp32":
            assert elem_err(host(gpu.grad_out[m]), dx) <= tol
    compare_grads(gpu.grad_dicts(0), ref["grads"][0], tol, "%s %s rank %d" % (name, scheme, rank))


@pytest.mark.parametrize("scheme", ["gpipe", "1f1b", "chimera_wave"])
def test_whole_pipeline_under_every_scheme_equals_the_model(scheme):
    """All P ranks' lists on one device with true dataflow: model outputs, input gradients and every stage's
    gradients against the oracle's non-pipelined model, and each rank's stash peak against the scheme's."""
    Wv = 1 if scheme == "chimera_wave" else 0
    wl = W["gpt_1024_bf16"].scaled(hidden=128, heads=2, ffn=512, seq=128, mb=1, n_blocks=1, P=4, W=Wv, M=6)
    S = hn.chunks_per_rank(Wv) * wl.P
    tol = TOL[wl.dtype] * max(1.0, (S * wl.n_blocks / 4.0) ** 0.5)      # depth rule of the pipeline tests
    lists = [hn.hanayo_schedule_scheme(SCHEME_ID[scheme], wl.P, Wv, wl.M, r) for r in range(wl.P)]
    gpu = GpuPipeline(wl, lists=lists)
    assert gpu.S == S
    peaks, _ = gpu.run(timing=True)
    torch.cuda.synchronize()
    if scheme == "gpipe":
        assert peaks == [wl.M] * wl.P
    elif scheme == "1f1b":
        assert peaks == [min(wl.P - r, wl.M) for r in range(wl.P)]
    params = [synth.stage_params(wl, s) for s in range(S)]
    xs = [synth.model_input(wl, m) for m in range(wl.M)]
    dys = [synth.loss_grad(wl, m) for m in range(wl.M)]
    ys, dxs, grads = OP.monolithic(oracle_cfg(wl), params, xs, dys, None)
    for m in range(wl.M):
        e = perr(host(gpu.act[m * S + S - 1]), ys[m])
        assert e <= tol, "output of micro-batch %d: %.3g" % (m, e)
        e = perr(host(gpu.grad[m * S]), dxs[m])
        assert e <= tol, "input gradient of micro-batch %d: %.3g" % (m, e)
    for s in range(S):
        compare_grads(gpu.grad_dicts(s), grads[s], tol, "%s stage %d" % (scheme, s))


def test_straight_placement_rejects_the_models_ends_on_a_split_rank_pair():
    wl = RANK_CASES["tiny_fp32"]
    tasks = hn.hanayo_schedule_scheme(hn.SCHEME_1F1B, wl.P, 0, wl.M, 0)
    gpu = GpuRank(wl, 0, tasks=tasks, ends=True)
    with pytest.raises(hn.HanayoError) as ei:
        gpu.run()
    assert ei.value.code == hn.EUNSUPPORTED
