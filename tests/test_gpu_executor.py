"""GPU parity of hanayo_executor_run: one rank's whole ordered task list against
the oracle's execution of the same list (all boundary outputs, all accumulated
gradients, stash peak against the plan)."""

import numpy as np
import pytest
import torch

from oracle import schedule as OS
from paper_2308_15762_amd import hanayo as hn
from paper_2308_15762_amd import synth
from helpers import TOL, GpuRank, compare_grads, elem_err, host, perr, oracle_rank

pytestmark = pytest.mark.gpu

W = synth.WORKLOADS

CASES = {
    # BASELINE configuration 1 in full: rank 0 of P=2, W=1, M=4 (16 tasks), and its rank 1
    "tiny_gpt_fp32_rank0": (W["tiny_gpt_fp32"], 0),
    "tiny_gpt_fp32_rank1": (W["tiny_gpt_fp32"], 1),
    # the other configurations' schedules on reduced chunk shapes
    "gpt_1024_sched_small": (W["gpt_1024_bf16"].scaled(hidden=128, heads=2, ffn=512, seq=128, mb=1), 0),
    "bert_sched_small": (W["bert_1024_bf16"].scaled(hidden=128, heads=2, ffn=512, seq=96, mb=2, n_blocks=2,
                                                    valid_len_range=(48, 96)), 0),
    # configuration 4's schedule in full (P = 16, W = 2, M = 32: 256 tasks) on a reduced chunk shape
    "gpt_4096_sched_small": (W["gpt_4096_bf16"].scaled(hidden=128, heads=1, ffn=512, seq=64, mb=1), 0),
    # configuration 5's schedule on rank 0 (P = 8, W = 4: 8 chunks, first and last stage, three local turns)
    "wave4_sched_small_rank0": (W["gpt_2560_wave4_bf16"].scaled(hidden=64, heads=1, ffn=256, seq=64, mb=1, M=24), 0),
    "wave4_sched_small_rank3": (W["gpt_2560_wave4_bf16"].scaled(hidden=160, heads=2, ffn=640, seq=64, mb=1, M=10), 3),
    "wave4_sched_small_last_rank": (W["gpt_2560_wave4_bf16"].scaled(hidden=64, heads=1, ffn=256, seq=64, mb=1, M=9), 7),
}


_ORACLE = {}


def oracle_of(name, tasks):
    """The oracle's run of a case, computed once per session."""
    if name not in _ORACLE:
        wl, rank = CASES[name]
        _ORACLE[name] = oracle_rank(wl, rank, tasks)
    return _ORACLE[name]


@pytest.mark.parametrize("lanes", [1, 2, 3])
@pytest.mark.parametrize("name", list(CASES))
def test_rank_list_matches_oracle(name, lanes):
    wl, rank = CASES[name]
    tol = TOL[wl.dtype]
    gpu = GpuRank(wl, rank, lanes=lanes)
    plan_peak, per_chunk, _ = hn.hanayo_stash_plan(gpu.tasks, wl.W)
    peak = gpu.run()
    torch.cuda.synchronize()
    assert peak == plan_peak == OS.stash_plan(OS.schedule(wl.P, wl.W, wl.M, rank), wl.W)[0]
    ref = oracle_of(name, gpu.tasks)
    assert ref["peak"] == peak
    nchunk = 2 * wl.W
    worst = 0.0
    for (m, c), y in ref["act_out"].items():
        e = perr(host(gpu.act_out[m * nchunk + c]), y)
        worst = max(worst, e)
        assert e <= tol, "act_out mb %d chunk %d: %.3g" % (m, c, e)
    for (m, c), dx in ref["grad_out"].items():
        e = perr(host(gpu.grad_out[m * nchunk + c]), dx)
        worst = max(worst, e)
        assert e <= tol, "grad_out mb %d chunk %d: %.3g" % (m, c, e)
    if wl.dtype == "fp32":   # fp32 storage: every entry at its own size as well (absolute floor = the tensor's rms)
        for (m, c), y in ref["act_out"].items():
            assert elem_err(host(gpu.act_out[m * nchunk + c]), y) <= tol
        for (m, c), dx in ref["grad_out"].items():
            assert elem_err(host(gpu.grad_out[m * nchunk + c]), dx) <= tol
    for c in range(nchunk):
        compare_grads(gpu.grad_dicts(c), ref["grads"][c], tol, "%s chunk %d" % (name, c))


def test_second_run_after_zeroing_grads_is_identical_enough():
    wl, rank = CASES["gpt_1024_sched_small"]
    gpu = GpuRank(wl, rank)
    gpu.run()
    torch.cuda.synchronize()
    first = [g.clone() for g in gpu.grads]
    out_first = gpu.act_out[-1].clone()
    gpu.zero_grads()
    gpu.run()
    torch.cuda.synchronize()
    assert torch.equal(out_first, gpu.act_out[-1])
    for a, b in zip(first, gpu.grads):
        assert perr(b.cpu().numpy(), a.cpu().numpy()) <= 1e-5


@pytest.mark.parametrize("lanes", [1, 4])
def test_gradients_repeat_bit_for_bit(lanes):
    """No kernel of the path adds with atomics (weight gradients start from the sums so far, bias gradients and
    LayerNorm parameter gradients are reduced in a fixed order): two runs give identical bits everywhere."""
    wl, rank = CASES["gpt_1024_sched_small"]
    gpu = GpuRank(wl, rank, lanes=lanes)
    snaps = []
    for _ in range(2):
        gpu.zero_grads()
        gpu.run()
        torch.cuda.synchronize()
        snaps.append([g.clone() for g in gpu.grads] + [t.clone() for t in gpu.grad_out])
    for a, b in zip(*snaps):
        assert torch.equal(a, b)


@pytest.mark.parametrize("name", ["gpt_1024_sched_small", "wave4_sched_small_rank3"])
def test_lanes_do_not_change_results(name):
    """Boundary outputs are bit-identical whatever the lane count; gradients differ only by the
    order of the bias-gradient atomics."""
    wl, rank = CASES[name]
    runs = []
    for lanes in (1, 2, 4):
        gpu = GpuRank(wl, rank, lanes=lanes)
        for _ in range(2):  # the second run reuses events and side streams
            gpu.zero_grads()
            gpu.run()
        torch.cuda.synchronize()
        runs.append(gpu)
    for other in runs[1:]:
        for a, b in zip(runs[0].act_out + runs[0].grad_out, other.act_out + other.grad_out):
            assert torch.equal(a, b)
        for a, b in zip(runs[0].grads, other.grads):
            assert perr(b.cpu().numpy(), a.cpu().numpy()) <= 1e-5


@pytest.mark.parametrize("lanes", [1, 3])
@pytest.mark.parametrize("name", ["tiny_gpt_fp32_rank0", "gpt_1024_sched_small", "bert_sched_small"])
def test_input_only_stash_recomputes_to_the_same_result(name, lanes):
    """Stash mode "input": entries hold the chunk input only and every backward recomputes its forward.
    The boundary outputs are bit-identical to the full-stash run, the gradients equal up to the order of
    the bias-gradient atomics, and the arena is the plan's entry count times one activation tensor."""
    wl, rank = CASES[name]
    full = GpuRank(wl, rank, lanes=lanes)
    full.run()
    lean = GpuRank(wl, rank, lanes=lanes, stash_mode=hn.STASH_INPUT)
    peak = lean.run()
    torch.cuda.synchronize()
    assert peak == hn.hanayo_stash_plan(lean.tasks, wl.W)[0]
    per_chunk = hn.hanayo_stash_plan(lean.tasks, wl.W)[1]
    act = hn.hanayo_act_bytes(lean.desc)
    assert lean.arena_bytes == sum(per_chunk) * ((act + 255) // 256 * 256) < full.arena_bytes
    for a, b in zip(full.act_out + full.grad_out, lean.act_out + lean.grad_out):
        assert torch.equal(a, b)
    for a, b in zip(full.grads, lean.grads):
        assert perr(b.cpu().numpy(), a.cpu().numpy()) <= 1e-5
    ref = oracle_of(name, lean.tasks)
    for c in range(2 * wl.W):
        compare_grads(lean.grad_dicts(c), ref["grads"][c], TOL[wl.dtype], "%s chunk %d" % (name, c))


def test_input_only_stash_needs_its_scratch():
    wl, rank = CASES["gpt_1024_sched_small"]
    gpu = GpuRank(wl, rank, stash_mode=hn.STASH_INPUT)
    gpu.scratch = None
    with pytest.raises(hn.HanayoError) as e:
        gpu.run()
    assert e.value.code == hn.EINVAL
    gpu.stash_mode = 7
    with pytest.raises(hn.HanayoError) as e:
        gpu.run()
    assert e.value.code == hn.EINVAL


def test_executor_rejects_too_many_lanes():
    wl, rank = CASES["gpt_1024_sched_small"]
    gpu = GpuRank(wl, rank, lanes=4)
    gpu.lanes = 5
    with pytest.raises(hn.HanayoError) as e:
        gpu.run()
    assert e.value.code == hn.EINVAL


def test_executor_rejects_bad_lists_without_touching_outputs():
    wl, rank = CASES["tiny_gpt_fp32_rank0"]
    gpu = GpuRank(wl, rank)
    marker = 123.0
    for t in gpu.act_out + gpu.grad_out:
        t.fill_(marker)
    tasks = gpu.tasks.copy()
    b_first = np.argmax(tasks["kind"] == hn.B)
    swapped = tasks.copy()
    swapped[[0, b_first]] = swapped[[b_first, 0]]             # a backward before its forward
    dup = tasks.copy()
    dup[1] = dup[0]                                           # a task twice, another missing
    wrong_stage = tasks.copy()
    wrong_stage["stage"][0] += 1
    for bad in (swapped, dup, wrong_stage, tasks[:-1]):
        with pytest.raises(hn.HanayoError) as ei:
            gpu.run(bad)
        assert ei.value.code == hn.ESTATE
    torch.cuda.synchronize()
    assert all(bool((t == marker).all()) for t in gpu.act_out + gpu.grad_out)


def test_executor_rejects_small_arena_and_missing_buffers():
    wl, rank = CASES["tiny_gpt_fp32_rank0"]
    gpu = GpuRank(wl, rank)
    keep = gpu.arena_bytes
    gpu.arena_bytes = keep - 1
    with pytest.raises(hn.HanayoError) as ei:
        gpu.run()
    assert ei.value.code == hn.ESTATE
    gpu.arena_bytes = keep
    gpu.act_in[0] = None
    with pytest.raises(hn.HanayoError) as ei:
        gpu.run()
    assert ei.value.code == hn.EINVAL
