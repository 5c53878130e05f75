#!/usr/bin/env python3
"""Emulated bubble ratio of a wave pipeline from task times measured on one GPU.

All P ranks' task lists of a workload are executed on this GPU with true dataflow
(hanayo_pipeline_run), every task bracketed by HIP events; the measured durations are
then replayed as P devices would run them (hanayo_replay: each rank in its own order,
a task starts when its producer has finished, transfers take no time).  That is the
paper's bubble analysis with measured T_F and T_B instead of the assumed T_B = 2 T_F,
and T_C = 0.  Printed next to it: the same schedule under the assumed costs, and the
closed form the paper gives for one unit of P micro-batches.

    python -m paper_2308_15762_amd.bubble --workload gpt_1024_bf16 [--M 4] [--repeat 3]
    python -m paper_2308_15762_amd.bubble --links [--link-workgroups 2]      (see report_links)

Prints one JSON line.
"""

import argparse
import json
import sys

import numpy as np


def printed_ratio(P, W):
    """The paper's simplified bubble ratio for M = P micro-batches, T_B = 2 T_F, T_C = 0."""
    return (2.0 * P - 2.0) / (3.0 * P * W + P - 1.0)


def paper_ratio(P, W, t_f, t_b, t_c):
    """The paper's bubble-ratio equation (theoretical analysis section) with communication time: t_f and t_b are
    the forward and backward times of ONE micro-batch through all 2W chunks of a device (the paper's T_F and T_B),
    t_c one transfer.  With t_b = 2 t_f and t_c = 0 it reduces to printed_ratio."""
    num = t_b / W + (1.0 + 2.0 * W + 2.0 / P + (P - 2.0) / 3.0) * t_c
    den = P / (P - 1.0) * t_f + (1.0 / (2.0 * W) + P / (P - 1.0)) * t_b + ((P - 2.0) / 2.0 + 4.0 * W) * t_c
    return num / den


def consistent_ratio(P, W):
    """Idle (P - 1) T_B / W per rank (the numerator of the paper's bubble equation) over idle plus the
    rank's own compute P (T_F + T_B), with T_B = 2 T_F: the ratio that equation gives once numerator and
    denominator use the same idle time."""
    return (2.0 * P - 2.0) / (3.0 * P * W + 2.0 * P - 2.0)


def measure(wl, repeat=3, ends=False):
    """Task durations [rank][task] in ms: the median over `repeat` timed runs after one warm-up."""
    import torch
    from .runner import GpuPipeline
    gpu = GpuPipeline(wl, ends=ends)
    gpu.run()
    torch.cuda.synchronize()
    runs = []
    for _ in range(repeat):
        gpu.zero_grads()
        _, ms = gpu.run(timing=True)
        runs.append(ms)
    return gpu.lists, [np.median(np.stack([r[k] for r in runs]), axis=0) for k in range(wl.P)]


def report(wl, repeat=3, ends=False):
    """ends: the model starts from token ids and ends in head + loss, which lengthens rank 0's forward task of
    stage 0 (embedding), its forward task of the last stage (head forward and backward) and its backward task
    of stage 0 (embedding backward)."""
    from . import hanayo as hn
    P, W, M = wl.P, wl.W, wl.M
    lists, ms = measure(wl, repeat, ends)
    makespan, idle = hn.hanayo_replay(lists, P, W, M, ms)
    unit_makespan, unit_idle = hn.hanayo_replay(lists, P, W, M)
    f = np.concatenate([m[t["kind"] == 0] for m, t in zip(ms, lists)])
    b = np.concatenate([m[t["kind"] == 1] for m, t in zip(ms, lists)])
    out = {
        "workload": wl.name, "P": P, "W": W, "M": M, "stages": 2 * W * P, "model_ends": bool(ends),
        "t_f_ms": float(f.mean()), "t_b_ms": float(b.mean()), "t_b_over_t_f": float(b.mean() / f.mean()),
        "makespan_ms": makespan, "idle_ms_per_rank": [float(v) for v in idle],
        "bubble_ratio_measured_times": float(np.mean(idle) / makespan),
        "bubble_ratio_assumed_costs": float(np.mean(unit_idle) / unit_makespan),
        "bubble_ratio_paper_closed_form_M_eq_P": printed_ratio(P, W),
        "bubble_ratio_paper_equation_measured_times_M_eq_P": paper_ratio(P, W, 2 * W * float(f.mean()), 2 * W * float(b.mean()), 0.0)
        if P > 1 else None,
        "bubble_ratio_numerator_form_M_eq_P": consistent_ratio(P, W),
        "one_gpu_total_ms": float(sum(m.sum() for m in ms)),
    }
    if ends:
        last = [m[(t["kind"] == 0) & (t["stage"] == 2 * W * P - 1)] for m, t in zip(ms, lists)]
        out["t_f_last_stage_with_head_ms"] = float(np.concatenate(last).mean())
        out["busy_ms_per_rank"] = [float(m.sum()) for m in ms]
    return out


def report_links(wl, link_workgroups=0, repeat=3):
    """The pipeline run from action lists with every send / receive pair carried out as a device copy
    (link_workgroups workgroups: the emulated link).  Measures the transfers, the whole run on this
    one GPU with blocking receives against overlapped ones, and replays the measured compute times
    and transfer time through the interpreter simulation with and without the paper's prefetch."""
    import time
    import torch
    from . import hanayo as hn
    from .runner import GpuPipeline
    P, W, M = wl.P, wl.W, wl.M
    gpu = GpuPipeline(wl)
    gpu.enable_links()
    wall = {}
    for mode, async_copies in (("blocking", False), ("overlapped", True)):
        gpu.run_actions(async_copies=async_copies, link_workgroups=link_workgroups)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(repeat):
            gpu.run_actions(async_copies=async_copies, link_workgroups=link_workgroups)
        torch.cuda.synchronize()
        wall[mode] = (time.perf_counter() - t0) / repeat * 1e3
    _, ms_block = gpu.run_actions(async_copies=False, link_workgroups=link_workgroups, timing=True)
    _, ms = gpu.run_actions(async_copies=True, link_workgroups=link_workgroups, timing=True)
    recv = [(a["kind"] == hn.RECV_ACT) | (a["kind"] == hn.RECV_GRAD) for a in gpu.actions]
    t_c_alone = float(np.concatenate([m[r] for m, r in zip(ms_block, recv)]).mean())
    t_c_overlapped = float(np.concatenate([m[r] for m, r in zip(ms, recv)]).mean())
    # compute durations from the blocking run (nothing shares the chip with them there)
    out = {"workload": wl.name, "P": P, "W": W, "M": M, "link_workgroups": link_workgroups,
           "message_mib": wl.mb * wl.seq * wl.hidden * (2 if wl.dtype == "bf16" else 4) / 2 ** 20,
           "messages": int(sum(r.sum() for r in recv)),
           "t_c_ms_alone": t_c_alone, "t_c_ms_overlapped": t_c_overlapped,
           "one_gpu_ms_blocking_receives": wall["blocking"], "one_gpu_ms_overlapped_transfers": wall["overlapped"]}
    for name, pre in (("no_prefetch", False), ("prefetch", True)):
        makespan, idle, waited = hn.hanayo_replay_actions(gpu.actions, P, W, M, 0.0, 0.0, t_c_alone, pre, ms_block)
        out["makespan_ms_" + name] = makespan
        out["bubble_ratio_" + name] = float(np.mean(idle) / makespan)
        out["waited_ms_per_rank_" + name] = [float(v) for v in waited]
    makespan0, idle0, _ = hn.hanayo_replay_actions(gpu.actions, P, W, M, 0.0, 0.0, 0.0, False, ms_block)
    out["makespan_ms_t_c_zero"] = makespan0
    comp = [(a["kind"] == hn.F, a["kind"] == hn.B) for a in gpu.actions]
    t_f = float(np.concatenate([m[c[0]] for m, c in zip(ms_block, comp)]).mean())
    t_b = float(np.concatenate([m[c[1]] for m, c in zip(ms_block, comp)]).mean())
    if P > 1:  # the paper's own equation for M = P micro-batches, with the measured times
        out["bubble_ratio_paper_equation_M_eq_P"] = paper_ratio(P, W, 2 * W * t_f, 2 * W * t_b, t_c_alone)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="gpt_1024_bf16")
    ap.add_argument("--M", type=int, default=None, help="micro-batches (default: the workload's)")
    ap.add_argument("--repeat", type=int, default=3)
    ap.add_argument("--ends", action="store_true", help="embedding in front of stage 0, head + loss behind the last stage")
    ap.add_argument("--links", action="store_true", help="run from action lists with the transfers carried out")
    ap.add_argument("--link-workgroups", type=int, default=0, help="workgroups of a transfer's copy kernel (0 = unrestricted)")
    args = ap.parse_args()
    import torch
    from . import synth
    if not torch.cuda.is_available():
        sys.exit("bubble: no GPU")
    wl = synth.WORKLOADS[args.workload]
    if args.M is not None:
        wl = wl.scaled(M=args.M)
    print(json.dumps(report_links(wl, args.link_workgroups, args.repeat) if args.links else report(wl, args.repeat, args.ends)))


if __name__ == "__main__":
    main()
