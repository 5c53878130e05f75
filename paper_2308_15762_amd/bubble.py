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
    python -m paper_2308_15762_amd.bubble --figure [--t-c 0.1]               (host only, see figure_table)

Prints one JSON line.
"""

import argparse
import json
import sys

import numpy as np


def printed_ratio(P, W):
    """The paper's simplified bubble ratio for M = P micro-batches, T_B = 2 T_F, T_C = 0 (hanayo_bubble_model)."""
    from . import hanayo as hn
    return hn.hanayo_bubble_model(hn.SCHEME_HANAYO, P, W, P, 1.0, 2.0, 0.0)[0] if P > 1 else 0.0


def paper_ratio(P, W, t_f, t_b, t_c):
    """The paper's bubble-ratio equation (theoretical analysis section) with communication time, from
    hanayo_bubble_model: t_f and t_b are the forward and backward times of ONE micro-batch through all 2W
    chunks of a device (the paper's T_F and T_B), t_c one transfer."""
    from . import hanayo as hn
    return hn.hanayo_bubble_model(hn.SCHEME_HANAYO, P, W, P, t_f, t_b, t_c)[0]


def consistent_ratio(P, W):
    """The same equation's idle time (its numerator) over idle plus the rank's own compute, T_B = 2 T_F."""
    from . import hanayo as hn
    return hn.hanayo_bubble_model(hn.SCHEME_HANAYO, P, W, P, 1.0, 2.0, 0.0)[2]


def figure_table(t_c=0.0, prefetch=True):
    """The curves of the paper's bubble-ratio figure, host only: for each device count P (B = P micro-batches,
    T_B = 2 T_F, transfers t_c in units of T_F) the ratio of GPipe, 1F1B, Chimera-wave and Hanayo with 2, 4
    and 8 waves, from the model (hanayo_bubble_model) and, in brackets, from the library's schedules replayed
    by the interpreter simulation (hanayo_replay_actions).  Returns the table as a list of rows."""
    from . import hanayo as hn
    cols = [("GPipe", hn.SCHEME_GPIPE, 0), ("1F1B", hn.SCHEME_1F1B, 0), ("Chimera-wave", hn.SCHEME_CHIMERA_WAVE, 1),
            ("Hanayo W=2", hn.SCHEME_HANAYO, 2), ("Hanayo W=4", hn.SCHEME_HANAYO, 4), ("Hanayo W=8", hn.SCHEME_HANAYO, 8)]
    rows = []
    for P in (2, 4, 8, 16, 32):
        row = {"P": P}
        for name, scheme, W in cols:
            model = hn.hanayo_bubble_model(scheme, P, W, P, 1.0, 2.0, t_c)
            tasks = [hn.hanayo_schedule_scheme(scheme, P, W, P, r) for r in range(P)]
            acts = [hn.hanayo_actions_of(tasks[r], P, W, r) for r in range(P)]
            # a task of a wave scheme is 1/2W of the device's forward or backward time
            n = hn.chunks_per_rank(W)
            makespan, idle, _ = hn.hanayo_replay_actions(acts, P, W, P, 1.0 / n, 2.0 / n, t_c, prefetch)
            row[name] = (model[0], model[2], float(np.mean(idle) / makespan))
        rows.append(row)
    return rows


def print_figure(t_c, prefetch):
    rows = figure_table(t_c, prefetch)
    names = [k for k in rows[0] if k != "P"]
    print("bubble ratio at B = P, T_B = 2 T_F, T_C = %g T_F: equation as printed / idle form / schedule simulated%s"
          % (t_c, " with prefetch" if prefetch else ""))
    print("| P | " + " | ".join(names) + " |")
    print("|---|" + "---|" * len(names))
    for row in rows:
        print("| %d | " % row["P"] + " | ".join("%.3f / %.3f / %.3f" % row[k] for k in names) + " |")


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
    ap.add_argument("--figure", action="store_true",
                    help="host only: the bubble-ratio curves of every scheme (model and simulated schedules)")
    ap.add_argument("--t-c", type=float, default=0.0, help="--figure: transfer time in units of T_F")
    args = ap.parse_args()
    if args.figure:
        print_figure(args.t_c, True)
        return
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
