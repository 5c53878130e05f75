"""Shared plumbing of the GPU parity tests."""

import numpy as np

from oracle import block as OB
from paper_2308_15762_amd import hanayo as hn
from paper_2308_15762_amd import synth
from paper_2308_15762_amd.runner import GpuChunk, GpuRank, dev, dev_bytes, host  # noqa: F401

TOL = {"fp32": 1e-4, "bf16": 2e-2}


def nerr(got, ref):
    """max |got - ref| / max |ref|  (the normalised error the tolerances refer to)."""
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def oracle_cfg(wl):
    return OB.BlockCfg(wl.hidden, wl.heads, wl.ffn, norm=wl.norm, causal=wl.causal)


def compare_grads(got, ref, tol, label=""):
    worst = 0.0
    for bi, (g, r) in enumerate(zip(got, ref)):
        for name in hn.PARAM_NAMES:
            e = nerr(g[name], r[name])
            worst = max(worst, e)
            assert e <= tol, "%s block %d %s: normalised error %.3g > %.3g" % (label, bi, name, e, tol)
    return worst


def oracle_rank(wl, rank, tasks):
    """The oracle's execution of the same list on the same seeded inputs."""
    from oracle import executor as OE
    params = [synth.chunk_params(wl, c) for c in range(2 * wl.W)]
    vl = (lambda m: synth.valid_lengths(wl, m)) if wl.valid_len_range is not None else None
    lst = [(int(t["kind"]), int(t["mb"]), int(t["chunk"]), int(t["stage"])) for t in tasks]
    return OE.run_rank(lst, wl.P, wl.W, rank, oracle_cfg(wl), params,
                       lambda m, c: synth.forward_input(wl, m, c), lambda m, c: synth.upstream_grad(wl, m, c), vl)
