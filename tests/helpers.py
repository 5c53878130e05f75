"""Shared plumbing of the GPU parity tests."""

import numpy as np

from oracle import block as OB
from paper_2308_15762_amd import hanayo as hn
from paper_2308_15762_amd import synth
from paper_2308_15762_amd.runner import GpuChunk, GpuRank, dev, dev_bytes, host  # noqa: F401

TOL = {"fp32": 1e-4, "bf16": 2e-2}


def nerr(got, ref):
    """max |got - ref| / max |ref|: the per-tensor normalised maximum error."""
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def rel_l2(got, ref):
    """||got - ref||_2 / ||ref||_2: sees a region of small entries that is wrong as a whole, which the
    maximum error normalised by the largest entry cannot."""
    ref = np.asarray(ref, dtype=np.float64).ravel()
    d = np.asarray(got, dtype=np.float64).ravel() - ref
    return float(np.sqrt(np.dot(d, d)) / max(np.sqrt(np.dot(ref, ref)), 1e-30))


def elem_err(got, ref):
    """Element-wise relative error with an absolute floor: max_i |got_i - ref_i| / (|ref_i| + rms(ref)).
    Every entry is judged at its own size, entries near zero at the tensor's typical size."""
    ref = np.asarray(ref, dtype=np.float64)
    d = np.abs(np.asarray(got, dtype=np.float64) - ref)
    floor = max(float(np.sqrt(np.mean(ref * ref))), 1e-30)
    return float((d / (np.abs(ref) + floor)).max())


def perr(got, ref):
    """The parity error the GPU tests hold against the tolerances: the larger of the normalised maximum
    error and the relative L2 error, so `perr <= tol` asserts both."""
    return max(nerr(got, ref), rel_l2(got, ref))


def oracle_cfg(wl):
    return OB.BlockCfg(wl.hidden, wl.heads, wl.ffn, norm=wl.norm, causal=wl.causal)


def compare_grads(got, ref, tol, label=""):
    worst = 0.0
    for bi, (g, r) in enumerate(zip(got, ref)):
        for name in hn.PARAM_NAMES:
            e = perr(g[name], r[name])
            worst = max(worst, e)
            assert e <= tol, "%s block %d %s: error %.3g (max-normalised %.3g, relative L2 %.3g) > %.3g" % (
                label, bi, name, e, nerr(g[name], r[name]), rel_l2(g[name], r[name]), tol)
            if tol <= 1e-4:   # fp32 storage: every entry at its own size as well
                ee = elem_err(g[name], r[name])
                assert ee <= tol, "%s block %d %s: element-wise error %.3g > %.3g" % (label, bi, name, ee, tol)
    return worst


def oracle_ends(wl, tied=True):
    """The `ends` argument of the oracle's rank walk for a workload (float64 copies of the seeded tables)."""
    p = synth.ends_params(wl)
    f = lambda a: np.asarray(a, dtype=np.float64)
    return {"wte": f(p["wte"]), "wpe": f(p["wpe"]), "head": None if tied else f(synth.untied_head(wl)),
            "lnf": None if p["lnf"] is None else (f(p["lnf"][0]), f(p["lnf"][1])),
            "tokens": lambda m: synth.token_ids(wl, m), "labels": lambda m: synth.labels(wl, m),
            "loss_scale": 1.0 / wl.M}


def oracle_rank(wl, rank, tasks, ends=None):
    """The oracle's execution of the same list on the same seeded inputs."""
    from oracle import executor as OE
    params = [synth.chunk_params(wl, c) for c in range(hn.chunks_per_rank(wl.W))]
    vl = (lambda m: synth.valid_lengths(wl, m)) if wl.valid_len_range is not None else None
    lst = [(int(t["kind"]), int(t["mb"]), int(t["chunk"]), int(t["stage"])) for t in tasks]
    return OE.run_rank(lst, wl.P, wl.W, rank, oracle_cfg(wl), params,
                       lambda m, c: synth.forward_input(wl, m, c), lambda m, c: synth.upstream_grad(wl, m, c), vl,
                       ends=ends if rank == 0 else None)
