"""Shared plumbing of the GPU parity tests: moves seeded host arrays to the
device, calls the library through its binding, brings results back."""

import numpy as np
import torch

from oracle import block as OB
from paper_2308_15762_amd import hanayo as hn
from paper_2308_15762_amd import synth

TOL = {"fp32": 1e-4, "bf16": 2e-2}


def nerr(got, ref):
    """max |got - ref| / max |ref|  (the normalised error the tolerances refer to)."""
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def dev(a, dtype):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.bfloat16() if dtype == "bf16" else t


def host(t):
    return t.float().cpu().numpy()


def dev_bytes(n):
    return torch.empty(int(n), dtype=torch.uint8, device="cuda")


def oracle_cfg(wl):
    return OB.BlockCfg(wl.hidden, wl.heads, wl.ffn, norm=wl.norm, causal=wl.causal)


class GpuChunk:
    """One chunk's device state: packed weights, fp32 grads, workspace."""

    def __init__(self, wl, params):
        self.wl = wl
        self.desc = hn.desc_for(wl)
        self.params = params
        self.weights = dev(hn.pack_params(self.desc, params), wl.dtype)
        assert self.weights.numel() * self.weights.element_size() <= hn.hanayo_weight_bytes(self.desc)
        self.grads = torch.zeros(hn.hanayo_grad_bytes(self.desc) // 4, dtype=torch.float32, device="cuda")
        self.work = dev_bytes(hn.hanayo_workspace_bytes(self.desc))

    def new_stash(self):
        return dev_bytes(hn.hanayo_stash_bytes(self.desc))

    def forward(self, x, valid_len=None, stash=None):
        wl = self.wl
        xd = dev(x, wl.dtype)
        y = torch.empty_like(xd)
        stash = self.new_stash() if stash is None else stash
        vl = None if valid_len is None else torch.from_numpy(np.asarray(valid_len, dtype=np.int32)).cuda()
        hn.hanayo_chunk_forward(self.desc, self.weights, xd, vl, y, stash, self.work)
        torch.cuda.synchronize()
        return host(y), (stash, vl)

    def backward(self, dy, stash):
        wl = self.wl
        st, vl = stash
        dyd = dev(dy, wl.dtype)
        dx = torch.empty_like(dyd)
        hn.hanayo_chunk_backward(self.desc, self.weights, self.grads, dyd, vl, st, dx, self.work)
        torch.cuda.synchronize()
        return host(dx)

    def grad_dicts(self):
        return hn.unpack_params(self.desc, self.grads.cpu().numpy(), self.params)


def compare_grads(got, ref, tol, label=""):
    worst = 0.0
    for bi, (g, r) in enumerate(zip(got, ref)):
        for name in hn.PARAM_NAMES:
            e = nerr(g[name], r[name])
            worst = max(worst, e)
            assert e <= tol, "%s block %d %s: normalised error %.3g > %.3g" % (label, bi, name, e, tol)
    return worst
