#!/usr/bin/env python3
"""What a plain device copy reaches at a given tensor size: the yardstick for the memory-bound kernels.

The LayerNorm kernels of the benchmark workload move 8 to 32 MiB per launch; at those sizes a launch is
over before the memory system is saturated, so the published HBM peak is not the right denominator for
them.  This prints the time and rate of the library's copy kernel (hanayo_op_copy) for several sizes,
rotating over enough buffer pairs (1 GiB) that nothing stays resident in the caches.

    python -m paper_2308_15762_amd.copybench [--mib 4 8 16 32 64 256]
"""

import argparse
import sys


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, nargs="+", default=[4, 8, 16, 32, 64, 256], help="MiB read (and as many written)")
    args = ap.parse_args()
    import torch
    from . import hanayo as hn
    if not torch.cuda.is_available():
        sys.exit("copybench: no GPU")
    for mib in args.mib:
        n = mib << 20
        pairs = max(2, (1024 << 20) // (2 * n))
        bufs = [(torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255),
                 torch.empty(n, dtype=torch.uint8, device="cuda")) for _ in range(pairs)]
        for a, b in bufs:
            hn.hanayo_op_copy(b, a, n)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        count = 0
        e0.record()
        for _ in range(4):
            for a, b in bufs:
                hn.hanayo_op_copy(b, a, n)
                count += 1
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / count
        print("copy_kernel %4d MiB read + %4d MiB written (%3d buffer pairs in rotation): %8.2f us  %7.1f GB/s"
              % (mib, mib, pairs, us, 2 * n / us / 1e3), flush=True)
        del bufs


if __name__ == "__main__":
    main()
