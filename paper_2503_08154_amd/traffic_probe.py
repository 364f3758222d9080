"""Launches, a few times each and in this order, a plain device-to-device copy
of known size and the forward and backward kernels on one layer of a workload,
so that a hardware-counter run can compare their memory traffic:

    rocprofv3 --pmc FETCH_SIZE  -d <dir> -- python3 paper_2503_08154_amd/traffic_probe.py --workload vit_l16
    rocprofv3 --pmc WRITE_SIZE  -d <dir> -- python3 paper_2503_08154_amd/traffic_probe.py --workload vit_l16

The copy moves exactly n*e bytes in and n*e bytes out (e = element size), which
calibrates what the counter reports per byte.  Buffers are distinct per
repetition so that no launch finds its data in a cache.
"""
from __future__ import annotations

import argparse
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2503_08154_amd import s2a  # noqa: E402
from paper_2503_08154_amd import workloads as wl  # noqa: E402


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="vit_l16", choices=sorted(wl.WORKLOADS))
    ap.add_argument("--reps", type=int, default=4)
    args = ap.parse_args()
    import torch

    w = wl.WORKLOADS[args.workload]
    x, dy = wl.layer_inputs(w, 0, 0)
    n = x.shape[0]
    s2a.qtable_init(16)
    st = torch.cuda.current_stream().cuda_stream
    sets = []
    for _ in range(args.reps):
        tx = torch.from_numpy(x.view(np.uint8)).cuda()
        tdy = torch.from_numpy(dy.view(np.uint8)).cuda()
        sets.append((tx, torch.empty_like(tx), torch.empty((n + 1) // 2, dtype=torch.uint8, device="cuda"),
                     tdy, torch.empty_like(tdy)))
    torch.cuda.synchronize()
    for tx, ty, tc, tdy, tdx in sets:      # plain copy: n*e bytes read, n*e bytes written
        ty.copy_(tx)
    torch.cuda.synchronize()
    for tx, ty, tc, tdy, tdx in sets:
        s2a.act_fwd(tx.data_ptr(), ty.data_ptr(), tc.data_ptr(), n, w.dtype, st)
    torch.cuda.synchronize()
    for tx, ty, tc, tdy, tdx in sets:
        s2a.act_bwd(tdy.data_ptr(), tc.data_ptr(), tdx.data_ptr(), n, w.dtype, st)
    torch.cuda.synchronize()
    print(f"traffic_probe {w.name}: n={n} copy_bytes_in={x.nbytes} copy_bytes_out={x.nbytes} reps={args.reps}")


if __name__ == "__main__":
    main()
