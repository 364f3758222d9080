"""Launches, a few times each and in this order, a plain device-to-device copy
of known size and the forward and backward kernels on one layer of a workload,
so that a hardware-counter run can compare their memory traffic:

    rocprofv3 --pmc FETCH_SIZE  -d <dir> -- python3 paper_2503_08154_amd/traffic_probe.py --workload vit_l16
    rocprofv3 --pmc WRITE_SIZE  -d <dir> -- python3 paper_2503_08154_amd/traffic_probe.py --workload vit_l16

The copy moves exactly n*e bytes in and n*e bytes out (e = element size), which
calibrates what the counter reports per byte.  Buffers are distinct per
repetition so that no launch finds its data in a cache.

With --extras the rows beyond the headline path follow, each on fresh buffers:
measured-range forward, ReLU mask forward / backward, softmax forward /
backward at the ViT-B/16 attention shape (bf16), CAP and LRP forward /
backward at [64, 197, 768] bf16.
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
    ap.add_argument("--extras", action="store_true", help="also launch the kernels of the rows beyond the headline path")
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
    if args.extras:
        extras(torch, w, x, dy, sets, st, args.reps)


def extras(torch, w, x, dy, sets, st, reps):
    n = x.shape[0]
    qs = [torch.empty(s2a.QSTATE_FLOATS, dtype=torch.float32, device="cuda") for _ in sets]
    masks = [torch.empty((n + 7) // 8, dtype=torch.uint8, device="cuda") for _ in sets]
    torch.cuda.synchronize()
    for (tx, ty, tc, tdy, tdx), q in zip(sets, qs):
        s2a.act_fwd_dyn(tx.data_ptr(), ty.data_ptr(), tc.data_ptr(), q.data_ptr(), n, w.dtype, st)
    torch.cuda.synchronize()
    for (tx, ty, tc, tdy, tdx), m in zip(sets, masks):
        s2a.relu_fwd(tx.data_ptr(), ty.data_ptr(), m.data_ptr(), n, w.dtype, st)
    torch.cuda.synchronize()
    for (tx, ty, tc, tdy, tdx), m in zip(sets, masks):
        s2a.relu_bwd(tdy.data_ptr(), m.data_ptr(), tdx.data_ptr(), n, w.dtype, st)
    torch.cuda.synchronize()
    # softmax at the ViT-B/16 attention shape, bf16
    rows, L = 64 * 12 * 197, 197
    rb = (L + 1) // 2
    logits = wl.draw_x(rows * L, "normal", 2.0, wl.BF16, seed=11)
    grads = wl.draw_dy(rows * L, 1e-2, wl.BF16, seed=12)
    sm = []
    for _ in range(reps):
        tl = torch.from_numpy(logits.view(np.uint8)).cuda()
        tg = torch.from_numpy(grads.view(np.uint8)).cuda()
        sm.append((tl, torch.empty_like(tl), torch.empty(rows * rb, dtype=torch.uint8, device="cuda"),
                   torch.empty(2 * rows, dtype=torch.float32, device="cuda"), tg, torch.empty_like(tg)))
    torch.cuda.synchronize()
    for tl, ty, tc, tq, tg, tdx in sm:
        s2a.softmax_fwd(tl.data_ptr(), ty.data_ptr(), tc.data_ptr(), tq.data_ptr(), rows, L, wl.BF16, st)
    torch.cuda.synchronize()
    for tl, ty, tc, tq, tg, tdx in sm:
        s2a.softmax_bwd(tg.data_ptr(), tc.data_ptr(), tq.data_ptr(), tdx.data_ptr(), rows, L, wl.BF16, st)
    torch.cuda.synchronize()
    # CAP and LRP at [64, 197, 768] bf16
    batch, N, C, rank, r_cap = 64, 197, 768, 30, 8
    m = batch * N * C
    tok = wl.draw_x(m, "normal", 1.5, wl.BF16, seed=13)
    A = torch.randn(N, rank, device="cuda") * 0.1
    B = torch.randn(rank, C, device="cuda") * 0.1
    cl = []
    for _ in range(reps):
        tt = torch.from_numpy(tok.view(np.uint8)).cuda()
        cl.append((tt, torch.empty(m // r_cap * 2, dtype=torch.uint8, device="cuda"), torch.empty_like(tt),
                   torch.empty(N, rank, device="cuda"), torch.empty(rank, C, device="cuda"), torch.empty(N, C, device="cuda")))
    torch.cuda.synchronize()
    for tt, ty, tfull, dA, dB, work in cl:
        s2a.cap_fwd(tt.data_ptr(), ty.data_ptr(), m // r_cap, r_cap, wl.BF16, st)
    torch.cuda.synchronize()
    for tt, ty, tfull, dA, dB, work in cl:
        s2a.cap_bwd(ty.data_ptr(), tfull.data_ptr(), m // r_cap, r_cap, wl.BF16, st)
    torch.cuda.synchronize()
    for tt, ty, tfull, dA, dB, work in cl:
        s2a.lrp_fwd(tt.data_ptr(), tfull.data_ptr(), A.data_ptr(), B.data_ptr(), batch, N, C, rank, wl.BF16, st)
    torch.cuda.synchronize()
    for tt, ty, tfull, dA, dB, work in cl:
        s2a.lrp_bwd(tt.data_ptr(), A.data_ptr(), B.data_ptr(), dA.data_ptr(), dB.data_ptr(), work.data_ptr(),
                    batch, N, C, rank, wl.BF16, st)
    torch.cuda.synchronize()
    print(f"traffic_probe extras: softmax rows={rows} L={L}; cap/lrp [{batch},{N},{C}] r={r_cap} rank={rank}")


if __name__ == "__main__":
    main()
