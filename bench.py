#!/usr/bin/env python3
"""Benchmark of the 4-bit GELU activation path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]
    python bench.py --probe [--workload NAME] [--extras]      (launches for counter runs, no timing)

A step is one pass of the whole hot path over one batch of synthetic
activations: the forward kernel over every layer (launch) of the workload,
then the backward kernel over the same layers in reverse, all enqueued on one
stream with no host synchronisation in between.  Every layer has its own
x / y / codes / dy / dx buffers, so each launch streams cold HBM (the working
set is several GB, far beyond the 256 MB on-die cache).  Inputs are resident
in HBM before the timed region starts.

The default workload is the ViT-L/16 MLP hidden layer, 24 layers back to back:
the largest per-step configuration, and one of the two shapes the bandwidth
target is stated on.  The other one (ViT-G/14, bf16 and fp32) and the remaining
configurations follow in `target_shapes`, each kernel with its own roofline
block; the rows beyond the headline path follow in `next_rows`.

Prints ONE JSON line.  `value` is algorithmic bytes moved per second, fwd+bwd:
(2*e + 0.5) bytes per element and direction, e = element size.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2503_08154_amd import s2a  # noqa: E402
from paper_2503_08154_amd import workloads as wl  # noqa: E402

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, vendor figure
METRIC = "GB/s and % of HBM peak for 4-bit GELU fwd+bwd (elements/s), 1xMI355X"

# HBM bytes per launch as the memory-side counters saw them (rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE, each scaled by what the same counter reads for a plain copy of known size) are
# measured offline -- a counter run cannot share a process with the timed region -- and kept as
# text summaries under profiles/.  They are read from those files at run time, so the JSON line
# and the committed evidence cannot drift apart.
TRAFFIC_FILES = ("profiles/fwd_bwd_kernels_hbm_traffic_pmc.txt", "profiles/other_rows_hbm_traffic_pmc.txt")


def load_traffic(root: str = ROOT):
    """{(row, kernel): bytes per launch} from the `traffic | row | kernel | read | written | algorithmic`
    lines of the counter summaries.  Missing files or rows simply give no entry (reported as null)."""
    table = {}
    for rel in TRAFFIC_FILES:
        path = os.path.join(root, rel)
        if not os.path.exists(path):
            continue
        for line in open(path):
            m = re.match(r"\s*traffic\s*\|\s*(\S+)\s*\|\s*(\S+)\s*\|\s*([\d,]+)\s*\|\s*([\d,]+)\s*\|\s*([\d,]+)", line)
            if m:
                rd, wr, alg = (int(m.group(k).replace(",", "")) for k in (3, 4, 5))
                table[(m.group(1), m.group(2))] = {"bytes": rd + wr, "read": rd, "written": wr, "algorithmic": alg,
                                                   "source": rel}
    return table


def esize(dtype: int) -> int:
    return 4 if dtype == wl.F32 else 2


def dname(dtype: int) -> str:
    return "bf16" if dtype == wl.BF16 else "f32"


def bytes_per_direction(n: int, dtype: int) -> float:
    return (2 * esize(dtype) + 0.5) * n


class Layer:
    """Device buffers of one launch (torch is used only to own memory)."""

    def __init__(self, torch, x: np.ndarray, dy: np.ndarray, dtype: int):
        self.n = int(x.shape[0])
        self.dtype = dtype
        self.x = torch.from_numpy(x.view(np.uint8)).cuda()
        self.dy = torch.from_numpy(dy.view(np.uint8)).cuda()
        self.y = torch.empty_like(self.x)
        self.dx = torch.empty_like(self.dy)
        self.codes = torch.empty((self.n + 1) // 2, dtype=torch.uint8, device="cuda")
        self.qstate = torch.empty(s2a.QSTATE_FLOATS, dtype=torch.float32, device="cuda")
        self.p = tuple(t.data_ptr() for t in (self.x, self.y, self.codes, self.dy, self.dx, self.qstate))
        # the ReLU mask (n/8 bytes) fits in the codes buffer (n/2 bytes)


def build_layers(torch, w: wl.Workload, distinct_seeds: bool):
    """One Layer per (layer, stage) of the workload, in forward order."""
    jobs = [(l, s) for l in range(w.layers) for s in range(len(w.shapes))]
    if distinct_seeds:
        with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
            host = list(ex.map(lambda j: wl.layer_inputs(w, j[0], j[1]), jobs))
    else:  # timing does not depend on the values: draw each stage once, reuse per layer
        per_stage = [wl.layer_inputs(w, 0, s) for s in range(len(w.shapes))]
        host = [per_stage[s] for (_, s) in jobs]
    return [Layer(torch, x, dy, w.dtype) for (x, dy) in host]


FWD = {"gelu": lambda L, st: s2a.act_fwd(L.p[0], L.p[1], L.p[2], L.n, L.dtype, st),
       "gelu_dyn": lambda L, st: s2a.act_fwd_dyn(L.p[0], L.p[1], L.p[2], L.p[5], L.n, L.dtype, st),
       "gelu_in_place": lambda L, st: s2a.act_fwd(L.p[0], L.p[0], L.p[2], L.n, L.dtype, st),
       "silu": lambda L, st: s2a.silu_fwd(L.p[0], L.p[1], L.p[2], L.n, L.dtype, st),
       "relu": lambda L, st: s2a.relu_fwd(L.p[0], L.p[1], L.p[2], L.n, L.dtype, st)}
BWD = {"gelu": lambda L, st: s2a.act_bwd(L.p[3], L.p[2], L.p[4], L.n, L.dtype, st),
       "gelu_dyn": lambda L, st: s2a.act_bwd_dyn(L.p[3], L.p[2], L.p[5], L.p[4], L.n, L.dtype, st),
       "gelu_in_place": lambda L, st: s2a.act_bwd(L.p[3], L.p[2], L.p[3], L.n, L.dtype, st),
       "silu": lambda L, st: s2a.silu_bwd(L.p[3], L.p[2], L.p[4], L.n, L.dtype, st),
       "relu": lambda L, st: s2a.relu_bwd(L.p[3], L.p[2], L.p[4], L.n, L.dtype, st)}


def run_step(layers, stream: int, ev=None, variant: str = "gelu"):
    """fwd over all layers, then bwd in reverse; optional (e0, e1, e2) events around the phases (e0
    may be None: the phase then starts at the event that ended the step before)."""
    fwd, bwd = FWD[variant], BWD[variant]
    if ev and ev[0] is not None:
        ev[0].record()
    for L in layers:
        fwd(L, stream)
    if ev:
        ev[1].record()
    for L in reversed(layers):
        bwd(L, stream)
    if ev:
        ev[2].record()


def time_workload(torch, w: wl.Workload, steps: int, warmup: int, distinct_seeds: bool, variant: str = "gelu"):
    layers = build_layers(torch, w, distinct_seeds)
    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(warmup):
        run_step(layers, stream, variant=variant)
    # the same steps once with nothing but the path's own launches on the stream: what the events
    # of the timed region cost (a record takes about 3 us on the stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        run_step(layers, stream, variant=variant)
    torch.cuda.synchronize()
    wall_plain = time.perf_counter() - t0
    # the timed region: exactly `steps` steps between two synchronisations, with an event after each
    # phase (the forward phase of a step starts at the event that ended the step before)
    events = [[None if k else torch.cuda.Event(enable_timing=True)] +
              [torch.cuda.Event(enable_timing=True) for _ in range(2)] for k in range(steps)]
    t1 = time.perf_counter()
    for k in range(steps):
        run_step(layers, stream, events[k], variant=variant)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t1
    for k in range(1, steps):
        events[k][0] = events[k - 1][2]
    fwd_steps = [e[0].elapsed_time(e[1]) for e in events]
    bwd_steps = [e[1].elapsed_time(e[2]) for e in events]
    fwd_ms, bwd_ms = sum(fwd_steps), sum(bwd_steps)
    launches = steps * len(layers)
    n_total = sum(L.n for L in layers)
    bytes_dir = sum(bytes_per_direction(L.n, L.dtype) for L in layers)
    res = {
        "ms_per_step": wall * 1e3 / steps,
        "ms_per_step_without_events": wall_plain * 1e3 / steps,
        "elements_per_step": n_total,
        "bytes_per_step": 2 * bytes_dir,
        "launches_per_phase": len(layers),
        "fwd_us_per_launch": fwd_ms * 1e3 / launches,
        "bwd_us_per_launch": bwd_ms * 1e3 / launches,
        "fwd_gbs": bytes_dir * steps / (fwd_ms * 1e-3) / 1e9,
        "bwd_gbs": bytes_dir * steps / (bwd_ms * 1e-3) / 1e9,
        "bytes_per_launch": bytes_dir / len(layers),
        # per launch, from the per-step phase times (a phase is one launch per layer)
        "fwd_us_median": float(np.median(fwd_steps)) * 1e3 / len(layers),
        "fwd_us_min": min(fwd_steps) * 1e3 / len(layers),
        "bwd_us_median": float(np.median(bwd_steps)) * 1e3 / len(layers),
        "bwd_us_min": min(bwd_steps) * 1e3 / len(layers),
    }
    del layers
    torch.cuda.empty_cache()
    return res


def time_tiny(torch, steps: int, warmup: int):
    """The smallest configuration over 64 buffer sets: the interval between launches enqueued one by
    one, and the same 128 launches captured once in a HIP graph and replayed (the launch-bound case
    that graphs are for; the entry points enqueue kernels only, so they can be captured)."""
    tw = wl.WORKLOADS["tiny"]
    tw = wl.Workload(tw.name, tw.index, tw.dtype, tw.shapes, 64, tw.dist, tw.scale, tw.dy_scale)
    layers = build_layers(torch, tw, False)
    launches = 2 * len(layers)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for _ in range(warmup):
            run_step(layers, side.cuda_stream)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run_step(layers, torch.cuda.current_stream().cuda_stream)
    stream = torch.cuda.current_stream().cuda_stream

    def wall(step):
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    eager = wall(lambda: run_step(layers, stream))
    replay = wall(graph.replay)
    res = {
        "workload": "tiny: f32 2x197x768, fwd then bwd over 64 buffer sets", "bound": "launch",
        "bytes_per_launch": int(bytes_per_direction(layers[0].n, layers[0].dtype)),
        "us_per_launch": round(eager * 1e6 / launches, 2),
        "us_per_launch_graph_replay": round(replay * 1e6 / launches, 2),
    }
    del graph, layers
    torch.cuda.empty_cache()
    return res


def time_copy_ceilings(torch, n: int, dtype: int, sets: int, steps: int, warmup: int):
    """Math-free kernels with the launch shape, the memory instructions and the traffic of the two
    activation kernels (s2a_stream_copy_shaped): the forward shape reads 16 bytes per lane and writes
    16 bytes plus the lane's share of the packed codes, the backward shape reads both and writes 16
    bytes.  They are timed in the sequence of a step -- a phase of forward-shaped launches over `sets`
    buffer sets, then a phase of backward-shaped ones in reverse -- because the rate of a phase depends
    on what ran before it: the first ten or so write-heavy launches after a read-heavy phase run 4 %
    faster than the same launches in an unbroken series (the chip's power management; an idle gap
    does not have the effect), and a ceiling measured in an unbroken series sits below the kernel
    it is meant to bound."""
    nbytes = n * esize(dtype) // 16 * 16
    side = 4 if dtype == wl.BF16 else 2
    bufs = [tuple(torch.empty(k, dtype=torch.uint8, device="cuda").fill_(v) for k, v in
                  ((nbytes, 0x3C), (nbytes, 0), (nbytes // 16 * side, 0x5A), (nbytes, 0x3C), (nbytes, 0)))
            for _ in range(sets)]
    P = [tuple(t.data_ptr() for t in b) for b in bufs]  # x, y, codes, dy, dx
    stream = torch.cuda.current_stream().cuda_stream

    def step(ev=None):
        if ev:
            ev[0].record()
        for p in P:
            s2a.stream_copy_shaped(p[0], p[1], p[2], nbytes, side, 0, stream)
        if ev:
            ev[1].record()
        for p in reversed(P):
            s2a.stream_copy_shaped(p[3], p[4], p[2], nbytes, side, 1, stream)
        if ev:
            ev[2].record()

    for _ in range(warmup):
        step()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    torch.cuda.synchronize()
    for k in range(steps):
        step(events[k])
    torch.cuda.synchronize()
    moved = 2 * nbytes + nbytes // 16 * side
    out = {}
    for shape, a, b in (("fwd", 0, 1), ("bwd", 1, 2)):
        us = sum(e[a].elapsed_time(e[b]) for e in events) * 1e3 / (steps * sets)
        gbs = moved / us / 1e3
        out[shape] = {"kernel": f"s2a::stream_copy_shaped_kernel<{side}, {'true' if shape == 'bwd' else 'false'}>",
                      "bytes_per_launch": moved, "us_per_launch": round(us, 2), "gbs": round(gbs, 1),
                      "frac": round(gbs / HBM_PEAK_GBS, 4), "buffer_sets": sets,
                      "sequence": "forward-shaped phase then backward-shaped phase, as in a step"}
    del bufs
    torch.cuda.empty_cache()
    return out


def kernel_block(res, w: wl.Workload, which: str, traffic, ceiling=None):
    """Roofline entry of one of the two kernels of a timed workload."""
    achieved = res[f"{which}_gbs"]
    kname = f"s2a::{which}_kernel<{dname(w.dtype)}>"
    tr = traffic.get((w.name, kname))
    out = {
        "kernel": kname,
        "bound": "hbm",
        "achieved": round(achieved, 1),
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4),
        "traffic": tr["bytes"] if tr else None,
        "traffic_source": (tr["source"] + " (offline counter run)") if tr else None,
        "us_per_launch": round(res[f"{which}_us_per_launch"], 2),
        "us_per_launch_median": round(res[f"{which}_us_median"], 2),
        "us_per_launch_min": round(res[f"{which}_us_min"], 2),
        "algorithmic_bytes_per_launch": res["bytes_per_launch"],
    }
    if ceiling is not None:
        out["copy_ceiling"] = ceiling
        out["frac_of_copy_ceiling"] = round(achieved / ceiling["gbs"], 4)
    return out


def roofline_of(res, w: wl.Workload, traffic, ceilings=None):
    """Roofline entry of the slower of the two kernels, the other one inside it."""
    which = "fwd" if res["fwd_us_per_launch"] >= res["bwd_us_per_launch"] else "bwd"
    other = "bwd" if which == "fwd" else "fwd"
    ceilings = ceilings or {}
    out = kernel_block(res, w, which, traffic, ceilings.get(which))
    out["other_kernel"] = kernel_block(res, w, other, traffic, ceilings.get(other))
    return out


# ---------------------------------------------------------------- rows beyond the headline path ----

WARM_MS = 40.0  # the rows beyond the headline path warm up by time: see time_ops


def time_ops(torch, ops, sets: int, steps: int, warmup: int):
    """ops: {name: fn(set_index)}; each timed alone over `sets` buffer sets, `steps` times, after
    `warmup` passes over the sets and at least WARM_MS of the same launches: the clocks take tens of
    milliseconds to settle after an idle period, and the kernels with real arithmetic (softmax: 26.5 us
    after 2 ms of warm-up, 23.5 us after 50 ms or 300 ms) show it far more than the streaming ones."""
    out = {}
    for name, fn in ops.items():
        t0 = time.perf_counter()
        k = 0
        while k < warmup or (time.perf_counter() - t0) * 1e3 < WARM_MS:
            for i in range(sets):
                fn(i)
            torch.cuda.synchronize()
            k += 1
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(steps):
            for i in range(sets):
                fn(i)
        e1.record()
        torch.cuda.synchronize()
        out[name] = e0.elapsed_time(e1) * 1e3 / (steps * sets)
    return out


def row_block(kernel: str, us: float, nbytes: float, traffic, row: str, note: str | None = None):
    tr = traffic.get((row, kernel.replace(" ", "")))  # several kernels of one call: their sum, under the joined name
    blk = {"kernel": kernel, "bound": "hbm", "us_per_launch": round(us, 2), "achieved": round(nbytes / us / 1e3, 1),
           "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4),
           "algorithmic_bytes_per_launch": int(nbytes),
           "traffic": tr["bytes"] if tr else None}
    if tr:
        blk["traffic_source"] = tr["source"] + " (offline counter run)"
    if note:
        blk["note"] = note
    return blk


def sets_for(nbytes: float, lo: int = 8, hi: int = 64) -> int:
    """Buffer sets so that at least ~2 GB go by between two uses of a buffer."""
    return int(min(hi, max(lo, 2e9 // max(nbytes, 1) + 1)))


def softmax_row(torch, row: str, rows: int, L: int, dtype: int, steps: int, warmup: int, traffic):
    """Softmax with 4-bit y on distinct buffer sets of [rows, L] logits (N(0, 2^2))."""
    n = rows * L
    rb = (L + 1) // 2
    g = np.random.Generator(np.random.Philox(wl.layer_seed(wl.WORKLOADS["vit_b16"], 0, 0) + 7))
    x = wl.to_storage(g.standard_normal(n) * 2.0, dtype)
    dy = wl.draw_dy(n, 1e-2, dtype, 4711)
    nbytes = 2 * esize(dtype) * n + rows * rb + 8 * rows
    sets = sets_for(nbytes, hi=16)
    bufs = []
    for _ in range(sets):
        tx = torch.from_numpy(x.view(np.uint8)).cuda()
        tdy = torch.from_numpy(dy.view(np.uint8)).cuda()
        bufs.append((tx, torch.empty_like(tx), torch.empty(rows * rb, dtype=torch.uint8, device="cuda"),
                     torch.empty(2 * rows, dtype=torch.float32, device="cuda"), tdy, torch.empty_like(tdy)))
    ptrs = [tuple(t.data_ptr() for t in b) for b in bufs]
    st = torch.cuda.current_stream().cuda_stream
    ops = {"fwd": lambda i: s2a.softmax_fwd(ptrs[i][0], ptrs[i][1], ptrs[i][2], ptrs[i][3], rows, L, dtype, st),
           "bwd": lambda i: s2a.softmax_bwd(ptrs[i][4], ptrs[i][2], ptrs[i][3], ptrs[i][5], rows, L, dtype, st)}
    us = time_ops(torch, ops, sets, steps, warmup)
    del bufs
    torch.cuda.empty_cache()
    return {"shape": f"[{rows}, {L}] {dname(dtype)}", "buffer_sets": sets,
            "fwd": row_block(f"s2a::softmax_fwd_staged<{dname(dtype)}>", us["fwd"], nbytes, traffic, row),
            "bwd": row_block(f"s2a::softmax_bwd_staged<{dname(dtype)}>", us["bwd"], nbytes, traffic, row)}


LRP_RANK = 30          # the rank of the Low-Rank Prompt rows; Sec. 4.3 scales it up to 100
LRP_RANK_SCALED = 100


def cap_lrp_row(torch, row: str, batch: int, N: int, C: int, steps: int, warmup: int, traffic, note=None,
                rank: int = LRP_RANK, lrp_only: bool = False):
    """Channel Average Pooling (r = 8) and Low-Rank Prompt on [batch, N, C] bf16 tokens."""
    r_cap = 8
    n = batch * N * C
    x = wl.draw_x(n, "normal", 1.5, wl.BF16, 31)
    dy = wl.draw_dy(n, 1e-2, wl.BF16, 32)
    g = np.random.Generator(np.random.Philox(33))
    A = torch.from_numpy((g.standard_normal((N, rank)) * 0.1).astype(np.float32)).cuda()
    B = torch.from_numpy((g.standard_normal((rank, C)) * 0.1).astype(np.float32)).cuda()
    sets = sets_for(4 * n, hi=48)
    bufs = []
    for _ in range(sets):
        tx = torch.from_numpy(x.view(np.uint8)).cuda()
        tdy = torch.from_numpy(dy.view(np.uint8)).cuda()
        bufs.append(dict(x=tx, y=torch.empty_like(tx), dy=tdy, dx=torch.empty_like(tdy),
                         pooled=torch.empty(n // r_cap * 2, dtype=torch.uint8, device="cuda"),
                         dpooled=tdy[: n // r_cap * 2].clone(),
                         dA=torch.empty(N, rank, device="cuda"), dB=torch.empty(rank, C, device="cuda"),
                         work=torch.empty(N, C, device="cuda")))
    st = torch.cuda.current_stream().cuda_stream
    P = [{k: v.data_ptr() for k, v in b.items()} for b in bufs]
    ops = {
        "cap_fwd": lambda i: s2a.cap_fwd(P[i]["x"], P[i]["pooled"], n // r_cap, r_cap, wl.BF16, st),
        "cap_bwd": lambda i: s2a.cap_bwd(P[i]["dpooled"], P[i]["dx"], n // r_cap, r_cap, wl.BF16, st),
        "lrp_fwd": lambda i: s2a.lrp_fwd(P[i]["x"], P[i]["y"], A.data_ptr(), B.data_ptr(), batch, N, C, rank, wl.BF16, st),
        "lrp_bwd": lambda i: s2a.lrp_bwd(P[i]["dy"], A.data_ptr(), B.data_ptr(), P[i]["dA"], P[i]["dB"], P[i]["work"],
                                         batch, N, C, rank, wl.BF16, st),
    }
    nbytes = {"cap_fwd": 2 * n + 2 * n // r_cap, "cap_bwd": 2 * n + 2 * n // r_cap, "lrp_fwd": 4 * n,
              "lrp_bwd": 2 * n + 4 * (2 * N * C + 2 * (N * rank + rank * C))}
    kernels = {"cap_fwd": "s2a::cap_fwd_kernel<bf16, 8>", "cap_bwd": "s2a::cap_bwd_kernel<bf16, 8>",
               "lrp_fwd": "s2a::lrp_fwd_kernel<bf16>", "lrp_bwd": "s2a::lrp_batch_sum_kernel<bf16> + s2a::lrp_grad_ab_kernel"}
    if lrp_only:
        ops = {k: v for k, v in ops.items() if k.startswith("lrp")}
    us = time_ops(torch, ops, sets, steps, warmup)
    del bufs
    torch.cuda.empty_cache()
    out = {"shape": f"[{batch}, {N}, {C}] bf16, " + ("" if lrp_only else f"CAP r={r_cap}, ") + f"LRP rank {rank}",
           "buffer_sets": sets}
    for k in ops:
        out[k] = row_block(kernels[k], us[k], nbytes[k], traffic, row, note)
    return out


def variant_row(torch, name: str, variant: str, steps: int, warmup: int, traffic, bytes_per_elem_fwd=None,
                w_override=None, row_key=None):
    """One of the element-wise variants (measured range, SiLU, ReLU mask) on a workload's layers."""
    tw = w_override or wl.WORKLOADS[name]
    if tw.layers == 1:
        tw = wl.Workload(tw.name, tw.index, tw.dtype, tw.shapes, 8, tw.dist, tw.scale, tw.dy_scale)
    r = time_workload(torch, tw, steps, warmup, distinct_seeds=False, variant=variant)
    n1 = tw.sizes()[0]
    e = esize(tw.dtype)
    side = 0.125 if variant == "relu" else 0.5
    fwd_bytes = (bytes_per_elem_fwd if bytes_per_elem_fwd is not None else 2 * e + side) * n1
    bwd_bytes = (2 * e + side) * n1
    dt = dname(tw.dtype)
    kn = {"gelu_dyn": (f"s2a::range_minmax_kernel<{dt}> + s2a::fwd_dyn_kernel<{dt}>", f"s2a::bwd_kernel<{dt}, dyn>"),
          "gelu_in_place": (f"s2a::fwd_kernel<{dt}>", f"s2a::bwd_kernel<{dt}>"),
          "silu": (f"s2a::fwd_kernel<{dt}, silu>", f"s2a::bwd_kernel<{dt}>"),
          "relu": (f"s2a::relu_fwd_kernel<{dt}>", f"s2a::relu_bwd_kernel<{dt}>")}[variant]
    return {"workload": name, "buffer_sets": tw.layers,
            "fwd": row_block(kn[0], r["fwd_us_per_launch"], fwd_bytes, traffic, row_key or f"{name}:{variant}"),
            "bwd": row_block(kn[1], r["bwd_us_per_launch"], bwd_bytes, traffic, row_key or f"{name}:{variant}")}


def cpu_baseline(w: wl.Workload, target_cpu_seconds: float = 12.0):
    """The CPU oracle, as it stands, over one layer of the workload, chunked over the host cores."""
    import oracle  # test infrastructure; used here only as the reported CPU baseline

    try:
        avail = len(os.sched_getaffinity(0))
    except AttributeError:
        avail = os.cpu_count() or 1
    # the GPU machines give one GPU's job a 16-core share whatever the machine shows, and set
    # OMP_NUM_THREADS to it: the oracle's chunks follow that setting
    share = int(os.environ.get("OMP_NUM_THREADS", "16"))
    cores = max(1, min(avail, share))
    x, dy = wl.layer_inputs(w, 0, 0)
    n = x.shape[0]
    edges = [(n * i // cores) & ~1 for i in range(cores)] + [n]  # even starts: no shared code byte
    oracle.table()  # load the library outside the timed region

    def work(i):
        a, b = edges[i], edges[i + 1]
        _, _, packed, _ = oracle.fwd(x[a:b], w.dtype, want_near=False)
        oracle.bwd(dy[a:b], w.dtype, packed)

    reps, cpu_seconds, wall = 0, 0.0, 0.0
    with ThreadPoolExecutor(max_workers=cores) as ex:
        while cpu_seconds < target_cpu_seconds and reps < 8:
            t0 = time.perf_counter()
            list(ex.map(work, range(cores)))
            dt = time.perf_counter() - t0
            wall += dt
            cpu_seconds += dt * cores
            reps += 1
    moved = 2 * bytes_per_direction(n, w.dtype) * reps
    # the same layer once on one core (the oracle is scalar code: no threads of its own)
    t0 = time.perf_counter()
    _, _, packed, _ = oracle.fwd(x, w.dtype, want_near=False)
    oracle.bwd(dy, w.dtype, packed)
    single = time.perf_counter() - t0
    return {
        "value": round(moved / wall / 1e9, 3),
        "unit": "GB/s",
        "cores": cores,
        "cores_available": avail,
        "kind": "oracle",
        "sample": f"one {w.name} layer ({n} elements) fwd+bwd, {reps} repetitions, "
                  f"split into {cores} contiguous chunks, one thread each "
                  f"(the box's core share for one GPU, OMP_NUM_THREADS={share}; the machine shows {avail})",
        "elements_per_s": round(n * reps / wall, 1),
        "single_core": {"value": round(2 * bytes_per_direction(n, w.dtype) / single / 1e9, 3), "unit": "GB/s",
                        "elements_per_s": round(n / single, 1), "sample": "the same layer once, one thread"},
    }


# ------------------------------------------------------------------------------- counter runs ----

def probe(torch, workload: str, reps: int, extras: bool):
    """Launches, `reps` times each on distinct (cold) buffers and in this order, a plain
    device-to-device copy of known size (n*e bytes in, n*e out: it calibrates what a counter reports
    per byte) and then the forward and the backward kernel on one layer of the workload; with
    `extras` the kernels of the rows beyond the headline path follow.  For rocprofv3 --pmc and
    --kernel-trace runs; nothing is timed here."""
    w = wl.WORKLOADS[workload]
    x, dy = wl.layer_inputs(w, 0, 0)
    n = x.shape[0]
    st = torch.cuda.current_stream().cuda_stream
    sets = []
    for _ in range(reps):
        tx = torch.from_numpy(x.view(np.uint8)).cuda()
        tdy = torch.from_numpy(dy.view(np.uint8)).cuda()
        sets.append((tx, torch.empty_like(tx), torch.empty((n + 1) // 2, dtype=torch.uint8, device="cuda"),
                     tdy, torch.empty_like(tdy)))

    def each(fn):
        torch.cuda.synchronize()
        for s in sets:
            fn(s)
        torch.cuda.synchronize()

    each(lambda s: s[1].copy_(s[0]))
    each(lambda s: s2a.act_fwd(s[0].data_ptr(), s[1].data_ptr(), s[2].data_ptr(), n, w.dtype, st))
    each(lambda s: s2a.act_bwd(s[3].data_ptr(), s[2].data_ptr(), s[4].data_ptr(), n, w.dtype, st))
    side = 4 if w.dtype == wl.BF16 else 2
    nb = x.nbytes // 16 * 16
    each(lambda s: s2a.stream_copy_shaped(s[0].data_ptr(), s[1].data_ptr(), s[2].data_ptr(), nb, side, 0, st))
    each(lambda s: s2a.stream_copy_shaped(s[3].data_ptr(), s[4].data_ptr(), s[2].data_ptr(), nb, side, 1, st))
    print(f"probe {w.name}: n={n} copy_bytes_in={x.nbytes} copy_bytes_out={x.nbytes} reps={reps}")
    if not extras:
        return
    qs = [torch.empty(s2a.QSTATE_FLOATS, dtype=torch.float32, device="cuda") for _ in sets]
    masks = [torch.empty((n + 7) // 8, dtype=torch.uint8, device="cuda") for _ in sets]
    sets[:] = [s + (qs[k], masks[k]) for k, s in enumerate(sets)]
    each(lambda s: s2a.act_fwd_dyn(s[0].data_ptr(), s[1].data_ptr(), s[2].data_ptr(), s[5].data_ptr(), n, w.dtype, st))
    each(lambda s: s2a.relu_fwd(s[0].data_ptr(), s[1].data_ptr(), s[6].data_ptr(), n, w.dtype, st))
    each(lambda s: s2a.relu_bwd(s[3].data_ptr(), s[6].data_ptr(), s[4].data_ptr(), n, w.dtype, st))
    del sets, qs, masks
    torch.cuda.empty_cache()
    for rows, L in SOFTMAX_SHAPES.values():
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
        for s in sm:
            s[1].copy_(s[0])
        torch.cuda.synchronize()
        for s in sm:
            s2a.softmax_fwd(s[0].data_ptr(), s[1].data_ptr(), s[2].data_ptr(), s[3].data_ptr(), rows, L, wl.BF16, st)
        torch.cuda.synchronize()
        for s in sm:
            s2a.softmax_bwd(s[4].data_ptr(), s[2].data_ptr(), s[3].data_ptr(), s[5].data_ptr(), rows, L, wl.BF16, st)
        torch.cuda.synchronize()
        del sm
        torch.cuda.empty_cache()
    for (batch, N, C), rank, lrp_only in [(v, LRP_RANK, False) for v in TOKEN_SHAPES.values()] + \
                                         [(TOKEN_SHAPES["vit_l16_tokens"], LRP_RANK_SCALED, True)]:
        r_cap = 8
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
        for s in cl:
            s[2].copy_(s[0])
        torch.cuda.synchronize()
        for tt, ty, tfull, dA, dB, work in cl:
            if not lrp_only:
                s2a.cap_fwd(tt.data_ptr(), ty.data_ptr(), m // r_cap, r_cap, wl.BF16, st)
        torch.cuda.synchronize()
        for tt, ty, tfull, dA, dB, work in cl:
            if not lrp_only:
                s2a.cap_bwd(ty.data_ptr(), tfull.data_ptr(), m // r_cap, r_cap, wl.BF16, st)
        torch.cuda.synchronize()
        for tt, ty, tfull, dA, dB, work in cl:
            s2a.lrp_fwd(tt.data_ptr(), tfull.data_ptr(), A.data_ptr(), B.data_ptr(), batch, N, C, rank, wl.BF16, st)
        torch.cuda.synchronize()
        for tt, ty, tfull, dA, dB, work in cl:
            s2a.lrp_bwd(tt.data_ptr(), A.data_ptr(), B.data_ptr(), dA.data_ptr(), dB.data_ptr(), work.data_ptr(),
                        batch, N, C, rank, wl.BF16, st)
        torch.cuda.synchronize()
        del cl
        torch.cuda.empty_cache()
    print("probe extras: softmax " + ", ".join(f"{k}=[{r},{L}]" for k, (r, L) in SOFTMAX_SHAPES.items())
          + "; cap/lrp " + ", ".join(f"{k}=[{b},{N},{C}]" for k, (b, N, C) in TOKEN_SHAPES.items())
          + f"; lrp rank {LRP_RANK_SCALED} at vit_l16_tokens")


# attention-shaped softmax rows: (rows, L).  ViT-B/16 and ViT-L/16: 197 tokens, 12 / 16 heads, batch 64;
# ViT-G/14: 257 tokens, 16 heads, batch 32; Swin-B stage 1: 7x7 windows, 64 windows x 4 heads per image
SOFTMAX_SHAPES = {"vit_b16_attention": (64 * 12 * 197, 197), "vit_l16_attention": (64 * 16 * 197, 197),
                  "vit_g14_attention": (32 * 16 * 257, 257), "swin_b_window_attention": (64 * 64 * 4 * 49, 49)}
# token tensors [batch, N, C] either side of the nonlinearity
TOKEN_SHAPES = {"vit_b16_tokens": (64, 197, 768), "vit_l16_tokens": (64, 197, 1024), "vit_g14_tokens": (32, 257, 1664),
                "vit_l16_hidden": (64, 197, 4096)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="vit_l16", choices=sorted(wl.WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-targets", action="store_true",
                    help="skip the per-kernel roofline entries at the other configurations")
    ap.add_argument("--no-extras", action="store_true", help="skip the rows beyond the headline path")
    ap.add_argument("--probe", action="store_true",
                    help="launch a calibrating copy and each kernel a few times on cold buffers and exit (for counter runs)")
    ap.add_argument("--extras", action="store_true", help="with --probe: also the kernels beyond the headline path")
    ap.add_argument("--reps", type=int, default=4, help="with --probe: launches per kernel")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this path is built and measured on ONE GPU; run with --gpus 1 "
                 "(the kernels are element-wise: more GPUs would each run the same launch on a shard)")

    import torch

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the activation path has no CPU fallback")
    torch.cuda.set_device(0)
    s2a.qtable_init(16)
    if args.probe:
        probe(torch, args.workload, args.reps, args.extras)
        return

    traffic = load_traffic()
    w = wl.WORKLOADS[args.workload]
    hw = w if w.layers > 1 else wl.Workload(w.name, w.index, w.dtype, w.shapes, 8, w.dist, w.scale, w.dy_scale)
    res = time_workload(torch, hw, args.steps, args.warmup, distinct_seeds=True)
    value = res["bytes_per_step"] / (res["ms_per_step"] * 1e-3) / 1e9
    sub = max(5, args.steps // 2)
    subw = max(5, args.warmup)
    n1 = w.sizes()[0]
    ceil_sets = max(8, min(24, res["launches_per_phase"]))
    ceilings = time_copy_ceilings(torch, n1, w.dtype, ceil_sets, sub, 3)
    out = {
        "metric": METRIC,
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(res["ms_per_step"], 4),
        "ms_per_step_without_events": round(res["ms_per_step_without_events"], 4),
        "value_without_events": round(res["bytes_per_step"] / (res["ms_per_step_without_events"] * 1e-3) / 1e9, 1),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",  # the type the path computes in; the storage type of the tensors is in config
        "data": "synthetic",
        "config": {
            "workload": f"{w.name}: {dname(w.dtype)} " + " + ".join("x".join(map(str, s)) for s in w.shapes)
                        + f", {hw.layers} layer(s) back to back, fwd then bwd",
            "storage_dtype": dname(w.dtype),
            "elements_per_step": res["elements_per_step"],
            "launches_per_step": 2 * res["launches_per_phase"],
        },
        "elements_per_s": round(res["elements_per_step"] / (res["ms_per_step"] * 1e-3), 1),
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "roofline": roofline_of(res, w, traffic, ceilings),
    }
    if not args.no_targets:
        targets = {}
        for name in ("vit_g14", "vit_g14_f32", "vit_l16", "vit_b16", "swin_b"):
            if name == w.name:
                continue
            tw = wl.WORKLOADS[name]
            # single-launch workloads get 8 buffer sets so that every launch reads cold HBM
            if tw.layers == 1:
                sets = 8 if len(tw.shapes) == 1 else 3     # swin_b: 4 stages x 3 sets, 2.6 GB per direction
                tw = wl.Workload(tw.name, tw.index, tw.dtype, tw.shapes, sets, tw.dist, tw.scale, tw.dy_scale)
            r = time_workload(torch, tw, sub, subw, distinct_seeds=False)
            cc = None
            if len(tw.shapes) == 1:
                cc = time_copy_ceilings(torch, tw.sizes()[0], tw.dtype, 8, sub, 3)
            targets[name] = {
                "workload": f"{name}: {dname(tw.dtype)} " + " + ".join("x".join(map(str, s)) for s in tw.shapes),
                "buffer_sets": tw.layers,
                "fwd": kernel_block(r, tw, "fwd", traffic, cc and cc["fwd"]),
                "bwd": kernel_block(r, tw, "bwd", traffic, cc and cc["bwd"]),
            }
        out["target_shapes"] = targets
        # the smallest configuration (2.6 MB per launch, 0.3 us at the roofline): reported, not a roofline figure
        out["tiny_config"] = time_tiny(torch, sub, subw)
    if not args.no_extras:
        rows = {}
        tl = wl.WORKLOADS["vit_l16"]
        e = esize(tl.dtype)
        # measured-range quantizer (Eq. 8 read literally), two regimes.  "saturating": the workload's own
        # activations reach both clip limits, so every wave of the range pass stops after its first loads:
        # 2e + 0.5 bytes per element.  "narrow": N(0, 0.3^2) stays inside the limits, so the range pass
        # reads all of x before the forward kernel reads it again: 3e + 0.5 bytes per element.
        narrow = wl.Workload(tl.name, tl.index, tl.dtype, tl.shapes, tl.layers, "normal", 0.3, tl.dy_scale)
        rows["measured_range_saturating_input"] = variant_row(torch, "vit_l16", "gelu_dyn", sub, subw, traffic)
        rows["measured_range_narrow_input"] = variant_row(torch, "vit_l16", "gelu_dyn", sub, subw, traffic,
                                                          bytes_per_elem_fwd=3 * e + 0.5, w_override=narrow,
                                                          row_key="vit_l16:gelu_dyn_narrow")
        rows["measured_range_vit_g14_f32"] = variant_row(torch, "vit_g14_f32", "gelu_dyn", sub, subw, traffic)
        # y written over x and dx over dy (the entry points allow exact aliasing): the same bytes, the
        # read and the write stream on the same DRAM pages.  Timing only: the values decay over the steps.
        rows["in_place_vit_l16"] = variant_row(torch, "vit_l16", "gelu_in_place", sub, subw, traffic)
        rows["silu"] = variant_row(torch, "vit_l16", "silu", sub, subw, traffic)
        rows["relu_mask_vit_l16"] = variant_row(torch, "vit_l16", "relu", sub, subw, traffic)
        rows["relu_mask_vit_g14_f32"] = variant_row(torch, "vit_g14_f32", "relu", sub, subw, traffic)
        sm = {}
        for key, (nrows, L) in SOFTMAX_SHAPES.items():
            sm[key + "_bf16"] = softmax_row(torch, key, nrows, L, wl.BF16, sub, 5, traffic)
        sm["vit_b16_attention_f32"] = softmax_row(torch, "vit_b16_attention_f32", *SOFTMAX_SHAPES["vit_b16_attention"],
                                                  wl.F32, sub, 5, traffic)
        rows["softmax_4bit"] = sm
        cl = {}
        for key, (b, N, C) in TOKEN_SHAPES.items():
            note = "launch- and fill/drain-bound at this size" if key == "vit_b16_tokens" else None
            cl[key] = cap_lrp_row(torch, key, b, N, C, sub, 5, traffic, note)
        key = "vit_l16_tokens"
        cl[f"{key}_rank_{LRP_RANK_SCALED}"] = cap_lrp_row(torch, f"{key}_rank_{LRP_RANK_SCALED}", *TOKEN_SHAPES[key], sub, 5, traffic,
                                                         rank=LRP_RANK_SCALED, lrp_only=True)
        rows["cap_lrp"] = cl
        out["next_rows"] = rows
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
