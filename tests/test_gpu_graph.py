"""Every entry point under HIP graph capture: every launch goes to the caller's
stream and nothing allocates or synchronises, so a captured forward+backward
must replay to the bits of the eager run, every time."""
import numpy as np
import pytest
import torch

from paper_2503_08154_amd import s2a
from paper_2503_08154_amd import workloads as wl

pytestmark = pytest.mark.gpu


def test_forward_backward_graph_replays_match_eager():
    s2a.qtable_init(16)
    w = wl.WORKLOADS["vit_b16"]
    n = 8192 * 37 + 5
    x, dy = wl.layer_inputs(w, 0, 0, n=n)
    rows, L = 1024, 197
    logits = wl.draw_x(rows * L, "normal", 2.0, wl.BF16, seed=3)
    tx = torch.from_numpy(x.view(np.uint8)).cuda()
    tdy = torch.from_numpy(dy.view(np.uint8)).cuda()
    tl = torch.from_numpy(logits.view(np.uint8)).cuda()
    out = {k: torch.empty_like(tx) for k in ("y", "dx", "y_dyn", "dx_dyn", "y_relu")}
    codes = torch.empty((n + 1) // 2, dtype=torch.uint8, device="cuda")
    codes_dyn = torch.empty_like(codes)
    mask = torch.empty((n + 7) // 8, dtype=torch.uint8, device="cuda")
    qstate = torch.empty(s2a.QSTATE_FLOATS, dtype=torch.float32, device="cuda")
    sm_y = torch.empty_like(tl)
    sm_dx = torch.empty_like(tl)
    sm_c = torch.empty(rows * ((L + 1) // 2), dtype=torch.uint8, device="cuda")
    sm_q = torch.empty(2 * rows, dtype=torch.float32, device="cuda")
    # CAP and LRP on a [batch, N, C] view of a prefix of x
    batch, N, C, rank, r_cap = 6, 19, 64, 30, 8
    m = batch * N * C
    cap_y = torch.empty(m // r_cap * 2, dtype=torch.uint8, device="cuda")
    cap_dx = torch.empty(m * 2, dtype=torch.uint8, device="cuda")
    lrp_y = torch.empty(m * 2, dtype=torch.uint8, device="cuda")
    A = torch.randn(N, rank, device="cuda")
    B = torch.randn(rank, C, device="cuda")
    dA, dB, work = torch.empty_like(A), torch.empty_like(B), torch.empty(N, C, device="cuda")
    out["dx_relu"] = torch.empty_like(tx)
    out["y_silu"] = torch.empty_like(tx)
    out["dx_silu"] = torch.empty_like(tx)
    codes_silu = torch.empty_like(codes)

    def run(stream):
        s2a.act_fwd(tx.data_ptr(), out["y"].data_ptr(), codes.data_ptr(), n, w.dtype, stream)
        s2a.act_bwd(tdy.data_ptr(), codes.data_ptr(), out["dx"].data_ptr(), n, w.dtype, stream)
        s2a.act_fwd_dyn(tx.data_ptr(), out["y_dyn"].data_ptr(), codes_dyn.data_ptr(), qstate.data_ptr(), n, w.dtype, stream)
        s2a.act_bwd_dyn(tdy.data_ptr(), codes_dyn.data_ptr(), qstate.data_ptr(), out["dx_dyn"].data_ptr(), n, w.dtype, stream)
        s2a.relu_fwd(tx.data_ptr(), out["y_relu"].data_ptr(), mask.data_ptr(), n, w.dtype, stream)
        s2a.relu_bwd(tdy.data_ptr(), mask.data_ptr(), out["dx_relu"].data_ptr(), n, w.dtype, stream)
        s2a.silu_fwd(tx.data_ptr(), out["y_silu"].data_ptr(), codes_silu.data_ptr(), n, w.dtype, stream)
        s2a.silu_bwd(tdy.data_ptr(), codes_silu.data_ptr(), out["dx_silu"].data_ptr(), n, w.dtype, stream)
        s2a.softmax_fwd(tl.data_ptr(), sm_y.data_ptr(), sm_c.data_ptr(), sm_q.data_ptr(), rows, L, wl.BF16, stream)
        s2a.softmax_bwd(tl.data_ptr(), sm_c.data_ptr(), sm_q.data_ptr(), sm_dx.data_ptr(), rows, L, wl.BF16, stream)
        s2a.cap_fwd(tx.data_ptr(), cap_y.data_ptr(), m // r_cap, r_cap, w.dtype, stream)
        s2a.cap_bwd(cap_y.data_ptr(), cap_dx.data_ptr(), m // r_cap, r_cap, w.dtype, stream)
        s2a.lrp_fwd(tx.data_ptr(), lrp_y.data_ptr(), A.data_ptr(), B.data_ptr(), batch, N, C, rank, w.dtype, stream)
        s2a.lrp_bwd(tdy.data_ptr(), A.data_ptr(), B.data_ptr(), dA.data_ptr(), dB.data_ptr(), work.data_ptr(),
                    batch, N, C, rank, w.dtype, stream)

    def snapshot():
        torch.cuda.synchronize()
        return [t.cpu().numpy().copy() for t in (*out.values(), codes, codes_dyn, codes_silu, mask, qstate, sm_y, sm_dx, sm_c, sm_q,
                                                 cap_y, cap_dx, lrp_y, dA, dB, work)]

    def scrub():
        for t in (*out.values(), codes, codes_dyn, codes_silu, mask, sm_y, sm_dx, sm_c, cap_y, cap_dx, lrp_y):
            t.fill_(0x5A)
        for t in (dA, dB, work):
            t.fill_(-1.0)
        qstate.fill_(-1.0)
        sm_q.fill_(-1.0)

    scrub()                                       # unwritten qstate slots keep the fill on both sides
    run(torch.cuda.current_stream().cuda_stream)
    eager = snapshot()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        run(side.cuda_stream)                     # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run(torch.cuda.current_stream().cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    for replay in range(3):
        scrub()                                   # the program's own eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for a, b in zip(got, eager):
            assert np.array_equal(a.view(np.uint8), b.view(np.uint8)), f"replay {replay} differs from the eager run"
