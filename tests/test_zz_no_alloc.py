"""GPU test of s2a_lrp_bwd_noalloc, the entry point for callers that cannot allocate: it must
give the results of s2a_lrp_bwd (same kernels, the working memory inside the library instead
of a caller's buffer) on calls in a row that share that memory, the later ones smaller."""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_08154_amd import s2a
from paper_2503_08154_amd import workloads as wl


def _case(batch, N, C, r, dtype, seed):
    n = batch * N * C
    dy = wl.draw_dy(n, 1.0, dtype, seed=seed)
    g = np.random.Generator(np.random.Philox(seed + 1))
    A = (g.standard_normal((N, r)) * 0.5).astype(np.float32)
    B = (g.standard_normal((r, C)) * 0.5).astype(np.float32)
    return dy, A, B


def _run(entry, dy, A, B, batch, N, C, r, dtype, with_work):
    st = torch.cuda.current_stream().cuda_stream
    tdy = torch.from_numpy(dy.view(np.uint8)).cuda()
    tA, tB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    dA = torch.full((N, r), float("nan"), device="cuda")
    dB = torch.full((r, C), float("nan"), device="cuda")
    if with_work:
        work = torch.full((N * C,), float("nan"), device="cuda")
        entry(tdy.data_ptr(), tA.data_ptr(), tB.data_ptr(), dA.data_ptr(), dB.data_ptr(), work.data_ptr(),
              batch, N, C, r, dtype, st)
    else:
        entry(tdy.data_ptr(), tA.data_ptr(), tB.data_ptr(), dA.data_ptr(), dB.data_ptr(), batch, N, C, r, dtype, st)
    torch.cuda.synchronize()
    return dA.cpu().numpy(), dB.cpu().numpy()


@pytest.mark.gpu
def test_noalloc_equals_lrp_bwd_on_calls_that_share_the_working_memory():
    assert torch.cuda.is_available()
    # large first (fills most of the library's array), then smaller ones that reuse its front
    cases = [(16, 257, 1664, 30, wl.BF16), (8, 197, 768, 30, wl.BF16), (3, 50, 64, 5, wl.F32), (2, 7, 8, 1, wl.BF16)]
    for k, (batch, N, C, r, dtype) in enumerate(cases):
        dy, A, B = _case(batch, N, C, r, dtype, seed=900 + 10 * k)
        dA1, dB1 = _run(s2a.lrp_bwd_noalloc, dy, A, B, batch, N, C, r, dtype, with_work=False)
        dA0, dB0 = _run(s2a.lrp_bwd, dy, A, B, batch, N, C, r, dtype, with_work=True)
        # the same kernels on the same inputs: bit-identical, which is within any tolerance
        np.testing.assert_array_equal(dA1.view(np.uint32), dA0.view(np.uint32))
        np.testing.assert_array_equal(dB1.view(np.uint32), dB0.view(np.uint32))
        # and against the oracle, with the tolerance of the Low-Rank-Prompt parity tests:
        # fp32 accumulation, |err| <= 2e-5 * sum |terms|
        if k > 0:       # the largest case would take the scalar oracle a minute
            dA_ref, dB_ref = oracle.lrp_bwd(dy, dtype, A, B, batch, N, C)
            g = np.abs(wl.storage_to_f64(dy, dtype)).reshape(batch, N, C).sum(axis=0)
            np.testing.assert_array_less(np.abs(dA1 - dA_ref), 2e-5 * (g @ np.abs(B.astype(np.float64)).T) + 1e-30)
            np.testing.assert_array_less(np.abs(dB1 - dB_ref), 2e-5 * (np.abs(A.astype(np.float64)).T @ g) + 1e-30)


def test_noalloc_rejects_what_does_not_fit():
    """Host-side: needs no GPU."""
    fake = 0x1000   # never dereferenced: the size check comes before any device work
    too_many = s2a.LRP_NOALLOC_MAX_FLOATS // 1024 + 1
    assert s2a.lrp_bwd_noalloc(fake, fake, fake, fake, fake, 4, too_many, 1024, 30, wl.BF16, check=False) == s2a.ERR_SIZE
    assert s2a.lrp_bwd_noalloc(fake, fake, fake, fake, fake, 4, 1024, 1024, 30, wl.BF16 + 5, check=False) == s2a.ERR_DTYPE
    assert s2a.lrp_bwd_noalloc(fake, fake, fake, None, fake, 4, 197, 768, 30, wl.BF16, check=False) == s2a.ERR_NULL
