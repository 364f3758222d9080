"""GPU parity of the Low-Rank Prompt kernels (s2a_lrp_fwd / s2a_lrp_bwd) against
the oracle.

Tolerances, from the fp32 arithmetic of the kernels (u = 2^-24):
  y   = x + sum_k a_k b_k : |err| <= 1e-6 * (|x| + sum_k |a_k b_k|)  (+ 1 bf16 ulp of y for bf16 storage)
  dA, dB are sums of up to batch + C (resp. batch + N) fp32 terms accumulated in sequence
        and by a tree: |err| <= 2e-5 * sum |terms|  (the bound (64 + 197) u = 1.6e-5 at ViT-B/16).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2503_08154_amd import s2a
from paper_2503_08154_amd import workloads as wl

import gpu_util as gu
import parity

pytestmark = pytest.mark.gpu
DTYPES = [wl.F32, wl.BF16]


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _check(batch, N, C, r, dtype, seed, inplace=False, b_offset=0, out_offset=0):
    g = np.random.Generator(np.random.Philox(seed))
    A = (g.standard_normal((N, r)) * 0.5).astype(np.float32)
    B = (g.standard_normal((r, C)) * 0.5).astype(np.float32)
    n = batch * N * C
    x = wl.draw_x(n, "normal", 1.5, dtype, seed=seed + 1)
    dy = wl.draw_dy(n, 1e-2, dtype, seed=seed + 2)
    es = gu.esize(dtype)
    st = torch.cuda.current_stream().cuda_stream
    tA = _dev(A)
    tB = torch.empty(r * C + b_offset, dtype=torch.float32, device="cuda")[b_offset:]   # b_offset floats off 16-byte alignment
    tB.copy_(torch.from_numpy(B.reshape(-1)))
    bx = gu.Buf(n * es).upload(x)
    by = bx if inplace else gu.Buf(n * es, fill=0xFF)
    s2a.lrp_fwd(bx.ptr, by.ptr, tA.data_ptr(), tB.data_ptr(), batch, N, C, r, dtype, st)
    torch.cuda.synchronize()
    assert bx.canaries_intact() and by.canaries_intact()
    y = wl.storage_to_f64(by.download(gu.storage_np(dtype)), dtype)
    y_ref = oracle.lrp_fwd(x, dtype, A, B, batch, N, C)
    mag = np.abs(A.astype(np.float64)) @ np.abs(B.astype(np.float64))            # sum_k |a_k b_k|, [N, C]
    tol = 1e-6 * (np.abs(wl.storage_to_f64(x, dtype)).reshape(batch, N, C) + mag[None]).reshape(-1)
    if dtype == wl.BF16:
        tol = tol + parity.bf16_ulp(y_ref)
    bad = ~(np.abs(y - y_ref) <= tol)
    if bad.any():
        b, i, c = np.nonzero(bad.reshape(batch, N, C))
        x_ok = inplace or bool((bx.download(gu.storage_np(dtype)).view(np.uint8) == x.view(np.uint8)).all())
        by2 = gu.Buf(n * es, fill=0xFF)   # the same launch once more, for the failure report only
        if not inplace:
            s2a.lrp_fwd(bx.ptr, by2.ptr, tA.data_ptr(), tB.data_ptr(), batch, N, C, r, dtype, st)
        again = int((~(np.abs(wl.storage_to_f64(by2.download(gu.storage_np(dtype)), dtype) - y_ref) <= tol)).sum())
        raise AssertionError(
            f"[x on the device intact: {x_ok}; a second launch leaves {again} elements out] "
            f"y: {int(bad.sum())} elements out, worst {np.nanmax(np.abs(y - y_ref) / tol):.2f}x the tolerance; "
            f"samples {np.unique(b)[:12]}, tokens {np.unique(i)[:12]}, channels {np.unique(c)[:24]} "
            f"({len(np.unique(b))} samples, {len(np.unique(i))} tokens, {len(np.unique(c))} channels); "
            f"first: y[{b[0]},{i[0]},{c[0]}] = {y.reshape(batch, N, C)[b[0], i[0], c[0]]!r} vs {y_ref.reshape(batch, N, C)[b[0], i[0], c[0]]!r}")

    bdy = gu.Buf(n * es).upload(dy)
    bA = gu.Buf(4 * N * r, fill=0xFF)
    bB = gu.Buf(4 * r * C, 4 * out_offset, fill=0xFF)      # out_offset floats off 16-byte alignment
    bw = gu.Buf(4 * N * C, 4 * out_offset, fill=0xFF)
    s2a.lrp_bwd(bdy.ptr, tA.data_ptr(), tB.data_ptr(), bA.ptr, bB.ptr, bw.ptr, batch, N, C, r, dtype, st)
    torch.cuda.synchronize()
    assert bA.canaries_intact() and bB.canaries_intact() and bw.canaries_intact() and bdy.canaries_intact()
    dA = bA.download(np.float32).reshape(N, r).astype(np.float64)
    dB = bB.download(np.float32).reshape(r, C).astype(np.float64)
    dA_ref, dB_ref = oracle.lrp_bwd(dy, dtype, A, B, batch, N, C)
    gabs = np.abs(wl.storage_to_f64(dy, dtype)).reshape(batch, N, C).sum(axis=0)   # sum_b |dy|, [N, C]
    tolA = 2e-5 * (gabs @ np.abs(B.astype(np.float64)).T) + 1e-30
    tolB = 2e-5 * (np.abs(A.astype(np.float64)).T @ gabs) + 1e-30
    assert (np.abs(dA - dA_ref) <= tolA).all(), f"dA: worst {np.max(np.abs(dA - dA_ref) / tolA):.2f}x the tolerance"
    assert (np.abs(dB - dB_ref) <= tolB).all(), f"dB: worst {np.max(np.abs(dB - dB_ref) / tolB):.2f}x the tolerance"


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("shape", [(1, 1, 8, 1), (2, 3, 16, 5), (3, 7, 24, 30), (5, 197, 768, 30), (64, 17, 256, 64),
                                   (1, 300, 1024, 2), (9, 50, 40, 30),
                                   # the 16 x 16 tiles of the backward products: exact, one past, rank limit on one token
                                   (2, 16, 64, 16), (2, 17, 72, 17), (1, 33, 136, 33), (1, 1, 8, 128), (3, 1, 1032, 1)])
def test_shapes(dtype, shape):
    batch, N, C, r = shape
    _check(batch, N, C, r, dtype, seed=sum(shape))


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("r", [5, 15, 30, 50, 70, 100, 127, 128])
def test_ranks_of_the_scaling_study(dtype, r):
    """Sec. 4.3 ("Scaling Tunable Parameters Up", Fig. 5) runs the prompt at ranks 5 .. 100; 128 is the
    library's limit.  Ranks above 64 take two rounds of the forward kernel's prompt sum, and every rank
    that is not a multiple of 16 leaves a ragged last rank tile in the backward products."""
    _check(4, 37, 256, r, dtype, seed=1000 + r)


@pytest.mark.parametrize("dtype", DTYPES)
def test_vit_l16_tokens_rank_100(dtype):
    _check(8, 197, 1024, 100, dtype, seed=4100)


def test_more_tokens_than_two_rounds():
    """N above 512: dB takes its tokens in a run-time number of rounds of 256 (one and two rounds are
    unrolled instantiations)."""
    _check(2, 1300, 64, 9, wl.BF16, seed=1300)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("vectors", [512, 513, 1024, 1025, 2049])
def test_wide_rows(dtype, vectors):
    """Rows of 512 .. 2049 16-byte vectors: dA contracts such rows in 2, 4 (unrolled) and a run-time
    number of rounds of 1024 channels, and the channel count is not a multiple of 64."""
    C = vectors * (8 if dtype == wl.BF16 else 4)
    _check(3, 2, C, 7, dtype, seed=vectors)


def test_swin_stage_shape():
    """Many tokens, few channels ([16, 3136, 128], the first Swin-B stage): 13 rounds of tokens in dB,
    196 token tiles in dA."""
    _check(16, 3136, 128, 30, wl.BF16, seed=3136)


@pytest.mark.parametrize("dtype", DTYPES)
def test_b_not_vector_aligned(dtype):
    """B only 4-byte aligned: the forward kernel's element loads of B."""
    _check(4, 21, 96, 30, dtype, seed=77, b_offset=1)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("off", [1, 2, 3])
def test_outputs_and_workspace_not_vector_aligned(dtype, off):
    """dB and the workspace only 4-byte aligned: element stores of dB, element loads of G in both products."""
    _check(3, 37, 200, 21, dtype, seed=500 + off, out_offset=off)


@pytest.mark.parametrize("dtype", DTYPES)
def test_vit_g14_tokens(dtype):
    """[.., 257, 1664]: two rounds of tokens in dB, two rounds of channels in dA, ragged tiles everywhere."""
    _check(2, 257, 1664, 30, dtype, seed=257)


@pytest.mark.parametrize("dtype", DTYPES)
def test_empty_batch_gives_zero_gradients(dtype):
    N, C, r = 5, 64, 9
    A = torch.randn(N, r, device="cuda")
    B = torch.randn(r, C, device="cuda")
    bA, bB, bw = gu.Buf(4 * N * r, fill=0xFF), gu.Buf(4 * r * C, fill=0xFF), gu.Buf(4 * N * C, fill=0xFF)
    s2a.lrp_bwd(0x1000, A.data_ptr(), B.data_ptr(), bA.ptr, bB.ptr, bw.ptr, 0, N, C, r, dtype,
                torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert not bA.download(np.float32).any() and not bB.download(np.float32).any()
    assert bA.canaries_intact() and bB.canaries_intact() and bw.canaries_intact()


@pytest.mark.parametrize("dtype", DTYPES)
def test_in_place(dtype):
    _check(6, 33, 128, 30, dtype, seed=9, inplace=True)


@pytest.mark.parametrize("dtype", DTYPES)
def test_vit_b16_full_size(dtype):
    """[64, 197, 768] tokens, rank 30: the paper's LRP setting on ViT-B/16."""
    _check(64, 197, 768, 30, dtype, seed=2030)


def test_identity_at_initialisation():
    """A = 0 leaves the activation bit-for-bit unchanged."""
    batch, N, C, r = 4, 19, 64, 30
    x = wl.draw_x(batch * N * C, "normal", 1.0, wl.BF16, seed=1)
    A = torch.zeros(N, r, device="cuda")
    B = torch.randn(r, C, device="cuda")
    bx = gu.Buf(x.nbytes).upload(x)
    by = gu.Buf(x.nbytes, fill=0xFF)
    s2a.lrp_fwd(bx.ptr, by.ptr, A.data_ptr(), B.data_ptr(), batch, N, C, r, wl.BF16, torch.cuda.current_stream().cuda_stream)
    np.testing.assert_array_equal(by.download(np.uint16), x)


def test_argument_errors():
    f = 0x1000
    assert s2a.lrp_fwd(f, f, f, f, 2, 3, 10, 4, s2a.BF16, check=False) == s2a.ERR_SIZE     # C not a multiple of 8
    assert s2a.lrp_fwd(f, f, f, f, 2, 3, 16, 0, s2a.BF16, check=False) == s2a.ERR_SIZE
    assert s2a.lrp_fwd(f, f, f, f, 2, 3, 16, 129, s2a.BF16, check=False) == s2a.ERR_SIZE
    assert s2a.lrp_fwd(f, f, f, f, 2, 3, 16, 4, 7, check=False) == s2a.ERR_DTYPE
    assert s2a.lrp_fwd(f, None, f, f, 2, 3, 16, 4, s2a.BF16, check=False) == s2a.ERR_NULL
    assert s2a.lrp_fwd(f + 2, f, f, f, 2, 3, 16, 4, s2a.BF16, check=False) == s2a.ERR_ALIGN
    assert s2a.lrp_bwd(f, f, f, f, f, None, 2, 3, 16, 4, s2a.F32, check=False) == s2a.ERR_NULL
    assert s2a.lrp_fwd(None, None, None, None, 0, 3, 16, 4, s2a.F32, check=False) == s2a.OK
