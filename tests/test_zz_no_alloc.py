"""The entry point that allocates nothing (lba_grad_static: the brick maps of the immediate estimator in device
memory that belongs to the library) against the entry point that takes them in a caller-given workspace
(lba_grad_ws), through the C ABI: two calls in a row, the second on a smaller input (the library's memory keeps the
first call's marks: they must not leak into the second), then a shape beyond the library's memory.  Bit for bit on
data whose sums are exactly representable; within the FP32 bound of the interface on general data."""
import numpy as np
import pytest
import torch

from paper_2401_14110_amd import binding as lb

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
QP, QA = (4, 7, 12, 0), (4, 7, 10, 0)                              # R_OF = 63.75


def codes(rng, shape, lo, hi):
    e = rng.integers(lo, hi + 1, shape); m = rng.integers(0, 8, shape); s = rng.integers(0, 2, shape)
    c = (s << 7) | (e << 3) | m
    return np.where((c & 0x7F) == 0x7F, c & 0xFE, c).astype(np.uint8)


def test_static_scratch_entry_point_matches_the_workspace_one(ref):
    from oracle import lba_grad_ref as gref
    rng = np.random.default_rng(2718)
    stream = torch.cuda.current_stream().cuda_stream
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)
    seen_blocked = 0
    # first a large input whose last third overflows everywhere, then a smaller one that overflows nowhere in its
    # first rows (marks left behind by the first call would send clean bricks to the wrong kernel: still correct,
    # so the second check is on the results AND on a third call with overflows in other places)
    for (M, N, K), loud, exact in [((600, 260, 900), "tail", True), ((130, 68, 260), "none", True), ((260, 132, 515), "head", True),
                                   ((300, 200, 600), "tail", False), ((70, 64, 100), "tail", False)]:
        A = codes(rng, (M, K), 2, 5); B = codes(rng, (N, K), 2, 5)
        if loud == "tail":
            A[:, K - K // 3:] = codes(rng, (M, K // 3), 6, 10); B[:, K - K // 3:] = codes(rng, (N, K // 3), 6, 10)
        if loud == "head":
            A[:, :K // 4] = codes(rng, (M, K // 4), 7, 10); B[:, :K // 4] = codes(rng, (N, K // 4), 7, 10)
        G = (rng.integers(-8, 9, (M, N)) / 4.0).astype(np.float32) if exact else rng.standard_normal((M, N)).astype(np.float32)
        tA, tB, tG = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV), torch.from_numpy(G).to(DEV)
        _, of, _ = lb.gemm_bwd(tA, tB, QP, QA, want_c=False)
        outs = []
        for entry in ("static", "ws"):
            dX = torch.full((M, K), float("nan"), device=DEV); dW = torch.full((N, K), float("nan"), device=DEV)
            args = (tG.data_ptr(), tA.data_ptr(), tB.data_ptr(), of.data_ptr(), None, dX.data_ptr(), dW.data_ptr(), M, N, K,
                    lb.STE_IMMEDIATE_OF)
            rc = lb.lba_grad_static(*args, stream) if entry == "static" else lb.lba_grad_ws(*args, ws.data_ptr(), ws.numel(), stream)
            assert rc == lb.OK, (entry, rc)
            torch.cuda.synchronize()
            outs.append((dX.cpu().numpy(), dW.cpu().numpy()))
        (sX, sW), (wX, wW) = outs
        oX, oW = gref.grad(G, A, B, ref.QFmt(*QP), ref.QFmt(*QA), 1)
        if exact:
            assert np.array_equal(sX, wX) and np.array_equal(sW, wW), (M, N, K, loud)
            assert np.array_equal(sX, oX.astype(np.float32)) and np.array_equal(sW, oW.astype(np.float32)), (M, N, K, loud)
        else:
            aX, aW = gref.grad_abs(G, A, B, ref.QFmt(*QP), ref.QFmt(*QA), 1)
            tolX, tolW = 2 * (N + 1) * 2.0 ** -24 * aX + 1e-30, 2 * (M + 1) * 2.0 ** -24 * aW + 1e-30
            for got in (sX, wX):
                assert (np.abs(got - oX) <= tolX).all(), (M, N, K, loud)
            for got in (sW, wW):
                assert (np.abs(got - oW) <= tolW).all(), (M, N, K, loud)
        seen_blocked += int(of.cpu().numpy().any())
    assert seen_blocked >= 3
    # a shape whose brick maps do not fit the library's memory is refused, and nothing is enqueued
    big = (1 << 17, 1 << 13, 1 << 12)
    assert lb.lba_grad_workspace_bytes(*big) > (1 << 20)
    p = ws.data_ptr()
    assert lb.lba_grad_static(p, p, p, p, None, p, p, *big, lb.STE_IMMEDIATE_OF, stream) == lb.ERR_SHAPE
    # the other estimators pass through unchanged
    M, N, K = 70, 64, 100
    A = codes(rng, (M, K), 5, 10); B = codes(rng, (N, K), 5, 10)
    G = (rng.integers(-8, 9, (M, N)) / 4.0).astype(np.float32)
    tA, tB, tG = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV), torch.from_numpy(G).to(DEV)
    dX = torch.empty((M, K), device=DEV); dW = torch.empty((N, K), device=DEV)
    assert lb.lba_grad_static(tG.data_ptr(), tA.data_ptr(), tB.data_ptr(), None, None, dX.data_ptr(), dW.data_ptr(), M, N, K,
                              lb.STE_IDENTITY, stream) == lb.OK
    torch.cuda.synchronize()
    oX, oW = gref.grad(G, A, B, ref.QFmt(*QP), ref.QFmt(*QA), 0)
    assert np.array_equal(dX.cpu().numpy(), oX.astype(np.float32)) and np.array_equal(dW.cpu().numpy(), oW.astype(np.float32))
