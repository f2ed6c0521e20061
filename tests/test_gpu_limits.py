"""GPU parity at the documented shape limits and at extreme aspect ratios: the largest M, operand
matrices beyond 2^31 and 2^32 bytes, chains of more than 2^24 steps, the largest N, and the shapes just
outside the limits (which must be refused, not run).  Operands are seeded; huge ones repeat a seeded
block with a prime period, so that an index that wraps at a power of two lands on different data."""
import numpy as np
import pytest
import torch

from paper_2401_14110_amd import binding as lb

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
PROD = (5, 7, 15)
ACC = (4, 7, 7)
PERIOD = 1000003                                                       # prime


def codes(rng, shape, lo_e=0, hi_e=15):
    e = rng.integers(lo_e, hi_e + 1, shape)
    c = (rng.integers(0, 2, shape) << 7) | (e << 3) | rng.integers(0, 8, shape)
    return np.where((c & 0x7F) == 0x7F, c & 0xFE, c).astype(np.uint8)


def periodic_rows(rng, M, K, lo_e=0, hi_e=15):
    """[M, K] codes on the GPU: row m is row m % PERIOD of a seeded block."""
    block = torch.from_numpy(codes(rng, (PERIOD, K), lo_e, hi_e)).to(DEV)
    reps = (M + PERIOD - 1) // PERIOD
    return block.repeat(reps, 1)[:M].contiguous()


def bits(x):
    return np.ascontiguousarray(x).view(np.uint32)


def test_largest_m(ref):
    # M = 2^30 - 64 (the limit: 2^24 - 1 workgroups of 256 lanes along grid x), N = K = 1: one FMAq per output,
    # so the whole 4.3 GB result is checked against the oracle's 256-entry table of Q_acc(Q_prod(a * b)); M one
    # larger is refused
    M = 2 ** 30 - 64
    rng = np.random.default_rng(2031)
    A = periodic_rows(rng, M, 1)
    b = np.array([[0x3A]], dtype=np.uint8)                             # 1.25
    for rnd in (0, 1):
        qp, qa = PROD + (rnd,), ACC + (rnd,)
        table = ref.gemm(np.arange(256, dtype=np.uint8).reshape(256, 1), b, ref.QFmt(*qp), ref.QFmt(*qa))
        tb = torch.from_numpy(table.view(np.int32).reshape(256)).to(DEV)
        C = lb.gemm(A, torch.from_numpy(b).to(DEV), qp, qa)
        torch.cuda.synchronize()
        got = C.view(torch.int32).reshape(-1)
        step = 1 << 28
        for s in range(0, M, step):
            want = tb[A[s:s + step, 0].long()]
            assert torch.equal(got[s:s + step], want), (rnd, s)
        del C, got
    with pytest.raises(lb.LbaError):
        lb.lba_plan_query(M + 1, 1, 1, PROD + (0,), ACC + (0,))


def test_operand_beyond_4_gib_and_its_planes(ref):
    # A of 2^25 + 3 rows x 136 bytes = 4.56e9 bytes: sampled rows (first, last, around byte offsets 2^31 and 2^32,
    # random) of C and of both event planes against the oracle, both roundings and both orders
    M, N, K = 2 ** 25 + 3, 2, 136
    rng = np.random.default_rng(2032)
    A = periodic_rows(rng, M, K, 3, 11)
    Bh = codes(rng, (N, K), 3, 11)
    B = torch.from_numpy(Bh).to(DEV)
    rows = {0, 1, 63, 64, M - 1, M - 2, M - 65, PERIOD - 1, PERIOD, PERIOD + 1}
    for off in (2 ** 31, 2 ** 32):
        rows |= {off // K + d for d in (-1, 0, 1, 2)}
    rows |= set(int(r) for r in rng.integers(0, M, 300))
    rows = np.array(sorted(rows))
    idx = torch.from_numpy(rows).to(DEV)
    Ah = A.index_select(0, idx).cpu().numpy()
    for rnd, order in ((0, 0), (1, 0), (0, 1), (1, 1)):
        qp, qa = PROD + (rnd,), ACC + (rnd,)
        wants = ref.gemm_bwd(Ah, Bh, ref.QFmt(*qp), ref.QFmt(*qa), order=order, level2=bool(order))
        C = lb.gemm(A, B, qp, qa, order=order)
        torch.cuda.synchronize()
        assert np.array_equal(bits(C.index_select(0, idx).cpu().numpy()), bits(wants[0])), (rnd, order, "C")
        del C
        gots = lb.gemm_bwd_chunked(A, B, qp, qa) if order else lb.gemm_bwd(A, B, qp, qa)
        torch.cuda.synchronize()
        assert np.array_equal(bits(gots[0].index_select(0, idx).cpu().numpy()), bits(wants[0])), (rnd, order, "C of the recompute call")
        for i in range(1, len(wants)):                                 # OF, UF [, second-level OF, UF]
            assert np.array_equal(gots[i].index_select(1, idx).cpu().numpy().view(np.uint32), wants[i]), (rnd, order, i)
        del gots


def test_chains_longer_than_2_to_24(ref):
    # K = 2^24 + 7 (odd: unaligned rows), 3 x 5 outputs: complete comparison, both roundings and orders; the
    # recompute call at K = 2^22 + 5 with complete planes
    rng = np.random.default_rng(2033)
    M, N, K = 3, 5, 2 ** 24 + 7
    A = codes(rng, (M, K), 2, 9); B = codes(rng, (N, K), 2, 9)
    tA, tB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    for rnd, order in ((0, 0), (1, 0), (0, 1), (1, 1)):
        qp, qa = PROD + (rnd,), (5, 10, 15, rnd)
        C = lb.gemm(tA, tB, qp, qa, order=order)
        torch.cuda.synchronize()
        want = ref.gemm(A, B, ref.QFmt(*qp), ref.QFmt(*qa), order=order)
        assert np.array_equal(bits(C.cpu().numpy()), bits(want)), (rnd, order)
    K2 = 2 ** 22 + 5
    A2, B2 = np.ascontiguousarray(A[:, :K2]), np.ascontiguousarray(B[:, :K2])
    tA2, tB2 = torch.from_numpy(A2).to(DEV), torch.from_numpy(B2).to(DEV)
    for rnd in (0, 1):
        qp, qa = PROD + (rnd,), ACC + (rnd,)
        C, of, uf = lb.gemm_bwd(tA2, tB2, qp, qa)
        torch.cuda.synchronize()
        want, wof, wuf = ref.gemm_bwd(A2, B2, ref.QFmt(*qp), ref.QFmt(*qa))
        assert np.array_equal(bits(C.cpu().numpy()), bits(want)), rnd
        assert np.array_equal(of.cpu().numpy().view(np.uint32), wof), rnd
        assert np.array_equal(uf.cpu().numpy().view(np.uint32), wuf), rnd


def test_largest_n(ref):
    # N = 2^21 (the limit) with M = 2, K = 3: complete comparison; N one larger is refused
    rng = np.random.default_rng(2034)
    M, N, K = 2, 2 ** 21, 3
    A = codes(rng, (M, K)); B = codes(rng, (N, K))
    for rnd in (0, 1):
        qp, qa = PROD + (rnd,), ACC + (rnd,)
        C = lb.gemm(torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV), qp, qa)
        torch.cuda.synchronize()
        want = ref.gemm(A, B, ref.QFmt(*qp), ref.QFmt(*qa))
        assert np.array_equal(bits(C.cpu().numpy()), bits(want)), rnd
    with pytest.raises(lb.LbaError):
        lb.lba_plan_query(M, N + 1, K, PROD + (0,), ACC + (0,))


def _grad_check(got, want, scale, terms, what):
    tol = 2 * (terms + 1) * 2.0 ** -24 * scale + 1e-30
    err = np.abs(got - want)
    assert (err <= tol).all(), "%s: worst error / tolerance %.3g" % (what, float((err / tol).max()))
    assert float((err / tol).max()) < 0.5


def test_gradient_products_at_the_largest_m_times_n(ref):
    # lba_grad with M * N = 2^30 (its limit; G is 4 GiB, the OF plane 8 GiB): sampled rows of dX and sampled
    # columns of dW for the three estimators; one more row is refused
    from oracle import lba_grad_ref as gref
    M, N, K = 2 ** 20, 2 ** 10, 64
    rng = np.random.default_rng(2035)
    Ah = codes(rng, (M, K), 3, 11); Bh = codes(rng, (N, K), 3, 11)
    A, B = torch.from_numpy(Ah).to(DEV), torch.from_numpy(Bh).to(DEV)
    torch.manual_seed(2035)
    G = torch.randn((M, N), dtype=torch.float32, device=DEV)
    qp, qa = PROD + (0,), ACC + (0,)
    fp, fa = ref.QFmt(*qp), ref.QFmt(*qa)
    _, of, _ = lb.gemm_bwd(A, B, qp, qa, want_c=False, want_uf=False)
    last = lb.last_overflow(of, K)
    rows = np.array(sorted({0, 1, 63, 64, M - 1, M - 2, M - 65, M // 2} | set(int(r) for r in rng.integers(0, M, 16))))
    cols = np.array([1, N - 1])                                        # each needs all 2^20 rows in the oracle
    idx, jdx = torch.from_numpy(rows).to(DEV), torch.from_numpy(cols).to(DEV)
    Gr = G.index_select(0, idx).cpu().numpy(); Gc = G.index_select(1, jdx).cpu().numpy()
    blocked = 0
    for ste in (lb.STE_IDENTITY, lb.STE_IMMEDIATE_OF, lb.STE_RECURSIVE_OF):
        dX, dW = lb.grad(G, A, B, ste, of_plane=of if ste == lb.STE_IMMEDIATE_OF else None,
                         last_of=last if ste == lb.STE_RECURSIVE_OF else None)
        torch.cuda.synchronize()
        c = gref.coefficients(Ah[rows], Bh, fp, fa, ste)
        blocked += int((~c).sum())
        wX, _ = gref.grad(Gr, Ah[rows], Bh, fp, fa, ste, c=c)
        aX, _ = gref.grad_abs(Gr, Ah[rows], Bh, fp, fa, ste, c=c)
        _grad_check(dX.index_select(0, idx).cpu().numpy(), wX, aX, N, "ste=%d dX rows" % ste)
        c = gref.coefficients(Ah, Bh[cols], fp, fa, ste)
        _, wW = gref.grad(Gc, Ah, Bh[cols], fp, fa, ste, c=c)
        _, aW = gref.grad_abs(Gc, Ah, Bh[cols], fp, fa, ste, c=c)
        _grad_check(dW.index_select(0, jdx).cpu().numpy(), wW, aW, M, "ste=%d dW columns" % ste)
        del dX, dW, c
    assert blocked > 0
    assert lb.lba_grad(G.data_ptr(), A.data_ptr(), B.data_ptr(), None, None, G.data_ptr(), None, M + 1, N, K,
                       lb.STE_IDENTITY) == lb.ERR_SHAPE            # refused before any pointer is used


def test_zero_fills_beyond_2_to_32_elements():
    # K == 0 stores +0 in all of C, M == 0 stores zeros in all of dW: both with more than 2^32 outputs
    M, N = 2 ** 22 + 1, 2 ** 10 + 3
    C = torch.full((M, N), 1.0, dtype=torch.float32, device=DEV)
    z = torch.empty((M, 0), dtype=torch.uint8, device=DEV)
    lb.gemm(z, torch.empty((N, 0), dtype=torch.uint8, device=DEV), PROD + (0,), ACC + (0,), out=C)
    torch.cuda.synchronize()
    assert int(C.view(torch.int32).count_nonzero()) == 0
    del C
    N, K = 2 ** 21, 2112
    dW = torch.full((N, K), 1.0, dtype=torch.float32, device=DEV)
    rc = lb.lba_grad(None, None, None, None, None, None, dW.data_ptr(), 0, N, K, lb.STE_IDENTITY)
    torch.cuda.synchronize()
    assert rc == lb.OK and int(dW.view(torch.int32).count_nonzero()) == 0


def test_plane_post_passes_at_two_to_31_outputs():
    # lba_last_overflow and lba_ste_plane with M * N = 2^31 (their limit) and K = 32 (one word per output, so
    # the expected values follow from each word alone): last = index of the highest set bit or -1; immediate
    # coefficients = complement; recursive (sequential) coefficients = the bits above `last`
    M, N, K = 2 ** 20, 2 ** 11, 32
    torch.manual_seed(2036)
    of = torch.randint(-2 ** 31, 2 ** 31, (1, M, N), dtype=torch.int32, device=DEV)
    of &= torch.randint(-2 ** 31, 2 ** 31, (1, M, N), dtype=torch.int32, device=DEV)
    of &= torch.randint(-2 ** 31, 2 ** 31, (1, M, N), dtype=torch.int32, device=DEV)     # sparser bits
    of.view(-1)[::7] = 0                                                                   # chains without overflow
    last = lb.last_overflow(of, K)
    imm = lb.ste_plane(of, K, lb.STE_IMMEDIATE_OF)
    rec = lb.ste_plane(of, K, lb.STE_RECURSIVE_OF)
    torch.cuda.synchronize()
    fo, fl, fi, fr = of.view(-1), last.view(-1), imm.view(-1), rec.view(-1)
    step = 1 << 27
    for s in range(0, M * N, step):
        w = fo[s:s + step].long() & 0xFFFFFFFF
        want_last = torch.where(w == 0, torch.full_like(w, -1), torch.log2(w.double()).floor().long())
        assert torch.equal(fl[s:s + step].long(), want_last), s
        assert torch.equal(fi[s:s + step].long() & 0xFFFFFFFF, w ^ 0xFFFFFFFF), s
        want_rec = (torch.full_like(w, 0xFFFFFFFF) << (want_last + 1)) & 0xFFFFFFFF
        assert torch.equal(fr[s:s + step].long() & 0xFFFFFFFF, want_rec), s
    assert lb.lba_last_overflow(of.data_ptr(), last.data_ptr(), M + 1, N, K) == lb.ERR_SHAPE


def test_largest_batch(ref):
    # lba_gemm_batched with 65535 members (the limit) sharing B: equals one product on the stacked rows
    rng = np.random.default_rng(2037)
    batch, M, N, K = 65535, 5, 7, 19
    A = codes(rng, (batch, M, K), 3, 11); B = codes(rng, (N, K), 3, 11)
    for rnd in (0, 1):
        qp, qa = PROD + (rnd,), ACC + (rnd,)
        C = lb.gemm_batched(torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV), qp, qa)
        torch.cuda.synchronize()
        want = ref.gemm(A.reshape(batch * M, K), B, ref.QFmt(*qp), ref.QFmt(*qa))
        assert np.array_equal(bits(C.cpu().numpy().reshape(batch * M, N)), bits(want)), rnd
    assert lb.lba_gemm_batched(1, 1, 1, 65536, M * K, 0, M * N, M, N, K, PROD + (0,), ACC + (0,)) == lb.ERR_SHAPE


def test_convolution_descriptor_limits(ref):
    # lba_conv2d at the descriptor's limits: c = 2^14 - 1 (bytes gathered one by one), the largest c that takes
    # the 16-byte path, kw = 2^14 - 1, and kh * kw * c just below 2^24; complete outputs against the oracle on the
    # written-out im2col matrix.  The descriptors just outside are refused.
    rng = np.random.default_rng(2038)
    cases = [(1, 3, 3, 16383, 5, 1, 1, 1, 0), (1, 4, 4, 16368, 8, 1, 1, 1, 0), (1, 2, 16390, 1, 4, 1, 16383, 1, 0),
             (2, 127, 127, 1023, 3, 127, 127, 1, 0)]
    for (n, h, w, c, cout, kh, kw, stride, pad) in cases:
        X = codes(rng, (n, h, w, c), 3, 10); W = codes(rng, (cout, kh, kw, c), 3, 10)
        A = ref.im2col_nhwc(X, kh, kw, stride, pad)
        B = W.reshape(cout, kh * kw * c)
        for rnd in (0, 1):
            qp, qa = PROD + (rnd,), (5, 10, 15, rnd)
            Y = lb.conv2d(torch.from_numpy(X).to(DEV), torch.from_numpy(W).to(DEV), qp, qa, stride=stride, pad=pad)
            torch.cuda.synchronize()
            want = ref.gemm(A, B, ref.QFmt(*qp), ref.QFmt(*qa))
            assert np.array_equal(bits(Y.cpu().numpy().reshape(want.shape)), bits(want)), ((n, h, w, c, cout, kh, kw), rnd)
    assert lb.lba_conv2d_out_shape((1, 128, 128, 1024, 128, 128, 1, 0))[0] == lb.ERR_SHAPE    # kh * kw * c = 2^24
    assert lb.lba_conv2d_out_shape((1, 1, 1 << 14, 1, 1, 1 << 14, 1, 0))[0] == lb.ERR_SHAPE   # kw = 2^14
    assert lb.lba_conv2d_out_shape((1 << 16, 128, 128, 1, 1, 1, 1, 0))[0] == lb.ERR_SHAPE     # 2^30 rows
    assert lb.lba_conv2d_out_shape((1 << 16, 128, 128, 1, 2, 2, 1, 0))[0] == lb.OK
