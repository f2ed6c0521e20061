"""GPU parity of the implicit-im2col convolution (lba_conv2d, lba_conv2d_bwd) against the oracle run on the
explicitly written-out im2col matrix."""
import itertools

import numpy as np
import pytest
import torch

from paper_2401_14110_amd import binding as lb
from paper_2401_14110_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def codes(rng, shape, lo=0, hi=15):
    e = rng.integers(lo, hi + 1, shape); m = rng.integers(0, 8, shape); s = rng.integers(0, 2, shape)
    c = (s << 7) | (e << 3) | m
    return np.where((c & 0x7F) == 0x7F, c & 0xFE, c).astype(np.uint8)


def bits(x):
    return np.ascontiguousarray(x).view(np.uint32)


CASES = [  # n, h, w, c, cout, kh, kw, stride, pad
    (2, 12, 10, 16, 24, 3, 3, 1, 1),
    (3, 9, 11, 64, 70, 3, 3, 2, 1),
    (2, 14, 14, 32, 64, 1, 1, 2, 0),       # a downsample convolution
    (2, 20, 18, 3, 64, 7, 7, 2, 3),        # the stem: c = 3, bytes gathered one by one
    (1, 8, 8, 48, 5, 3, 3, 1, 0),
    (2, 7, 9, 20, 33, 3, 2, 1, 2),         # c % 16 != 0, padding wider than the filter's reach
    (1, 5, 5, 16, 16, 5, 5, 1, 2),
]


def test_out_shape_and_limits():
    assert lb.lba_conv2d_out_shape((32, 56, 56, 64, 3, 3, 1, 1)) == (lb.OK, 56, 56)
    assert lb.lba_conv2d_out_shape((64, 224, 224, 3, 7, 7, 2, 3)) == (lb.OK, 112, 112)
    assert lb.lba_conv2d_out_shape((1, 5, 5, 8, 7, 7, 1, 0))[0] == lb.ERR_SHAPE        # filter larger than the image
    assert lb.lba_conv2d_out_shape((1, 5, 5, 0, 3, 3, 1, 0))[0] == lb.ERR_SHAPE
    assert lb.lba_conv2d_out_shape((1, 5, 5, 1 << 14, 3, 3, 1, 1))[0] == lb.ERR_SHAPE
    assert lb.lba_conv2d_out_shape((1, 5, 5, 8, 3, 3, 0, 1))[0] == lb.ERR_SHAPE


@pytest.mark.parametrize("rnd", [0, 1])
def test_conv2d_against_explicit_im2col(ref, rnd):
    rng = np.random.default_rng(120 + rnd)
    for (n, h, w, c, cout, kh, kw, stride, pad) in CASES:
        X = codes(rng, (n, h, w, c), 3, 12); W = codes(rng, (cout, kh, kw, c), 3, 12)
        A = ref.im2col_nhwc(X, kh, kw, stride, pad)
        B = W.reshape(cout, kh * kw * c)
        tX, tW = torch.from_numpy(X).to(DEV), torch.from_numpy(W).to(DEV)
        for (qp, qa), order in itertools.product([((5, 7, 15), (4, 7, 7)), ((4, 7, 12), (4, 7, 10)), ((5, 4, 15), (4, 7, 7))], (0, 1)):
            qpf, qaf = qp + (rnd,), qa + (rnd,)
            Y = lb.conv2d(tX, tW, qpf, qaf, stride=stride, pad=pad, order=order)
            torch.cuda.synchronize()
            want = ref.gemm(A, B, ref.QFmt(*qpf), ref.QFmt(*qaf), order=order)
            assert Y.shape[-1] == cout and Y.numel() == want.size
            assert np.array_equal(bits(Y.cpu().numpy().reshape(want.shape)), bits(want)), ((n, h, w, c, cout, kh, kw, stride, pad), qpf, qaf, order)
            # and it is what lba_gemm gives on the written-out matrix
            C = lb.gemm(torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV), qpf, qaf, order=order)
            assert torch.equal(C, Y.reshape(C.shape))
        # the recompute call
        qpf, qaf = (5, 7, 15, rnd), (4, 7, 7, rnd)
        Y, of, uf = lb.conv2d(tX, tW, qpf, qaf, stride=stride, pad=pad, planes=True)
        torch.cuda.synchronize()
        wc, wof, wuf = ref.gemm_bwd(A, B, ref.QFmt(*qpf), ref.QFmt(*qaf))
        assert np.array_equal(bits(Y.cpu().numpy().reshape(wc.shape)), bits(wc))
        assert np.array_equal(of.cpu().numpy().view(np.uint32), wof) and np.array_equal(uf.cpu().numpy().view(np.uint32), wuf)


def test_conv2d_on_every_lane_block_and_on_mixed_grids(ref):
    # E4M3 tensors take the kernels of the row-major product with the gather in place of A's fetch, on the same
    # tiles and grids: 2 x 4 and 4 x 4 lane blocks, whole rounds of 48 x 64 workgroups with a 32 x 32 tail, and full
    # rounds of 64 x 64 followed by a round of 48 x 64 and the tail (the small cases above run the 2 x 2 block)
    rng = np.random.default_rng(126)
    seen, rounded = set(), set()
    for (n, h, w, c, cout, kh, kw, stride, pad), want_plan in [
            ((3, 76, 76, 16, 64, 3, 3, 1, 1), "2x4"), ((8, 64, 64, 16, 64, 1, 1, 1, 0), "4x4"),
            ((5, 23, 167, 16, 64, 3, 3, 1, 1), "mid"), ((4, 112, 112, 16, 256, 3, 3, 2, 1), "mid"),
            ((1, 625, 97, 16, 64, 3, 3, 1, 1), "main+mid"), ((1, 360, 383, 3, 60, 3, 3, 2, 1), "tail")]:
        X = codes(rng, (n, h, w, c), 3, 12); W = codes(rng, (cout, kh, kw, c), 3, 12)
        A = ref.im2col_nhwc(X, kh, kw, stride, pad)
        B = W.reshape(cout, kh * kw * c)
        tX, tW = torch.from_numpy(X).to(DEV), torch.from_numpy(W).to(DEV)
        for rnd, order in ((0, 0), (1, 0), (0, 1), (1, 1)):
            qpf, qaf = (5, 7, 15, rnd), (4, 7, 7, rnd)
            plan = lb.lba_plan_query(A.shape[0], cout, A.shape[1], qpf, qaf, order)
            main = plan["grid_x"] - plan["mid_blocks"] - plan["tail_blocks"]
            got = ("%dx%d" % (plan["thread_m"], plan["thread_n"]) if plan["mid_blocks"] + plan["tail_blocks"] == 0
                   else ("main+mid" if main > 0 and plan["mid_blocks"] > 0 else ("mid" if plan["mid_blocks"] > 0 else "tail")))
            assert plan["kernel"] == 0 and got == want_plan, (A.shape, cout, plan)
            seen.add(got)
            Y = lb.conv2d(tX, tW, qpf, qaf, stride=stride, pad=pad, order=order)
            torch.cuda.synchronize()
            want = ref.gemm(A, B, ref.QFmt(*qpf), ref.QFmt(*qaf), order=order)
            assert np.array_equal(bits(Y.cpu().numpy().reshape(want.shape)), bits(want)), ((n, h, w, c, cout, kh, kw, stride, pad), rnd, order)
        # a Q_prod that rounds the products (5 mantissa bits): the kernels for other operand formats, which gather
        # by themselves, on their mixed grids
        for rnd in (0, 1):
            qpf, qaf = (5, 4, 15, rnd), (4, 7, 7, rnd)
            plan = lb.lba_plan_query(A.shape[0], cout, A.shape[1], qpf, qaf, 0)
            assert plan["kernel"] == 0
            rounded.add((plan["grid_x"] - plan["mid_blocks"] - plan["tail_blocks"] > 0, plan["mid_blocks"] > 0, plan["tail_blocks"] > 0))
            Y = lb.conv2d(tX, tW, qpf, qaf, stride=stride, pad=pad)
            torch.cuda.synchronize()
            want = ref.gemm(A, B, ref.QFmt(*qpf), ref.QFmt(*qaf))
            assert np.array_equal(bits(Y.cpu().numpy().reshape(want.shape)), bits(want)), ((n, h, w, c, cout, kh, kw, stride, pad), qpf)
        # the recompute call: 4 x 4 workgroups, with the 32 x 32 tail where the forward call's grid has one
        qpf, qaf = (5, 7, 15, 0), (4, 7, 7, 0)
        plan = lb.lba_plan_query(A.shape[0], cout, A.shape[1], qpf, qaf, 0, 1)
        assert plan["kernel"] == 0 and plan["mid_blocks"] == 0
        seen.add("planes, tail" if plan["tail_blocks"] > 0 else "planes")
        Y, of, uf = lb.conv2d(tX, tW, qpf, qaf, stride=stride, pad=pad, planes=True)
        torch.cuda.synchronize()
        wc, wof, wuf = ref.gemm_bwd(A, B, ref.QFmt(*qpf), ref.QFmt(*qaf))
        assert np.array_equal(bits(Y.cpu().numpy().reshape(wc.shape)), bits(wc))
        assert np.array_equal(of.cpu().numpy().view(np.uint32), wof) and np.array_equal(uf.cpu().numpy().view(np.uint32), wuf)
        assert wof.any() and wuf.any()
    assert seen == {"2x4", "4x4", "mid", "main+mid", "tail", "planes", "planes, tail"}
    assert {(False, True, True), (True, True, True), (True, False, True)} <= rounded, rounded


def test_conv2d_unaligned_tensor_and_status_codes(ref):
    rng = np.random.default_rng(125)
    n, h, w, c, cout = 2, 10, 10, 32, 40
    X = codes(rng, (n, h, w, c), 3, 12); W = codes(rng, (cout, 3, 3, c), 3, 12)
    buf = torch.zeros(X.size + 3, dtype=torch.uint8, device=DEV)
    buf[3:] = torch.from_numpy(X).to(DEV).reshape(-1)
    tX = buf[3:].view(n, h, w, c)                                  # 3 bytes off a 16-byte boundary
    tW = torch.from_numpy(W).to(DEV)
    Y = lb.conv2d(tX, tW, (5, 7, 15, 0), (4, 7, 7, 0), stride=1, pad=1)
    torch.cuda.synchronize()
    want = ref.gemm(ref.im2col_nhwc(X, 3, 3, 1, 1), W.reshape(cout, -1), ref.QFmt(5, 7, 15, 0), ref.QFmt(4, 7, 7, 0))
    assert np.array_equal(bits(Y.cpu().numpy().reshape(want.shape)), bits(want))
    d = (n, h, w, c, 3, 3, 1, 1)
    y = Y.data_ptr()
    assert lb.lba_conv2d(None, tW.data_ptr(), y, d, cout, (5, 7, 15, 0), (4, 7, 7, 0)) == lb.ERR_NULL
    assert lb.lba_conv2d(tX.data_ptr(), tW.data_ptr(), y, (n, h, w, c, 13, 3, 1, 1), cout, (5, 7, 15, 0), (4, 7, 7, 0)) == lb.ERR_SHAPE
    assert lb.lba_conv2d(tX.data_ptr(), tW.data_ptr(), y, d, cout, (5, 0, 15, 0), (4, 7, 7, 0)) == lb.ERR_FORMAT
    assert lb.lba_conv2d_bwd(tX.data_ptr(), tW.data_ptr(), y, y, None, d, cout, (5, 7, 15, 0), (4, 7, 7, 0), order=1) == lb.ERR_UNSUPPORTED


def test_resnet18_conv_at_full_size(ref):
    # the benchmark's conv configuration from its NHWC activation tensor: batch 32, 56 x 56 x 64, 3 x 3, 64 filters;
    # sampled output pixels against the oracle (their im2col rows are written out on the host)
    n, h, w, c, cout = 32, 56, 56, 64, 64
    X, ta = inputs.make_operand("relu", n * h * w, c, 1, 0, device=DEV)
    Wt, tb = inputs.make_operand("normal", cout, 9 * c, 1, 1, device=DEV, std=(2.0 / (9 * c)) ** 0.5)
    qp, qa, _ = inputs.folded_formats(ta, tb, (5, 7, 15), (4, 7, 7), 0)
    tX = X.view(n, h, w, c)
    Y = lb.conv2d(tX, Wt.view(cout, 3, 3, c), qp, qa, stride=1, pad=1)
    torch.cuda.synchronize()
    Yh = Y.cpu().numpy().reshape(n * h * w, cout)
    Xh = tX.cpu().numpy()
    rng = np.random.default_rng(3)
    rows = sorted(set([0, 1, 55, 56, 57, h * w - 1, h * w, n * h * w - 1]) | set(int(r) for r in rng.integers(0, n * h * w, 40)))
    A = np.zeros((len(rows), 9 * c), dtype=np.uint8)
    for t, r in enumerate(rows):
        img, rem = divmod(r, h * w)
        oh, ow = divmod(rem, w)
        for i in range(3):
            for j in range(3):
                ih, iw = oh - 1 + i, ow - 1 + j
                if 0 <= ih < h and 0 <= iw < w:
                    A[t, (i * 3 + j) * c:(i * 3 + j + 1) * c] = Xh[img, ih, iw]
    want = ref.gemm(A, Wt.cpu().numpy(), ref.QFmt(*qp), ref.QFmt(*qa))
    assert np.array_equal(bits(Yh[rows]), bits(want))
    assert np.count_nonzero(want) > want.size // 2


def im2col_rows(Xh, rows, desc, oh_ow):
    """The im2col rows `rows` of the NHWC tensor Xh, written out on the host (k = (i*kw + j)*c + ch, +0 outside)."""
    n, h, w, c, kh, kw, stride, pad = desc
    oh_n, ow_n = oh_ow
    A = np.zeros((len(rows), kh * kw * c), dtype=np.uint8)
    for t, r in enumerate(rows):
        img, rem = divmod(r, oh_n * ow_n)
        oh, ow = divmod(rem, ow_n)
        for i in range(kh):
            for j in range(kw):
                ih, iw = oh * stride - pad + i, ow * stride - pad + j
                if 0 <= ih < h and 0 <= iw < w:
                    A[t, (i * kw + j) * c:(i * kw + j + 1) * c] = Xh[img, ih, iw]
    return A


def test_resnet50_convolutions_at_full_size(ref):
    # every distinct convolution of the benchmark's ResNet-50 sweep from its NHWC tensor, in the launch configuration
    # bench.py --implicit times: sampled output pixels (first and last rows, the rows around the seams of the mixed
    # grid's regions, random ones) against the oracle on their written-out im2col rows; for three layers (the stem
    # with its byte-wise gather, a strided 3 x 3 layer, a layer whose recompute grid is mixed) also the recompute call
    layers = inputs.make_conv_workload("resnet50", DEV)
    rng = np.random.default_rng(7)
    seen, with_planes, hosts = set(), 0, {}
    for l in layers:
        key = (l["desc"], l["cout"])
        if key in seen:
            continue
        seen.add(key)
        n, h, w, c, kh, kw, stride, pad = l["desc"]
        M, N, K = l["M"], l["N"], l["K"]
        rc, oh, ow = lb.lba_conv2d_out_shape(l["desc"])
        assert rc == lb.OK and n * oh * ow == M
        qp, qa, _ = inputs.folded_formats(l["ta"], l["tb"], (5, 7, 15), (4, 7, 7), 0)
        plan = lb.lba_plan_query(M, N, K, qp, qa, 0)
        main_rows = 64 * ((plan["grid_x"] - plan["mid_blocks"] - plan["tail_blocks"]) // max(1, (N + 63) // 64))
        mid_rows = main_rows + 48 * (plan["mid_blocks"] // max(1, (N + 63) // 64))
        rows = {0, 1, M - 1, M - 2, ow - 1, ow, oh * ow - 1, oh * ow % M}
        for seam in (main_rows, mid_rows):
            rows |= {r for r in range(seam - 2, seam + 3) if 0 <= r < M}
        rows |= set(int(r) for r in rng.integers(0, M, 24))
        rows = sorted(rows)
        xk = id(l["X"])
        if xk not in hosts:
            hosts = {xk: l["X"].cpu().numpy()}                   # one tensor on the host at a time
        A = im2col_rows(hosts[xk], rows, l["desc"], (oh, ow))
        Bh = l["B"].cpu().numpy()
        Wt = l["B"].view(N, kh, kw, c)
        planes = l["name"] in ("conv1", "layer2.0.conv2", "layer3.0.conv2")
        if planes:
            Y, of, uf = lb.conv2d(l["X"], Wt, qp, qa, stride=stride, pad=pad, planes=True)
            torch.cuda.synchronize()
            wc, wof, wuf = ref.gemm_bwd(A, Bh, ref.QFmt(*qp), ref.QFmt(*qa))
            idx = torch.tensor(rows, device=DEV)
            assert np.array_equal(of[:, idx, :].cpu().numpy().view(np.uint32), wof), l["name"]
            assert np.array_equal(uf[:, idx, :].cpu().numpy().view(np.uint32), wuf), l["name"]
            assert wuf.any()
            with_planes += 1
            del of, uf
        else:
            Y = lb.conv2d(l["X"], Wt, qp, qa, stride=stride, pad=pad)
            torch.cuda.synchronize()
            wc = ref.gemm(A, Bh, ref.QFmt(*qp), ref.QFmt(*qa))
        got = Y.view(M, N)[torch.tensor(rows, device=DEV)].cpu().numpy()
        assert np.array_equal(bits(got), bits(wc)), (l["name"], l["desc"])
        assert np.count_nonzero(wc) > wc.size // 4, l["name"]
        del Y
    assert len(seen) >= 20 and with_planes == 3
