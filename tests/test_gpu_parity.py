"""GPU parity: the HIP library (called through the C ABI binding) against the CPU oracle, element
by element and bit for bit, on the same seeded inputs.  Run with -m gpu on an MI355X."""
import itertools
import os
import random

import numpy as np
import pytest
import torch

from paper_2401_14110_amd import binding as lb
from paper_2401_14110_amd import inputs

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def fm(ref, f):
    return ref.QFmt(*f)


def rand_codes(rng, shape, lo_e=0, hi_e=15, nan_free=True):
    e = rng.integers(lo_e, hi_e + 1, shape)
    m = rng.integers(0, 8, shape)
    s = rng.integers(0, 2, shape)
    c = (s << 7) | (e << 3) | m
    if nan_free:
        c = np.where((c & 0x7F) == 0x7F, c & 0xFE, c)
    return c.astype(np.uint8)


def bits(x):
    return np.ascontiguousarray(x).view(np.uint32)


def run_gpu(A, B, qp, qa, order=0):
    C = lb.gemm(torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV), qp, qa, order=order)
    torch.cuda.synchronize()
    return C.cpu().numpy()


def check(ref, A, B, qp, qa, what="", order=0):
    got = run_gpu(A, B, qp, qa, order)
    want = ref.gemm(A, B, fm(ref, qp), fm(ref, qa), order=order)
    bad = bits(got) != bits(want)
    if bad.any():
        i, j = np.argwhere(bad)[0]
        raise AssertionError("%s qp=%s qa=%s shape=%s: %d mismatches, first at [%d,%d]: gpu %r oracle %r (plan %s)"
                             % (what, qp, qa, (A.shape, B.shape), int(bad.sum()), i, j, got[i, j], want[i, j],
                                lb.lba_plan_query(A.shape[0], B.shape[0], A.shape[1], qp, qa)))
    return got


# formats: (qprod, qacc) as (E, M, b); rounding appended per test
FMT_PAPER = [((5, 7, 15), (4, 7, 7)),        # default biases in real units
             ((5, 7, -1), (4, 7, -9)),       # the same moved into code units of scaled operands
             ((4, 7, 12), (4, 7, 10)),       # b_acc, b_prod = 10, 12 (Sec. 3.1)
             ((4, 7, 9), (4, 7, 7)),         # 7, 9 (Table 4)
             ((6, 7, 20), (4, 7, 7))]        # Q_prod cannot change a product: fused path
FMT_SWEEP = [((5, 7, 15), (E, M, (1 << (E - 1)) - 1)) for M in (3, 5, 8, 10) for E in (4, 5, 6)]
FMT_ODD = [((5, 4, 15), (4, 7, 7)),          # product mantissa is rounded
           ((3, 4, 6), (3, 4, 6)),           # 8-bit accumulator M4E3 (Sec. 4), b = 6 (App. C.4)
           ((3, 4, 5), (3, 4, 5)),           # b = 5 (App. C.3)
           ((5, 9, 15), (4, 8, 7)),          # wider product mantissa than accumulator
           ((5, 7, 40), (4, 7, -9)),         # products far below the accumulator's range
           ((7, 23, 64), (7, 23, 64)),       # widest formats
           ((5, 7, 15), (4, 22, 7)), ((5, 7, 15), (4, 23, 7)), ((5, 7, 15), (5, 11, 15)),
           ((2, 1, 0), (2, 1, 0)), ((7, 7, 126), (7, 7, 126)), ((4, 7, -112), (4, 7, -112)),
           ((5, 7, -30), (4, 7, 7)), ((5, 7, 15), (4, 7, -30))]


def test_k1_every_code_pair(ref):
    # C[a, b] = Q_acc(Q_prod(a * b)) for all 256 x 256 codes (NaN codes included: read as +-480)
    codes = np.arange(256, dtype=np.uint8).reshape(256, 1)
    for (qp, qa), rnd in itertools.product(FMT_PAPER + FMT_SWEEP[::3] + FMT_ODD, (0, 1)):
        check(ref, codes, codes, qp + (rnd,), qa + (rnd,), "K=1")


def test_hand_worked_chain_and_exact_sum(ref):
    tab = [l.split("#")[0].split() for l in open(os.path.join(GOLD, "chain_p1b.txt"))]
    tab = [r for r in tab if r]
    a = np.array([[int(r[1], 16) for r in tab]], dtype=np.uint8)
    b = np.array([[int(r[2], 16) for r in tab]], dtype=np.uint8)
    for rnd, col in ((0, 3), (1, 6)):
        for k in range(1, 5):
            got = run_gpu(a[:, :k], b[:, :k], (5, 7, 16, rnd), (4, 7, 7, rnd))
            assert got[0, 0] == float(tab[k - 1][col])
    # 256 - 2^-18: floor must give 255 (sum exact before rounding), nearest-even 256
    a = np.array([[0x58, 0x81]], dtype=np.uint8)
    b = np.array([[0x58, 0x01]], dtype=np.uint8)
    assert run_gpu(a, b, (5, 7, 18, 0), (4, 7, 7, 0))[0, 0] == 255.0
    assert run_gpu(a, b, (5, 7, 18, 1), (4, 7, 7, 1))[0, 0] == 256.0


def test_config1_single_gemm(ref):
    # M = N = 64, K = 256, N(0,1) operands scaled to max|x| = 448, seed 0; Q_prod 1-5-7, Q_acc 1-4-7
    A = inputs.normal(0, 0, 64 * 256)
    B = inputs.normal(0, 1, 64 * 256)
    Ac, ta = inputs.quantize_tensor(A, "exact448")
    Bc, tb = inputs.quantize_tensor(B, "exact448")
    Ac = Ac.reshape(64, 256).numpy(); Bc = Bc.reshape(64, 256).numpy()
    for rnd in (1, 0):
        # biases as written (code units: saturates nearly everywhere) and folded to real units
        check(ref, Ac, Bc, (5, 7, 15, rnd), (4, 7, 7, rnd), "config1 literal")
        qp, qa, _ = inputs.folded_formats(ta, tb, rnd=rnd)
        got = check(ref, Ac, Bc, qp, qa, "config1 folded")
        assert np.count_nonzero(got) > 3000


SHAPES = [(1, 1, 1), (3, 5, 7), (17, 9, 31), (65, 67, 33), (130, 70, 147), (257, 129, 100), (64, 1000, 64),
          (200, 64, 576), (128, 128, 16), (129, 257, 48), (64, 64, 1025)]


@pytest.mark.parametrize("rnd", [0, 1])
def test_ragged_shapes_paper_formats(ref, rnd):
    rng = np.random.default_rng(20 + rnd)
    for (M, N, K) in SHAPES:
        A = rand_codes(rng, (M, K), 3, 12)
        B = rand_codes(rng, (N, K), 3, 12)
        for qp, qa in FMT_PAPER:
            check(ref, A, B, qp + (rnd,), qa + (rnd,), "ragged")


@pytest.mark.parametrize("rnd", [0, 1])
def test_accumulator_width_sweep_and_odd_formats(ref, rnd):
    rng = np.random.default_rng(30 + rnd)
    A = rand_codes(rng, (150, 200)); B = rand_codes(rng, (70, 200))
    A2 = rand_codes(rng, (70, 96), 5, 10); B2 = rand_codes(rng, (66, 96), 5, 10)
    for qp, qa in FMT_SWEEP + FMT_ODD:
        check(ref, A, B, qp + (rnd,), qa + (rnd,), "sweep full-range operands")
        check(ref, A2, B2, qp + (rnd,), qa + (rnd,), "sweep mid-range operands")


def test_synthetic_workload_distributions(ref):
    # ReLU activations x Kaiming weights (conv as im2col) and N(0,1) x N(0,0.02) (BERT linear),
    # power-of-two per-tensor scaling, biases folded; sizes span several tiles with ragged tails
    for kind_a, std_b, (M, N, K), seed in (("relu", None, (300, 64, 576), 2), ("relu", None, (200, 130, 147), 3),
                                           ("normal", 0.02, (260, 200, 768), 4)):
        std = (2.0 / K) ** 0.5 if std_b is None else std_b
        A, ta = inputs.make_operand(kind_a, M, K, seed, 0)
        B, tb = inputs.make_operand("normal", N, K, seed, 1, std=std)
        for rnd in (0, 1):
            qp, qa, _ = inputs.folded_formats(ta, tb, rnd=rnd)
            got = check(ref, A.numpy(), B.numpy(), qp, qa, "workload")
            assert np.count_nonzero(got) > got.size // 2


@pytest.mark.parametrize("rnd", [0, 1])
def test_chunked_order(ref, rnd):
    # chunks of 16 then a second-level chain (Sec. 3): K below, at and across chunk and tile
    # boundaries, fast and general kernels, saturating and non-saturating formats
    rng = np.random.default_rng(60 + rnd)
    for (M, N, K) in [(5, 7, 1), (9, 3, 15), (17, 9, 16), (33, 20, 17), (65, 67, 31), (70, 64, 32), (64, 70, 33),
                      (130, 66, 48), (40, 40, 147), (66, 130, 576)]:
        A = rand_codes(rng, (M, K), 3, 12)
        B = rand_codes(rng, (N, K), 3, 12)
        for qp, qa in FMT_PAPER + [FMT_ODD[0], FMT_ODD[1], FMT_ODD[3], FMT_SWEEP[0], FMT_SWEEP[5], FMT_ODD[5]]:
            check(ref, A, B, qp + (rnd,), qa + (rnd,), "chunk16", order=1)
    A, ta = inputs.make_operand("relu", 200, 576, 5, 0)
    B, tb = inputs.make_operand("normal", 64, 576, 5, 1, std=(2.0 / 576) ** 0.5)
    # the paper's bias pairs (b_acc, b_prod) = (10, 12), (7, 9), (8, 10) in real units, folded
    for ba, bp in ((10, 12), (7, 9), (8, 10)):
        qp, qa, _ = inputs.folded_formats(ta, tb, (4, 7, bp), (4, 7, ba), rnd)
        got = check(ref, A.numpy(), B.numpy(), qp, qa, "chunk16 paper biases", order=1)
        assert np.count_nonzero(got) > got.size // 2


def test_chunked_order_with_chunks_side_by_side(ref):
    # launches with few outputs run several chunks of an output side by side (first-level chains are independent;
    # the second level stays an ordered chain): ragged K below, at and across the depth of a k-tile of each shape of
    # that kernel (64 and 256), ragged M and N, both workgroup shapes, clamped and clamp-free first levels,
    # both roundings and the bfloat16 shortcut (M = 7), every product mode.  Bit for bit the oracle's chunked order.
    rng = np.random.default_rng(161)
    shapes = [(70, 66), (5, 3), (33, 130), (300, 200), (1100, 530), (17, 1000)]
    seen = set()
    for (M, N) in shapes:
        for K in (17, 147, 530, 64, 127, 256, 1100):
            if M * N * K > 4e8:
                continue
            A = rand_codes(rng, (M, K), 2, 13); B = rand_codes(rng, (N, K), 2, 13)
            for qp, qa in [((5, 7, 15), (4, 7, 7)), ((4, 7, 12), (4, 7, 10)), ((6, 7, 20), (6, 7, 31)), ((5, 7, 15), (5, 10, 15)),
                           ((6, 7, 20), (4, 5, 7)), ((5, 7, -1), (4, 7, -9))]:
                for rnd in (0, 1):
                    qpf, qaf = qp + (rnd,), qa + (rnd,)
                    name = lb.lba_plan_kernel_name(M, N, K, qpf, qaf, 1, 0)
                    if "kpar" not in name:
                        continue
                    seen.add(name)
                    check(ref, A, B, qpf, qaf, "chunks side by side %s" % name, order=1)
    shapes_seen = {n.split("<")[1].split(",")[0] + n.split(",")[2] for n in seen}
    assert shapes_seen == {"4 1", "2 4"}, seen
    assert {n.rstrip(">").split(", ")[3] for n in seen} == {"0", "1", "2"} and {n.rstrip(">").split(", ")[4] for n in seen} == {"0", "1", "2"}, seen


def test_no_underflow_flag(ref):
    # FMAq "excluding underflow events" (Sec. 3): the flag on either quantizer or both, all kernels
    NOUF = 0x100
    rng = np.random.default_rng(80)
    A = rand_codes(rng, (90, 150), 0, 12); B = rand_codes(rng, (70, 150), 0, 12)
    A2 = rand_codes(rng, (40, 64), 0, 6); B2 = rand_codes(rng, (50, 64), 0, 6)          # mostly below R_UF
    for (qp, qa), rnd, (fp, fa), order in itertools.product(
            [FMT_PAPER[0], FMT_PAPER[1], FMT_PAPER[2], FMT_PAPER[4], FMT_ODD[0], FMT_ODD[1], FMT_SWEEP[0], FMT_SWEEP[11]],
            (0, 1), ((NOUF, 0), (0, NOUF), (NOUF, NOUF)), (0, 1)):
        check(ref, A, B, qp + (rnd | fp,), qa + (rnd | fa,), "no-underflow", order=order)
        check(ref, A2, B2, qp + (rnd | fp,), qa + (rnd | fa,), "no-underflow small", order=order)
    # event planes with the flag
    for (qp, qa), rnd, (fp, fa) in itertools.product([FMT_PAPER[0], FMT_PAPER[1], FMT_ODD[1]], (0, 1),
                                                     ((NOUF, 0), (0, NOUF), (NOUF, NOUF))):
        qpf, qaf = qp + (rnd | fp,), qa + (rnd | fa,)
        C, of, uf = lb.gemm_bwd(torch.from_numpy(A2).to(DEV), torch.from_numpy(B2).to(DEV), qpf, qaf)
        torch.cuda.synchronize()
        wc, wof, wuf = ref.gemm_bwd(A2, B2, fm(ref, qpf), fm(ref, qaf))
        assert np.array_equal(bits(C.cpu().numpy()), bits(wc)), (qpf, qaf)
        assert np.array_equal(of.cpu().numpy().view(np.uint32), wof), (qpf, qaf)
        assert np.array_equal(uf.cpu().numpy().view(np.uint32), wuf), (qpf, qaf)
    # at a workload's scale: ReLU x Kaiming with folded biases, the paper's first fine-tuning stage
    A, ta = inputs.make_operand("relu", 300, 576, 6, 0)
    B, tb = inputs.make_operand("normal", 128, 576, 6, 1, std=(2.0 / 576) ** 0.5)
    qp, qa, _ = inputs.folded_formats(ta, tb, (4, 7, 12), (4, 7, 10), 0)
    qp = qp[:3] + (qp[3] | NOUF,); qa = qa[:3] + (qa[3] | NOUF,)
    for order in (0, 1):
        check(ref, A.numpy(), B.numpy(), qp, qa, "no-underflow workload", order=order)


def test_batched_products(ref):
    # attention-shaped batched products (scores Q.K^T and context P.V as A.B^T), a shared B, and
    # strides that break 16-byte alignment
    rng = np.random.default_rng(90)
    for (batch, M, N, K), shared in (((12, 128, 128, 64), False), ((12, 128, 64, 128), False),
                                     ((5, 70, 33, 50), False), ((7, 40, 66, 96), True)):
        A = rand_codes(rng, (batch, M, K), 3, 11)
        B = rand_codes(rng, (N, K) if shared else (batch, N, K), 3, 11)
        for (qp, qa), rnd, order in itertools.product([FMT_PAPER[1], FMT_PAPER[3], FMT_ODD[1]], (0, 1), (0, 1)):
            qpf, qaf = qp + (rnd,), qa + (rnd,)
            C = lb.gemm_batched(torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV), qpf, qaf, order=order)
            torch.cuda.synchronize()
            got = C.cpu().numpy()
            for z in range(batch):
                want = ref.gemm(A[z], B if shared else B[z], fm(ref, qpf), fm(ref, qaf), order=order)
                assert np.array_equal(bits(got[z]), bits(want)), (batch, M, N, K, shared, qpf, qaf, order, z)
    # batch limits and the empty batch
    d = torch.zeros((1, 8, 8), dtype=torch.uint8, device=DEV)
    assert lb.lba_gemm_batched(d.data_ptr(), d.data_ptr(), None, 0, 64, 64, 64, 8, 8, 8, (5, 7, 15, 0), (4, 7, 7, 0)) == lb.OK
    assert lb.lba_gemm_batched(d.data_ptr(), d.data_ptr(), None, 65536, 64, 64, 64, 8, 8, 8, (5, 7, 15, 0), (4, 7, 7, 0)) == lb.ERR_SHAPE
    assert lb.lba_gemm_batched(d.data_ptr(), d.data_ptr(), None, 2, -1, 64, 64, 8, 8, 8, (5, 7, 15, 0), (4, 7, 7, 0)) == lb.ERR_SHAPE


def test_every_lane_block(ref):
    # output counts that select each lane block of the fast kernel (2x2, 2x4, 4x4), ragged on both
    # sides, both roundings and both orders; all outputs compared.  The smallest grids of the sequential order take
    # 32 x 16 tiles (2 x 1 per lane) throughout.
    rng = np.random.default_rng(70)
    small = set()
    for (M, N, K), want_tile in (((130, 70, 70), (32, 16)), ((700, 650, 70), (32, 32)), ((1530, 2045, 70), (32, 64)),
                                 ((2100, 2110, 70), (64, 64))):
        A = rand_codes(rng, (M, K), 3, 12)
        B = rand_codes(rng, (N, K), 3, 12)
        for (qp, qa), rnd, order in itertools.product([FMT_PAPER[1], FMT_PAPER[3], FMT_PAPER[4]], (0, 1), (0, 1)):
            plan = lb.lba_plan_query(M, N, K, qp + (rnd,), qa + (rnd,), order)
            assert plan["kernel"] == 0
            if want_tile == (32, 16):
                if order == 0 and plan["tail_blocks"] > 0:         # (the chunked order has the K-parallel kernel there;
                    assert plan["tail_blocks"] == 5 * 5 == plan["grid_x"]      # formats with two sums per step keep 2 x 2)
                    small.add(rnd)
            else:
                assert (plan["tile_m"], plan["tile_n"]) == want_tile
            check(ref, A, B, qp + (rnd,), qa + (rnd,), "lane block %s" % (want_tile,), order=order)
    assert small == {0, 1}


TINY = [0x00, 0x80, 0x01, 0x81, 0x08, 0x38, 0xB8, 0x39, 0x3F, 0x47, 0x58, 0xDA, 0x7E, 0xFE, 0x77, 0x0F]


def test_brute_force_short_sequences(ref):
    # every pair of the 16-code subset at K = 2 against every other pair (65536 chains), and random
    # K = 3, 4 sequences: all outputs of the cross product are compared
    pairs = np.array(list(itertools.product(TINY, TINY)), dtype=np.uint8)          # [256, 2]
    rnd_gen = random.Random(5)
    seq3 = np.array([[rnd_gen.choice(TINY) for _ in range(3)] for _ in range(300)], dtype=np.uint8)
    seq4 = np.array([[rnd_gen.choice(TINY) for _ in range(4)] for _ in range(300)], dtype=np.uint8)
    for (qp, qa), rnd in itertools.product([FMT_PAPER[0], FMT_PAPER[1], FMT_ODD[1], FMT_ODD[3], FMT_SWEEP[0]], (0, 1)):
        for S in (pairs, seq3, seq4):
            check(ref, S, S, qp + (rnd,), qa + (rnd,), "brute")


def test_unaligned_pointers_and_views(ref):
    rng = np.random.default_rng(40)
    for K in (16, 64, 147, 50):
        base_a = torch.from_numpy(rand_codes(rng, (40 * K + 13,), 4, 11)).to(DEV)
        base_b = torch.from_numpy(rand_codes(rng, (33 * K + 7,), 4, 11)).to(DEV)
        for oa, ob in ((0, 0), (1, 3), (5, 2), (13, 7)):
            A = base_a[oa:oa + 40 * K].view(40, K)
            B = base_b[ob:ob + 33 * K].view(33, K)
            Cbuf = torch.empty(40 * 33 + 3, dtype=torch.float32, device=DEV)
            C = Cbuf[1:1 + 40 * 33].view(40, 33)               # 4-byte aligned only
            lb.gemm(A, B, (5, 7, 15, 0), (4, 7, 7, 0), out=C)
            torch.cuda.synchronize()
            want = ref.gemm(A.cpu().numpy(), B.cpu().numpy(), ref.QFmt(5, 7, 15, 0), ref.QFmt(4, 7, 7, 0))
            assert np.array_equal(bits(C.cpu().numpy()), bits(want)), (K, oa, ob)


def test_degenerate_sizes(ref):
    A = torch.zeros((5, 0), dtype=torch.uint8, device=DEV)
    B = torch.zeros((7, 0), dtype=torch.uint8, device=DEV)
    C = torch.full((5, 7), 3.0, device=DEV)
    lb.gemm(A, B, (5, 7, 15, 0), (4, 7, 7, 0), out=C)
    torch.cuda.synchronize()
    assert (C.cpu().numpy().view(np.uint32) == 0).all()                 # K = 0: +0 everywhere
    E = torch.zeros((0, 9), dtype=torch.uint8, device=DEV)
    assert lb.gemm(E, torch.zeros((4, 9), dtype=torch.uint8, device=DEV), (5, 7, 15, 0), (4, 7, 7, 0)).shape == (0, 4)
    # all-zero operands, negative zeros
    Z = np.full((70, 40), 0x80, dtype=np.uint8)
    got = check(ref, Z, Z, (5, 7, 15, 0), (4, 7, 7, 0), "zeros")
    assert (bits(got) == 0).all()
    # maximum-magnitude operands: saturates at once
    X = np.full((66, 40), 0x7E, dtype=np.uint8)
    got = check(ref, X, X, (5, 7, 15, 1), (4, 7, 7, 1), "max")
    assert (got == 510.0).all()


def test_event_planes_and_c_of_the_recompute_call(ref):
    rng = np.random.default_rng(50)
    cases = [((70, 66, 100), 0, 15), ((33, 130, 64), 3, 12), ((5, 3, 31), 0, 15), ((64, 64, 33), 5, 10)]
    for (M, N, K), lo, hi in cases:
        A = rand_codes(rng, (M, K), lo, hi); B = rand_codes(rng, (N, K), lo, hi)
        for (qp, qa), rnd in itertools.product([FMT_PAPER[0], FMT_PAPER[1], FMT_ODD[1], FMT_ODD[0], FMT_SWEEP[1]], (0, 1)):
            qpf, qaf = qp + (rnd,), qa + (rnd,)
            C, of, uf = lb.gemm_bwd(torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV), qpf, qaf)
            torch.cuda.synchronize()
            wc, wof, wuf = ref.gemm_bwd(A, B, fm(ref, qpf), fm(ref, qaf))
            assert np.array_equal(bits(C.cpu().numpy()), bits(wc)), (M, N, K, qpf, qaf)
            assert np.array_equal(of.cpu().numpy().view(np.uint32), wof), (M, N, K, qpf, qaf, "OF")
            assert np.array_equal(uf.cpu().numpy().view(np.uint32), wuf), (M, N, K, qpf, qaf, "UF")
            fwd = run_gpu(A, B, qpf, qaf)                                  # same C as the forward call
            assert np.array_equal(bits(fwd), bits(wc))
    # planes alone, one plane alone
    A = torch.from_numpy(rand_codes(rng, (20, 40))).to(DEV); B = torch.from_numpy(rand_codes(rng, (24, 40))).to(DEV)
    C, of, uf = lb.gemm_bwd(A, B, (5, 7, 15, 0), (4, 7, 7, 0), want_c=False)
    torch.cuda.synchronize()
    _, wof, wuf = ref.gemm_bwd(A.cpu().numpy(), B.cpu().numpy(), ref.QFmt(5, 7, 15, 0), ref.QFmt(4, 7, 7, 0))
    assert C is None and np.array_equal(of.cpu().numpy().view(np.uint32), wof)
    assert np.array_equal(uf.cpu().numpy().view(np.uint32), wuf)


def test_nearest_even_below_seven_mantissa_bits_keeps_ties_right(ref):
    # K = 2 chains: a first product of any small size, then every product of two codes (many are exact
    # midpoints of a 4..7-bit grid): the tie must be broken by the small partial sum, also when that sum
    # is far below the 24-bit window of the add.  Formats on both sides of the planner's exactness rule.
    rng = np.random.default_rng(70)
    codes = np.arange(256, dtype=np.uint8)
    codes = np.where((codes & 0x7F) == 0x7F, codes & 0xFE, codes).astype(np.uint8)
    A = np.stack([rand_codes(rng, (256,), 0, 6), codes], axis=1)
    B = np.stack([rand_codes(rng, (256,), 0, 6), codes], axis=1)
    variants = set()
    for qp, qa in [((5, 7, 15), (4, 3, 7)), ((5, 7, 15), (4, 6, 7)), ((5, 7, 18), (4, 5, 7)), ((5, 7, 15), (5, 4, 15)),
                   ((5, 7, 15), (6, 6, 31)), ((6, 7, 20), (5, 3, -2)), ((5, 7, 4), (4, 4, -6)), ((4, 7, 7), (4, 5, 7)),
                   ((4, 9, 7), (4, 6, 7)), ((5, 7, 15), (3, 6, 2)), ((5, 7, 15), (7, 5, 40))]:
        qpf, qaf = qp + (1,), qa + (1,)
        plan = lb.lba_plan_query(256, 256, 2, qpf, qaf)
        plain = lb.lba_plan_query(256, 256, 2, qpf, (4, 8, 7, 1))          # a format that needs one FP32 rounding only
        variants.add((plan["kernel"], plan["valu_per_mac_x100"] - plain["valu_per_mac_x100"]))
        check(ref, A, B, qpf, qaf, "rne small M, K=2")
        check(ref, A, B, qpf, qaf, "rne small M, K=2, chunked", order=1)
        check(ref, A, B, qpf, (qa[0], qa[1], qa[2], 0x101), "rne small M, no underflow")
    assert {(0, 0), (0, 400)} <= variants                   # the plain scaled kernel and its two-directed-sums variant
    # mantissas between 11 and 21 bits take that variant too (22 and 23: the general kernel)
    for qa in ((5, 11, 15), (4, 16, 7), (5, 21, 15), (6, 13, 31), (4, 22, 7)):
        check(ref, A, B, (5, 7, 15, 1), qa + (1,), "rne wide M, K=2")
    # longer chains with the full exponent range
    A = rand_codes(rng, (130, 100)); B = rand_codes(rng, (70, 100))
    for M in (3, 4, 5, 6, 12, 19, 21):
        for E, b in ((4, 7), (4, 0), (4, -6), (5, 15), (3, 3), (6, 31)):
            check(ref, A, B, (5, 7, 15, 1), (E, M, b, 1), "rne M=%d" % M)
            if M in (5, 12):
                check(ref, A, B, (5, 7, 15, 1), (E, M, b, 1), "rne M=%d chunked" % M, order=1)
                check(ref, A, B, (6, 7, 20, 1), (E, M, b, 1), "rne M=%d, Q_prod identity" % M)


def test_random_formats(ref):
    # a seeded sweep over the whole format space the ABI admits (E 2..7, M 1..23, biases that keep every value an
    # FP32 normal, both roundings, the no-underflow flag, both orders): whichever kernel the planner picks
    # (scaled, its round-to-odd variant, general) must give the oracle's bits
    rng = np.random.default_rng(2024)
    pyr = random.Random(2024)
    A = rand_codes(rng, (40, 70)); B = rand_codes(rng, (36, 70))
    picked = set()
    done = 0
    while done < 90:
        fmts = []
        for _ in range(2):
            E = pyr.randint(2, 7); M = pyr.choice([1, 2, 3, 4, 5, 6, 7, 8, 10, 11, 13, 16, 20, 21, 22, 23])
            lo, hi = (1 << E) - 128, 126                       # 2^E - b - 1 <= 127 and b <= 126
            b = pyr.randint(max(lo, -20), min(hi, 40))
            fmts.append((E, M, b))
        rnd = pyr.randint(0, 1)
        flags = pyr.choice([0, 0, 0, 0x100])
        qpf, qaf = fmts[0] + (rnd | flags,), fmts[1] + (rnd | pyr.choice([0, 0, 0, 0x100]),)
        order = pyr.randint(0, 1)
        try:
            plan = lb.lba_plan_query(40, 36, 70, qpf, qaf, order)
        except lb.LbaError:
            continue
        picked.add((plan["kernel"], rnd, plan["valu_per_mac_x100"] >= 1000))
        check(ref, A, B, qpf, qaf, "random format %d" % done, order=order)
        done += 1
    assert {(0, 0, False), (0, 1, False), (0, 1, True), (1, 1, True)} <= picked, picked


def test_no_underflow_accumulators_with_a_tiny_range(ref):
    # the no-underflow flag on an accumulator whose R_OF lies far below every product (top exponent -75 and
    # -123): every non-zero step saturates at +-R_OF, whichever kernel runs it
    rng = np.random.default_rng(2025)
    A = rand_codes(rng, (40, 70)); B = rand_codes(rng, (36, 70))
    for qa in ((4, 7, 90, 0x100), (2, 7, 126, 0x100), (4, 7, 81, 0x100), (4, 7, 82, 0x101), (3, 3, 100, 0x100)):
        for order in (0, 1):
            got = check(ref, A, B, (5, 7, 15, qa[3] & 1), qa, "tiny no-underflow accumulator", order=order)
            top = (1 << qa[0]) - qa[2] - 1
            rof = 2.0 ** top * (2 - 2.0 ** -qa[1])
            assert set(np.unique(np.abs(got)).tolist()) <= {0.0, rof}
            assert (np.abs(got) == rof).any()


def test_random_formats_over_the_whole_bias_range(ref):
    # the same sweep with the biases drawn from the whole documented range (2^E - b - 1 <= 127, b <= 126): most
    # of these formats flush or saturate everything, which is where a domain of the scaled kernel can run out of
    # FP32's own exponent range
    pyr = random.Random(77)
    rng = np.random.default_rng(77)
    A = rand_codes(rng, (40, 70)); B = rand_codes(rng, (36, 70))
    done = 0
    kernels = set()
    while done < 80:
        fmts = []
        for _ in range(2):
            E = pyr.randint(2, 7); M = pyr.choice([1, 3, 5, 7, 8, 10, 12, 20, 23])
            b = pyr.randint((1 << E) - 128, 126)
            if done % 2:                                       # every other case: near the operands' own range
                b = pyr.randint(max((1 << E) - 128, -30), 60)
            fmts.append((E, M, b))
        rnd = pyr.randint(0, 1)
        qpf, qaf = fmts[0] + (rnd | pyr.choice([0, 0, 0x100]),), fmts[1] + (rnd | pyr.choice([0, 0, 0x100]),)
        order = pyr.randint(0, 1)
        if ref.carrier_bits(fm(ref, qpf), fm(ref, qaf)) == 0:
            continue
        plan = lb.lba_plan_query(40, 36, 70, qpf, qaf, order)
        kernels.add(plan["kernel"])
        check(ref, A, B, qpf, qaf, "random format (full bias range) %d" % done, order=order)
        done += 1
    assert kernels == {0, 1}


def test_event_planes_of_the_chunked_order(ref):
    # first-level planes (bit k: step k of its own chunk's chain) and second-level planes (bit j: the add
    # of chunk j) for K below, at and across chunk, tile and second-level-word (512) boundaries; scaled
    # and general kernels; ragged M, N
    rng = np.random.default_rng(80)
    cases = [((5, 3, 1), 0, 15), ((20, 9, 16), 3, 12), ((33, 70, 17), 3, 12), ((70, 66, 100), 0, 15),
             ((64, 64, 512), 4, 11), ((37, 68, 530), 2, 12), ((16, 24, 1100), 5, 10)]
    fmts = [FMT_PAPER[0], FMT_PAPER[1], FMT_PAPER[2], FMT_ODD[1], FMT_ODD[0], FMT_SWEEP[1]]
    seen = np.zeros(4, dtype=np.int64)
    kernels = set()
    for (M, N, K), lo, hi in cases:
        A = rand_codes(rng, (M, K), lo, hi); B = rand_codes(rng, (N, K), lo, hi)
        tA, tB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
        for (qp, qa), rnd in itertools.product(fmts, (0, 1)):
            qpf, qaf = qp + (rnd,), qa + (rnd,)
            kernels.add(lb.lba_plan_query(M, N, K, qpf, qaf, 1, 1)["kernel"])
            got = lb.gemm_bwd_chunked(tA, tB, qpf, qaf)
            torch.cuda.synchronize()
            want = ref.gemm_bwd(A, B, fm(ref, qpf), fm(ref, qaf), order=ref.ORDER_CHUNK16, level2=True)
            assert np.array_equal(bits(got[0].cpu().numpy()), bits(want[0])), (M, N, K, qpf, qaf)
            for name, g, w in zip(("OF", "UF", "OF2", "UF2"), got[1:], want[1:]):
                assert np.array_equal(g.cpu().numpy().view(np.uint32), w), (M, N, K, qpf, qaf, name)
            seen += [int(np.count_nonzero(w)) for w in want[1:]]
            assert np.array_equal(bits(run_gpu(A, B, qpf, qaf, order=1)), bits(want[0]))
    assert kernels == {0, 1} and (seen[:3] > 0).all(), seen
    # a second-level underflow (cancellation between two grid values): chunk 0 = 1.5 * 2^-7, chunk 1 = -2^-7
    A = np.zeros((3, 20), dtype=np.uint8); B = np.zeros((2, 20), dtype=np.uint8)
    A[:, 0], B[:, 0] = 0x3C, 0x04
    A[:, 16], B[:, 16] = 0xB8, 0x04
    for rnd in (0, 1):
        qpf, qaf = (5, 7, 15, rnd), (4, 7, 7, rnd)
        got = lb.gemm_bwd_chunked(torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV), qpf, qaf)
        torch.cuda.synchronize()
        want = ref.gemm_bwd(A, B, fm(ref, qpf), fm(ref, qaf), order=ref.ORDER_CHUNK16, level2=True)
        assert (want[4] == 2).all()
        for g, w in zip(got[1:], want[1:]):
            assert np.array_equal(g.cpu().numpy().view(np.uint32), w)
        assert (got[0].cpu().numpy() == 0).all()
    # a single plane, no C; lba_gemm_bwd itself refuses the chunked order
    tA = torch.from_numpy(rand_codes(rng, (20, 40))).to(DEV); tB = torch.from_numpy(rand_codes(rng, (24, 40))).to(DEV)
    of2 = torch.full((1, 20, 24), -1, dtype=torch.int32, device=DEV)
    rc = lb.lba_gemm_bwd_chunked(tA.data_ptr(), tB.data_ptr(), None, None, None, of2.data_ptr(), None, 20, 24, 40,
                                 (5, 7, 15, 0), (4, 7, 7, 0))
    torch.cuda.synchronize()
    assert rc == lb.OK
    want = ref.gemm_bwd(tA.cpu().numpy(), tB.cpu().numpy(), ref.QFmt(5, 7, 15, 0), ref.QFmt(4, 7, 7, 0),
                        order=ref.ORDER_CHUNK16, level2=True)
    assert np.array_equal(of2.cpu().numpy().view(np.uint32), want[3])
    assert lb.lba_gemm_bwd_chunked(tA.data_ptr(), tB.data_ptr(), None, None, None, None, None, 20, 24, 40,
                                   (5, 7, 15, 0), (4, 7, 7, 0)) == lb.ERR_NULL
    assert lb.lba_gemm_bwd(tA.data_ptr(), tB.data_ptr(), None, of2.data_ptr(), None, 20, 24, 40,
                           (5, 7, 15, 0), (4, 7, 7, 0), order=1) == lb.ERR_UNSUPPORTED


def test_product_underflow_at_the_boundary_of_the_class_test(ref):
    # Where the smallest non-zero product (2^-18: two smallest subnormal codes) is still an FP32 denormal number in the
    # kernel's product domain, an underflowed product is found by its class; one bias further down it would round to
    # zero and the kernel tests the operands and the product for zero instead.  Q_prod biases on both sides of that
    # line (-5 | -6), operands full of subnormal codes and zeros, both orders: C and all planes against the oracle.
    rng = np.random.default_rng(4243)
    M, N, K = 70, 40, 150
    A = rand_codes(rng, (M, K), 0, 3); B = rand_codes(rng, (N, K), 0, 3)
    A[rng.random((M, K)) < 0.1] = 0x01; B[rng.random((N, K)) < 0.1] = 0x81            # the smallest magnitudes
    A[rng.random((M, K)) < 0.05] = 0x00; B[rng.random((N, K)) < 0.05] = 0x80           # zeros of both signs
    A[:, 128:] = rand_codes(rng, (M, K - 128), 6, 12)
    tA, tB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    slots = set()
    for bp in (-3, -4, -5, -6, -7, -9):
        for (Ea, Ma, ba), order in itertools.product([(4, 7, 7), (5, 10, bp - 2)], (0, 1)):
            qpf, qaf = (5, 7, bp, 0), (Ea, Ma, ba, 0)
            plan = lb.lba_plan_query(M, N, K, qpf, qaf, order, 1)
            if plan["kernel"] == 0:
                slots.add((bp >= -5, (plan["valu_per_mac_x100"] // 100) % 2 == 1))       # 9 slots per MAC with the class test, 10 without
            if order == 1:
                got = lb.gemm_bwd_chunked(tA, tB, qpf, qaf)
                want = ref.gemm_bwd(A, B, fm(ref, qpf), fm(ref, qaf), order=ref.ORDER_CHUNK16, level2=True)
            else:
                got = lb.gemm_bwd(tA, tB, qpf, qaf)
                want = ref.gemm_bwd(A, B, fm(ref, qpf), fm(ref, qaf))
            torch.cuda.synchronize()
            assert np.array_equal(bits(got[0].cpu().numpy()), bits(want[0])), (qpf, qaf, order, "C")
            for i in range(1, len(want)):
                assert np.array_equal(got[i].cpu().numpy().view(np.uint32), want[i]), (qpf, qaf, order, "plane %d" % i)
            assert want[2].any()                                                     # products do underflow
    assert (True, True) in slots and (False, False) in slots and len(slots) == 2, slots   # the planner's line is where the test says


def test_random_formats_event_planes(ref):
    # a seeded sweep of the recompute call over formats (both roundings, both orders, with and without the
    # underflow plane) whose ranges lie near the operands' own, so that overflows, product underflows and
    # accumulator underflows all occur; operands quiet at the start of the chains and loud at the end, so that
    # k-tiles with and without a possible overflow both run.  Whichever kernel the planner picks must give the
    # oracle's C and planes.
    pyr = random.Random(4242)
    rng = np.random.default_rng(4242)
    A = rand_codes(rng, (70, 150), 2, 9); B = rand_codes(rng, (40, 150), 2, 9)
    A[:, 96:] = rand_codes(rng, (70, 54), 6, 14)
    tA, tB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    picked, events = set(), [0, 0, 0]
    done = 0
    while done < 70:
        Ep, Ea = pyr.randint(3, 6), pyr.choice([3, 3, 4, 4, 4, 5, 6])
        Mp, Ma = pyr.choice([7, 7, 8, 10, 12]), pyr.choice([3, 5, 7, 7, 8, 10, 11, 16, 23])
        ba = pyr.randint(-6, 12)
        bp = ba + pyr.choice([-3, 0, 2, 2, 5, 8, 8, 12, 20, 23, 24, 30])
        if bp > 126 or (1 << Ep) - bp - 1 > 127 or (1 << Ea) - ba - 1 > 127:
            continue
        rnd, order, want_uf = pyr.randint(0, 1), pyr.randint(0, 1), pyr.random() < 0.75
        qpf, qaf = (Ep, Mp, bp, rnd), (Ea, Ma, ba, rnd)
        plan = lb.lba_plan_query(70, 40, 150, qpf, qaf, order, 1 if want_uf else 3)
        picked.add((plan["kernel"], rnd, order))
        what = (qpf, qaf, order, want_uf, plan["kernel"])
        if order == 1:
            got = lb.gemm_bwd_chunked(tA, tB, qpf, qaf, want_uf=want_uf)
            want = ref.gemm_bwd(A, B, fm(ref, qpf), fm(ref, qaf), order=ref.ORDER_CHUNK16, level2=True)
        else:
            got = lb.gemm_bwd(tA, tB, qpf, qaf, want_uf=want_uf)
            want = ref.gemm_bwd(A, B, fm(ref, qpf), fm(ref, qaf))
        torch.cuda.synchronize()
        assert np.array_equal(bits(got[0].cpu().numpy()), bits(want[0])), what + ("C",)
        for i in range(1, len(want)):
            if got[i] is None:
                assert not want_uf and i % 2 == 0
                continue
            assert np.array_equal(got[i].cpu().numpy().view(np.uint32), want[i]), what + ("plane %d" % i,)
        events[0] += int(want[1].any()); events[1] += int(want[2].any()); events[2] += int((want[1] == 0).all(axis=(1, 2)).any())
        done += 1
    assert {(0, 0, 0), (0, 0, 1), (0, 1, 0), (0, 1, 1), (1, 1, 0)} <= picked, picked
    assert events[0] > 15 and events[1] > 20 and events[2] > 10, events


def test_overflow_plane_alone(ref):
    # without an underflow plane the recompute call runs its overflow-only variant; under the sequential
    # order k-tiles that cannot overflow take the forward kernel's tile.  Small operands (no event at all),
    # full-range operands (events in most tiles) and a mix (quiet start, loud end) must all give the
    # oracle's OF plane and C.
    rng = np.random.default_rng(85)
    for (M, N, K), lo, hi in [((70, 66, 200), 0, 6), ((70, 66, 200), 0, 15), ((64, 64, 96), 3, 9), ((33, 130, 530), 2, 10),
                              ((5, 3, 31), 0, 15)]:
        A = rand_codes(rng, (M, K), lo, hi); B = rand_codes(rng, (N, K), lo, hi)
        if (lo, hi) == (3, 9):
            A[:, 64:] = rand_codes(rng, (M, K - 64), 10, 15)           # loud last tile
        tA, tB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
        for qp, qa in [FMT_PAPER[0], FMT_PAPER[1], FMT_PAPER[2], FMT_ODD[1]]:
            qpf, qaf = qp + (0,), qa + (0,)
            C, of, none = lb.gemm_bwd(tA, tB, qpf, qaf, want_uf=False)
            torch.cuda.synchronize()
            wc, wof, _ = ref.gemm_bwd(A, B, fm(ref, qpf), fm(ref, qaf))
            assert none is None
            assert np.array_equal(bits(C.cpu().numpy()), bits(wc)), (M, N, K, qpf, qaf)
            assert np.array_equal(of.cpu().numpy().view(np.uint32), wof), (M, N, K, qpf, qaf)
            got = lb.gemm_bwd_chunked(tA, tB, qpf, qaf, want_uf=False)
            torch.cuda.synchronize()
            want = ref.gemm_bwd(A, B, fm(ref, qpf), fm(ref, qaf), order=ref.ORDER_CHUNK16, level2=True)
            assert got[2] is None and got[4] is None
            assert np.array_equal(bits(got[0].cpu().numpy()), bits(want[0]))
            assert np.array_equal(got[1].cpu().numpy().view(np.uint32), want[1])
            assert np.array_equal(got[3].cpu().numpy().view(np.uint32), want[3])


def test_diff_plane(ref):
    # lba_gemm_bwd_diff: 1 - STE^DIFF per step (Sec. 4 "Immediate / DIFF", App. D) for several thresholds, both
    # roundings, both orders; ragged shapes across tile and word boundaries; operands from full range (overflow
    # and swamping), small (product underflow) and mixed.  The planes must differ between thresholds (the
    # comparison is live) and C must be the forward call's.
    rng = np.random.default_rng(123)
    cases = [((70, 66, 100), 0, 15), ((33, 130, 64), 3, 12), ((5, 3, 31), 0, 15), ((64, 64, 33), 5, 10), ((130, 20, 530), 0, 9)]
    fmts = [FMT_PAPER[0], FMT_PAPER[1], FMT_PAPER[2], FMT_ODD[0], FMT_ODD[1], FMT_ODD[3], FMT_SWEEP[1], FMT_SWEEP[5],
            ((7, 23, 64), (7, 23, 64)), ((5, 7, 15), (4, 23, 7))]
    distinct = 0
    for ci, ((M, N, K), lo, hi) in enumerate(cases):
        A = rand_codes(rng, (M, K), lo, hi); B = rand_codes(rng, (N, K), lo, hi)
        tA, tB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
        for fi, ((qp, qa), rnd) in enumerate(itertools.product(fmts, (0, 1))):
            if (ci + fi) % 2:                                          # half of the grid: keeps the oracle's time down
                continue
            qpf, qaf = qp + (rnd,), qa + (rnd,)
            for order in (0, 1):
                prev = None
                for eps2 in (0.0, 2.0 ** -6, 0.5, 0.75, 1.0):
                    C, diff = lb.gemm_bwd_diff(tA, tB, qpf, qaf, eps2, order=order)
                    torch.cuda.synchronize()
                    wc, wd = ref.gemm_diff(A, B, fm(ref, qpf), fm(ref, qaf), eps2, order=order)
                    assert np.array_equal(bits(C.cpu().numpy()), bits(wc)), (M, N, K, qpf, qaf, order, eps2)
                    got = diff.cpu().numpy().view(np.uint32)
                    bad = got != wd
                    assert not bad.any(), (M, N, K, qpf, qaf, order, eps2, int(bad.sum()), np.argwhere(bad)[0])
                    distinct += int(prev is not None and not np.array_equal(prev, got))
                    prev = got
    assert distinct > 100
    # the plane alone; a threshold with 12 significant bits
    C, diff = lb.gemm_bwd_diff(tA, tB, (5, 7, 15, 0), (4, 7, 7, 0), 2731 * 2.0 ** -13, want_c=False)
    torch.cuda.synchronize()
    _, wd = ref.gemm_diff(A, B, ref.QFmt(5, 7, 15, 0), ref.QFmt(4, 7, 7, 0), 2731 * 2.0 ** -13)
    assert C is None and np.array_equal(diff.cpu().numpy().view(np.uint32), wd)
    # other operand formats (the paper's M4E3 weights and activations with per-tensor biases): lba_gemm_bwd_diff_in
    A = rng.integers(0, 256, (70, 100)).astype(np.uint8); B = rng.integers(0, 256, (66, 100)).astype(np.uint8)
    tA, tB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    for (ia, ib), (qp, qa), rnd, order in [(((3, 4, 3), (3, 4, 5)), ((5, 7, 15), (4, 7, 7)), 0, 0),
                                           (((3, 4, 2), (4, 3, 7)), ((5, 7, 15), (4, 7, 7)), 1, 1),
                                           (((2, 5, 0), (5, 2, 12)), ((5, 5, 12), (5, 9, 14)), 1, 0),
                                           (((3, 4, 4), (3, 4, 4)), ((3, 4, 6), (3, 4, 6)), 0, 1)]:
        for eps2 in (0.0, 0.25, 0.875):
            C, diff = lb.gemm_bwd_diff(tA, tB, qp + (rnd,), qa + (rnd,), eps2, order=order, fmt_a=ia, fmt_b=ib)
            torch.cuda.synchronize()
            wc, wd = ref.gemm_diff(A, B, fm(ref, qp + (rnd,)), fm(ref, qa + (rnd,)), eps2, order=order,
                                   fmt_a=ref.InFmt(*ia), fmt_b=ref.InFmt(*ib))
            assert np.array_equal(bits(C.cpu().numpy()), bits(wc)), (ia, ib, qp, qa, rnd, order, eps2)
            assert np.array_equal(diff.cpu().numpy().view(np.uint32), wd), (ia, ib, qp, qa, rnd, order, eps2)
    # empty chains and empty outputs
    z = torch.empty((4, 0), dtype=torch.uint8, device=DEV)
    C, diff = lb.gemm_bwd_diff(z, z, (5, 7, 15, 0), (4, 7, 7, 0), 0.5)
    torch.cuda.synchronize()
    assert diff.numel() == 0 and (C == 0).all() and tuple(C.shape) == (4, 4)


def test_operand_code_formats(ref):
    # lba_gemm_in / lba_gemm_bwd_in: operands in other 8-bit formats (the paper's M4E3 with a per-tensor
    # bias, E5M2, E2M5, mixed with E4M3).  Products have up to 12 significant bits, so Q_prod's mantissa
    # rounding is active: truncation runs in the scaled kernel, nearest-even in the general one.
    rng = np.random.default_rng(110)
    shapes = [(70, 66, 100), (33, 130, 64), (5, 3, 31), (64, 64, 200)]
    combos = [((3, 4, 3), (3, 4, 3), (5, 7, 15), (4, 7, 7)),        # canonical biases
              ((3, 4, 6), (3, 4, 1), (5, 7, 15), (4, 7, 7)),        # flex biases: folded into the quantizers
              ((3, 4, -2), (4, 3, 9), (4, 7, 12), (4, 7, 10)),      # mixed with E4M3; the paper's (10, 12) pair
              ((5, 2, 15), (5, 2, 17), (5, 7, 15), (4, 7, 7)),      # E5M2: 6-bit products
              ((2, 5, 1), (2, 5, 0), (5, 7, 15), (4, 7, 7)),        # E2M5: 12-bit products
              ((3, 4, 3), (3, 4, 3), (6, 9, 20), (4, 7, 7)),        # Q_prod wide enough: no product rounding
              ((3, 4, 3), (3, 4, 3), (5, 5, 15), (5, 10, 15)),      # narrow Q_prod, wide accumulator
              ((3, 4, 4), (3, 4, 4), (3, 4, 6), (3, 4, 6))]         # 8-bit accumulator
    for (M, N, K) in shapes:
        A = rng.integers(0, 256, (M, K)).astype(np.uint8); B = rng.integers(0, 256, (N, K)).astype(np.uint8)
        tA, tB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
        for (fa, fb, qp, qa), rnd, order in itertools.product(combos, (0, 1), (0, 1)):
            qpf, qaf = qp + (rnd,), qa + (rnd,)
            got = lb.gemm_in(tA, tB, fa, fb, qpf, qaf, order=order)
            torch.cuda.synchronize()
            want = ref.gemm_in(A, B, ref.InFmt(*fa), ref.InFmt(*fb), fm(ref, qpf), fm(ref, qaf), order=order)
            bad = bits(got.cpu().numpy()) != bits(want)
            assert not bad.any(), ((M, N, K), fa, fb, qpf, qaf, order, int(bad.sum()), got.cpu().numpy()[bad][:3], want[bad][:3])
        # the recompute call (sequential order)
        for (fa, fb, qp, qa), rnd in itertools.product(combos[:3], (0, 1)):
            qpf, qaf = qp + (rnd,), qa + (rnd,)
            C, of, uf = lb.gemm_in(tA, tB, fa, fb, qpf, qaf, planes=True)
            torch.cuda.synchronize()
            wc, wof, wuf = ref.gemm_in(A, B, ref.InFmt(*fa), ref.InFmt(*fb), fm(ref, qpf), fm(ref, qaf), planes=True)
            assert np.array_equal(bits(C.cpu().numpy()), bits(wc)), (fa, fb, qpf, qaf)
            assert np.array_equal(of.cpu().numpy().view(np.uint32), wof) and np.array_equal(uf.cpu().numpy().view(np.uint32), wuf)
    # E4M3 through the general entry point is lba_gemm
    A = rand_codes(rng, (40, 50)); B = rand_codes(rng, (30, 50))
    tA, tB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    assert torch.equal(lb.gemm_in(tA, tB, (4, 3, 7), (4, 3, 7), (5, 7, 15, 0), (4, 7, 7, 0)), lb.gemm(tA, tB, (5, 7, 15, 0), (4, 7, 7, 0)))
    # limits
    a, b = tA.data_ptr(), tB.data_ptr()
    c = torch.empty((40, 30), dtype=torch.float32, device=DEV).data_ptr()
    assert lb.lba_gemm_in(a, b, c, 40, 30, 50, (3, 3, 3), (3, 4, 3), (5, 7, 15, 0), (4, 7, 7, 0)) == lb.ERR_FORMAT
    assert lb.lba_gemm_in(a, b, c, 40, 30, 50, (3, 4, 33), (3, 4, 3), (5, 7, 15, 0), (4, 7, 7, 0)) == lb.ERR_FORMAT
    assert lb.lba_gemm_in(a, b, c, 40, 30, 50, (3, 4, 32), (3, 4, 32), (5, 7, 120, 0), (4, 7, 7, 0)) == lb.OK
    assert lb.lba_gemm_in(a, b, c, 40, 30, 50, (3, 4, -32), (3, 4, -32), (5, 7, 120, 0), (4, 7, 7, 0)) == lb.ERR_FORMAT   # folded bias 190
    assert lb.lba_gemm_bwd_in(a, b, c, c, None, 40, 30, 50, (3, 4, 3), (3, 4, 3), (5, 7, 15, 0), (4, 7, 7, 0), order=1) == lb.ERR_UNSUPPORTED
    torch.cuda.synchronize()


def test_operand_code_formats_on_mixed_grids(ref):
    # lba_gemm_in on the grids of the E4M3 product: 64 x 64 workgroups with a 32 x 32 tail, whole rounds of 48 x 64, full
    # rounds followed by one of 48 x 64, and small grids as 32 x 32 workgroups throughout; the product modes that only
    # these kernels have (truncated and nearest-even products), both orders, both roundings; and lba_gemm_bwd_in on its
    # mixed grids (floor, sequential order)
    rng = np.random.default_rng(111)
    combos = [((3, 4, 3), (3, 4, 3), (5, 7, 15), (4, 7, 7)),        # 10-bit products into an 8-bit Q_prod mantissa
              ((3, 4, 6), (4, 3, 9), (4, 7, 12), (4, 7, 10)),       # flex bias, mixed with E4M3
              ((3, 4, 3), (3, 4, 3), (6, 9, 20), (4, 7, 7))]        # Q_prod wide enough: no product rounding
    kinds, bwd_kinds = set(), set()
    for (M, N, K) in [(64 * 420 + 17, 60, 40), (12544, 256, 40), (64 * 947 + 17, 64, 40), (70, 50, 96), (34560, 60, 27)]:
        A = rng.integers(0, 256, (M, K)).astype(np.uint8); B = rng.integers(0, 256, (N, K)).astype(np.uint8)
        tA, tB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
        for (fa, fb, qp, qa), rnd, order in itertools.product(combos, (0, 1), (0, 1)):
            qpf, qaf = qp + (rnd,), qa + (rnd,)
            plan = lb.lba_plan_query_in(M, N, K, fa, fb, qpf, qaf, order)
            if plan["kernel"] == 0:
                main = plan["grid_x"] - plan["mid_blocks"] - plan["tail_blocks"]
                assert plan["mid_blocks"] + plan["tail_blocks"] > 0, ((M, N, K), plan)
                kinds.add((main > 0, plan["mid_blocks"] > 0, plan["tail_blocks"] > 0))
            got = lb.gemm_in(tA, tB, fa, fb, qpf, qaf, order=order)
            torch.cuda.synchronize()
            want = ref.gemm_in(A, B, ref.InFmt(*fa), ref.InFmt(*fb), fm(ref, qpf), fm(ref, qaf), order=order)
            bad = bits(got.cpu().numpy()) != bits(want)
            assert not bad.any(), ((M, N, K), fa, fb, qpf, qaf, order, int(bad.sum()))
            if rnd == 0 and order == 0:                        # the recompute call: 64 x 64 workgroups and the 32 x 32 tail
                wc, wof, wuf = ref.gemm_in(A, B, ref.InFmt(*fa), ref.InFmt(*fb), fm(ref, qpf), fm(ref, qaf), planes=True)
                for with_masks in (1, 3):                      # both planes; the OF plane alone (truncated products: this one only)
                    plan = lb.lba_plan_query_in(M, N, K, fa, fb, qpf, qaf, order, with_masks=with_masks)
                    if plan["kernel"] == 0 and plan["tail_blocks"] > 0:    # (three full rounds and most of a fourth: plain grid)
                        assert plan["mid_blocks"] == 0, ((M, N, K), plan)
                        bwd_kinds.add((with_masks, plan["grid_x"] > plan["tail_blocks"]))
                    C, of, uf = lb.gemm_in(tA, tB, fa, fb, qpf, qaf, planes=True, uf_plane=with_masks == 1)
                    torch.cuda.synchronize()
                    assert np.array_equal(bits(C.cpu().numpy()), bits(wc)), ((M, N, K), fa, fb, qpf, qaf)
                    assert np.array_equal(of.cpu().numpy().view(np.uint32), wof), ((M, N, K), fa, fb, qpf, qaf)
                    assert uf is None or np.array_equal(uf.cpu().numpy().view(np.uint32), wuf), ((M, N, K), fa, fb, qpf, qaf)
    assert {(True, False, True), (False, True, True), (True, True, True), (False, False, True)} <= kinds, kinds
    assert bwd_kinds == {(1, True), (1, False), (3, True), (3, False)}, bwd_kinds


def test_mixed_grid(ref):
    # launches whose last round of 64 x 64 workgroups would be mostly empty finish their last rows with
    # 32 x 32 workgroups: both regions, their seam and the ragged edges against the oracle
    rng = np.random.default_rng(130)
    mixed = 0
    for (M, N, K) in [(64 * 420 + 17, 60, 100), (64 * 392, 64, 40), (64 * 150 + 33, 130, 64)]:
        A = rand_codes(rng, (M, K), 3, 12); B = rand_codes(rng, (N, K), 3, 12)
        for (qp, qa), rnd, order in itertools.product([FMT_PAPER[0], FMT_PAPER[2], FMT_PAPER[4], FMT_SWEEP[4]], (0, 1), (0, 1)):
            qpf, qaf = qp + (rnd,), qa + (rnd,)
            plan = lb.lba_plan_query(M, N, K, qpf, qaf, order)
            two_sums = rnd == 1 and plan["valu_per_mac_x100"] >= 1000      # the round-to-odd variant has no mixed grid
            assert plan["kernel"] == 1 or two_sums or (plan["tail_blocks"] + plan["mid_blocks"] > 0 and plan["grid_y"] == 1), plan
            mixed += plan["tail_blocks"] + plan["mid_blocks"] > 0
            check(ref, A, B, qpf, qaf, "mixed grid", order=order)
    assert mixed >= 36
    # whole rounds of 48 x 64 workgroups (3 x 4 outputs per lane; the forward call): one, two and four rounds of them
    # in front of the 32 x 32 tail, and one round of them behind three rounds of 64 x 64
    for (M, N, K), main in [((64 * 300 + 5, 64, 40), False), ((64 * 392, 64, 40), False), ((12544, 256, 40), False), ((64 * 947 + 17, 64, 40), True)]:
        A = rand_codes(rng, (M, K), 3, 12); B = rand_codes(rng, (N, K), 3, 12)
        for (qp, qa), rnd, order in itertools.product([FMT_PAPER[0], FMT_SWEEP[4]], (0, 1), (0, 1)):
            qpf, qaf = qp + (rnd,), qa + (rnd,)
            plan = lb.lba_plan_query(M, N, K, qpf, qaf, order)
            if plan["kernel"] == 0 and plan["valu_per_mac_x100"] < 1000:
                assert plan["mid_blocks"] > 0 and (205 <= plan["mid_blocks"] <= 256 if main else plan["mid_blocks"] % 256 == 0), plan
                assert (plan["grid_x"] - plan["mid_blocks"] - plan["tail_blocks"] > 0) == main, plan
            check(ref, A, B, qpf, qaf, "48-row rounds", order=order)
        assert lb.lba_plan_query(M, N, K, FMT_PAPER[0][0] + (0,), FMT_PAPER[0][1] + (0,), 0, 1)["mid_blocks"] == 0   # recompute: none
    # not used where it cannot help: exact multiples of a round, tiny and huge grids (for the recompute call too)
    assert lb.lba_plan_query(64 * 256, 64, 64, (5, 7, 15, 0), (4, 7, 7, 0))["tail_blocks"] == 0
    assert lb.lba_plan_query(64 * 40, 64, 64, (5, 7, 15, 0), (4, 7, 7, 0))["tail_blocks"] == 0
    # up to 384 workgroups of 64 x 64 a CU would run a single wave per SIMD (half rate): finer plain tiles instead
    small = lb.lba_plan_query(64 * 270, 64, 64, (5, 7, 15, 0), (4, 7, 7, 0))
    assert small["tail_blocks"] + small["mid_blocks"] == 0 and (small["thread_m"], small["thread_n"]) == (2, 4)
    assert lb.lba_plan_query(64 * 100, 64, 64, (5, 7, 15, 0), (4, 7, 7, 0))["thread_n"] == 2
    assert lb.lba_plan_query(64 * 12544, 64, 64, (5, 7, 15, 0), (4, 7, 7, 0))["tail_blocks"] == 0
    assert lb.lba_plan_query(64 * 300, 64, 64, (5, 7, 15, 0), (4, 7, 7, 0), 0, 1)["tail_blocks"] == 0
    # the recompute call has the mixed grid under the sequential order (both planes, or the overflow plane alone): quiet
    # operands (k-tiles that take the forward tile), loud ones, and a quiet start with a loud end
    for (M, N, K), lo, hi in [((64 * 420 + 17, 60, 100), 3, 8), ((64 * 392, 64, 72), 0, 15), ((64 * 150 + 33, 130, 96), 3, 9)]:
        A = rand_codes(rng, (M, K), lo, hi); B = rand_codes(rng, (N, K), lo, hi)
        if (lo, hi) == (3, 9):
            A[:, 64:] = rand_codes(rng, (M, K - 64), 10, 15)
        tA, tB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
        for qp, qa in (FMT_PAPER[0], FMT_PAPER[2], FMT_SWEEP[4]):
            qpf, qaf = qp + (0,), qa + (0,)
            plan = lb.lba_plan_query(M, N, K, qpf, qaf, 0, 3)
            assert plan["kernel"] == 0 and plan["tail_blocks"] > 0 and plan["grid_y"] == 1, plan
            assert lb.lba_plan_query(M, N, K, qpf, qaf, 0, 1)["tail_blocks"] > 0         # both planes: the same grid
            assert lb.lba_plan_query(M, N, K, qpf, qaf, 1, 1)["tail_blocks"] == 0        # chunked recompute: plain grid
            C, of, uf = lb.gemm_bwd(tA, tB, qpf, qaf)
            torch.cuda.synchronize()
            wc, wof, wuf = ref.gemm_bwd(A, B, fm(ref, qpf), fm(ref, qaf))
            assert np.array_equal(bits(C.cpu().numpy()), bits(wc)), (M, N, K, qpf, qaf)
            assert np.array_equal(of.cpu().numpy().view(np.uint32), wof) and np.array_equal(uf.cpu().numpy().view(np.uint32), wuf)
            C, of, _ = lb.gemm_bwd(tA, tB, qpf, qaf, want_uf=False)
            torch.cuda.synchronize()
            wc, wof, _ = ref.gemm_bwd(A, B, fm(ref, qpf), fm(ref, qaf))
            assert np.array_equal(bits(C.cpu().numpy()), bits(wc)), (M, N, K, qpf, qaf)
            assert np.array_equal(of.cpu().numpy().view(np.uint32), wof), (M, N, K, qpf, qaf)
            _, of2, _ = lb.gemm_bwd(tA, tB, qpf, qaf, want_uf=False, want_c=False)       # the plane alone
            torch.cuda.synchronize()
            assert torch.equal(of, of2)
            # the DIFF plane on the same grid, both orders
            for order in (0, 1):
                assert lb.lba_plan_query(M, N, K, qpf, qaf, order, 2)["tail_blocks"] > 0
                C, diff = lb.gemm_bwd_diff(tA, tB, qpf, qaf, 0.25, order=order)
                torch.cuda.synchronize()
                wc, wd = ref.gemm_diff(A, B, fm(ref, qpf), fm(ref, qaf), 0.25, order=order)
                assert np.array_equal(bits(C.cpu().numpy()), bits(wc)), (M, N, K, qpf, qaf, order)
                assert np.array_equal(diff.cpu().numpy().view(np.uint32), wd), (M, N, K, qpf, qaf, order)


def test_calls_on_side_streams(ref):
    # Every kernel of a call runs on the caller's stream: a chain of dependent calls (recompute call -> last
    # overflow -> coefficient plane -> gradient products with their zero fill and atomic adds) is queued on a
    # non-default stream without any synchronisation in between, twice at once on two streams with different
    # operands.  The integer results equal the oracle's; the gradients equal those of the same calls on the
    # default stream up to the summation order.
    rng = np.random.default_rng(321)
    qp, qa = (5, 7, 15, 0), (4, 7, 7, 0)
    jobs = []
    for (M, N, K) in ((520, 260, 500), (300, 516, 260)):
        A = rand_codes(rng, (M, K), 3, 11); B = rand_codes(rng, (N, K), 3, 11)
        G = rng.standard_normal((M, N)).astype(np.float32)
        jobs.append((A, B, G, torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV), torch.from_numpy(G).to(DEV)))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = []
    for (A, B, G, tA, tB, tG), st in zip(jobs, streams):
        K = A.shape[1]
        with torch.cuda.stream(st):                                    # allocations of the binding follow the stream
            C, of, uf = lb.gemm_bwd(tA, tB, qp, qa, stream=st)
            last = lb.last_overflow(of, K, stream=st)
            coef = lb.ste_plane(of, K, lb.STE_RECURSIVE_OF, stream=st)
            dX, dW = lb.grad(tG, tA, tB, lb.STE_COEF_PLANE, of_plane=coef, stream=st)
            dX2, dW2 = lb.grad(tG, tA, tB, lb.STE_RECURSIVE_OF, last_of=last, stream=st)
        outs.append((C, of, uf, last, coef, dX, dW, dX2, dW2))
    for st in streams:
        st.synchronize()
    for (A, B, G, tA, tB, tG), (C, of, uf, last, coef, dX, dW, dX2, dW2) in zip(jobs, outs):
        K = A.shape[1]
        wc, wof, wuf = ref.gemm_bwd(A, B, fm(ref, qp), fm(ref, qa))
        assert np.array_equal(bits(C.cpu().numpy()), bits(wc))
        assert np.array_equal(of.cpu().numpy().view(np.uint32), wof) and np.array_equal(uf.cpu().numpy().view(np.uint32), wuf)
        last0 = lb.last_overflow(of, K)
        dXr, dWr = lb.grad(tG, tA, tB, lb.STE_RECURSIVE_OF, last_of=last0)
        torch.cuda.synchronize()
        assert torch.equal(last, last0) and int((last >= 0).sum()) > 0
        scale = float(dXr.abs().max()) + float(dWr.abs().max())
        for got, want in ((dX, dXr), (dX2, dXr), (dW, dWr), (dW2, dWr)):
            assert float((got - want).abs().max()) <= 1e-4 * scale


def test_hip_graph_replays(ref):
    # The library only launches kernels (no allocation, no memset, no synchronisation), so a sequence of calls can
    # be captured into a HIP graph.  The graph is replayed three times with new operands written into the same
    # buffers, with eager work and synchronisations between the replays; every replay is checked against the
    # oracle (integers) and against the eager gradient products.
    rng = np.random.default_rng(322)
    qp, qa = (5, 7, 15, 0), (4, 7, 7, 0)
    M, N, K = 200, 132, 300
    tA = torch.zeros((M, K), dtype=torch.uint8, device=DEV); tB = torch.zeros((N, K), dtype=torch.uint8, device=DEV)
    tG = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    C = torch.empty((M, N), dtype=torch.float32, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                                      # one eager pass before the capture
        lb.gemm(tA, tB, qp, qa, out=C)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lb.gemm(tA, tB, qp, qa, out=C)
        Cc = lb.gemm(tA, tB, qp, qa, order=1)
        C2, of, uf = lb.gemm_bwd(tA, tB, qp, qa)
        last = lb.last_overflow(of, K)
        dX, dW = lb.grad(tG, tA, tB, lb.STE_RECURSIVE_OF, last_of=last)
        dXi, dWi = lb.grad(tG, tA, tB, lb.STE_IMMEDIATE_OF, of_plane=of)
        C3, of3, _, ws = lb.gemm_bwd_ws(tA, tB, qp, qa, want_uf=False)         # the recompute call that also leaves the brick maps
        dXp, dWp = lb.grad_premapped(tG, tA, tB, of3, ws)
    for rep in range(3):
        A = rand_codes(rng, (M, K), 3, 11); B = rand_codes(rng, (N, K), 3, 11)
        G = rng.standard_normal((M, N)).astype(np.float32)
        tA.copy_(torch.from_numpy(A)); tB.copy_(torch.from_numpy(B)); tG.copy_(torch.from_numpy(G))
        for t in (C, Cc, C2, dX, dW, dXi, dWi, C3, dXp, dWp):
            t.fill_(7.0)                                               # stale values must not survive
        ws.fill_(1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        wc, wof, wuf = ref.gemm_bwd(A, B, fm(ref, qp), fm(ref, qa))
        assert np.array_equal(bits(C.cpu().numpy()), bits(wc)) and np.array_equal(bits(C2.cpu().numpy()), bits(wc)), rep
        assert np.array_equal(bits(Cc.cpu().numpy()), bits(ref.gemm(A, B, fm(ref, qp), fm(ref, qa), order=1))), rep
        assert np.array_equal(of.cpu().numpy().view(np.uint32), wof) and np.array_equal(uf.cpu().numpy().view(np.uint32), wuf), rep
        last0 = lb.last_overflow(of, K)
        eX, eW = lb.grad(tG, tA, tB, lb.STE_RECURSIVE_OF, last_of=last0)
        eXi, eWi = lb.grad(tG, tA, tB, lb.STE_IMMEDIATE_OF, of_plane=of)
        torch.cuda.synchronize()
        assert torch.equal(last, last0), rep
        scale = float(eX.abs().max()) + float(eW.abs().max())
        assert torch.equal(of3, of) and np.array_equal(bits(C3.cpu().numpy()), bits(wc)), rep
        for got, want in ((dX, eX), (dW, eW), (dXi, eXi), (dWi, eWi), (dXp, eXi), (dWp, eWi)):
            assert float((got - want).abs().max()) <= 1e-4 * scale, rep
