"""Pins for the CPU oracle: everything here runs without a GPU and compares the oracle with
facts fixed by the paper and by mathematics (hand-worked values, closed forms, library rounding
routines, exact arithmetic, brute force), never with the HIP path."""
import itertools
import math
import os
import random
from fractions import Fraction

import numpy as np
import pytest
import torch

import frac_model as FM

GOLD = os.path.join(os.path.dirname(__file__), "golden")
TINY = [0x00, 0x80, 0x01, 0x81, 0x08, 0x38, 0xB8, 0x39, 0x3F, 0x47, 0x58, 0xDA, 0x7E, 0xFE, 0x77, 0x0F]


def rows(name):
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                yield line.split()


# ------------------------------------------------------------------------------------------
# the scalar quantizer (Sec. 2.3)
# ------------------------------------------------------------------------------------------

def test_hand_worked_roundings(ref):
    n = 0
    for xs, fl, rn in rows("q_m7e4_b7_roundings.txt"):
        x = float(eval(xs))
        assert ref.quantize(x, ref.QFmt(4, 7, 7, ref.FLOOR)) == float(fl), xs
        assert ref.quantize(x, ref.QFmt(4, 7, 7, ref.RNE)) == float(rn), xs
        n += 1
    assert n >= 15


def test_range_closed_forms(ref):
    for M, E, b, rof, ufexp in rows("r_of_closed_forms.txt"):
        M, E, b = int(M), int(E), int(b)
        for rnd in (ref.FLOOR, ref.RNE):
            f = ref.QFmt(E, M, b, rnd)
            v, ev = ref.quantize(1e30, f, with_events=True)
            assert v == float(rof) and ev == ref.EV_OF
            assert ref.quantize(float(rof), f) == float(rof)
            ruf = 2.0 ** int(ufexp)
            assert ref.quantize(ruf, f) == ruf
            below = np.nextafter(ruf, 0.0)
            assert ref.quantize(below, f, with_events=True) == (0.0, ref.EV_UF)
            # the largest value below R_OF that floor keeps below R_OF
            assert ref.quantize(np.nextafter(float(rof), 0.0), ref.QFmt(E, M, b, ref.FLOOR)) < float(rof)


def test_default_bias_is_half_range(ref):
    # Sec. 3: the default bias of FP16-like formats is b = 2^(E-1); for E=4 that is 8 (App. B)
    f = ref.QFmt(4, 7, 8, ref.FLOOR)
    assert ref.quantize(1e9, f) == 255.0 and ref.quantize(2.0 ** -8, f) == 2.0 ** -8


def test_matches_ieee_half_cast(ref):
    # M10 E5 b=14 on [2^-14, 65504) is IEEE binary16 rounding (a library routine)
    rng = np.random.default_rng(1)
    xs = np.concatenate([rng.uniform(2.0 ** -14, 1.0, 2000), rng.uniform(1.0, 65000.0, 2000),
                         np.ldexp(1.0 + rng.integers(0, 1 << 13, 2000) / float(1 << 12), rng.integers(-14, 14, 2000))])
    xs = xs[(xs >= 2.0 ** -14) & (xs < 65504.0)]
    f = ref.QFmt(5, 10, 14, ref.RNE)
    for x in xs:
        for s in (1.0, -1.0):
            assert ref.quantize(s * x, f) == float(np.float16(s * x))


def test_matches_bfloat16_cast_and_float32_bitmask(ref):
    # M7 E7 b=64: nearest-even equals the float32->bfloat16 cast; floor equals masking the low
    # 16 bits of the float32 word (the paper's "floor ... via bit-mask", Sec. 3)
    g = torch.Generator().manual_seed(2)
    x = (torch.randn(4000, generator=g) * torch.exp2(torch.randint(-40, 40, (4000,), generator=g).float()))
    bf = x.bfloat16().float()
    fl = (x.view(torch.int32) & ~0xFFFF).view(torch.float32)
    for i in range(x.numel()):
        xi = float(x[i])
        assert ref.quantize(xi, ref.QFmt(7, 7, 64, ref.RNE)) == float(bf[i])
        assert ref.quantize(xi, ref.QFmt(7, 7, 64, ref.FLOOR)) == float(fl[i])
    # other mantissa widths: mask the low 23-M bits
    for M in (1, 3, 10, 22, 23):
        mask = ~((1 << (23 - M)) - 1)
        fl = (x.view(torch.int32) & mask).view(torch.float32)
        for i in range(0, x.numel(), 7):
            assert ref.quantize(float(x[i]), ref.QFmt(7, M, 64, ref.FLOOR)) == float(fl[i])


def test_quantizer_invariants_and_error_bounds(ref):
    # Table 1: swamping relative error < 2^-M (floor) / <= 2^-(M+1) (nearest); underflow absolute
    # error < 2^-b; plus idempotence, sign symmetry, monotonicity, floor never grows magnitude
    rnd = random.Random(3)
    for _ in range(300):
        E = rnd.randint(2, 7); M = rnd.randint(1, 23)
        b = rnd.randint(max((1 << E) - 128, -20), 40)
        top = (1 << E) - b - 1
        for r in (ref.FLOOR, ref.RNE):
            f = ref.QFmt(E, M, b, r)
            prev_x, prev_q = None, None
            xs = sorted(math.ldexp(rnd.uniform(1, 2), rnd.randint(-b - 3, top + 2)) for _ in range(12))
            for x in xs:
                q, ev = ref.quantize(x, f, with_events=True)
                assert ref.quantize(q, f) == q                       # idempotent
                assert ref.quantize(-x, f) == -q                     # odd
                if prev_x is not None:
                    assert q >= prev_q                               # monotone
                prev_x, prev_q = x, q
                if ev == 0:
                    rel = abs(Fraction(q) - Fraction(x)) / Fraction(x)
                    if r == ref.FLOOR:
                        assert q <= x and rel < Fraction(1, 2 ** M)
                    else:
                        assert rel <= Fraction(1, 2 ** (M + 1))
                elif ev == ref.EV_UF:
                    assert q == 0.0 and x < 2.0 ** -b
                else:
                    assert x >= q and q == math.ldexp(2 - 2.0 ** -M, top)


def test_underflow_is_decided_before_rounding(ref):
    # nearest-even must not round a value just below 2^-b up to 2^-b
    f = ref.QFmt(4, 7, 7, ref.RNE)
    assert ref.quantize(2.0 ** -7 * (1 - 2.0 ** -12), f) == 0.0


def test_quantizer_against_fraction_model(ref):
    rnd = random.Random(4)
    for _ in range(400):
        E = rnd.randint(2, 7); M = rnd.randint(1, 12)
        b = rnd.randint(max((1 << E) - 128, -10), 30)
        r = rnd.randint(0, 1)
        top = (1 << E) - b - 1
        x = math.ldexp(rnd.randint(1, 1 << 20), rnd.randint(-b - 24, top - 16))
        x = -x if rnd.random() < 0.5 else x
        want, _ = FM.quant(Fraction(x), E, M, b, r)
        assert Fraction(ref.quantize(x, ref.QFmt(E, M, b, r))) == want


def test_no_underflow_flag(ref):
    # FMAq "excluding underflow events" (Sec. 3, Fig. 2b): below R_UF the mantissa is still rounded
    # to M bits instead of flushing; everything else is unchanged.  M7 pins: bfloat16 cast
    # (nearest-even) and the float32 bit-mask (floor), far below R_UF = 2^-7.
    g = torch.Generator().manual_seed(12)
    x = torch.randn(3000, generator=g) * torch.exp2(torch.randint(-60, 8, (3000,), generator=g).float())
    bf = x.bfloat16().float()
    fl = (x.view(torch.int32) & ~0xFFFF).view(torch.float32)
    fr = ref.QFmt(4, 7, 7, ref.RNE | ref.NO_UNDERFLOW)
    ff = ref.QFmt(4, 7, 7, ref.FLOOR | ref.NO_UNDERFLOW)
    for i in range(x.numel()):
        xi = float(x[i])
        if abs(xi) >= 509.0:
            continue
        assert ref.quantize(xi, fr) == float(bf[i])
        assert ref.quantize(xi, ff) == float(fl[i])
    assert ref.quantize(1e9, fr) == 510.0 and ref.quantize(-1e9, ff) == -510.0      # overflow unchanged
    assert ref.quantize(2.0 ** -30, ref.QFmt(4, 7, 7, ref.RNE)) == 0.0              # without the flag: flushed
    # a chain: sequential bfloat16 accumulation of small products (most are below 2^-7), no overflow
    rng = np.random.default_rng(13)
    A = _rand_codes(rng, (10, 100), 0, 7); B = _rand_codes(rng, (9, 100), 0, 7)
    a = torch.from_numpy(A).view(torch.float8_e4m3fn).float()
    b = torch.from_numpy(B).view(torch.float8_e4m3fn).float()
    s = torch.zeros(10, 9)
    for k in range(100):
        s = (s + a[:, k:k + 1] * b[:, k:k + 1].T).bfloat16().float()
    assert float(s.abs().max()) < 500
    assert (torch.from_numpy(ref.gemm(A, B, fr, fr)) == s).all()
    with_uf = ref.gemm(A, B, ref.QFmt(4, 7, 7, ref.RNE), ref.QFmt(4, 7, 7, ref.RNE))
    assert not (torch.from_numpy(with_uf) == s).all()                              # the flag matters here
    # no underflow events are reported by a flagged quantizer
    _, of, uf = ref.gemm_bwd(A, B, fr, fr)
    assert not uf.any()
    # brute force against the Fraction model, flag on either or both quantizers
    rnd_gen = random.Random(14)
    for fp, fa in (((5, 7, 15, 0 | 0x100), (4, 7, 7, 0)), ((5, 7, 15, 1), (4, 7, 7, 1 | 0x100)),
                   ((4, 4, 6, 1 | 0x100), (3, 4, 3, 0 | 0x100))):
        for _ in range(150):
            K = rnd_gen.randint(1, 5)
            sa = [rnd_gen.choice(TINY) for _ in range(K)]; sb = [rnd_gen.choice(TINY) for _ in range(K)]
            want, evs = FM.chain(sa, sb, fp, fa)
            C, of, uf = ref.gemm_bwd(np.array([sa], dtype=np.uint8), np.array([sb], dtype=np.uint8),
                                     ref.QFmt(*fp), ref.QFmt(*fa))
            assert Fraction(float(C[0, 0])) == want
            for k, (o, u_) in enumerate(evs):
                assert (int(of[0, 0, 0]) >> k) & 1 == int(o) and (int(uf[0, 0, 0]) >> k) & 1 == int(u_)


# ------------------------------------------------------------------------------------------
# decoding and products
# ------------------------------------------------------------------------------------------

def test_decode_table_against_torch_float8(ref):
    codes = torch.arange(256, dtype=torch.uint8)
    want = codes.view(torch.float8_e4m3fn).double()
    for c in range(256):
        if (c & 0x7F) == 0x7F:
            assert abs(ref.decode(c)) == 480.0            # NaN codes read as the normal pattern
            continue
        assert ref.decode(c) == float(want[c]), c
        assert Fraction(ref.decode(c)) == FM.e4m3_value(c)
    assert ref.decode(0x7E) == 448.0 and ref.decode(0x01) == 2.0 ** -9


def test_all_products_exact_and_at_most_8_bits(ref):
    wide_p = ref.QFmt(7, 23, 40, ref.FLOOR)
    wide_a = ref.QFmt(7, 23, 40, ref.FLOOR)
    vals = [ref.decode(c) for c in range(256)]
    mn, mx = 1e9, 0.0
    for a in range(0, 256):
        for b in range(a, 256, 3 if a % 5 else 1):
            got, ev = ref.fmaq(a, b, 0.0, wide_p, wide_a)
            p = vals[a] * vals[b]                                # exact in double
            assert got == p and ev == 0
            if p != 0:
                n = Fraction(abs(p)).numerator
                while n % 2 == 0:
                    n //= 2
                assert n.bit_length() <= 8
                mn, mx = min(mn, abs(p)), max(mx, abs(p))
    assert mn == 2.0 ** -18 and mx == 480.0 * 480.0


# ------------------------------------------------------------------------------------------
# FMAq and the sequential chain (Sec. 3, App. D)
# ------------------------------------------------------------------------------------------

def test_hand_worked_chain(ref):
    qp = (5, 7, 16)
    qa = (4, 7, 7)
    tab = list(rows("chain_p1b.txt"))
    a = np.array([[int(r[1], 16) for r in tab]], dtype=np.uint8)
    b = np.array([[int(r[2], 16) for r in tab]], dtype=np.uint8)
    for rnd, col in ((ref.FLOOR, 3), (ref.RNE, 6)):
        fp, fa = ref.QFmt(*qp, rnd), ref.QFmt(*qa, rnd)
        s = 0.0
        for k, r in enumerate(tab):
            s, ev = ref.fmaq(int(r[1], 16), int(r[2], 16), s, fp, fa)
            assert s == float(r[col]), (rnd, k)
            assert bool(ev & ref.EV_OF) == bool(int(r[col + 1])) and bool(ev & ref.EV_UF) == bool(int(r[col + 2]))
            # every prefix of the chain through the GEMM entry point
            C, of, uf = ref.gemm_bwd(a[:, :k + 1], b[:, :k + 1], fp, fa)
            assert C[0, 0] == float(r[col])
            assert (int(of[0, 0, 0]) >> k) & 1 == int(r[col + 1])
            assert (int(uf[0, 0, 0]) >> k) & 1 == int(r[col + 2])
        assert ref.gemm(a, b, fp, fa)[0, 0] == 510.0


def test_sum_is_exact_before_the_accumulator_rounds(ref):
    # 256 + (-2^-18): floor keeps 255 (the exact sum is below 256), nearest-even gives 256.
    # An FP32 add in front of the quantizer would give 256 in both cases.
    a = np.array([[0x58, 0x81]], dtype=np.uint8)
    b = np.array([[0x58, 0x01]], dtype=np.uint8)
    qp = (5, 7, 18)
    assert ref.gemm(a, b, ref.QFmt(*qp, ref.FLOOR), ref.QFmt(4, 7, 7, ref.FLOOR))[0, 0] == 255.0
    assert ref.gemm(a, b, ref.QFmt(*qp, ref.RNE), ref.QFmt(4, 7, 7, ref.RNE))[0, 0] == 256.0


def _rand_codes(rng, shape, lo_e=0, hi_e=15):
    e = rng.integers(lo_e, hi_e + 1, shape)
    m = rng.integers(0, 8, shape)
    s = rng.integers(0, 2, shape)
    c = (s << 7) | (e << 3) | m
    c = np.where((c & 0x7F) == 0x7F, c & 0xFE, c)
    return c.astype(np.uint8)


def test_wide_accumulator_equals_exact_dot_product(ref):
    rng = np.random.default_rng(5)
    A = _rand_codes(rng, (9, 300))
    B = _rand_codes(rng, (7, 300))
    va = np.vectorize(ref.decode)(A)
    vb = np.vectorize(ref.decode)(B)
    want = np.array([[math.fsum(va[i] * vb[j]) for j in range(7)] for i in range(9)])
    exact = np.array([[float(sum(Fraction(x) * Fraction(y) for x, y in zip(va[i], vb[j])))
                       for j in range(7)] for i in range(9)])
    assert (want == exact).all()
    for rnd in (ref.FLOOR, ref.RNE):
        f = ref.QFmt(7, 23, 40, rnd)
        # sums of <= 300 products of magnitude < 2^18 with unit 2^-18 need at most 45 bits > 24:
        # restrict to operands whose products all share a narrow exponent window instead
        A2 = _rand_codes(rng, (9, 200), 7, 10); B2 = _rand_codes(rng, (7, 200), 7, 10)
        va2 = np.vectorize(ref.decode)(A2); vb2 = np.vectorize(ref.decode)(B2)
        want2 = va2 @ vb2.T                                        # exact: < 24 bits everywhere
        assert ref.carrier_bits(f, f) == 320
        C = ref.gemm(A2, B2, f, f)
        assert (C.astype(np.float64) == want2).all()
        assert (ref.gemm(A2, B2, f, f, order=ref.ORDER_CHUNK16).astype(np.float64) == want2).all()


def test_chain_equals_sequential_bfloat16_accumulation(ref):
    # Q_prod = Q_acc = M7 E7 b=64 with nearest-even: products (<= 8 significant bits) are bfloat16
    # values and s <- bf16(s + p) is one correctly rounded bfloat16 add (float32 add then cast is
    # an innocuous double rounding since 24 >= 2*8+2).
    rng = np.random.default_rng(6)
    A = _rand_codes(rng, (16, 257)); B = _rand_codes(rng, (12, 257))
    a = torch.from_numpy(A).view(torch.float8_e4m3fn).float()
    b = torch.from_numpy(B).view(torch.float8_e4m3fn).float()
    s = torch.zeros(16, 12)
    for k in range(257):
        p = a[:, k:k + 1] * b[:, k:k + 1].T
        assert (p.bfloat16().float() == p).all()
        s = (s + p).bfloat16().float()
    f = ref.QFmt(7, 7, 64, ref.RNE)
    C = ref.gemm(A, B, f, f)
    assert (torch.from_numpy(C) == s).all()


def test_chain_equals_sequential_half_accumulation(ref):
    # M10 E5 b=14 nearest-even vs numpy float16 adds; operands chosen so that no partial sum is
    # subnormal in binary16 (sums are multiples of 2^-12) or overflows it
    rng = np.random.default_rng(7)
    A = _rand_codes(rng, (8, 150), 4, 11); B = _rand_codes(rng, (8, 150), 4, 11)
    va = np.vectorize(ref.decode)(A); vb = np.vectorize(ref.decode)(B)
    s = np.zeros((8, 8), dtype=np.float16)
    for k in range(150):
        p = np.outer(va[:, k], vb[:, k])
        ph = p.astype(np.float16)
        assert (ph.astype(np.float64) == p).all()
        s = (s + ph).astype(np.float16)
        assert np.isfinite(s).all()
    f = ref.QFmt(5, 10, 14, ref.RNE)
    C = ref.gemm(A, B, f, f)
    assert (C.astype(np.float64) == s.astype(np.float64)).all()


@pytest.mark.parametrize("rnd", [0, 1])
def test_brute_force_tiny_k_against_fraction_model(ref, rnd):
    fmts = [((5, 7, 15), (4, 7, 7)), ((5, 7, 16), (4, 3, 2)), ((4, 4, 6), (3, 4, 3)), ((5, 7, -1), (4, 7, -9)),
            ((6, 2, 10), (5, 10, 12))]
    rng = random.Random(8)
    for qp, qa in fmts:
        fp, fa = ref.QFmt(*qp, rnd), ref.QFmt(*qa, rnd)
        # K = 1: every pair of the subset; K = 2..4: random sequences from the subset
        seqs = [([a], [b]) for a in TINY for b in TINY]
        for K in (2, 3, 4):
            seqs += [([rng.choice(TINY) for _ in range(K)], [rng.choice(TINY) for _ in range(K)])
                     for _ in range(120)]
        for sa, sb in seqs:
            want, evs = FM.chain(sa, sb, qp + (rnd,), qa + (rnd,))
            A = np.array([sa], dtype=np.uint8); B = np.array([sb], dtype=np.uint8)
            C, of, uf = ref.gemm_bwd(A, B, fp, fa)
            assert Fraction(float(C[0, 0])) == want, (qp, qa, sa, sb)
            for k, (o, u) in enumerate(evs):
                assert (int(of[0, 0, 0]) >> k) & 1 == int(o)
                assert (int(uf[0, 0, 0]) >> k) & 1 == int(u)
            assert np.array_equal(C, ref.gemm(A, B, fp, fa))


def test_chain_invariants(ref):
    rng = np.random.default_rng(9)
    A = _rand_codes(rng, (6, 96)); B = _rand_codes(rng, (5, 96))
    for rnd in (ref.FLOOR, ref.RNE):
        fp, fa = ref.QFmt(5, 7, 15, rnd), ref.QFmt(4, 7, 7, rnd)
        rof = 510.0
        C, of, uf = ref.gemm_bwd(A, B, fp, fa)
        for i in range(6):
            for j in range(5):
                s = 0.0
                for k in range(96):
                    s2, ev = ref.fmaq(int(A[i, k]), int(B[j, k]), s, fp, fa)
                    assert ref.quantize(s2, fa) == s2                    # S_k stays on the grid
                    if ref.decode(int(A[i, k])) * ref.decode(int(B[j, k])) == 0:
                        assert s2 == s or abs(s) == rof                  # a zero product changes nothing
                    if ev & ref.EV_OF:
                        assert abs(s2) == rof
                    assert (int(of[k // 32, i, j]) >> (k % 32)) & 1 == (1 if ev & ref.EV_OF else 0)
                    assert (int(uf[k // 32, i, j]) >> (k % 32)) & 1 == (1 if ev & ref.EV_UF else 0)
                    s = s2
                assert C[i, j] == np.float32(s)
        # zero-length chain, zero stored as +0
        Z = ref.gemm(A[:, :0], B[:, :0], fp, fa)
        assert Z.shape == (6, 5) and (Z.view(np.uint32) == 0).all()


def test_threads_and_row_slabs_agree(ref):
    rng = np.random.default_rng(10)
    A = _rand_codes(rng, (37, 70)); B = _rand_codes(rng, (11, 70))
    fp, fa = ref.QFmt(5, 7, 15, 0), ref.QFmt(4, 7, 7, 0)
    C1 = ref.gemm(A, B, fp, fa, nthreads=1)
    C8 = ref.gemm(A, B, fp, fa, nthreads=8)
    assert np.array_equal(C1.view(np.uint32), C8.view(np.uint32))
    assert np.array_equal(ref.gemm(A[5:9], B, fp, fa), C1[5:9])
    r1 = ref.gemm_bwd(A, B, fp, fa, nthreads=1); r8 = ref.gemm_bwd(A, B, fp, fa, nthreads=5)
    for x, y in zip(r1, r8):
        assert np.array_equal(x, y)


def test_chunked_order(ref):
    rng = np.random.default_rng(11)
    fp, fa = (5, 7, 15), (4, 7, 7)
    for rnd in (0, 1):
        qp, qa = ref.QFmt(*fp, rnd), ref.QFmt(*fa, rnd)
        # K <= 16: one chunk, the second level adds it to zero and re-quantizes a grid value
        A = _rand_codes(rng, (5, 16)); B = _rand_codes(rng, (4, 16))
        assert np.array_equal(ref.gemm(A, B, qp, qa, order=ref.ORDER_CHUNK16), ref.gemm(A, B, qp, qa))
        # general K against the Fraction model, including a short last chunk
        A = _rand_codes(rng, (3, 41), 5, 12); B = _rand_codes(rng, (2, 41), 5, 12)
        C = ref.gemm(A, B, qp, qa, order=ref.ORDER_CHUNK16)
        for i in range(3):
            for j in range(2):
                want = FM.chain_chunk16([int(c) for c in A[i]], [int(c) for c in B[j]], fp + (rnd,), fa + (rnd,))
                assert Fraction(float(C[i, j])) == want


def test_chunked_order_event_planes(ref):
    """First- and second-level event bits of the two-level order against the Fraction model."""
    rng = np.random.default_rng(12)

    def bit(plane, idx, i, j):
        return bool((int(plane[idx // 32, i, j]) >> (idx % 32)) & 1)

    for (fp, fa), rnd, K, lo, hi in [(((5, 7, 15), (4, 7, 7)), 0, 41, 3, 12), (((5, 7, 15), (4, 7, 7)), 1, 50, 0, 15),
                                     (((4, 7, 9), (4, 3, 7)), 0, 530, 2, 11), (((3, 4, 6), (3, 4, 6)), 1, 37, 4, 10)]:
        qp, qa = ref.QFmt(*fp, rnd), ref.QFmt(*fa, rnd)
        A = _rand_codes(rng, (2, K), lo, hi); B = _rand_codes(rng, (2, K), lo, hi)
        C, of, uf, of2, uf2 = ref.gemm_bwd(A, B, qp, qa, order=ref.ORDER_CHUNK16, level2=True)
        assert np.array_equal(C.view(np.uint32), ref.gemm(A, B, qp, qa, order=ref.ORDER_CHUNK16).view(np.uint32))
        nchunk = (K + 15) // 16
        assert of.shape[0] == (K + 31) // 32 and of2.shape[0] == (nchunk + 31) // 32
        seen = [0, 0, 0, 0]
        for i in range(2):
            for j in range(2):
                want, ev1, ev2 = FM.chain_chunk16([int(c) for c in A[i]], [int(c) for c in B[j]],
                                                  fp + (rnd,), fa + (rnd,), with_events=True)
                assert Fraction(float(C[i, j])) == want
                for k in range(K):
                    assert (bit(of, k, i, j), bit(uf, k, i, j)) == ev1[k], (fp, fa, rnd, i, j, k)
                    seen[0] += ev1[k][0]; seen[1] += ev1[k][1]
                for c in range(nchunk):
                    assert (bit(of2, c, i, j), bit(uf2, c, i, j)) == ev2[c], (fp, fa, rnd, i, j, c)
                    seen[2] += ev2[c][0]; seen[3] += ev2[c][1]
                # padding bits are zero
                for k in range(K, 32 * of.shape[0]):
                    assert not bit(of, k, i, j) and not bit(uf, k, i, j)
                for c in range(nchunk, 32 * of2.shape[0]):
                    assert not bit(of2, c, i, j) and not bit(uf2, c, i, j)
        print(fp, fa, rnd, "events seen (OF, UF, OF2, UF2):", seen)
    # a second-level underflow needs cancellation between two values of the grid: chunk 0 sums to
    # 1.5 * 2^-7, chunk 1 to -2^-7; T_2 = 2^-8 is below R_UF = 2^-7 and not zero
    A = np.zeros((1, 20), dtype=np.uint8); B = np.zeros((1, 20), dtype=np.uint8)
    A[0, 0], B[0, 0] = 0x3C, 0x04            # 1.5 * 2^-7
    A[0, 16], B[0, 16] = 0xB8, 0x04          # -1 * 2^-7
    for rnd in (0, 1):
        C, of, uf, of2, uf2 = ref.gemm_bwd(A, B, ref.QFmt(5, 7, 15, rnd), ref.QFmt(4, 7, 7, rnd),
                                           order=ref.ORDER_CHUNK16, level2=True)
        assert C[0, 0] == 0.0 and int(uf2[0, 0, 0]) == 0b10 and int(of2[0, 0, 0]) == 0
        assert int(uf[0, 0, 0]) == 0 and int(of[0, 0, 0]) == 0


def test_hand_worked_diff_estimator(ref):
    qp, qa = (5, 7, 16), (4, 7, 7)
    tab = list(rows("chain_diff.txt"))
    a = np.array([[int(r[1], 16) for r in tab]], dtype=np.uint8)
    b = np.array([[int(r[2], 16) for r in tab]], dtype=np.uint8)
    for rnd, col in ((ref.FLOOR, 3), (ref.RNE, 6)):
        fp, fa = ref.QFmt(*qp, rnd), ref.QFmt(*qa, rnd)
        for c, eps2 in enumerate((0.0, 0.5, 0.75)):
            C, diff = ref.gemm_diff(a, b, fp, fa, eps2)
            assert C[0, 0] == 510.0
            for k, r in enumerate(tab):
                assert (int(diff[0, 0, 0]) >> k) & 1 == 1 - int(r[col + c]), (rnd, eps2, k)   # the plane holds 1 - STE
            assert int(diff[0, 0, 0]) >> len(tab) == 0
        # a ratio equal to the threshold does not pass (strict inequality): step 0 has ratio exactly 1
        assert int(ref.gemm_diff(a, b, fp, fa, 1.0)[1][0, 0, 0]) & 1 == 1
        assert int(ref.gemm_diff(a, b, fp, fa, 0.999)[1][0, 0, 0]) & 1 == 0


@pytest.mark.parametrize("rnd", [0, 1])
def test_diff_estimator_against_fraction_model(ref, rnd):
    """The DIFF plane against the ratio written out with Fractions, for dyadic and non-dyadic thresholds; a
    finite eps1 far below every quantity in play gives the same bits as the limit the oracle implements."""
    fmts = [((5, 7, 15), (4, 7, 7)), ((5, 7, 16), (4, 3, 2)), ((4, 4, 6), (3, 4, 3)), ((5, 7, -1), (4, 7, -9)),
            ((6, 2, 10), (5, 10, 12)), ((5, 7, 15), (4, 7, 7 | 0)), ((5, 7, 12), (4, 7, 10))]
    rng = random.Random(21)
    seen = {0: 0, 1: 0}
    for qp, qa in fmts:
        fp, fa = ref.QFmt(*qp, rnd), ref.QFmt(*qa, rnd)
        seqs = [([x], [y]) for x in TINY[::2] for y in TINY[::3]]
        for K in (2, 3, 5):
            seqs += [([rng.choice(TINY) for _ in range(K)], [rng.choice(TINY) for _ in range(K)]) for _ in range(60)]
        for eps2 in (0.0, 2.0 ** -6, 0.3, 0.5, 1.0, 1.75):
            for sa, sb in seqs:
                want_s, ste = FM.chain_diff(sa, sb, qp + (rnd,), qa + (rnd,), Fraction(eps2))
                _, ste_e1 = FM.chain_diff(sa, sb, qp + (rnd,), qa + (rnd,), Fraction(eps2), Fraction(1, 2 ** 90))
                if eps2 > 0:
                    assert ste == ste_e1
                A = np.array([sa], dtype=np.uint8); B = np.array([sb], dtype=np.uint8)
                C, diff = ref.gemm_diff(A, B, fp, fa, eps2)
                assert Fraction(float(C[0, 0])) == want_s
                for k, v in enumerate(ste):
                    assert (int(diff[0, 0, 0]) >> k) & 1 == 1 - v, (qp, qa, eps2, sa, sb, k)
                    seen[v] += 1
    assert seen[0] > 500 and seen[1] > 500


def test_diff_plane_properties(ref):
    """eps2 = 0 marks exactly the steps that leave the sum unchanged; the blocked set grows with eps2; product
    underflows are always blocked; the value C does not depend on eps2; under the chunked order the bits are
    those of each chunk's own chain from zero."""
    rng = np.random.default_rng(5)
    A = rng.integers(0, 256, size=(6, 70), dtype=np.uint8); A[(A & 0x7F) == 0x7F] = 0x3A
    B = rng.integers(0, 256, size=(5, 70), dtype=np.uint8); B[(B & 0x7F) == 0x7F] = 0x41
    for rnd in (ref.FLOOR, ref.RNE):
        fp, fa = ref.QFmt(5, 7, 12, rnd), ref.QFmt(4, 7, 10, rnd)
        C0, of, uf = ref.gemm_bwd(A, B, fp, fa)
        prev = None
        for eps2 in (0.0, 2.0 ** -8, 0.125, 0.5, 1.0, 4.0):
            C, diff = ref.gemm_diff(A, B, fp, fa, eps2)
            assert np.array_equal(C, C0)
            if prev is not None:
                assert (prev & ~diff).max() == 0 and (diff & ~prev).max() > 0
            prev = diff
        # eps2 = 0: replay every chain one step at a time and mark the steps that did not move the sum
        _, nc = ref.gemm_diff(A, B, fp, fa, 0.0)
        for m in range(A.shape[0]):
            for n in range(B.shape[0]):
                s = 0.0
                for k in range(A.shape[1]):
                    z, ev = ref.fmaq(int(A[m, k]), int(B[n, k]), s, fp, fa)
                    assert (int(nc[k // 32, m, n]) >> (k % 32)) & 1 == int(z == s)
                    if ev & ref.EV_UF and ref.decode(A[m, k]) * ref.decode(B[n, k]) != 0 and z == s:
                        assert (int(prev[k // 32, m, n]) >> (k % 32)) & 1
                    s = z
        assert nc.max() > 0
        # chunked order: chunk j's bits = the bits of the product of columns 16j .. 16j+15 alone
        _, dch = ref.gemm_diff(A, B, fp, fa, 0.25, order=ref.ORDER_CHUNK16)
        for j in range(0, 70, 16):
            _, dj = ref.gemm_diff(A[:, j:j + 16], B[:, j:j + 16], fp, fa, 0.25)
            got = (dch[j // 32] >> (j % 32)) & ((1 << min(16, 70 - j)) - 1)
            assert np.array_equal(got, dj[0])
        assert np.array_equal(ref.gemm_diff(A, B, fp, fa, 0.25, order=ref.ORDER_CHUNK16)[0],
                              ref.gemm(A, B, fp, fa, order=ref.ORDER_CHUNK16))


def test_input_code_formats(ref):
    """Operands in other 8-bit formats (the paper's M4E3 with a per-tensor bias, Sec. 3.1)."""
    import torch
    # decode: library casts where a standard format exists, the closed form everywhere
    for c in range(256):
        if (c & 0x7F) != 0x7F:
            t = torch.tensor([c], dtype=torch.uint8).view(torch.float8_e4m3fn).float().item()
            assert ref.decode_in(c, ref.InFmt(4, 3, 7)) == t == ref.decode(c)
        if ((c >> 2) & 31) != 31:                                    # binary8 E5M2: e = 31 is inf / NaN there
            t = torch.tensor([c], dtype=torch.uint8).view(torch.float8_e5m2).float().item()
            assert ref.decode_in(c, ref.InFmt(5, 2, 15)) == t
        for (E, M, b) in ((3, 4, 3), (3, 4, -2), (2, 5, 1), (5, 2, 20), (4, 3, 0)):
            assert Fraction(ref.decode_in(c, ref.InFmt(E, M, b))) == FM.code_value(c, E, M, b)
    assert ref.decode_in(0x7F, ref.InFmt(3, 4, 3)) == 31.0 and ref.decode_in(0x01, ref.InFmt(3, 4, 3)) == 2.0 ** -6
    # a 10-bit product that Q_prod (M = 7) must round: (1 + 13/16)(1 + 11/16) = 783/256 = 1100001111b * 2^-8
    A = np.array([[0x3D]], dtype=np.uint8); B = np.array([[0x3B]], dtype=np.uint8)   # e = 3 -> 2^0 with bias 3
    f = ref.InFmt(3, 4, 3)
    wide = ref.QFmt(6, 12, 20, 0)
    assert ref.gemm_in(A, B, f, f, ref.QFmt(5, 7, 15, 0), wide)[0, 0] == 195 / 64      # floor
    assert ref.gemm_in(A, B, f, f, ref.QFmt(5, 7, 15, 1), wide)[0, 0] == 196 / 64      # nearest
    assert ref.gemm_in(A, B, f, f, ref.QFmt(5, 9, 15, 0), wide)[0, 0] == 783 / 256     # wide enough: exact
    # brute force against the Fraction model, events included, product rounding active
    rng = np.random.default_rng(21)
    for (ia, ib), (fp, fa), rnd, K in [(((3, 4, 3), (3, 4, 5)), ((5, 7, 15), (4, 7, 7)), 0, 30),
                                       (((3, 4, 2), (4, 3, 7)), ((5, 7, 15), (4, 7, 7)), 1, 30),
                                       (((2, 5, 0), (5, 2, 12)), ((5, 5, 12), (5, 9, 14)), 1, 24),
                                       (((3, 4, 4), (3, 4, 4)), ((3, 4, 6), (3, 4, 6)), 0, 20)]:
        A = rng.integers(0, 256, (3, K)).astype(np.uint8); B = rng.integers(0, 256, (2, K)).astype(np.uint8)
        C, of, uf = ref.gemm_in(A, B, ref.InFmt(*ia), ref.InFmt(*ib), ref.QFmt(*fp, rnd), ref.QFmt(*fa, rnd), planes=True)
        for i in range(3):
            for j in range(2):
                want, evs = FM.chain([int(c) for c in A[i]], [int(c) for c in B[j]], fp + (rnd,), fa + (rnd,), ia, ib)
                assert Fraction(float(C[i, j])) == want, (ia, ib, fp, fa, rnd, i, j)
                for k in range(K):
                    got = (bool((int(of[0, i, j]) >> k) & 1), bool((int(uf[0, i, j]) >> k) & 1))
                    assert got == evs[k], (ia, ib, k)
        # the DIFF plane with these operand formats: the un-quantized product is the one of the decoded codes
        for eps2 in (0.0, 0.25, 0.875):
            Cd, diff = ref.gemm_diff(A, B, ref.QFmt(*fp, rnd), ref.QFmt(*fa, rnd), eps2, fmt_a=ref.InFmt(*ia), fmt_b=ref.InFmt(*ib))
            assert np.array_equal(Cd, C)
            for i in range(3):
                for j in range(2):
                    _, ste = FM.chain_diff([int(c) for c in A[i]], [int(c) for c in B[j]], fp + (rnd,), fa + (rnd,),
                                           Fraction(eps2), None, ia, ib)
                    for k in range(K):
                        assert (int(diff[0, i, j]) >> k) & 1 == 1 - ste[k], (ia, ib, eps2, i, j, k)
    # the exponent biases are power-of-two scales: moving them moves the quantizers' biases and the result
    A = rng.integers(0, 256, (6, 50)).astype(np.uint8); B = rng.integers(0, 256, (5, 50)).astype(np.uint8)
    base = ref.gemm_in(A, B, ref.InFmt(3, 4, 3), ref.InFmt(3, 4, 3), ref.QFmt(5, 7, 15, 0), ref.QFmt(4, 7, 7, 0))
    moved = ref.gemm_in(A, B, ref.InFmt(3, 4, 5), ref.InFmt(3, 4, 0), ref.QFmt(5, 7, 14, 0), ref.QFmt(4, 7, 6, 0))
    assert np.array_equal(moved, base * 2.0) and np.count_nonzero(base) > 20
    with pytest.raises(ValueError):
        ref.gemm_in(A, B, ref.InFmt(3, 3, 3), ref.InFmt(3, 4, 3), ref.QFmt(5, 7, 15, 0), ref.QFmt(4, 7, 7, 0))
    with pytest.raises(ValueError):
        ref.gemm_in(A, B, ref.InFmt(3, 4, 40), ref.InFmt(3, 4, 3), ref.QFmt(5, 7, 15, 0), ref.QFmt(4, 7, 7, 0))


def test_im2col_against_the_definition(ref):
    """The written-out convolution operand, element by element from the definition of a padded, strided window,
    and against torch's unfold (channel-major there, so the taps are compared after a transpose)."""
    import torch
    rng = np.random.default_rng(31)
    for (n, h, w, c, kh, kw, stride, pad) in [(2, 4, 5, 3, 3, 3, 2, 1), (1, 6, 6, 2, 1, 1, 2, 0), (2, 5, 7, 4, 3, 2, 1, 2)]:
        X = rng.integers(0, 256, (n, h, w, c)).astype(np.uint8)
        A = ref.im2col_nhwc(X, kh, kw, stride, pad)
        oh = (h + 2 * pad - kh) // stride + 1
        ow = (w + 2 * pad - kw) // stride + 1
        assert A.shape == (n * oh * ow, kh * kw * c)
        for m in range(A.shape[0]):
            img, rem = divmod(m, oh * ow)
            y, x = divmod(rem, ow)
            for i in range(kh):
                for j in range(kw):
                    ih, iw = y * stride - pad + i, x * stride - pad + j
                    inside = 0 <= ih < h and 0 <= iw < w
                    for ch in range(c):
                        assert A[m, (i * kw + j) * c + ch] == (X[img, ih, iw, ch] if inside else 0)
        U = torch.nn.functional.unfold(torch.from_numpy(X).permute(0, 3, 1, 2).float(), (kh, kw), padding=pad, stride=stride)
        U = U.reshape(n, c, kh * kw, oh * ow).permute(0, 3, 2, 1).reshape(n * oh * ow, kh * kw * c)     # (c, tap) -> (tap, c)
        assert np.array_equal(U.numpy().astype(np.uint8), A)


def test_oracle_rejects_bad_arguments(ref):
    A = np.zeros((2, 4), dtype=np.uint8)
    good = ref.QFmt(4, 7, 7, 0)
    for bad in (ref.QFmt(4, 0, 7, 0), ref.QFmt(8, 7, 7, 0), ref.QFmt(4, 7, 127, 0), ref.QFmt(4, 7, 7, 2),
                ref.QFmt(7, 7, -1, 0), ref.QFmt(1, 7, 0, 0), ref.QFmt(4, 24, 7, 0)):
        with pytest.raises(ValueError):
            ref.gemm(A, A, bad, good)
        with pytest.raises(ValueError):
            ref.gemm(A, A, good, bad)
    with pytest.raises(ValueError):
        ref.gemm(A, A, good, good, order=7)
