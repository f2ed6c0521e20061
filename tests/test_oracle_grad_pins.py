"""Pins of the gradient oracle (oracle/lba_grad_ref.py) to things other than itself: a library matmul
for the identity estimator, hand-worked coefficient patterns, an independently written Fraction model
(events and exact rational sums) on tiny cases, and the structural relations between the estimators
(Sec. 4 and App. D of the paper)."""
from fractions import Fraction

import numpy as np
import pytest

import frac_model as FM


@pytest.fixture(scope="module")
def gref(ref):
    from oracle import lba_grad_ref
    return lba_grad_ref


def _codes(rng, shape, lo=0, hi=15):
    e = rng.integers(lo, hi + 1, shape); m = rng.integers(0, 8, shape); s = rng.integers(0, 2, shape)
    c = (s << 7) | (e << 3) | m
    return np.where((c & 0x7F) == 0x7F, c & 0xFE, c).astype(np.uint8)


def test_identity_estimator_is_the_plain_matmul_backward(ref, gref):
    rng = np.random.default_rng(1)
    A = _codes(rng, (9, 40)); B = _codes(rng, (7, 40))
    G = rng.standard_normal((9, 7))
    tab = np.array([ref.decode(c) for c in range(256)])
    dX, dW = gref.grad(G, A, B, ref.QFmt(5, 7, 15, 0), ref.QFmt(4, 7, 7, 0), gref.STE_IDENTITY)
    assert np.allclose(dX, G @ tab[B], rtol=1e-13, atol=0) and np.allclose(dW, G.T @ tab[A], rtol=1e-13, atol=0)
    # formats too wide to overflow: every estimator is the identity
    for ste in (gref.STE_IMMEDIATE_OF, gref.STE_RECURSIVE_OF):
        for order in (ref.ORDER_SEQ, ref.ORDER_CHUNK16):
            dX2, dW2 = gref.grad(G, A, B, ref.QFmt(6, 7, 20, 0), ref.QFmt(7, 12, 40, 0), ste, order)
            assert np.array_equal(dX2, dX) and np.array_equal(dW2, dW)


def test_hand_worked_coefficient_patterns(ref, gref):
    # Q_acc = M7E4 b=7: R_OF = 510.  448 * 448 overflows when added; -448 brings the sum back to 62.
    P, N448, ONE, Z = 0x7E, 0xFE, 0x38, 0x00          # +448, -448, 1.0, 0
    qp, qa = ref.QFmt(5, 7, 15, 0), ref.QFmt(4, 7, 7, 0)
    cases = [  # (a codes, b codes, OF pattern, immediate c, recursive c)
        ([P, N448, ONE], [P, ONE, ONE], [1, 0, 0], [0, 1, 1], [0, 1, 1]),
        ([ONE, P, N448], [ONE, P, ONE], [0, 1, 0], [1, 0, 1], [0, 0, 1]),
        ([ONE, ONE, P], [ONE, ONE, P], [0, 0, 1], [1, 1, 0], [0, 0, 0]),
        ([ONE, Z, ONE], [ONE, P, ONE], [0, 0, 0], [1, 1, 1], [1, 1, 1]),
    ]
    g = 0.75
    tab = np.array([ref.decode(c) for c in range(256)])
    for a, b, of_want, c_imm, c_rec in cases:
        A = np.array([a], dtype=np.uint8); B = np.array([b], dtype=np.uint8)
        _, of, _ = ref.gemm_bwd(A, B, qp, qa)
        assert [int(of[0, 0, 0] >> k) & 1 for k in range(3)] == of_want
        last = gref.last_overflow(of, 3)[0, 0]
        assert last == max([k for k in range(3) if of_want[k]], default=-1)
        for ste, c in ((gref.STE_IMMEDIATE_OF, c_imm), (gref.STE_RECURSIVE_OF, c_rec), (gref.STE_IDENTITY, [1, 1, 1])):
            assert gref.coefficients(A, B, qp, qa, ste)[0, 0].astype(int).tolist() == c
            dX, dW = gref.grad(np.array([[g]]), A, B, qp, qa, ste)
            assert dX[0].tolist() == [g * tab[b[k]] * c[k] for k in range(3)]
            assert dW[0].tolist() == [g * tab[a[k]] * c[k] for k in range(3)]


def _frac_grad(G, A, B, qp, qa, ste, chunked):
    """Exact rational dX, dW with events from the Fraction model."""
    M, K = A.shape
    N = B.shape[0]
    dX = [[Fraction(0)] * K for _ in range(M)]
    dW = [[Fraction(0)] * K for _ in range(N)]
    for m in range(M):
        for n in range(N):
            a = [int(c) for c in A[m]]; b = [int(c) for c in B[n]]
            if chunked:
                _, ev1, ev2 = FM.chain_chunk16(a, b, qp, qa, with_events=True)
            else:
                _, ev1 = FM.chain(a, b, qp, qa)
                ev2 = []
            for k in range(K):
                if ste == 0:
                    c = 1
                elif ste == 1:
                    c = 0 if ev1[k][0] else 1
                else:
                    if chunked:
                        j = k // 16
                        path = [ev1[i][0] for i in range(k, min(K, 16 * j + 16))] + [ev2[jj][0] for jj in range(j, len(ev2))]
                    else:
                        path = [ev1[i][0] for i in range(k, K)]
                    c = 0 if any(path) else 1
                g = Fraction(float(G[m, n]))
                dX[m][k] += g * FM.e4m3_value(b[k]) * c
                dW[n][k] += g * FM.e4m3_value(a[k]) * c
    return dX, dW


@pytest.mark.parametrize("chunked", [False, True])
def test_brute_force_against_fraction_model(ref, gref, chunked):
    rng = np.random.default_rng(2 + chunked)
    order = ref.ORDER_CHUNK16 if chunked else ref.ORDER_SEQ
    for (fp, fa), rnd, K, lo, hi in [(((5, 7, 15), (4, 7, 7)), 0, 37, 3, 12), (((4, 7, 9), (4, 3, 7)), 1, 50, 2, 12),
                                     (((3, 4, 6), (3, 4, 6)), 0, 20, 4, 10)]:
        A = _codes(rng, (3, K), lo, hi); B = _codes(rng, (2, K), lo, hi)
        G = rng.integers(-8, 9, (3, 2)) / 4.0                       # exact in binary
        zeros = 0
        for ste in (0, 1, 2):
            dX, dW = gref.grad(G, A, B, ref.QFmt(*fp, rnd), ref.QFmt(*fa, rnd), ste, order)
            wX, wW = _frac_grad(G, A, B, fp + (rnd,), fa + (rnd,), ste, chunked)
            for m in range(3):
                for k in range(K):
                    assert Fraction(float(dX[m, k])) == wX[m][k], (fp, fa, ste, m, k)
            for n in range(2):
                for k in range(K):
                    assert Fraction(float(dW[n, k])) == wW[n][k], (fp, fa, ste, n, k)
            zeros += int((~gref.coefficients(A, B, ref.QFmt(*fp, rnd), ref.QFmt(*fa, rnd), ste, order)).sum())
        assert zeros > 0                                            # the case exercises overflow events


def test_relations_between_the_estimators(ref, gref):
    rng = np.random.default_rng(4)
    A = _codes(rng, (12, 100), 3, 12); B = _codes(rng, (10, 100), 3, 12)
    qp, qa = ref.QFmt(5, 7, 15, 0), ref.QFmt(4, 7, 7, 0)
    for order in (ref.ORDER_SEQ, ref.ORDER_CHUNK16):
        c_imm = gref.coefficients(A, B, qp, qa, gref.STE_IMMEDIATE_OF, order)
        c_rec = gref.coefficients(A, B, qp, qa, gref.STE_RECURSIVE_OF, order)
        assert (c_rec <= c_imm).all() and c_imm.sum() < c_imm.size and c_rec.sum() < c_imm.sum()
        # a recursive coefficient is non-increasing when walking back from the end of a path
        if order == ref.ORDER_SEQ:
            assert (np.diff(c_rec.astype(int), axis=2) >= 0).all()
            _, of, _ = ref.gemm_bwd(A, B, qp, qa)
            last = gref.last_overflow(of, 100)
            assert np.array_equal(c_rec, np.arange(100)[None, None, :] > last[:, :, None])
    # linear in g
    G1 = rng.standard_normal((12, 10)); G2 = rng.standard_normal((12, 10))
    d1 = gref.grad(G1, A, B, qp, qa, 2); d2 = gref.grad(G2, A, B, qp, qa, 2); d3 = gref.grad(G1 + 2 * G2, A, B, qp, qa, 2)
    assert np.allclose(d3[0], d1[0] + 2 * d2[0], rtol=1e-12, atol=1e-9) and np.allclose(d3[1], d1[1] + 2 * d2[1], rtol=1e-12, atol=1e-9)


def test_immediate_diff_coefficients_against_fraction_model(ref, gref):
    """'Immediate / DIFF' (Sec. 4): the coefficients are STE^DIFF itself, step by step, from the ratio written
    with Fractions; they block at least every overflow that moved the sum by less than eps2 |x w|, every fully
    swamped step and every product underflow, and the gradient is the plain sum over the kept terms."""
    rng = np.random.default_rng(12)
    for (fp, fa), rnd, K, lo, hi, eps2 in [(((5, 7, 15), (4, 7, 7)), 0, 37, 3, 12, 0.25), (((4, 7, 9), (4, 3, 7)), 1, 40, 2, 12, 0.5),
                                           (((3, 4, 6), (3, 4, 6)), 0, 20, 4, 10, 0.0)]:
        A = _codes(rng, (3, K), lo, hi); B = _codes(rng, (2, K), lo, hi)
        qp, qa = ref.QFmt(*fp, rnd), ref.QFmt(*fa, rnd)
        c = gref.coefficients(A, B, qp, qa, gref.STE_IMMEDIATE_DIFF, eps2=eps2)
        for m in range(3):
            for n in range(2):
                _, ste = FM.chain_diff([int(x) for x in A[m]], [int(x) for x in B[n]], fp + (rnd,), fa + (rnd,), Fraction(eps2))
                assert [int(v) for v in c[m, n]] == ste, (fp, fa, m, n)
        assert 0 < c.sum() < c.size
        G = rng.integers(-8, 9, (3, 2)) / 4.0
        dX, dW = gref.grad(G, A, B, qp, qa, gref.STE_IMMEDIATE_DIFF, c=c)
        tab = gref.decode_table()
        for m in range(3):
            for k in range(K):
                assert dX[m, k] == sum(G[m, n] * tab[B[n, k]] * c[m, n, k] for n in range(2))
        for n in range(2):
            for k in range(K):
                assert dW[n, k] == sum(G[m, n] * tab[A[m, k]] * c[m, n, k] for m in range(3))


def test_sum_of_magnitudes_that_scales_the_fp32_tolerance(ref, gref):
    """grad_abs (sum over the kept terms of |g| * |value|) sets the tolerance of every floating-point gradient
    parity test, so it is pinned like the sums themselves: hand-worked single chains from the coefficient
    patterns above, a library matmul of magnitudes for the identity estimator, the Fraction model on a case
    with overflows, and the inequalities that any sum of magnitudes satisfies."""
    P, N448, ONE, Z = 0x7E, 0xFE, 0x38, 0x00          # +448, -448, 1.0, 0
    qp, qa = ref.QFmt(5, 7, 15, 0), ref.QFmt(4, 7, 7, 0)
    # (a codes, b codes, immediate c, recursive c): the patterns of test_hand_worked_coefficient_patterns
    cases = [([P, N448, ONE], [P, ONE, ONE], [0, 1, 1], [0, 1, 1]),
             ([ONE, P, N448], [ONE, P, ONE], [1, 0, 1], [0, 0, 1]),
             ([ONE, ONE, P], [ONE, ONE, P], [1, 1, 0], [0, 0, 0])]
    val = {P: 448.0, N448: 448.0, ONE: 1.0, Z: 0.0}    # magnitudes, typed by hand
    for a, b, c_imm, c_rec in cases:
        A = np.array([a], dtype=np.uint8); B = np.array([b], dtype=np.uint8)
        for g in (0.75, -0.75):
            for ste, c in ((gref.STE_IMMEDIATE_OF, c_imm), (gref.STE_RECURSIVE_OF, c_rec), (gref.STE_IDENTITY, [1, 1, 1])):
                aX, aW = gref.grad_abs(np.array([[g]]), A, B, qp, qa, ste)
                assert aX.shape == (1, 3) and aW.shape == (1, 3)
                assert aX[0].tolist() == [0.75 * val[b[k]] * c[k] for k in range(3)]
                assert aW[0].tolist() == [0.75 * val[a[k]] * c[k] for k in range(3)]
    # identity estimator: |G| times the matrix of magnitudes (library matmul)
    rng = np.random.default_rng(21)
    A = _codes(rng, (9, 40)); B = _codes(rng, (7, 40))
    G = rng.standard_normal((9, 7))
    tab = np.array([abs(ref.decode(c)) for c in range(256)])
    aX, aW = gref.grad_abs(G, A, B, qp, qa, gref.STE_IDENTITY)
    assert np.allclose(aX, np.abs(G) @ tab[B], rtol=1e-13, atol=0) and np.allclose(aW, np.abs(G).T @ tab[A], rtol=1e-13, atol=0)
    # with overflows, both orders: exact rational sums of magnitudes from the Fraction model's events
    # (all-positive gradients and operands make the plain sums of _frac_grad sums of magnitudes)
    for chunked in (False, True):
        order = ref.ORDER_CHUNK16 if chunked else ref.ORDER_SEQ
        K = 37
        A = _codes(rng, (3, K), 3, 12); B = _codes(rng, (2, K), 3, 12)
        G = rng.integers(-8, 9, (3, 2)) / 4.0
        for ste in (0, 1, 2):
            aX, aW = gref.grad_abs(G, A, B, qp, qa, ste, order)
            dX, dW = gref.grad(G, A, B, qp, qa, ste, order)
            assert (aX >= np.abs(dX)).all() and (aW >= np.abs(dW)).all()            # triangle inequality
            # same events (they depend on the signed operands), magnitudes summed exactly
            M_, N_ = 3, 2
            wX = [[Fraction(0)] * K for _ in range(M_)]; wW = [[Fraction(0)] * K for _ in range(N_)]
            for m in range(M_):
                for n in range(N_):
                    a = [int(c) for c in A[m]]; b = [int(c) for c in B[n]]
                    if chunked:
                        _, ev1, ev2 = FM.chain_chunk16(a, b, (5, 7, 15, 0), (4, 7, 7, 0), with_events=True)
                    else:
                        _, ev1 = FM.chain(a, b, (5, 7, 15, 0), (4, 7, 7, 0)); ev2 = []
                    for k in range(K):
                        if ste == 0:
                            c = 1
                        elif ste == 1:
                            c = 0 if ev1[k][0] else 1
                        else:
                            j = k // 16
                            path = ([ev1[i][0] for i in range(k, min(K, 16 * j + 16))] + [ev2[jj][0] for jj in range(j, len(ev2))]
                                    if chunked else [ev1[i][0] for i in range(k, K)])
                            c = 0 if any(path) else 1
                        g = abs(Fraction(float(G[m, n])))
                        wX[m][k] += g * abs(FM.e4m3_value(b[k])) * c
                        wW[n][k] += g * abs(FM.e4m3_value(a[k])) * c
            assert all(Fraction(float(aX[m, k])) == wX[m][k] for m in range(M_) for k in range(K))
            assert all(Fraction(float(aW[n, k])) == wW[n][k] for n in range(N_) for k in range(K))
    # a sign flip of g or of an operand column that leaves the events alone leaves the magnitudes alone:
    # identity estimator, any signs
    aX2, aW2 = gref.grad_abs(-G, A, B, qp, qa, gref.STE_IDENTITY)
    aX1, aW1 = gref.grad_abs(G, A, B, qp, qa, gref.STE_IDENTITY)
    assert np.array_equal(aX1, aX2) and np.array_equal(aW1, aW2)
    assert np.array_equal(gref.grad_abs(G, A ^ 0x80, B, qp, qa, gref.STE_IDENTITY)[1], aW1)
