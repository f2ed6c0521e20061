"""Collected first among the GPU tests (file name): the arithmetic of the scaled-domain kernels leans on the wave's
FP32 mode register (rounding toward zero for the paper's floor rounding, flushed denormals), which inline
assembly sets around ordinary compiler-generated multiplies and fused multiply-adds.  If a compiler ever folded,
reassociated or moved those across the mode writes, the cheapest place to see it is one FMAq step on every pair of
codes: C[a, b] = Q_acc(Q_prod(a * b)) for all 256 x 256 pairs, once per product mode of the kernels (identity,
flush, flush + clamp, truncated mantissa with and without clamp, nearest-even mantissa with and without clamp), floor
and nearest-even, both orders, plus a two-step chain whose second product is far below the first (the case where
rounding the exact sum toward zero and to nearest differ).  Everything against the oracle, bit for bit."""
import numpy as np
import pytest
import torch

from paper_2401_14110_amd import binding as lb

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

# (Q_prod, Q_acc) that select each product mode of the scaled kernel for E4M3 operands (prod_mode of the plan)
MODES = {0: ((6, 7, 20), (4, 7, 7)), 1: ((5, 7, -1), (4, 7, -9)), 2: ((5, 7, 15), (4, 7, 7))}
# ... and for the paper's M4E3 operands (10-bit products: Q_prod's mantissa takes part)
MODES_IN = {3: ((6, 4, 20), (4, 7, 7), 0), 4: ((5, 4, 23), (4, 7, 7), 0), 5: ((6, 4, 20), (4, 7, 7), 1), 6: ((5, 4, 23), (4, 7, 7), 1)}


def bits(x):
    return np.ascontiguousarray(x).view(np.uint32)


def test_one_step_on_every_code_pair_per_product_mode(ref):
    codes = np.arange(256, dtype=np.uint8).reshape(256, 1)
    t = torch.from_numpy(codes).to(DEV)
    for mode, (qp, qa) in MODES.items():
        for rnd in (0, 1):
            for order in (0, 1):
                qpf, qaf = qp + (rnd,), qa + (rnd,)
                assert lb.lba_plan_query(256, 256, 1, qpf, qaf, order)["prod_mode"] == mode
                got = lb.gemm(t, t, qpf, qaf, order=order)
                torch.cuda.synchronize()
                want = ref.gemm(codes, codes, ref.QFmt(*qpf), ref.QFmt(*qaf), order=order)
                assert np.array_equal(bits(got.cpu().numpy()), bits(want)), (mode, rnd, order)
    m4e3 = (3, 4, 3)
    for mode, (qp, qa, rnd) in MODES_IN.items():
        qpf, qaf = qp + (rnd,), qa + (rnd,)
        assert lb.lba_plan_query_in(256, 256, 1, m4e3, m4e3, qpf, qaf)["prod_mode"] == mode
        got = lb.gemm_in(t, t, m4e3, m4e3, qpf, qaf)
        torch.cuda.synchronize()
        want = ref.gemm_in(codes, codes, ref.InFmt(*m4e3), ref.InFmt(*m4e3), ref.QFmt(*qpf), ref.QFmt(*qaf))
        assert np.array_equal(bits(got.cpu().numpy()), bits(want)), (mode, rnd)


def test_two_steps_where_the_rounding_direction_shows(ref):
    # S_1 = a0 * b0 for every pair, then a tiny second product of either sign: under floor the exact sum is
    # truncated toward zero (256 - 2^-18 -> 255), under nearest-even it is not (-> 256)
    codes = np.arange(256, dtype=np.uint8)
    codes = np.where((codes & 0x7F) == 0x7F, codes & 0xFE, codes).astype(np.uint8)
    for tiny in (0x01, 0x81, 0x09):
        A = np.stack([codes, np.full(256, tiny, dtype=np.uint8)], axis=1)
        B = np.stack([codes, np.full(256, 0x01, dtype=np.uint8)], axis=1)
        tA, tB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
        for qp, qa in (((5, 7, 18), (4, 7, 7)), ((6, 7, 20), (5, 10, 15)), ((5, 7, 18), (4, 3, 7))):
            for rnd in (0, 1):
                qpf, qaf = qp + (rnd,), qa + (rnd,)
                got = lb.gemm(tA, tB, qpf, qaf)
                torch.cuda.synchronize()
                want = ref.gemm(A, B, ref.QFmt(*qpf), ref.QFmt(*qaf))
                assert np.array_equal(bits(got.cpu().numpy()), bits(want)), (tiny, qpf, qaf)
    a = torch.tensor([[0x58, 0x81]], dtype=torch.uint8, device=DEV)
    b = torch.tensor([[0x58, 0x01]], dtype=torch.uint8, device=DEV)
    assert float(lb.gemm(a, b, (5, 7, 18, 0), (4, 7, 7, 0))[0, 0]) == 255.0
    assert float(lb.gemm(a, b, (5, 7, 18, 1), (4, 7, 7, 1))[0, 0]) == 256.0
