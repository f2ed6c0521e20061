"""CPU oracle for the gradient side of the LBA product: the fine-grained straight-through
estimators of Sec. 4 and App. D of the paper, written out from their definitions in float64.

TEST INFRASTRUCTURE ONLY (same rule as lba_ref.py): imported by tests/, the smoke check and the
benchmark's CPU-baseline leg; nothing in the product package imports it and it imports nothing
from there.  It builds on the forward oracle's event planes (lba_ref.gemm_bwd) and on numpy.

With y = LBA(A . B^T) computed by the chain z_k = FMAq(a_k, b_k, s_k) and g = dL/dy, the
estimators give every step k of every output (m, n) a coefficient c[m, n, k] in {0, 1}:

    dX[m, k] = sum_n g[m, n] * value(B[n, k]) * c[m, n, k]
    dW[n, k] = sum_m g[m, n] * value(A[m, k]) * c[m, n, k]

  identity      c = 1                                  (the plain GEMM backward)
  immediate/OF  c_k = STE^OF_k = 1 - OF_k              (dz/ds = 1; the product pair sees the STE)
  recursive/OF  c_k = prod_{i >= k on k's path to the output} STE^OF_i
                sequential order: 1 iff no overflow at any step i >= k, i.e. k > last overflow index
                chunked order: the path of step k is the rest of its chunk's chain, then the
                second-level adds of chunks j >= k // 16 (App. D, last paragraph: the tree of Fig. 1
                with the arrows reversed)
  immediate/DIFF c_k = STE^DIFF_k = 1 - DIFF_k         (Sec. 4: zero on overflow, underflow and full swamping,
                detected as |z - s| <= eps2 |x w|; lba_ref.gemm_diff; first-level steps under either order)
"""
import numpy as np

from . import lba_ref

STE_IDENTITY, STE_IMMEDIATE_OF, STE_RECURSIVE_OF = 0, 1, 2
STE_IMMEDIATE_DIFF = 4         # oracle-side name only: the library consumes the DIFF plane like an OF plane


def decode_table():
    """value(code) for the 256 E4M3 codes (NaN codes read as +-480, as in the forward oracle)."""
    return np.array([lba_ref.decode(c) for c in range(256)], dtype=np.float64)


def unpack_plane(plane, K):
    """uint32 [W, M, N] plane (bit k % 32 of word k // 32) -> bool [M, N, K']  with K' = K."""
    W, M, N = plane.shape
    bits = ((plane[:, :, :, None] >> np.arange(32, dtype=np.uint32)) & 1).astype(bool)   # [W, M, N, 32]
    return np.moveaxis(bits, 0, 2).reshape(M, N, W * 32)[:, :, :K]


def last_overflow(of_plane, K):
    """int32 [M, N]: the largest k with OF_k set, -1 if the chain never overflowed (App. D: all the
    recursive correction needs under the sequential order)."""
    of = unpack_plane(of_plane, K)
    idx = np.where(of, np.arange(K, dtype=np.int64), -1)
    return idx.max(axis=2).astype(np.int32) if K > 0 else np.full(of.shape[:2], -1, dtype=np.int32)


def coefficients(A, B, qprod, qacc, ste, order=lba_ref.ORDER_SEQ, eps2=None):
    """bool [M, N, K] coefficient tensor c of the chosen estimator (eps2: the DIFF threshold)."""
    M, K = A.shape
    N = B.shape[0]
    if ste == STE_IDENTITY:
        return np.ones((M, N, K), dtype=bool)
    if ste == STE_IMMEDIATE_DIFF:
        _, diff = lba_ref.gemm_diff(A, B, qprod, qacc, eps2, order=order)
        return ~unpack_plane(diff, K)
    if order == lba_ref.ORDER_SEQ:
        _, of, _ = lba_ref.gemm_bwd(A, B, qprod, qacc, order=order)
        ok = ~unpack_plane(of, K)
        if ste == STE_IMMEDIATE_OF:
            return ok
        if ste == STE_RECURSIVE_OF:
            # c_k = ok_k and ok_{k+1} and ... and ok_{K-1}
            return np.logical_and.accumulate(ok[:, :, ::-1], axis=2)[:, :, ::-1]
    elif order == lba_ref.ORDER_CHUNK16:
        _, of, _, of2, _ = lba_ref.gemm_bwd(A, B, qprod, qacc, order=order, level2=True)
        ok = ~unpack_plane(of, K)
        if ste == STE_IMMEDIATE_OF:
            return ok                                  # second-level adds have no product pair
        if ste == STE_RECURSIVE_OF:
            nchunk = (K + 15) // 16
            ok2 = ~unpack_plane(of2, nchunk)
            tail2 = np.logical_and.accumulate(ok2[:, :, ::-1], axis=2)[:, :, ::-1]   # chunks j' >= j
            c = np.empty_like(ok)
            for j in range(nchunk):
                seg = ok[:, :, 16 * j:16 * j + 16]
                c[:, :, 16 * j:16 * j + 16] = (np.logical_and.accumulate(seg[:, :, ::-1], axis=2)[:, :, ::-1]
                                               & tail2[:, :, j:j + 1])
            return c
    raise ValueError("unknown estimator / order")


def grad(G, A, B, qprod, qacc, ste, order=lba_ref.ORDER_SEQ, c=None):
    """(dX [M, K], dW [N, K]) in float64 from g = G [M, N] and the uint8 operand codes.
    c: the coefficient tensor if the caller already has it (coefficients(...) of the same arguments)."""
    G = np.asarray(G, dtype=np.float64)
    tab = decode_table()
    X = tab[np.asarray(A, dtype=np.uint8)]             # [M, K]
    Wv = tab[np.asarray(B, dtype=np.uint8)]            # [N, K]
    if c is None:
        c = coefficients(A, B, qprod, qacc, ste, order)
    gc = G[:, :, None] * c                              # [M, N, K]
    dX = np.einsum("mnk,nk->mk", gc, Wv)
    dW = np.einsum("mnk,mk->nk", gc, X)
    return dX, dW


def grad_abs(G, A, B, qprod, qacc, ste, order=lba_ref.ORDER_SEQ, c=None):
    """Sums of |terms| of dX and dW: the scale of a float32 accumulation's rounding error."""
    G = np.abs(np.asarray(G, dtype=np.float64))
    tab = np.abs(decode_table())
    if c is None:
        c = coefficients(A, B, qprod, qacc, ste, order)
    gc = G[:, :, None] * c
    return (np.einsum("mnk,nk->mk", gc, tab[np.asarray(B, dtype=np.uint8)]),
            np.einsum("mnk,mk->nk", gc, tab[np.asarray(A, dtype=np.uint8)]))
