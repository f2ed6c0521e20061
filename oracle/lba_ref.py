"""ctypes loader for the CPU oracle (oracle/lba_ref.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
CPU-baseline leg.  Nothing in the product package imports this module, and this module imports
nothing from the product package.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lba_ref.cpp")
_LIB = os.path.join(_HERE, "liblba_ref.so")

FLOOR, RNE = 0, 1
NO_UNDERFLOW = 0x100          # OR-ed into QFmt.round: this quantizer never flushes to zero
ORDER_SEQ, ORDER_CHUNK16 = 0, 1
EV_OF, EV_UF = 1, 2


class QFmt(ctypes.Structure):
    """(E, M, b, round) of the floating-point quantizer, Sec. 2.3 of the paper."""
    _fields_ = [("exp_bits", ctypes.c_int32), ("man_bits", ctypes.c_int32),
                ("bias", ctypes.c_int32), ("round", ctypes.c_int32)]

    def __repr__(self):
        return "QFmt(E=%d, M=%d, b=%d, %s%s)" % (self.exp_bits, self.man_bits, self.bias,
                                                 "RNE" if self.round & 1 else "FLOOR",
                                                 ", no underflow" if self.round & NO_UNDERFLOW else "")


class InFmt(ctypes.Structure):
    """8-bit operand code format: 1 sign, E exponent, M = 7 - E mantissa bits, integer exponent bias
    (the paper's weights / activations: M4E3 with a per-tensor "flex" bias, Sec. 3.1)."""
    _fields_ = [("exp_bits", ctypes.c_int32), ("man_bits", ctypes.c_int32), ("bias", ctypes.c_int32)]

    def __repr__(self):
        return "InFmt(E=%d, M=%d, bias=%d)" % (self.exp_bits, self.man_bits, self.bias)


def _compiler():
    for c in ("/opt/rocm/lib/llvm/bin/clang++", "/opt/rocm/llvm/bin/clang++", "clang++"):
        if os.path.sep not in c or os.path.exists(c):
            return c
    raise RuntimeError("no clang++ found for the oracle build")


def build(force=False):
    """Compile the oracle into oracle/liblba_ref.so (host code only)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = [_compiler(), "-O2", "-std=c++17", "-shared", "-fPIC", "-pthread", _SRC, "-o", _LIB]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        u8p = ctypes.c_void_p
        L.lba_ref_gemm.restype = ctypes.c_int
        L.lba_ref_gemm.argtypes = [u8p, u8p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                   ctypes.c_int64, QFmt, QFmt, ctypes.c_int32, ctypes.c_int32]
        L.lba_ref_gemm_bwd.restype = ctypes.c_int
        L.lba_ref_gemm_bwd.argtypes = [u8p, u8p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                       QFmt, QFmt, ctypes.c_int32, ctypes.c_int32]
        L.lba_ref_gemm_diff.restype = ctypes.c_int
        L.lba_ref_gemm_diff.argtypes = [u8p, u8p, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                        QFmt, QFmt, ctypes.c_int32, ctypes.c_double, ctypes.c_int32]
        L.lba_ref_gemm_diff_in.restype = ctypes.c_int
        L.lba_ref_gemm_diff_in.argtypes = [u8p, u8p, ctypes.c_void_p, ctypes.c_void_p,
                                           ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, InFmt, InFmt,
                                           QFmt, QFmt, ctypes.c_int32, ctypes.c_double, ctypes.c_int32]
        L.lba_ref_gemm_in.restype = ctypes.c_int
        L.lba_ref_gemm_in.argtypes = [u8p, u8p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                      ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, InFmt, InFmt,
                                      QFmt, QFmt, ctypes.c_int32, ctypes.c_int32]
        L.lba_ref_decode_in.restype = ctypes.c_double
        L.lba_ref_decode_in.argtypes = [ctypes.c_uint8, InFmt]
        L.lba_ref_decode.restype = ctypes.c_double
        L.lba_ref_decode.argtypes = [ctypes.c_uint8]
        L.lba_ref_quantize.restype = ctypes.c_int
        L.lba_ref_quantize.argtypes = [ctypes.c_double, QFmt, ctypes.POINTER(ctypes.c_double),
                                       ctypes.POINTER(ctypes.c_int32)]
        L.lba_ref_fmaq.restype = ctypes.c_int
        L.lba_ref_fmaq.argtypes = [ctypes.c_uint8, ctypes.c_uint8, ctypes.c_double, QFmt, QFmt,
                                   ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)]
        L.lba_ref_carrier_bits.restype = ctypes.c_int
        L.lba_ref_carrier_bits.argtypes = [QFmt, QFmt]
        _lib = L
    return _lib


def _threads(nthreads):
    if nthreads is None:
        nthreads = min(16, os.cpu_count() or 1)
    return int(nthreads)


def _u8(x):
    a = np.ascontiguousarray(np.asarray(x, dtype=np.uint8))
    return a


def decode(code):
    return lib().lba_ref_decode(int(code) & 0xFF)


def quantize(x, fmt, with_events=False):
    out = ctypes.c_double()
    ev = ctypes.c_int32()
    rc = lib().lba_ref_quantize(float(x), fmt, ctypes.byref(out), ctypes.byref(ev))
    if rc != 0:
        raise ValueError("lba_ref_quantize error %d for %r" % (rc, fmt))
    return (out.value, ev.value) if with_events else out.value


def fmaq(a_code, b_code, s, qprod, qacc):
    """One FMAq step (Sec. 3 of the paper); returns (value, event bits)."""
    out = ctypes.c_double()
    ev = ctypes.c_int32()
    rc = lib().lba_ref_fmaq(int(a_code) & 0xFF, int(b_code) & 0xFF, float(s), qprod, qacc,
                            ctypes.byref(out), ctypes.byref(ev))
    if rc != 0:
        raise ValueError("lba_ref_fmaq error %d" % rc)
    return out.value, ev.value


def gemm(A, B, qprod, qacc, order=ORDER_SEQ, nthreads=None):
    """C = LBA(A . B^T): A [M,K] uint8 E4M3 codes, B [N,K] uint8 codes -> C [M,N] float32."""
    A = _u8(A)
    B = _u8(B)
    M, K = A.shape
    N, K2 = B.shape
    assert K == K2
    C = np.empty((M, N), dtype=np.float32)
    rc = lib().lba_ref_gemm(A.ctypes.data, B.ctypes.data, C.ctypes.data, M, N, K, qprod, qacc,
                            order, _threads(nthreads))
    if rc != 0:
        raise ValueError("lba_ref_gemm error %d" % rc)
    return C


def decode_in(code, fmt):
    return lib().lba_ref_decode_in(int(code) & 0xFF, fmt)


def gemm_in(A, B, fmt_a, fmt_b, qprod, qacc, order=ORDER_SEQ, nthreads=None, planes=False):
    """gemm (or, with planes, gemm_bwd under the sequential order) for operands coded in fmt_a / fmt_b."""
    A = _u8(A)
    B = _u8(B)
    M, K = A.shape
    N, K2 = B.shape
    assert K == K2
    C = np.empty((M, N), dtype=np.float32)
    of = uf = None
    if planes:
        W = (K + 31) // 32
        of = np.empty((W, M, N), dtype=np.uint32)
        uf = np.empty((W, M, N), dtype=np.uint32)
    rc = lib().lba_ref_gemm_in(A.ctypes.data, B.ctypes.data, C.ctypes.data,
                               of.ctypes.data if planes else None, uf.ctypes.data if planes else None,
                               M, N, K, fmt_a, fmt_b, qprod, qacc, order, _threads(nthreads))
    if rc != 0:
        raise ValueError("lba_ref_gemm_in error %d" % rc)
    return (C, of, uf) if planes else C


def im2col_nhwc(X, kh, kw, stride=1, pad=0):
    """The GEMM operand of a convolution, written out: X [n, h, w, c] uint8 codes -> [n*oh*ow, kh*kw*c] with
    k = (i*kw + j)*c + ch and code 0 (the value +0) for taps outside the image (App. A of the paper: a
    convolution is the same dot product with shared weights)."""
    X = np.asarray(X, dtype=np.uint8)
    n, h, w, c = X.shape
    oh = (h + 2 * pad - kh) // stride + 1
    ow = (w + 2 * pad - kw) // stride + 1
    Xp = np.zeros((n, h + 2 * pad, w + 2 * pad, c), dtype=np.uint8)
    Xp[:, pad:pad + h, pad:pad + w, :] = X
    cols = np.empty((n, oh, ow, kh, kw, c), dtype=np.uint8)
    for i in range(kh):
        for j in range(kw):
            cols[:, :, :, i, j, :] = Xp[:, i:i + stride * (oh - 1) + 1:stride, j:j + stride * (ow - 1) + 1:stride, :]
    return cols.reshape(n * oh * ow, kh * kw * c)


def mask_words(M, N, K):
    return ((K + 31) // 32) * M * N


def gemm_bwd(A, B, qprod, qacc, order=ORDER_SEQ, nthreads=None, level2=False):
    """Returns (C, OF plane, UF plane[, OF2, UF2]); planes are uint32 [ceil(K/32), M, N]."""
    A = _u8(A)
    B = _u8(B)
    M, K = A.shape
    N, K2 = B.shape
    assert K == K2
    W = (K + 31) // 32
    C = np.empty((M, N), dtype=np.float32)
    of = np.empty((W, M, N), dtype=np.uint32)
    uf = np.empty((W, M, N), dtype=np.uint32)
    of2 = uf2 = None
    p_of2 = p_uf2 = None
    if level2:
        W2 = ((K + 15) // 16 + 31) // 32
        of2 = np.empty((W2, M, N), dtype=np.uint32)
        uf2 = np.empty((W2, M, N), dtype=np.uint32)
        p_of2, p_uf2 = of2.ctypes.data, uf2.ctypes.data
    rc = lib().lba_ref_gemm_bwd(A.ctypes.data, B.ctypes.data, C.ctypes.data, of.ctypes.data,
                                uf.ctypes.data, p_of2, p_uf2, M, N, K, qprod, qacc, order,
                                _threads(nthreads))
    if rc != 0:
        raise ValueError("lba_ref_gemm_bwd error %d" % rc)
    if level2:
        return C, of, uf, of2, uf2
    return C, of, uf


def gemm_diff(A, B, qprod, qacc, eps2, order=ORDER_SEQ, nthreads=None, fmt_a=None, fmt_b=None):
    """(C, DIFF plane): bit k of an output's words is 1 - STE^DIFF of step k (Sec. 4, App. D of the paper) for
    the threshold eps2 >= 0 (eps1 -> 0+), first-level steps under either order; uint32 [ceil(K/32), M, N].
    fmt_a / fmt_b: operand code formats (default E4M3)."""
    A = _u8(A)
    B = _u8(B)
    M, K = A.shape
    N, K2 = B.shape
    assert K == K2
    C = np.empty((M, N), dtype=np.float32)
    diff = np.empty(((K + 31) // 32, M, N), dtype=np.uint32)
    if fmt_a is not None or fmt_b is not None:
        rc = lib().lba_ref_gemm_diff_in(A.ctypes.data, B.ctypes.data, C.ctypes.data, diff.ctypes.data, M, N, K,
                                        fmt_a or InFmt(4, 3, 7), fmt_b or InFmt(4, 3, 7),
                                        qprod, qacc, order, float(eps2), _threads(nthreads))
    else:
        rc = lib().lba_ref_gemm_diff(A.ctypes.data, B.ctypes.data, C.ctypes.data, diff.ctypes.data, M, N, K,
                                     qprod, qacc, order, float(eps2), _threads(nthreads))
    if rc != 0:
        raise ValueError("lba_ref_gemm_diff error %d" % rc)
    return C, diff


def carrier_bits(qprod, qacc):
    return lib().lba_ref_carrier_bits(qprod, qacc)
