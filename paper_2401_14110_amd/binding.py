"""Thin ctypes binding over the C ABI in include/lba.h (argument marshalling only).

Every step of the computation runs in the HIP library; there is no CPU fallback: if the library
has not been built, loading raises.  torch is used for device memory and for the current stream.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIBPATH = os.path.join(_HERE, "liblba_hip.so")

ROUND_FLOOR, ROUND_RNE = 0, 1
STE_IDENTITY, STE_IMMEDIATE_OF, STE_RECURSIVE_OF, STE_COEF_PLANE = 0, 1, 2, 3
ORDER_SEQ, ORDER_CHUNK16 = 0, 1
OK, ERR_NULL, ERR_SHAPE, ERR_FORMAT, ERR_UNSUPPORTED, ERR_ALIGN, ERR_LAUNCH = range(7)


class lba_qfmt(ctypes.Structure):
    _fields_ = [("exp_bits", ctypes.c_int32), ("man_bits", ctypes.c_int32),
                ("bias", ctypes.c_int32), ("round", ctypes.c_int32)]


class lba_infmt(ctypes.Structure):
    _fields_ = [("exp_bits", ctypes.c_int32), ("man_bits", ctypes.c_int32), ("bias", ctypes.c_int32)]


def infmt(f):
    return f if isinstance(f, lba_infmt) else lba_infmt(*[int(v) for v in f])


class lba_conv2d_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("n", "h", "w", "c", "kh", "kw", "stride", "pad")]


class lba_plan_info(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "kernel", "prod_mode", "round", "tile_m", "tile_n", "tile_k", "thread_m", "thread_n",
        "grid_x", "grid_y", "valu_per_mac_x100", "tail_blocks", "mid_blocks")]


class LbaError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("lba error %d: %s" % (code, text))
        self.code = code


_lib = None


def lib(path=None):
    """Load paper_2401_14110_amd/liblba_hip.so (built by __graft_entry__.build()).  `path`: another build of
    the same library, honoured only on the first call of a process (A/B measurements)."""
    global _lib
    if _lib is None:
        libpath = path or _LIBPATH
        if not os.path.exists(libpath):
            raise RuntimeError("HIP library %s is missing: run `python __graft_entry__.py` "
                               "(there is no fallback path)" % libpath)
        L = ctypes.CDLL(libpath)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
        L.lba_gemm.restype = ctypes.c_int
        L.lba_gemm.argtypes = [vp, vp, vp, i64, i64, i64, lba_qfmt, lba_qfmt, i32, vp]
        L.lba_gemm_bwd.restype = ctypes.c_int
        L.lba_gemm_bwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, lba_qfmt, lba_qfmt, i32, vp]
        L.lba_gemm_batched.restype = ctypes.c_int
        L.lba_gemm_batched.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, i64, i64, lba_qfmt, lba_qfmt, i32, vp]
        L.lba_gemm_bwd_diff.restype = ctypes.c_int
        L.lba_gemm_bwd_diff.argtypes = [vp, vp, vp, vp, i64, i64, i64, lba_qfmt, lba_qfmt, i32, ctypes.c_float, vp]
        L.lba_gemm_bwd_diff_in.restype = ctypes.c_int
        L.lba_gemm_bwd_diff_in.argtypes = [vp, vp, vp, vp, i64, i64, i64, lba_infmt, lba_infmt, lba_qfmt, lba_qfmt, i32,
                                           ctypes.c_float, vp]
        L.lba_gemm_bwd_chunked.restype = ctypes.c_int
        L.lba_gemm_bwd_chunked.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, lba_qfmt, lba_qfmt, vp]
        L.lba_mask_words_level2.restype = ctypes.c_size_t
        L.lba_mask_words_level2.argtypes = [i64, i64, i64]
        L.lba_gemm_in.restype = ctypes.c_int
        L.lba_gemm_in.argtypes = [vp, vp, vp, i64, i64, i64, lba_infmt, lba_infmt, lba_qfmt, lba_qfmt, i32, vp]
        L.lba_gemm_bwd_in.restype = ctypes.c_int
        L.lba_gemm_bwd_in.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, lba_infmt, lba_infmt, lba_qfmt, lba_qfmt, i32, vp]
        L.lba_conv2d.restype = ctypes.c_int
        L.lba_conv2d.argtypes = [vp, vp, vp, lba_conv2d_desc, i64, lba_qfmt, lba_qfmt, i32, vp]
        L.lba_conv2d_bwd.restype = ctypes.c_int
        L.lba_conv2d_bwd.argtypes = [vp, vp, vp, vp, vp, lba_conv2d_desc, i64, lba_qfmt, lba_qfmt, i32, vp]
        L.lba_conv2d_out_shape.restype = ctypes.c_int
        L.lba_conv2d_out_shape.argtypes = [lba_conv2d_desc, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
        L.lba_plan_query_in.restype = ctypes.c_int
        L.lba_plan_query_in.argtypes = [i64, i64, i64, lba_infmt, lba_infmt, lba_qfmt, lba_qfmt, i32, i32,
                                        ctypes.POINTER(lba_plan_info)]
        L.lba_last_overflow.restype = ctypes.c_int
        L.lba_last_overflow.argtypes = [vp, vp, i64, i64, i64, vp]
        L.lba_ste_plane.restype = ctypes.c_int
        L.lba_ste_plane.argtypes = [vp, vp, vp, i64, i64, i64, i32, i32, vp]
        L.lba_grad.restype = ctypes.c_int
        L.lba_grad.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i32, vp]
        L.lba_grad_ws.restype = ctypes.c_int
        L.lba_grad_ws.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i32, vp, ctypes.c_size_t, vp]
        L.lba_gemm_bwd_ws.restype = ctypes.c_int
        L.lba_gemm_bwd_ws.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, lba_qfmt, lba_qfmt, vp, ctypes.c_size_t, vp]
        L.lba_grad_premapped.restype = ctypes.c_int
        L.lba_grad_premapped.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, vp, ctypes.c_size_t, vp]
        L.lba_grad_static.restype = ctypes.c_int
        L.lba_grad_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i32, vp]
        L.lba_grad_workspace_bytes.restype = ctypes.c_size_t
        L.lba_grad_workspace_bytes.argtypes = [i64, i64, i64]
        L.lba_grad_workspace_bytes_fast.restype = ctypes.c_size_t
        L.lba_grad_workspace_bytes_fast.argtypes = [i64, i64, i64]
        L.lba_mask_words.restype = ctypes.c_size_t
        L.lba_mask_words.argtypes = [i64, i64, i64]
        L.lba_strerror.restype = ctypes.c_char_p
        L.lba_strerror.argtypes = [ctypes.c_int]
        L.lba_plan_kernel_name_in.restype = ctypes.c_int
        L.lba_plan_kernel_name_in.argtypes = [i64, i64, i64, lba_infmt, lba_infmt, lba_qfmt, lba_qfmt, i32, i32, ctypes.c_char_p,
                                              ctypes.c_size_t]
        L.lba_plan_kernel_name.restype = ctypes.c_int
        L.lba_plan_kernel_name.argtypes = [i64, i64, i64, lba_qfmt, lba_qfmt, i32, i32, ctypes.c_char_p, ctypes.c_size_t]
        L.lba_plan_query.restype = ctypes.c_int
        L.lba_plan_query.argtypes = [i64, i64, i64, lba_qfmt, lba_qfmt, i32, i32,
                                     ctypes.POINTER(lba_plan_info)]
        _lib = L
    return _lib


def qfmt(f):
    """(E, M, b, round) tuple or lba_qfmt -> lba_qfmt."""
    return f if isinstance(f, lba_qfmt) else lba_qfmt(*[int(v) for v in f])


def lba_strerror(code):
    return lib().lba_strerror(int(code)).decode()


strerror = lba_strerror


def _check(rc):
    if rc != OK:
        raise LbaError(rc, strerror(rc))


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


# ---- raw calls: same names and argument order as include/lba.h ------------------------------

def lba_gemm(A, B, C, M, N, K, qprod, qacc, order=ORDER_SEQ, hip_stream=None):
    """Raw call: A, B, C are device addresses (ints) or None; returns the status code."""
    return lib().lba_gemm(A, B, C, M, N, K, qfmt(qprod), qfmt(qacc), order,
                          ctypes.c_void_p(hip_stream) if isinstance(hip_stream, int) else hip_stream)


def lba_gemm_bwd(A, B, C, of_mask, uf_mask, M, N, K, qprod, qacc, order=ORDER_SEQ, hip_stream=None):
    return lib().lba_gemm_bwd(A, B, C, of_mask, uf_mask, M, N, K, qfmt(qprod), qfmt(qacc), order,
                              ctypes.c_void_p(hip_stream) if isinstance(hip_stream, int) else hip_stream)


def lba_gemm_batched(A, B, C, batch, stride_a, stride_b, stride_c, M, N, K, qprod, qacc,
                     order=ORDER_SEQ, hip_stream=None):
    return lib().lba_gemm_batched(A, B, C, batch, stride_a, stride_b, stride_c, M, N, K, qfmt(qprod),
                                  qfmt(qacc), order,
                                  ctypes.c_void_p(hip_stream) if isinstance(hip_stream, int) else hip_stream)


def lba_gemm_bwd_diff(A, B, C, diff_mask, M, N, K, qprod, qacc, order, eps2, hip_stream=None):
    return lib().lba_gemm_bwd_diff(A, B, C, diff_mask, M, N, K, qfmt(qprod), qfmt(qacc), order, float(eps2), hip_stream)


def lba_gemm_bwd_diff_in(A, B, C, diff_mask, M, N, K, fmt_a, fmt_b, qprod, qacc, order, eps2, hip_stream=None):
    return lib().lba_gemm_bwd_diff_in(A, B, C, diff_mask, M, N, K, infmt(fmt_a), infmt(fmt_b), qfmt(qprod), qfmt(qacc),
                                      order, float(eps2), hip_stream)


def lba_gemm_bwd_chunked(A, B, C, of_mask, uf_mask, of_mask2, uf_mask2, M, N, K, qprod, qacc, hip_stream=None):
    return lib().lba_gemm_bwd_chunked(A, B, C, of_mask, uf_mask, of_mask2, uf_mask2, M, N, K, qfmt(qprod),
                                      qfmt(qacc),
                                      ctypes.c_void_p(hip_stream) if isinstance(hip_stream, int) else hip_stream)


def lba_gemm_in(A, B, C, M, N, K, fmt_a, fmt_b, qprod, qacc, order=ORDER_SEQ, hip_stream=None):
    return lib().lba_gemm_in(A, B, C, M, N, K, infmt(fmt_a), infmt(fmt_b), qfmt(qprod), qfmt(qacc), order,
                             ctypes.c_void_p(hip_stream) if isinstance(hip_stream, int) else hip_stream)


def lba_gemm_bwd_in(A, B, C, of_mask, uf_mask, M, N, K, fmt_a, fmt_b, qprod, qacc, order=ORDER_SEQ, hip_stream=None):
    return lib().lba_gemm_bwd_in(A, B, C, of_mask, uf_mask, M, N, K, infmt(fmt_a), infmt(fmt_b), qfmt(qprod),
                                 qfmt(qacc), order,
                                 ctypes.c_void_p(hip_stream) if isinstance(hip_stream, int) else hip_stream)


def _desc(d):
    return d if isinstance(d, lba_conv2d_desc) else lba_conv2d_desc(*[int(v) for v in d])


def lba_conv2d(X, W, Y, desc, cout, qprod, qacc, order=ORDER_SEQ, hip_stream=None):
    return lib().lba_conv2d(X, W, Y, _desc(desc), cout, qfmt(qprod), qfmt(qacc), order,
                            ctypes.c_void_p(hip_stream) if isinstance(hip_stream, int) else hip_stream)


def lba_conv2d_bwd(X, W, Y, of_mask, uf_mask, desc, cout, qprod, qacc, order=ORDER_SEQ, hip_stream=None):
    return lib().lba_conv2d_bwd(X, W, Y, of_mask, uf_mask, _desc(desc), cout, qfmt(qprod), qfmt(qacc), order,
                                ctypes.c_void_p(hip_stream) if isinstance(hip_stream, int) else hip_stream)


def lba_conv2d_out_shape(desc):
    """(status, oh, ow)"""
    oh, ow = ctypes.c_int32(0), ctypes.c_int32(0)
    rc = lib().lba_conv2d_out_shape(_desc(desc), ctypes.byref(oh), ctypes.byref(ow))
    return rc, oh.value, ow.value


def lba_last_overflow(of_mask, last_of, M, N, K, hip_stream=None):
    return lib().lba_last_overflow(of_mask, last_of, M, N, K,
                                   ctypes.c_void_p(hip_stream) if isinstance(hip_stream, int) else hip_stream)


def lba_ste_plane(of_mask, of_mask2, coef, M, N, K, ste, order, hip_stream=None):
    return lib().lba_ste_plane(of_mask, of_mask2, coef, M, N, K, ste, order,
                               ctypes.c_void_p(hip_stream) if isinstance(hip_stream, int) else hip_stream)


def lba_grad(G, A, B, of_mask, last_of, dX, dW, M, N, K, ste, hip_stream=None):
    return lib().lba_grad(G, A, B, of_mask, last_of, dX, dW, M, N, K, ste,
                          ctypes.c_void_p(hip_stream) if isinstance(hip_stream, int) else hip_stream)


def lba_grad_ws(G, A, B, of_mask, last_of, dX, dW, M, N, K, ste, workspace, workspace_bytes, hip_stream=None):
    return lib().lba_grad_ws(G, A, B, of_mask, last_of, dX, dW, M, N, K, ste, workspace, workspace_bytes,
                             ctypes.c_void_p(hip_stream) if isinstance(hip_stream, int) else hip_stream)


def lba_grad_static(G, A, B, of_mask, last_of, dX, dW, M, N, K, ste, hip_stream=None):
    return lib().lba_grad_static(G, A, B, of_mask, last_of, dX, dW, M, N, K, ste,
                                 ctypes.c_void_p(hip_stream) if isinstance(hip_stream, int) else hip_stream)


def lba_gemm_bwd_ws(A, B, C, of_mask, uf_mask, M, N, K, qprod, qacc, workspace, workspace_bytes, hip_stream=None):
    return lib().lba_gemm_bwd_ws(A, B, C, of_mask, uf_mask, M, N, K, qfmt(qprod), qfmt(qacc), workspace, workspace_bytes,
                                 ctypes.c_void_p(hip_stream) if isinstance(hip_stream, int) else hip_stream)


def lba_grad_premapped(G, A, B, of_mask, dX, dW, M, N, K, workspace, workspace_bytes, hip_stream=None):
    return lib().lba_grad_premapped(G, A, B, of_mask, dX, dW, M, N, K, workspace, workspace_bytes,
                                    ctypes.c_void_p(hip_stream) if isinstance(hip_stream, int) else hip_stream)


def lba_grad_workspace_bytes(M, N, K):
    return int(lib().lba_grad_workspace_bytes(M, N, K))


def lba_grad_workspace_bytes_fast(M, N, K):
    return int(lib().lba_grad_workspace_bytes_fast(M, N, K))


def lba_mask_words(M, N, K):
    return int(lib().lba_mask_words(M, N, K))


def lba_mask_words_level2(M, N, K):
    return int(lib().lba_mask_words_level2(M, N, K))


def lba_plan_query_in(M, N, K, fmt_a, fmt_b, qprod, qacc, order=ORDER_SEQ, with_masks=0):
    info = lba_plan_info()
    _check(lib().lba_plan_query_in(M, N, K, infmt(fmt_a), infmt(fmt_b), qfmt(qprod), qfmt(qacc), order, with_masks,
                                   ctypes.byref(info)))
    return {n: getattr(info, n) for n, _ in lba_plan_info._fields_}


def lba_plan_query(M, N, K, qprod, qacc, order=ORDER_SEQ, with_masks=0):
    info = lba_plan_info()
    _check(lib().lba_plan_query(M, N, K, qfmt(qprod), qfmt(qacc), order, with_masks, ctypes.byref(info)))
    return {n: getattr(info, n) for n, _ in lba_plan_info._fields_}


def lba_plan_kernel_name(M, N, K, qprod, qacc, order=ORDER_SEQ, with_masks=0):
    buf = ctypes.create_string_buffer(128)
    _check(lib().lba_plan_kernel_name(M, N, K, qfmt(qprod), qfmt(qacc), order, with_masks, buf, len(buf)))
    return buf.value.decode()


def lba_plan_kernel_name_in(M, N, K, fmt_a, fmt_b, qprod, qacc, order=ORDER_SEQ, with_masks=0):
    buf = ctypes.create_string_buffer(128)
    _check(lib().lba_plan_kernel_name_in(M, N, K, infmt(fmt_a), infmt(fmt_b), qfmt(qprod), qfmt(qacc), order, with_masks, buf,
                                         len(buf)))
    return buf.value.decode()


# ---- tensor conveniences --------------------------------------------------------------------

def _ops(A, B):
    if A.dtype != torch.uint8 or B.dtype != torch.uint8:
        raise TypeError("A and B must be uint8 E4M3 codes")
    if not (A.is_cuda and B.is_cuda):
        raise ValueError("A and B must be device tensors")
    if A.dim() != 2 or B.dim() != 2 or A.shape[1] != B.shape[1]:
        raise ValueError("A must be [M, K] and B [N, K]")
    return A.contiguous(), B.contiguous()


def gemm(A, B, qprod, qacc, order=ORDER_SEQ, out=None, stream=None):
    """C[M,N] (float32, device) = LBA product of A [M,K] and B [N,K] uint8 E4M3 device tensors."""
    A, B = _ops(A, B)
    M, K = A.shape
    N = B.shape[0]
    C = out if out is not None else torch.empty((M, N), dtype=torch.float32, device=A.device)
    _check(lib().lba_gemm(A.data_ptr() or None, B.data_ptr() or None, C.data_ptr() or None,
                          M, N, K, qfmt(qprod), qfmt(qacc), order, _stream(stream)))
    return C


def gemm_batched(A, B, qprod, qacc, order=ORDER_SEQ, stream=None):
    """A [batch, M, K], B [batch, N, K] or [N, K] (shared) uint8 device tensors -> C [batch, M, N]."""
    if A.dtype != torch.uint8 or B.dtype != torch.uint8 or not (A.is_cuda and B.is_cuda):
        raise TypeError("A and B must be uint8 device tensors")
    A = A.contiguous()
    B = B.contiguous()
    batch, M, K = A.shape
    shared = B.dim() == 2
    N = B.shape[-2]
    if B.shape[-1] != K or (not shared and B.shape[0] != batch):
        raise ValueError("shape mismatch")
    C = torch.empty((batch, M, N), dtype=torch.float32, device=A.device)
    _check(lib().lba_gemm_batched(A.data_ptr() or None, B.data_ptr() or None, C.data_ptr() or None, batch,
                                  M * K, 0 if shared else N * K, M * N, M, N, K,
                                  qfmt(qprod), qfmt(qacc), order, _stream(stream)))
    return C


def gemm_bwd(A, B, qprod, qacc, order=ORDER_SEQ, want_c=True, stream=None, want_uf=True):
    """Returns (C or None, OF plane, UF plane or None); planes are int32 tensors [ceil(K/32), M, N]."""
    A, B = _ops(A, B)
    M, K = A.shape
    N = B.shape[0]
    W = (K + 31) // 32
    C = torch.empty((M, N), dtype=torch.float32, device=A.device) if want_c else None
    of = torch.empty((W, M, N), dtype=torch.int32, device=A.device)
    uf = torch.empty((W, M, N), dtype=torch.int32, device=A.device) if want_uf else None
    _check(lib().lba_gemm_bwd(A.data_ptr() or None, B.data_ptr() or None,
                              (C.data_ptr() or None) if want_c else None,
                              of.data_ptr() or None, (uf.data_ptr() or None) if want_uf else None,
                              M, N, K, qfmt(qprod), qfmt(qacc), order, _stream(stream)))
    return C, of, uf


def _workspace(workspace):
    if workspace.dtype != torch.uint8 or not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous uint8 device tensor")
    return workspace


def gemm_bwd_ws(A, B, qprod, qacc, workspace=None, want_c=True, stream=None, want_uf=True):
    """lba_gemm_bwd_ws: as gemm_bwd (sequential order), and `workspace` (allocated here if None: a uint8 device tensor
    of lba_grad_workspace_bytes_fast(M, N, K) bytes: the maps, and behind them the scratch memory in which
    grad_premapped combines its split sums) receives the brick maps of the OF plane for grad_premapped.
    Returns (C or None, OF plane, UF plane or None, workspace)."""
    A, B = _ops(A, B)
    M, K = A.shape
    N = B.shape[0]
    W = (K + 31) // 32
    if workspace is None:
        workspace = torch.empty(max(256, lba_grad_workspace_bytes_fast(M, N, K)), dtype=torch.uint8, device=A.device)
    workspace = _workspace(workspace)
    C = torch.empty((M, N), dtype=torch.float32, device=A.device) if want_c else None
    of = torch.empty((W, M, N), dtype=torch.int32, device=A.device)
    uf = torch.empty((W, M, N), dtype=torch.int32, device=A.device) if want_uf else None
    _check(lib().lba_gemm_bwd_ws(A.data_ptr() or None, B.data_ptr() or None,
                                 (C.data_ptr() or None) if want_c else None,
                                 of.data_ptr() or None, (uf.data_ptr() or None) if want_uf else None,
                                 M, N, K, qfmt(qprod), qfmt(qacc), workspace.data_ptr() or None, workspace.numel(),
                                 _stream(stream)))
    return C, of, uf, workspace


def grad_premapped(G, A, B, of_plane, workspace, want_dx=True, want_dw=True, stream=None):
    """lba_grad_premapped: the immediate estimator's dX, dW from the OF plane and the workspace of gemm_bwd_ws."""
    A, B = _ops(A, B)
    M, K = A.shape
    N = B.shape[0]
    if G.dtype != torch.float32 or tuple(G.shape) != (M, N) or not G.is_cuda:
        raise ValueError("G must be a float32 device tensor [M, N]")
    G = G.contiguous()
    of_plane = _plane(of_plane, K, M, N, "of_plane")
    workspace = _workspace(workspace)
    dX = torch.empty((M, K), dtype=torch.float32, device=A.device) if want_dx else None
    dW = torch.empty((N, K), dtype=torch.float32, device=A.device) if want_dw else None
    ptr = lambda t: (t.data_ptr() or None) if t is not None else None
    _check(lib().lba_grad_premapped(ptr(G), ptr(A), ptr(B), ptr(of_plane), ptr(dX), ptr(dW), M, N, K,
                                    ptr(workspace), workspace.numel(), _stream(stream)))
    return dX, dW


def gemm_bwd_diff(A, B, qprod, qacc, eps2, order=ORDER_SEQ, want_c=True, stream=None, fmt_a=None, fmt_b=None):
    """Returns (C or None, DIFF plane [ceil(K/32), M, N] int32): bit k is 1 - STE^DIFF of step k.
    With fmt_a / fmt_b: lba_gemm_bwd_diff_in."""
    A, B = _ops(A, B)
    M, K = A.shape
    N = B.shape[0]
    C = torch.empty((M, N), dtype=torch.float32, device=A.device) if want_c else None
    diff = torch.empty(((K + 31) // 32, M, N), dtype=torch.int32, device=A.device)
    if fmt_a is not None or fmt_b is not None:
        _check(lib().lba_gemm_bwd_diff_in(A.data_ptr() or None, B.data_ptr() or None,
                                          (C.data_ptr() or None) if want_c else None, diff.data_ptr() or None, M, N, K,
                                          infmt(fmt_a or (4, 3, 7)), infmt(fmt_b or (4, 3, 7)), qfmt(qprod), qfmt(qacc),
                                          order, float(eps2), _stream(stream)))
        return C, diff
    _check(lib().lba_gemm_bwd_diff(A.data_ptr() or None, B.data_ptr() or None, (C.data_ptr() or None) if want_c else None,
                                   diff.data_ptr() or None, M, N, K, qfmt(qprod), qfmt(qacc), order, float(eps2),
                                   _stream(stream)))
    return C, diff


def gemm_bwd_chunked(A, B, qprod, qacc, want_c=True, stream=None, want_uf=True):
    """Chunked order.  Returns (C or None, OF, UF, OF2, UF2): first-level planes [ceil(K/32), M, N] and
    second-level planes [ceil(ceil(K/16)/32), M, N], int32 tensors (UF, UF2 are None without want_uf)."""
    A, B = _ops(A, B)
    M, K = A.shape
    N = B.shape[0]
    W = (K + 31) // 32
    W2 = ((K + 15) // 16 + 31) // 32
    C = torch.empty((M, N), dtype=torch.float32, device=A.device) if want_c else None
    planes = [torch.empty((w, M, N), dtype=torch.int32, device=A.device) if (want_uf or i % 2 == 0) else None
              for i, w in enumerate((W, W, W2, W2))]
    _check(lib().lba_gemm_bwd_chunked(A.data_ptr() or None, B.data_ptr() or None,
                                      (C.data_ptr() or None) if want_c else None,
                                      *[(t.data_ptr() or None) if t is not None else None for t in planes],
                                      M, N, K, qfmt(qprod), qfmt(qacc), _stream(stream)))
    return (C, *planes)


def _plane(t, K, M=None, N=None, what="plane"):
    """An event / coefficient plane as the library reads it: int32 [ceil(K/32), M, N], contiguous, on the device."""
    if t.dtype not in (torch.int32, torch.uint32) or not t.is_cuda or t.dim() != 3:
        raise ValueError("%s must be a 3-d int32 device tensor [ceil(K/32), M, N]" % what)
    if t.shape[0] != (K + 31) // 32 or (M is not None and tuple(t.shape[1:]) != (M, N)):
        raise ValueError("%s has shape %s, expected [%d, M, N]" % (what, tuple(t.shape), (K + 31) // 32))
    return t.contiguous()


def last_overflow(of_plane, K, stream=None):
    """int32 [M, N] index of the last overflowing step of every chain (-1: none) from an OF plane."""
    of_plane = _plane(of_plane, K, what="of_plane")
    W, M, N = of_plane.shape
    out = torch.empty((M, N), dtype=torch.int32, device=of_plane.device)
    _check(lib().lba_last_overflow(of_plane.data_ptr() or None, out.data_ptr() or None, M, N, K, _stream(stream)))
    return out


def grad(G, A, B, ste, of_plane=None, last_of=None, want_dx=True, want_dw=True, stream=None, workspace=None):
    """Masked gradient products: returns (dX [M, K] or None, dW [N, K] or None), float32 device tensors.
    workspace: a uint8 device tensor of at least lba_grad_workspace_bytes(M, N, K) bytes: lba_grad_ws."""
    A, B = _ops(A, B)
    M, K = A.shape
    N = B.shape[0]
    if G.dtype != torch.float32 or tuple(G.shape) != (M, N) or not G.is_cuda:
        raise ValueError("G must be a float32 device tensor [M, N]")
    G = G.contiguous()
    if of_plane is not None:
        of_plane = _plane(of_plane, K, M, N, "of_plane")
    if last_of is not None:
        if last_of.dtype != torch.int32 or tuple(last_of.shape) != (M, N) or not last_of.is_cuda:
            raise ValueError("last_of must be an int32 device tensor [M, N]")
        last_of = last_of.contiguous()
    dX = torch.empty((M, K), dtype=torch.float32, device=A.device) if want_dx else None
    dW = torch.empty((N, K), dtype=torch.float32, device=A.device) if want_dw else None
    ptr = lambda t: (t.data_ptr() or None) if t is not None else None
    if workspace is not None:
        if workspace.dtype != torch.uint8 or not workspace.is_cuda or not workspace.is_contiguous():
            raise ValueError("workspace must be a contiguous uint8 device tensor")
        _check(lib().lba_grad_ws(ptr(G), ptr(A), ptr(B), ptr(of_plane), ptr(last_of), ptr(dX), ptr(dW), M, N, K, ste,
                                 ptr(workspace), workspace.numel(), _stream(stream)))
        return dX, dW
    _check(lib().lba_grad(ptr(G), ptr(A), ptr(B), ptr(of_plane), ptr(last_of), ptr(dX), ptr(dW), M, N, K, ste,
                          _stream(stream)))
    return dX, dW


def ste_plane(of_plane, K, ste, order=ORDER_SEQ, of_plane2=None, stream=None):
    """Coefficient plane (int32 [ceil(K/32), M, N], bit = 1: passes) of an estimator from the OF plane(s)."""
    of_plane = _plane(of_plane, K, what="of_plane")
    W, M, N = of_plane.shape
    if of_plane2 is not None:
        if of_plane2.dtype not in (torch.int32, torch.uint32) or not of_plane2.is_cuda or \
                tuple(of_plane2.shape) != (((K + 15) // 16 + 31) // 32, M, N):
            raise ValueError("of_plane2 must be an int32 device tensor [ceil(ceil(K/16)/32), M, N]")
        of_plane2 = of_plane2.contiguous()
    out = torch.empty_like(of_plane)
    _check(lib().lba_ste_plane(of_plane.data_ptr() or None,
                               (of_plane2.data_ptr() or None) if of_plane2 is not None else None,
                               out.data_ptr() or None, M, N, K, ste, order, _stream(stream)))
    return out


def gemm_in(A, B, fmt_a, fmt_b, qprod, qacc, order=ORDER_SEQ, planes=False, stream=None, uf_plane=True):
    """lba_gemm_in (or, with planes, lba_gemm_bwd_in: returns (C, OF, UF); UF is None without uf_plane) on uint8
    device tensors."""
    A, B = _ops(A, B)
    M, K = A.shape
    N = B.shape[0]
    C = torch.empty((M, N), dtype=torch.float32, device=A.device)
    if not planes:
        _check(lib().lba_gemm_in(A.data_ptr() or None, B.data_ptr() or None, C.data_ptr() or None, M, N, K,
                                 infmt(fmt_a), infmt(fmt_b), qfmt(qprod), qfmt(qacc), order, _stream(stream)))
        return C
    W = (K + 31) // 32
    of = torch.empty((W, M, N), dtype=torch.int32, device=A.device)
    uf = torch.empty((W, M, N), dtype=torch.int32, device=A.device) if uf_plane else None
    _check(lib().lba_gemm_bwd_in(A.data_ptr() or None, B.data_ptr() or None, C.data_ptr() or None,
                                 of.data_ptr() or None, (uf.data_ptr() or None) if uf_plane else None, M, N, K,
                                 infmt(fmt_a), infmt(fmt_b), qfmt(qprod), qfmt(qacc), order, _stream(stream)))
    return C, of, uf


def conv2d(X, W, qprod, qacc, stride=1, pad=0, order=ORDER_SEQ, planes=False, stream=None):
    """X [n, h, w, c] and W [cout, kh, kw, c] uint8 device tensors -> Y [n, oh, ow, cout] float32
    (with planes: also the OF and UF planes [ceil(K/32), n*oh*ow, cout] of the recompute call)."""
    if X.dtype != torch.uint8 or W.dtype != torch.uint8 or not (X.is_cuda and W.is_cuda):
        raise TypeError("X and W must be uint8 device tensors")
    X = X.contiguous()
    W = W.contiguous()
    n, h, w, c = X.shape
    cout, kh, kw, c2 = W.shape
    if c != c2:
        raise ValueError("channel mismatch")
    desc = lba_conv2d_desc(n, h, w, c, kh, kw, stride, pad)
    rc, oh, ow = lba_conv2d_out_shape(desc)
    _check(rc)
    Y = torch.empty((n, oh, ow, cout), dtype=torch.float32, device=X.device)
    if not planes:
        _check(lib().lba_conv2d(X.data_ptr() or None, W.data_ptr() or None, Y.data_ptr() or None, desc, cout,
                                qfmt(qprod), qfmt(qacc), order, _stream(stream)))
        return Y
    M, K = n * oh * ow, kh * kw * c
    of = torch.empty(((K + 31) // 32, M, cout), dtype=torch.int32, device=X.device)
    uf = torch.empty_like(of)
    _check(lib().lba_conv2d_bwd(X.data_ptr() or None, W.data_ptr() or None, Y.data_ptr() or None,
                                of.data_ptr() or None, uf.data_ptr() or None, desc, cout,
                                qfmt(qprod), qfmt(qacc), order, _stream(stream)))
    return Y, of, uf
