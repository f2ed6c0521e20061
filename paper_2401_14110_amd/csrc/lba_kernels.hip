// lba_kernels.hip -- host side of the HIP library: plan -> launch, and the C ABI of include/lba.h.
// The device code is in lba_device.h; its instantiations are in lba_fast_*.hip, lba_bwd.hip, lba_gen.hip.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "lba_internal.h"
#include "lba_launch.h"

namespace lba {

// C[0..n) = +0 with a grid-stride loop (n may exceed what one grid dimension holds, 2^32 - 1 lanes)
__global__ void lba_fill_zero_kernel(float* C, int64_t n) {
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += step) C[i] = 0.0f;
}

static hipError_t launch_plan(const Plan& pl, hipStream_t st) {
    if (pl.kernel == KERNEL_FAST && pl.kpar > 0) return launch_kpar(pl, st);
    if (pl.kernel == KERNEL_FAST && pl.events == 2) return launch_fast_diff(pl, st);
    if (pl.kernel == KERNEL_FAST && pl.events) return launch_fast_bwd(pl, st);
    if (pl.kernel == KERNEL_FAST && pl.rne_odd) return launch_fast_odd(pl, st);
    if (pl.kernel == KERNEL_FAST && pl.amode == 2) return launch_fast_conv(pl, st);
    if (pl.kernel == KERNEL_FAST && pl.amode == 1 && pl.mix_tail > 0)
        return pl.order == LBA_ORDER_CHUNK16 ? launch_fast_in_mixed_chunk(pl, st) : launch_fast_in_mixed_seq(pl, st);
    if (pl.kernel == KERNEL_FAST && pl.amode) return launch_fast_amode(pl, st);   // 4 x 4 workgroups on a plain grid
    if (pl.kernel == KERNEL_FAST && pl.mix_tail > 0) return launch_fast_mixed(pl, st);
    if (pl.kernel == KERNEL_FAST) {
        if (pl.tm == 2 && pl.tn == 2) return launch_fast_22(pl, st);
        if (pl.tm == 2) return launch_fast_24(pl, st);
        return launch_fast_44(pl, st);
    }
    return launch_gen(pl, st);
}

// The kernel launch_plan starts for a plan, named as a profiler prints the template instantiation
// ("lba_fast_mixed_kernel<32, 1, 0, 0>"): benchmark reports use it to find the counter records of the kernel
// that actually ran.  uf: the call asks for an underflow plane.  Mirrors launch_plan and the launchers.
static void plan_kernel_name(const Plan& pl, bool uf, char* buf, size_t n) {
    const int pm = pl.prod_mode, ord = pl.order;
    const char* b = uf ? (pl.uf_class ? "2" : "1") : "0";      // the UF argument of the recompute kernels
    if (pl.kernel == KERNEL_GEN) {
        snprintf(buf, n, "lba_gen_kernel<%d, %s, %d, %s>", pl.round, pl.events == 1 ? "true" : "false", ord,
                 pl.events == 2 ? "true" : "false");
        return;
    }
    if (pl.kpar > 0) {
        const int rnd = pl.round == LBA_ROUND_FLOOR ? 0 : (pl.kp.sh_a == 16 ? 2 : 1);
        snprintf(buf, n, "lba_kpar_kernel<%d, 4, %d, %d, %d>", pl.kpar == 3 ? 2 : 4, pl.kpar == 1 ? 1 : 4, pm, rnd);
    } else if (pl.events == 2) {
        snprintf(buf, n, pl.mix_tail > 0 ? "lba_fast_diff_mixed_kernel<%d, %d, %d>" : "lba_fast_diff_kernel<%d, %d, %d>", pm, pl.round, ord);
    } else if (pl.events) {
        if (pl.amode == 2 && pl.mix_tail > 0) snprintf(buf, n, "lba_fast_bwd_conv_mixed_kernel<%d, 0, %s>", pm, b);
        else if (pl.amode == 2)   snprintf(buf, n, "lba_fast_bwd_kernel<%d, 0, 0, %s, 2>", pm, b);
        else if (pl.amode && pl.mix_tail > 0) snprintf(buf, n, "lba_fast_bwd_in_mixed_kernel<%d, 0, %s>", pm, b);
        else if (pl.amode)        snprintf(buf, n, "lba_fast_bwd_kernel<%d, 0, 0, %s, 1>", pm, b);
        else if (pl.mix_tail > 0) snprintf(buf, n, "lba_fast_bwd_mixed_kernel<%d, %d, %s>", pm, pl.round, b);
        else                      snprintf(buf, n, "lba_fast_bwd_kernel<%d, %d, %d, %s, 0>", pm, pl.round, ord, b);
    } else if (pl.rne_odd) {
        snprintf(buf, n, "lba_fast_kernel<4, 4, %d, %d, 3, %d, 0>", pl.bk, pm, ord);
    } else {
        // rounding code of the instantiation: 0 floor, 1 nearest-even by bfe / add3 / and, 2 by the bfloat16 conversion (M = 7)
        const int rnd = pl.round == LBA_ROUND_FLOOR ? 0 : ((pl.kp.sh_a == 16 && pl.amode != 1) ? 2 : 1);
        if (pl.amode == 2 && pl.mix_tail > 0) snprintf(buf, n, "lba_fast_conv_mixed_kernel<%d, %d, %d, %d>", pl.bk, pm, rnd, ord);
        else if (pl.amode == 2)   snprintf(buf, n, "lba_fast_kernel<%d, %d, %d, %d, %d, %d, 2>", pl.tm, pl.tn, pl.bk, pm, rnd, ord);
        else if (pl.amode && pl.mix_tail > 0) snprintf(buf, n, "lba_fast_in_mixed_kernel<%d, %d, %d, %d>", pl.bk, pm, rnd, ord);
        else if (pl.amode)        snprintf(buf, n, "lba_fast_kernel<4, 4, %d, %d, %d, %d, 1>", pl.bk, pm, rnd, ord);
        else if (pl.mix_tail > 0) snprintf(buf, n, "lba_fast_mixed_kernel<%d, %d, %d, %d>", pl.bk, pm, rnd, ord);
        else                      snprintf(buf, n, "lba_fast_kernel<%d, %d, %d, %d, %d, %d, 0>", pl.tm, pl.tn, pl.bk, pm, rnd, ord);
    }
}

static int gcd_align(const void* ptr, int64_t K) {
    const uintptr_t a = (uintptr_t)ptr;
    if ((a % 16) == 0 && (K % 16) == 0) return 16;
    return 1;
}

static int run(const uint8_t* A, const uint8_t* B, float* C, uint32_t* of_mask, uint32_t* uf_mask,
               int64_t M, int64_t N, int64_t K, const lba_qfmt& qprod, const lba_qfmt& qacc,
               int order, int events, void* stream,
               int64_t batch = 1, int64_t stride_a = 0, int64_t stride_b = 0, int64_t stride_c = 0,
               uint32_t* of_mask2 = nullptr, uint32_t* uf_mask2 = nullptr, const InSpec* in = nullptr,
               const lba_conv2d_desc* conv = nullptr, int conv_oh = 0, int conv_ow = 0, float diff_eps = 0.0f,
               void* brick_ws = nullptr) {
    Plan pl;
    if (batch < 0 || batch > 65535 || stride_a < 0 || stride_b < 0 || stride_c < 0) return LBA_ERR_SHAPE;
    int rc = make_plan(M, N, K, qprod, qacc, order, events, &pl, batch, in, conv != nullptr);
    if (rc != LBA_OK) return rc;
    if (in) pl.kp.out_exp -= in->delta;                        // the operand biases' power-of-two scale
    if (M == 0 || N == 0 || batch == 0) return LBA_OK;
    if (!events && !C) return LBA_ERR_NULL;
    if (events && K > 0 && !of_mask && !uf_mask && !of_mask2 && !uf_mask2) return LBA_ERR_NULL;   // K = 0: planes have no words
    hipStream_t st = (hipStream_t)stream;
    if (K == 0) {                                              // empty chains: S_0 = 0; no mask words
        if (C) {
            const int64_t n = M * N, blocks = (n + 255) / 256;
            for (int64_t z = 0; z < batch; ++z) {
                hipLaunchKernelGGL(lba_fill_zero_kernel, dim3((unsigned)(blocks < (1 << 20) ? blocks : (1 << 20))), dim3(256), 0, st,
                                   C + z * stride_c, n);
                if (hipGetLastError() != hipSuccess) return LBA_ERR_LAUNCH;
            }
        }
        return LBA_OK;
    }
    if (!A || !B) return LBA_ERR_NULL;
    KParams& kp = pl.kp;
    kp.A = A; kp.B = B; kp.C = C; kp.of_mask = of_mask; kp.uf_mask = uf_mask;
    kp.of_mask2 = of_mask2; kp.uf_mask2 = uf_mask2;
    kp.diff_eps = diff_eps;
    if (brick_ws) brick_map_params(brick_ws, M, N, K, &kp);    // the recompute kernel marks the bricks it finds dirty
    kp.batch = (int32_t)batch; kp.stride_a = stride_a; kp.stride_b = stride_b; kp.stride_c = stride_c;
    int la = gcd_align(A, K);
    const int lb = gcd_align(B, K);
    if (conv) {                                                // A is gathered; only B's rows need the alignment
        kp.conv = 1;
        kp.cv_h = conv->h; kp.cv_w = conv->w; kp.cv_c = conv->c; kp.cv_kw = conv->kw;
        kp.cv_stride = conv->stride; kp.cv_pad = conv->pad; kp.cv_oh = conv_oh; kp.cv_ow = conv_ow;
        kp.cv_vec = ((conv->c % 16) == 0 && ((uintptr_t)A % 16) == 0) ? 1 : 0;
        kp.cv_magic_c = (((uint64_t)1 << 40) + (uint64_t)conv->c - 1) / (uint64_t)conv->c;
        kp.cv_magic_kw = (((uint64_t)1 << 40) + (uint64_t)conv->kw - 1) / (uint64_t)conv->kw;
        la = lb;
    }
    kp.ld_align = (la < lb ? la : lb);
    if ((stride_a % 16) != 0 || (stride_b % 16) != 0) kp.ld_align = 1;
    const bool c_ok = (!C || ((uintptr_t)C % 16) == 0) && (stride_c % 4) == 0;
    const bool o_ok = !of_mask || ((uintptr_t)of_mask % 16) == 0;
    const bool u_ok = !uf_mask || ((uintptr_t)uf_mask % 16) == 0;
    const bool l2_ok = ((uintptr_t)of_mask2 % 16) == 0 && ((uintptr_t)uf_mask2 % 16) == 0;
    kp.c_vec = ((N % 4) == 0 && c_ok && o_ok && u_ok && l2_ok) ? 1 : 0;
    return launch_plan(pl, st) == hipSuccess ? LBA_OK : LBA_ERR_LAUNCH;
}

}  // namespace lba

// ---------------------------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------------------------
extern "C" {

int lba_gemm(const uint8_t* A, const uint8_t* B, float* C, int64_t M, int64_t N, int64_t K,
             lba_qfmt qprod, lba_qfmt qacc, int32_t order, void* hip_stream) {
    return lba::run(A, B, C, nullptr, nullptr, M, N, K, qprod, qacc, order, 0, hip_stream);
}

int lba_gemm_bwd(const uint8_t* A, const uint8_t* B, float* C, uint32_t* of_mask, uint32_t* uf_mask,
                 int64_t M, int64_t N, int64_t K, lba_qfmt qprod, lba_qfmt qacc, int32_t order,
                 void* hip_stream) {
    if (order == LBA_ORDER_CHUNK16) {                          // has second-level planes: lba_gemm_bwd_chunked
        lba::Plan pl;
        const int rc = lba::make_plan(M, N, K, qprod, qacc, order, 1, &pl);
        return rc != LBA_OK ? rc : LBA_ERR_UNSUPPORTED;
    }
    // 3: the overflow plane alone (the planner may then cut the last rows finer)
    return lba::run(A, B, C, of_mask, uf_mask, M, N, K, qprod, qacc, order, (of_mask && !uf_mask) ? 3 : 1, hip_stream);
}

int lba_gemm_bwd_ws(const uint8_t* A, const uint8_t* B, float* C, uint32_t* of_mask, uint32_t* uf_mask,
                    int64_t M, int64_t N, int64_t K, lba_qfmt qprod, lba_qfmt qacc,
                    void* workspace, size_t workspace_bytes, void* hip_stream) {
    const int events = (of_mask && !uf_mask) ? 3 : 1;
    lba::Plan pl;
    int rc = lba::make_plan(M, N, K, qprod, qacc, LBA_ORDER_SEQ, events, &pl);
    if (rc != LBA_OK) return rc;
    if (M == 0 || N == 0 || K == 0)                            // no plane words, no bricks
        return lba::run(A, B, C, of_mask, uf_mask, M, N, K, qprod, qacc, LBA_ORDER_SEQ, events, hip_stream);
    const size_t need = lba_grad_workspace_bytes(M, N, K);
    if (need == 0) return LBA_ERR_SHAPE;                       // beyond what lba_grad takes
    if (!of_mask || !workspace) return LBA_ERR_NULL;           // the maps describe the overflow plane
    if (((uintptr_t)workspace % 256) != 0) return LBA_ERR_ALIGN;
    if (workspace_bytes < need) return LBA_ERR_SHAPE;
    if (!A || !B) return LBA_ERR_NULL;
    hipStream_t st = (hipStream_t)hip_stream;
    // the scaled-domain recompute kernel marks the bricks itself; after the general kernel one pass over the plane
    // does (or, where that pass cannot read the plane in 16-byte groups, every brick is marked)
    const bool fused = pl.kernel == lba::KERNEL_FAST;
    if (fused) {
        rc = lba::brick_maps_fill(workspace, M, N, K, false, st);
        if (rc != LBA_OK) return rc;
    }
    rc = lba::run(A, B, C, of_mask, uf_mask, M, N, K, qprod, qacc, LBA_ORDER_SEQ, events, hip_stream,
                  1, 0, 0, 0, nullptr, nullptr, nullptr, nullptr, 0, 0, 0.0f, fused ? workspace : nullptr);
    if (rc != LBA_OK || fused) return rc;
    if ((N % 4) == 0 && ((uintptr_t)of_mask % 16) == 0) return lba::brick_maps_scan(of_mask, workspace, M, N, K, 0u, st);
    return lba::brick_maps_fill(workspace, M, N, K, true, st);
}

// eps2 must make eps2 * |x w| exact in FP32: at most 12 significant bits, and a range that keeps the
// product of any non-zero |x w| in [2^-18, 2^18] an FP32 normal.
static bool diff_eps_ok(float eps2) {
    if (eps2 == 0.0f) return true;
    if (!(eps2 >= 0x1p-32f && eps2 <= 16.0f)) return false;    // also refuses NaN and negative values
    uint32_t u;
    __builtin_memcpy(&u, &eps2, 4);
    return (u & 0xFFFu) == 0u;
}

int lba_gemm_bwd_diff(const uint8_t* A, const uint8_t* B, float* C, uint32_t* diff_mask,
                      int64_t M, int64_t N, int64_t K, lba_qfmt qprod, lba_qfmt qacc, int32_t order,
                      float eps2, void* hip_stream) {
    lba::Plan pl;
    const int rc = lba::make_plan(M, N, K, qprod, qacc, order, 2, &pl);
    if (rc != LBA_OK) return rc;
    if (!diff_eps_ok(eps2)) return LBA_ERR_FORMAT;
    if (!diff_mask && M > 0 && N > 0 && K > 0) return LBA_ERR_NULL;
    return lba::run(A, B, C, diff_mask, nullptr, M, N, K, qprod, qacc, order, 2, hip_stream,
                    1, 0, 0, 0, nullptr, nullptr, nullptr, nullptr, 0, 0, eps2);
}

int lba_gemm_bwd_chunked(const uint8_t* A, const uint8_t* B, float* C,
                         uint32_t* of_mask, uint32_t* uf_mask, uint32_t* of_mask2, uint32_t* uf_mask2,
                         int64_t M, int64_t N, int64_t K, lba_qfmt qprod, lba_qfmt qacc, void* hip_stream) {
    return lba::run(A, B, C, of_mask, uf_mask, M, N, K, qprod, qacc, LBA_ORDER_CHUNK16, 1, hip_stream,
                    1, 0, 0, 0, of_mask2, uf_mask2);
}

// Operand biases are one power-of-two scale 2^-delta: C = 2^-delta * LBA(codes at canonical biases) with
// both quantizer biases lowered by delta (Sec. 2.3: Q_{M,E,b}(2^-T y) = 2^-T Q_{M,E,b-T}(y)).
static int run_in(const uint8_t* A, const uint8_t* B, float* C, uint32_t* of_mask, uint32_t* uf_mask,
                  int64_t M, int64_t N, int64_t K, lba_infmt fmt_a, lba_infmt fmt_b, lba_qfmt qprod, lba_qfmt qacc,
                  int32_t order, int events, void* hip_stream, float diff_eps = 0.0f) {
    lba::InSpec in;
    int rc = lba::make_in_spec(fmt_a, fmt_b, &in);
    if (rc != LBA_OK) return rc;
    if ((rc = lba::validate_fmt(qprod)) != LBA_OK || (rc = lba::validate_fmt(qacc)) != LBA_OK) return rc;
    qprod.bias -= in.delta;
    qacc.bias -= in.delta;
    return lba::run(A, B, C, of_mask, uf_mask, M, N, K, qprod, qacc, order, events, hip_stream, 1, 0, 0, 0,
                    nullptr, nullptr, &in, nullptr, 0, 0, diff_eps);
}

int lba_gemm_in(const uint8_t* A, const uint8_t* B, float* C, int64_t M, int64_t N, int64_t K,
                lba_infmt fmt_a, lba_infmt fmt_b, lba_qfmt qprod, lba_qfmt qacc, int32_t order, void* hip_stream) {
    return run_in(A, B, C, nullptr, nullptr, M, N, K, fmt_a, fmt_b, qprod, qacc, order, 0, hip_stream);
}

int lba_gemm_bwd_in(const uint8_t* A, const uint8_t* B, float* C, uint32_t* of_mask, uint32_t* uf_mask,
                    int64_t M, int64_t N, int64_t K, lba_infmt fmt_a, lba_infmt fmt_b,
                    lba_qfmt qprod, lba_qfmt qacc, int32_t order, void* hip_stream) {
    if (order == LBA_ORDER_CHUNK16) return LBA_ERR_UNSUPPORTED;
    return run_in(A, B, C, of_mask, uf_mask, M, N, K, fmt_a, fmt_b, qprod, qacc, order, 1, hip_stream);
}

int lba_gemm_bwd_diff_in(const uint8_t* A, const uint8_t* B, float* C, uint32_t* diff_mask,
                         int64_t M, int64_t N, int64_t K, lba_infmt fmt_a, lba_infmt fmt_b,
                         lba_qfmt qprod, lba_qfmt qacc, int32_t order, float eps2, void* hip_stream) {
    if (!diff_eps_ok(eps2)) {                                  // reported after a format error, like lba_gemm_bwd_diff
        const int rc = run_in(nullptr, nullptr, nullptr, nullptr, nullptr, 0, 0, 0, fmt_a, fmt_b, qprod, qacc, order, 2, hip_stream);
        return rc != LBA_OK ? rc : LBA_ERR_FORMAT;
    }
    return run_in(A, B, C, diff_mask, nullptr, M, N, K, fmt_a, fmt_b, qprod, qacc, order, 2, hip_stream, eps2);
}

int lba_conv2d_out_shape(lba_conv2d_desc d, int32_t* oh, int32_t* ow) {
    if (d.n < 1 || d.h < 1 || d.w < 1 || d.c < 1 || d.kh < 1 || d.kw < 1 || d.stride < 1 || d.pad < 0) return LBA_ERR_SHAPE;
    if (d.c >= (1 << 14) || d.kw >= (1 << 14) || d.kh >= (1 << 14)) return LBA_ERR_SHAPE;
    if ((int64_t)d.kh * d.kw * d.c >= ((int64_t)1 << 24)) return LBA_ERR_SHAPE;
    const int64_t eh = (int64_t)d.h + 2 * (int64_t)d.pad - d.kh, ew = (int64_t)d.w + 2 * (int64_t)d.pad - d.kw;
    if (eh < 0 || ew < 0) return LBA_ERR_SHAPE;
    const int64_t o_h = eh / d.stride + 1, o_w = ew / d.stride + 1;
    if ((int64_t)d.n * o_h * o_w > (((int64_t)1 << 30) - 64)) return LBA_ERR_SHAPE;   // the rows of the product
    if (oh) *oh = (int32_t)o_h;
    if (ow) *ow = (int32_t)o_w;
    return LBA_OK;
}

static int run_conv(const uint8_t* X, const uint8_t* W, float* Y, uint32_t* of_mask, uint32_t* uf_mask,
                    const lba_conv2d_desc& d, int64_t cout, lba_qfmt qprod, lba_qfmt qacc, int32_t order, int events,
                    void* hip_stream) {
    int32_t oh = 0, ow = 0;
    const int rc = lba_conv2d_out_shape(d, &oh, &ow);
    if (rc != LBA_OK) return rc;
    return lba::run(X, W, Y, of_mask, uf_mask, (int64_t)d.n * oh * ow, cout, (int64_t)d.kh * d.kw * d.c, qprod, qacc,
                    order, events, hip_stream, 1, 0, 0, 0, nullptr, nullptr, nullptr, &d, oh, ow);
}

int lba_conv2d(const uint8_t* X, const uint8_t* W, float* Y, lba_conv2d_desc desc, int64_t cout,
               lba_qfmt qprod, lba_qfmt qacc, int32_t order, void* hip_stream) {
    return run_conv(X, W, Y, nullptr, nullptr, desc, cout, qprod, qacc, order, 0, hip_stream);
}

int lba_conv2d_bwd(const uint8_t* X, const uint8_t* W, float* Y, uint32_t* of_mask, uint32_t* uf_mask,
                   lba_conv2d_desc desc, int64_t cout, lba_qfmt qprod, lba_qfmt qacc, int32_t order,
                   void* hip_stream) {
    if (order == LBA_ORDER_CHUNK16) return LBA_ERR_UNSUPPORTED;
    return run_conv(X, W, Y, of_mask, uf_mask, desc, cout, qprod, qacc, order, 1, hip_stream);
}

int lba_gemm_batched(const uint8_t* A, const uint8_t* B, float* C, int64_t batch,
                     int64_t stride_a, int64_t stride_b, int64_t stride_c,
                     int64_t M, int64_t N, int64_t K,
                     lba_qfmt qprod, lba_qfmt qacc, int32_t order, void* hip_stream) {
    return lba::run(A, B, C, nullptr, nullptr, M, N, K, qprod, qacc, order, 0, hip_stream,
                    batch, stride_a, stride_b, stride_c);
}

// groups * M * N, saturated at SIZE_MAX (a caller sizing a buffer from a wrapped count would under-allocate)
static size_t plane_words(int64_t groups, int64_t M, int64_t N) {
    size_t mn = 0, words = 0;
    if (__builtin_mul_overflow((size_t)M, (size_t)N, &mn) || __builtin_mul_overflow(mn, (size_t)groups, &words))
        return SIZE_MAX;
    return words;
}

size_t lba_mask_words(int64_t M, int64_t N, int64_t K) {
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    return plane_words(K / 32 + (K % 32 != 0), M, N);
}

size_t lba_mask_words_level2(int64_t M, int64_t N, int64_t K) {
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    const int64_t chunks = K / 16 + (K % 16 != 0);
    return plane_words(chunks / 32 + (chunks % 32 != 0), M, N);
}

const char* lba_strerror(int code) {
    switch (code) {
        case LBA_OK: return "ok";
        case LBA_ERR_NULL: return "a required pointer is NULL";
        case LBA_ERR_SHAPE: return "invalid shape (negative, M > 2^30 - 64, K > 2^31 - 64, N > 2^21, or beyond the call's own limit)";
        case LBA_ERR_FORMAT: return "quantizer format outside the supported limits";
        case LBA_ERR_UNSUPPORTED: return "unknown or unimplemented accumulation order";
        case LBA_ERR_ALIGN: return "alignment (reserved)";
        case LBA_ERR_LAUNCH: return "HIP kernel launch failed";
        default: return "unknown status code";
    }
}

static int plan_query(int64_t M, int64_t N, int64_t K, lba_qfmt qprod, lba_qfmt qacc, int32_t order,
                      int32_t with_masks, const lba::InSpec* in, lba_plan_info* out) {
    if (!out) return LBA_ERR_NULL;
    lba::Plan pl;
    int rc = lba::make_plan(M, N, K, qprod, qacc, order, with_masks, &pl, 1, in);
    if (rc != LBA_OK) return rc;
    out->kernel = pl.kernel; out->prod_mode = pl.prod_mode; out->round = pl.round;
    out->tile_m = 16 * pl.tm; out->tile_n = 16 * pl.tn; out->tile_k = pl.bk;
    if (pl.kpar > 0) {                                         // outputs per workgroup and depth of a k-tile (chunks in flight x 16)
        out->tile_m = pl.kpar == 1 ? 32 : 8;
        out->tile_n = pl.kpar == 1 ? 32 : 16;
        out->tile_k = pl.kpar == 1 ? 64 : 256;
    }
    out->thread_m = pl.tm; out->thread_n = pl.tn;
    out->grid_x = pl.grid_x; out->grid_y = pl.grid_y;
    out->valu_per_mac_x100 = pl.valu_per_mac_x100;
    out->tail_blocks = pl.mix_tail > 0 ? pl.mix_tail - pl.kp.mix_half : 0;
    out->mid_blocks = pl.mix_tail > 0 ? pl.kp.mix_half : 0;
    return LBA_OK;
}

int lba_plan_query(int64_t M, int64_t N, int64_t K, lba_qfmt qprod, lba_qfmt qacc, int32_t order,
                   int32_t with_masks, lba_plan_info* out) {
    return plan_query(M, N, K, qprod, qacc, order, with_masks, nullptr, out);
}

int lba_plan_kernel_name(int64_t M, int64_t N, int64_t K, lba_qfmt qprod, lba_qfmt qacc, int32_t order,
                         int32_t with_masks, char* buf, size_t buf_len) {
    if (!buf || buf_len == 0) return LBA_ERR_NULL;
    lba::Plan pl;
    const int rc = lba::make_plan(M, N, K, qprod, qacc, order, with_masks, &pl);
    if (rc != LBA_OK) return rc;
    lba::plan_kernel_name(pl, with_masks == 1, buf, buf_len);
    return LBA_OK;
}

int lba_plan_query_in(int64_t M, int64_t N, int64_t K, lba_infmt fmt_a, lba_infmt fmt_b,
                      lba_qfmt qprod, lba_qfmt qacc, int32_t order, int32_t with_masks, lba_plan_info* out) {
    lba::InSpec in;
    int rc = lba::make_in_spec(fmt_a, fmt_b, &in);
    if (rc != LBA_OK) return rc;
    if ((rc = lba::validate_fmt(qprod)) != LBA_OK || (rc = lba::validate_fmt(qacc)) != LBA_OK) return rc;
    qprod.bias -= in.delta;
    qacc.bias -= in.delta;
    return plan_query(M, N, K, qprod, qacc, order, with_masks, &in, out);
}

int lba_plan_kernel_name_in(int64_t M, int64_t N, int64_t K, lba_infmt fmt_a, lba_infmt fmt_b,
                            lba_qfmt qprod, lba_qfmt qacc, int32_t order, int32_t with_masks, char* buf, size_t buf_len) {
    if (!buf || buf_len == 0) return LBA_ERR_NULL;
    lba::InSpec in;
    int rc = lba::make_in_spec(fmt_a, fmt_b, &in);
    if (rc != LBA_OK) return rc;
    if ((rc = lba::validate_fmt(qprod)) != LBA_OK || (rc = lba::validate_fmt(qacc)) != LBA_OK) return rc;
    qprod.bias -= in.delta;
    qacc.bias -= in.delta;
    lba::Plan pl;
    if ((rc = lba::make_plan(M, N, K, qprod, qacc, order, with_masks, &pl, 1, &in)) != LBA_OK) return rc;
    lba::plan_kernel_name(pl, with_masks == 1, buf, buf_len);
    return LBA_OK;
}

}  // extern "C"
