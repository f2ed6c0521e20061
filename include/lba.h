/* lba.h -- C ABI of the MI355X (gfx950) simulated low-bit-width-accumulator matrix product.
 *
 * The library computes, for FP8 (OCP E4M3) operand matrices, the matrix product in which every
 * fused multiply-add is replaced by the quantized one of arXiv 2401.14110, Sec. 3:
 *
 *      FMAq(x, w, s) = Q_acc( Q_prod(x * w) + s )
 *
 * where x*w and the sum are exact and Q_prod / Q_acc are the floating-point quantizer of Sec. 2.3
 * (M mantissa bits, E exponent bits, exponent bias b):
 *
 *      R_OF = 2^(2^E - b - 1) * (2 - 2^-M),    R_UF = 2^-b
 *      |v| >= R_OF  ->  sign(v) * R_OF           (saturation)
 *      |v| <  R_UF  ->  0                        (flush to zero, decided before rounding)
 *      otherwise       sign(v) * 2^e * (1 + m),  e = floor(log2 |v|), m rounded to M bits
 *
 * with the mantissa rounded by truncation of the magnitude ("floor ... via bit-mask", Sec. 3) or
 * to nearest, ties to even.  The format has 2^E exponent values, no subnormals, no inf, no NaN.
 *
 * Layout follows App. A (Y = X W^T): A is [M, K] and B is [N, K], both row-major with the
 * reduction index contiguous; C is [M, N] row-major float32:  C[m, n] = S_K of the recursion
 * S_0 = 0, S_{k+1} = FMAq(A[m, k], B[n, k], S_k)  (App. D), k = 0 .. K-1 in that order.
 *
 * All pointers are DEVICE pointers owned by the caller.  Calls enqueue work on `hip_stream`
 * (a hipStream_t passed as void*; NULL = the default stream) and return without synchronising.
 * A and B are only read; C and the masks are fully overwritten.  The library keeps no state
 * between calls and allocates no device memory.  On any error nothing is enqueued.
 */
#ifndef LBA_H_
#define LBA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* One quantizer Q_{M,E,b} (Sec. 2.3).  bias is the paper's b (signed): R_UF = 2^-bias and the
 * top exponent is 2^exp_bits - bias - 1.  A per-tensor power-of-two scale of the operands is
 * folded by the caller into bias:  Q_{M,E,b}(2^-T y) = 2^-T Q_{M,E,b-T}(y).
 * Limits (else LBA_ERR_FORMAT): 1 <= man_bits <= 23, 2 <= exp_bits <= 7, round in {0, 1} (+ flag),
 * bias <= 126 and 2^exp_bits - bias - 1 <= 127, i.e. every value of the format is an FP32 normal. */
typedef struct {
    int32_t exp_bits;   /* E */
    int32_t man_bits;   /* M */
    int32_t bias;       /* b */
    int32_t round;      /* LBA_ROUND_FLOOR or LBA_ROUND_RNE, optionally | LBA_NO_UNDERFLOW */
} lba_qfmt;

enum { LBA_ROUND_FLOOR = 0,   /* truncate the magnitude's mantissa (the paper's LBA rounding) */
       LBA_ROUND_RNE = 1,     /* nearest, ties to even (the generic Round of the quantizer)   */
       LBA_NO_UNDERFLOW = 0x100 }; /* flag OR-ed into `round`: this quantizer never flushes to zero
                                 (FMAq "excluding underflow events", the first fine-tuning stage of
                                 Sec. 3 and Fig. 2b): values below R_UF keep an M-bit mantissa as
                                 if the exponent range had no lower end; R_OF is unchanged */

enum { LBA_ORDER_SEQ = 0,       /* k = 0 .. K-1 in one chain (App. D)                           */
       LBA_ORDER_CHUNK16 = 1 }; /* chunks of 16, then a chain over the chunk sums (Sec. 3, Fig. 1) */

enum { LBA_OK = 0,
       LBA_ERR_NULL = 1,         /* a required pointer is NULL                                  */
       LBA_ERR_SHAPE = 2,        /* negative or too large M, N, K (or M*N, where a call says so)  */
       LBA_ERR_FORMAT = 3,       /* a quantizer format outside the limits above                 */
       LBA_ERR_UNSUPPORTED = 4,  /* unknown order, or lba_gemm_bwd with the chunked order        */
       LBA_ERR_ALIGN = 5,        /* reserved: no entry point requires alignment                 */
       LBA_ERR_LAUNCH = 6 };     /* the HIP runtime refused the launch                          */

/* Forward product (Sec. 3, App. A, App. D).
 *   A   [M, K] uint8 E4M3 codes (device), B [N, K] uint8 E4M3 codes (device), C [M, N] float32 (device).
 *   E4M3: 1 sign, 4 exponent (bias 7), 3 mantissa bits; e = 0 is subnormal, m * 2^-9; no inf.
 *   The two NaN codes 0x7f / 0xff are outside the contract; they are read as +-480.
 *   Zero results are stored as +0.0f.  K == 0 stores +0.0f everywhere; M*N == 0 does nothing.
 *   No alignment is required of A, B, C or of K.  Shape limits: M <= 2^30 - 64, K <= 2^31 - 64,
 *   N <= 2^21 (else LBA_ERR_SHAPE).
 *   order: LBA_ORDER_SEQ, or LBA_ORDER_CHUNK16 = chunks of 16 consecutive k, each summed by its own
 *   chain from 0, then T_0 = 0, T_{j+1} = Q_acc(T_j + chunk_j) over the chunks in order (a short last
 *   chunk when 16 does not divide K; no Q_prod at the second level). */
int lba_gemm(const uint8_t* A, const uint8_t* B, float* C,
             int64_t M, int64_t N, int64_t K,
             lba_qfmt qprod, lba_qfmt qacc, int32_t order, void* hip_stream);

/* Operand code format for the *_in calls: 8-bit codes with 1 sign bit, exp_bits exponent bits and
 * man_bits = 7 - exp_bits mantissa bits; e == 0: (-1)^s * m * 2^(1 - bias - man_bits), e > 0:
 * (-1)^s * (1 + m / 2^man_bits) * 2^(e - bias); every code is a finite number.  bias is an integer per
 * tensor: the paper's weights and activations are M4E3 (exp_bits 3, man_bits 4) with the largest bias
 * that avoids overflow of the tensor ("flex-bias", Sec. 3.1).  {4, 3, 7} is the E4M3 of lba_gemm.
 * Limits (else LBA_ERR_FORMAT): 2 <= exp_bits <= 5, man_bits == 7 - exp_bits, -32 <= bias <= 32. */
typedef struct {
    int32_t exp_bits;
    int32_t man_bits;
    int32_t bias;
} lba_infmt;

/* lba_gemm for operands coded in fmt_a (A) and fmt_b (B).  A product of two such values can have up to
 * man_a + man_b + 2 significant bits, so Q_prod's mantissa rounding takes part (with E4M3 operands and
 * the usual 7-bit Q_prod mantissa it never does).  The two biases act as one power-of-two scale
 * 2^-(bias_a + bias_b) and are folded into the quantizers' biases (Q_{M,E,b}(2^-T y) = 2^-T Q_{M,E,b-T}(y));
 * the folded biases must stay inside lba_qfmt's limits (else LBA_ERR_FORMAT).  Everything else as lba_gemm. */
int lba_gemm_in(const uint8_t* A, const uint8_t* B, float* C, int64_t M, int64_t N, int64_t K,
                lba_infmt fmt_a, lba_infmt fmt_b, lba_qfmt qprod, lba_qfmt qacc, int32_t order,
                void* hip_stream);

/* lba_gemm_bwd (sequential order) for operands coded in fmt_a / fmt_b. */
int lba_gemm_bwd_in(const uint8_t* A, const uint8_t* B, float* C, uint32_t* of_mask, uint32_t* uf_mask,
                    int64_t M, int64_t N, int64_t K, lba_infmt fmt_a, lba_infmt fmt_b,
                    lba_qfmt qprod, lba_qfmt qacc, int32_t order, void* hip_stream);

/* Convolution straight from the activation tensor (implicit im2col; App. A: a convolution is the same
 * dot product with shared weights).  X [n, h, w, c] codes (NHWC), W [cout, kh, kw, c] codes,
 * Y [n, oh, ow, cout] float32 with oh = (h + 2 pad - kh) / stride + 1, ow likewise; all device pointers.
 * It is lba_gemm with M = n*oh*ow rows, N = cout, K = kh*kw*c, where row (n, oh, ow) holds
 * X[n, oh*stride - pad + i, ow*stride - pad + j, ch] at k = (i*kw + j)*c + ch (c fastest: this IS the
 * accumulation order of every output's chain), and taps outside the image hold code 0 (the value +0).
 * Limits (else LBA_ERR_SHAPE): every field >= 1 (pad >= 0), c < 2^14, kw < 2^14, K < 2^24, oh, ow >= 1,
 * n*oh*ow <= 2^30 - 64.  Everything else as lba_gemm. */
typedef struct {
    int32_t n, h, w, c;     /* activation tensor */
    int32_t kh, kw;         /* filter taps */
    int32_t stride, pad;    /* same in both directions; dilation 1 */
} lba_conv2d_desc;

int lba_conv2d(const uint8_t* X, const uint8_t* W, float* Y, lba_conv2d_desc desc, int64_t cout,
               lba_qfmt qprod, lba_qfmt qacc, int32_t order, void* hip_stream);

/* lba_gemm_bwd of the same product (sequential order): planes of lba_mask_words(n*oh*ow, cout, kh*kw*c) words. */
int lba_conv2d_bwd(const uint8_t* X, const uint8_t* W, float* Y, uint32_t* of_mask, uint32_t* uf_mask,
                   lba_conv2d_desc desc, int64_t cout, lba_qfmt qprod, lba_qfmt qacc, int32_t order,
                   void* hip_stream);

/* oh, ow of a descriptor (LBA_ERR_SHAPE if it is outside the limits above). */
int lba_conv2d_out_shape(lba_conv2d_desc desc, int32_t* oh, int32_t* ow);

/* `batch` independent forward products in one launch (batched matrix multiplication, e.g. the
 * attention products of a transformer, which the paper also runs through its LBA GEMM, App. C.2):
 * member z uses A + z*stride_a, B + z*stride_b (bytes) and C + z*stride_c (floats); a stride of 0
 * shares that operand between members.  batch <= 65535; everything else as for lba_gemm. */
int lba_gemm_batched(const uint8_t* A, const uint8_t* B, float* C, int64_t batch,
                     int64_t stride_a, int64_t stride_b, int64_t stride_c,
                     int64_t M, int64_t N, int64_t K,
                     lba_qfmt qprod, lba_qfmt qacc, int32_t order, void* hip_stream);

/* Forward product re-run for the fine-grained gradient estimators (Sec. 4, App. C.3, App. D): the
 * same deterministic chain, additionally writing one bit per FMAq step and event:
 *   OF_k = [ |Q_prod(x_k w_k) + S_k| >= R_OF of Q_acc ]         (1 - STE^OF of App. D)
 *   UF_k = [ x_k w_k != 0 and Q_prod(x_k w_k) == 0 ]  or  [ t_k != 0 and |t_k| < R_UF of Q_acc ]
 * Each plane holds lba_mask_words(M, N, K) uint32 words: word index ((k / 32) * M + m) * N + n,
 * bit k % 32; bits for k >= K are zero.  C may be NULL (then only the planes are written); either
 * plane may be NULL but not both.  C, when given, equals lba_gemm's bit for bit.
 * LBA_ORDER_SEQ only (LBA_ERR_UNSUPPORTED otherwise: the chunked order has second-level planes too and is
 * served by lba_gemm_bwd_chunked below). */
int lba_gemm_bwd(const uint8_t* A, const uint8_t* B, float* C,
                 uint32_t* of_mask, uint32_t* uf_mask,
                 int64_t M, int64_t N, int64_t K,
                 lba_qfmt qprod, lba_qfmt qacc, int32_t order, void* hip_stream);

/* The DIFF plane of the same re-run (Sec. 4, "Immediate / DIFF"; App. D, STE^DIFF): with
 * z_k = FMAq(x_k, w_k, S_k), the paper's estimator is STE^DIFF_k = [ |z_k - S_k| / (|x_k w_k| + eps1) > eps2 ]:
 * zero on overflow, product underflow and full swamping, whatever the FMAq does inside.  The paper
 * gives no values for its two constants and adds eps1 only to keep the denominator valid; this call
 * takes eps1 -> 0+ (a zero product has ratio 0) and eps2 from the caller:
 *   DIFF_k = 1 - STE^DIFF_k = [ |S_{k+1} - S_k| <= eps2 * |x_k w_k| ]      (exact reals; x_k w_k un-quantized)
 * written with the layout and polarity of the OF plane (1 = the gradient of that product pair is
 * blocked), so lba_grad (LBA_STE_IMMEDIATE_OF), lba_ste_plane and lba_last_overflow take it in place of
 * an OF plane.  eps2 = 0 gives the "no change" plane [ S_{k+1} == S_k ].  Either order; under
 * LBA_ORDER_CHUNK16 the bits are those of the first-level steps (S_k is the sum of k's own chunk; the
 * second level has no product pair).  C may be NULL, else it equals lba_gemm's bit for bit.
 * eps2 must be 0, or in [2^-32, 16] with at most 12 significant bits (so that eps2 * |x w| is exact in
 * the kernel's arithmetic): anything else is LBA_ERR_FORMAT.  Operand scales: the ratio is scale-free,
 * fold them into the biases as for lba_gemm. */
int lba_gemm_bwd_diff(const uint8_t* A, const uint8_t* B, float* C, uint32_t* diff_mask,
                      int64_t M, int64_t N, int64_t K,
                      lba_qfmt qprod, lba_qfmt qacc, int32_t order, float eps2, void* hip_stream);

/* lba_gemm_bwd_diff for operands coded in fmt_a / fmt_b (x_k w_k is the product of the decoded codes). */
int lba_gemm_bwd_diff_in(const uint8_t* A, const uint8_t* B, float* C, uint32_t* diff_mask,
                         int64_t M, int64_t N, int64_t K, lba_infmt fmt_a, lba_infmt fmt_b,
                         lba_qfmt qprod, lba_qfmt qacc, int32_t order, float eps2, void* hip_stream);

/* The same re-run for the chunked order (Sec. 3: chunks of 16, Fig. 1 right; App. D, last paragraph: the
 * recompute follows the same tree).  First-level planes of_mask / uf_mask: as for lba_gemm_bwd, with S_k the
 * partial sum of k's own chunk (a chain that starts from 0 at every multiple of 16).  Second-level planes
 * of_mask2 / uf_mask2, lba_mask_words_level2(M, N, K) words each: for chunk j = 0 .. ceil(K / 16) - 1, with
 * T_0 = 0 and T_{j+1} = Q_acc(T_j + chunk_j), bit j % 32 of word ((j / 32) * M + m) * N + n is
 *   OF2_j = [ |T_j + chunk_j| >= R_OF of Q_acc ]
 *   UF2_j = [ T_j + chunk_j != 0 and |T_j + chunk_j| < R_UF of Q_acc ]    (no Q_prod at the second level)
 * and bits for j >= ceil(K / 16) are zero.  C may be NULL; any of the four planes may be NULL, but not all
 * of them (unless K == 0, when the planes have no words).  C, when given, equals lba_gemm's with
 * LBA_ORDER_CHUNK16 bit for bit.  The second-level OF plane is what lba_ste_plane needs for the recursive
 * estimator under this order.  Errors as for lba_gemm_bwd. */
int lba_gemm_bwd_chunked(const uint8_t* A, const uint8_t* B, float* C,
                         uint32_t* of_mask, uint32_t* uf_mask, uint32_t* of_mask2, uint32_t* uf_mask2,
                         int64_t M, int64_t N, int64_t K,
                         lba_qfmt qprod, lba_qfmt qacc, void* hip_stream);

/* Number of uint32 words in one event plane: ceil(K / 32) * M * N (0 if any size is <= 0; SIZE_MAX if the
 * count does not fit in size_t, which no shape inside the limits of the calls above reaches). */
size_t lba_mask_words(int64_t M, int64_t N, int64_t K);

/* Number of uint32 words in one second-level plane of lba_gemm_bwd_chunked: ceil(ceil(K / 16) / 32) * M * N
 * (one bit per chunk of 16 steps, Sec. 3; 0 if any size is <= 0, SIZE_MAX on overflow of size_t). */
size_t lba_mask_words_level2(int64_t M, int64_t N, int64_t K);

/* ---- gradient side: the fine-grained straight-through estimators of Sec. 4 and App. D ---------
 *
 * With g = dL/dC, every FMAq step k of output (m, n) gets a coefficient c[m, n, k] in {0, 1} and
 *   dX[m, k] = sum_n g[m, n] * value(B[n, k]) * c[m, n, k]      (gradient w.r.t. the codes' values of A)
 *   dW[n, k] = sum_m g[m, n] * value(A[m, k]) * c[m, n, k]      (gradient w.r.t. the codes' values of B)
 * value() is the E4M3 value of a code (operand scales are the caller's: scale g).
 *   LBA_STE_IDENTITY      c = 1
 *   LBA_STE_IMMEDIATE_OF  c_k = 1 - OF_k: the estimator that treats the partial sum with the identity
 *                         and the product pair with STE^OF.  Needs of_mask, the first-level OF plane of
 *                         lba_gemm_bwd or lba_gemm_bwd_chunked (the second level has no product pair).
 *   LBA_STE_RECURSIVE_OF  c_k = product of STE^OF over all steps i >= k of the sequential chain, i.e.
 *                         [k > last_of[m, n]].  Needs last_of from lba_last_overflow.  (Chunked order:
 *                         the path also runs through the second level: build the coefficient plane
 *                         with lba_ste_plane and pass it with LBA_STE_COEF_PLANE.)
 *   LBA_STE_COEF_PLANE    c is read from of_mask as it is (a plane written by lba_ste_plane).
 * Arithmetic: FP32 products and FP32 sums.  The order of the summation is unspecified (the sum may be
 * split across workgroups and combined with atomic adds), so results are reproducible up to FP32
 * rounding: |error| <= (terms + 1) * 2^-24 * sum of |terms| to first order.  The identity and the
 * recursive estimator run on the matrix cores when G (and last_of) are 16-byte aligned and N % 4 == 0
 * (recursive: K <= 12288): g is split exactly into three bfloat16
 * pieces whose products with the FP8 values are exact; gradient values below about 2^-100 may lose
 * pieces to the flush of subnormal numbers there.
 */
enum { LBA_STE_IDENTITY = 0, LBA_STE_IMMEDIATE_OF = 1, LBA_STE_RECURSIVE_OF = 2,
       LBA_STE_COEF_PLANE = 3 };   /* lba_grad only: of_mask holds the coefficients themselves (lba_ste_plane) */

/* Coefficient plane of an estimator from the event planes of the recompute call: bit k % 32 of word
 * ((k/32)*M + m)*N + n is c[m, n, k] (1: the gradient of that step passes); bits for k >= K are 0.
 *   ste = LBA_STE_IMMEDIATE_OF: c_k = 1 - OF_k (either order; of_mask2 is ignored).
 *   ste = LBA_STE_RECURSIVE_OF, order = LBA_ORDER_SEQ: c_k = 1 iff no step i >= k overflowed.
 *   ste = LBA_STE_RECURSIVE_OF, order = LBA_ORDER_CHUNK16: the path of step k is the rest of its chunk's
 *     chain and then the second-level adds of the chunks j >= k / 16 (App. D, last paragraph: the tree of
 *     Fig. 1 with the arrows reversed): c_k = 1 iff none of them overflowed.  Needs of_mask2, the
 *     second-level OF plane of lba_gemm_bwd_chunked.
 * coef has lba_mask_words(M, N, K) words and may be the same buffer as of_mask (in place).  The plane is
 * consumed by lba_grad with ste = LBA_STE_COEF_PLANE.  M * N <= 2^31 (else LBA_ERR_SHAPE).
 * Returns LBA_OK, LBA_ERR_NULL, LBA_ERR_SHAPE, LBA_ERR_UNSUPPORTED (ste or order) or LBA_ERR_LAUNCH. */
int lba_ste_plane(const uint32_t* of_mask, const uint32_t* of_mask2, uint32_t* coef,
                  int64_t M, int64_t N, int64_t K, int32_t ste, int32_t order, void* hip_stream);

/* The recursive estimator's post-pass (App. D): last_of[m*N + n] = the largest k whose bit is set in the
 * OF plane of lba_gemm_bwd, or -1 when the chain never overflowed.  of_mask: lba_mask_words(M, N, K)
 * words, last_of: M*N int32, both device pointers owned by the caller.  K == 0 writes -1 everywhere.
 * M * N <= 2^31 (else LBA_ERR_SHAPE).
 * Returns LBA_OK, LBA_ERR_NULL, LBA_ERR_SHAPE or LBA_ERR_LAUNCH. */
int lba_last_overflow(const uint32_t* of_mask, int32_t* last_of, int64_t M, int64_t N, int64_t K,
                      void* hip_stream);

/* The masked gradient products.  G [M, N] float32, A [M, K] and B [N, K] uint8 codes, dX [M, K] and
 * dW [N, K] float32, all device pointers owned by the caller; either output may be NULL (then its
 * operand, B for dX and A for dW, may be NULL too) but not both.  of_mask / last_of as required by
 * `ste`, else ignored.  Outputs are overwritten.  K <= 64 * 65535 and M * N <= 2^30 (else LBA_ERR_SHAPE).
 * M == 0 or N == 0 stores zeros.
 * Returns LBA_OK, LBA_ERR_NULL, LBA_ERR_SHAPE, LBA_ERR_UNSUPPORTED (unknown ste) or LBA_ERR_LAUNCH;
 * nothing is enqueued on error. */
int lba_grad(const float* G, const uint8_t* A, const uint8_t* B,
             const uint32_t* of_mask, const int32_t* last_of,
             float* dX, float* dW, int64_t M, int64_t N, int64_t K, int32_t ste, void* hip_stream);

/* lba_grad with a workspace (Sec. 4, App. D: the immediate estimator is the plain backward product wherever no
 * step of a region overflowed).  Same arguments, results and error bound as lba_grad; with ste =
 * LBA_STE_IMMEDIATE_OF or LBA_STE_COEF_PLANE (and G 16-byte aligned, N % 4 == 0) the work is split by bricks of
 * 128 rows x 32 summed indices x 256 k: one pass over the plane marks, in the workspace, the bricks that hold a
 * blocked coefficient; all other bricks are dense products and run on the matrix cores, the marked ones in the
 * kernel that applies the plane bit by bit.  Where the accumulator format fits the data (few or no overflows)
 * this is close to the cost of the identity estimator plus one read of the plane.
 * workspace: device memory owned by the caller, 256-byte aligned (else LBA_ERR_ALIGN), at least
 * lba_grad_workspace_bytes(M, N, K) bytes (else LBA_ERR_SHAPE), NULL is LBA_ERR_NULL; its contents on return are
 * unspecified, and calls that share a workspace must not overlap.  What a workspace holds beyond that size is
 * scratch memory for every estimator that runs on the matrix cores (identity, recursive, the clean bricks of the
 * immediate one): where a sum over m or n is cut across workgroups, its slices are stored there and added up in a
 * fixed order instead of meeting in atomic adds (faster; with the identity estimator no atomic add is left and every
 * run gives the same bits); from
 * lba_grad_workspace_bytes_fast(M, N, K) bytes on every such sum of the call fits.  A smaller workspace is not an
 * error: sums whose slices do not fit take the atomic adds. */
int lba_grad_ws(const float* G, const uint8_t* A, const uint8_t* B,
                const uint32_t* of_mask, const int32_t* last_of,
                float* dX, float* dW, int64_t M, int64_t N, int64_t K, int32_t ste,
                void* workspace, size_t workspace_bytes, void* hip_stream);

/* The recompute call and the immediate estimator as a pair that reads the overflow plane once less (Sec. 4
 * "Immediate / OF", App. C.3: the planes are written by the recompute and read by the backward products).
 * lba_gemm_bwd_ws is lba_gemm_bwd under the sequential order (same C and planes, same errors) and also leaves in
 * `workspace` the brick maps of the overflow plane it wrote, which lba_grad_ws would otherwise build with a pass of
 * its own over that plane: the recompute kernel knows which words it stores are non-zero.  of_mask must not be NULL
 * (LBA_ERR_NULL); workspace: device memory, 256-byte aligned (LBA_ERR_ALIGN), at least
 * lba_grad_workspace_bytes(M, N, K) bytes (LBA_ERR_SHAPE; also for shapes beyond lba_grad's limits, for which that
 * count is 0 although M, N, K > 0); its layout is the library's own.
 * lba_grad_premapped is lba_grad_ws with ste = LBA_STE_IMMEDIATE_OF for exactly that plane and that workspace,
 * both unchanged since lba_gemm_bwd_ws wrote them (same shape; any stream order that makes the recompute call
 * complete first): it skips the pass over the plane.  A workspace that does not describe the plane gives wrong
 * gradients without an error.  The maps are read only; what the workspace holds beyond them is used as lba_grad_ws
 * uses it (slices of split sums).  Results (FP32 sums, order unspecified) and errors as lba_grad_ws. */
int lba_gemm_bwd_ws(const uint8_t* A, const uint8_t* B, float* C,
                    uint32_t* of_mask, uint32_t* uf_mask,
                    int64_t M, int64_t N, int64_t K, lba_qfmt qprod, lba_qfmt qacc,
                    void* workspace, size_t workspace_bytes, void* hip_stream);
int lba_grad_premapped(const float* G, const uint8_t* A, const uint8_t* B, const uint32_t* of_mask,
                       float* dX, float* dW, int64_t M, int64_t N, int64_t K,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* lba_grad_ws for callers that cannot allocate device memory (code under HIP graph capture, serving loops,
 * harnesses that forbid hipMalloc): the brick maps live in 1 MiB of device memory that belongs to the library
 * itself (one copy per GPU, held until the process ends), so the call takes no workspace and allocates nothing.
 * Shapes whose maps would not fit, lba_grad_workspace_bytes(M, N, K) > 2^20 (about M * N * K > 5 * 10^11), are
 * refused with LBA_ERR_SHAPE: use lba_grad_ws.  Results and every other error as lba_grad_ws.  All calls on one GPU
 * share that memory (its maps are cleared by each call that uses them; what they leave of the 1 MiB serves as
 * lba_grad_ws's scratch memory for split sums that fit): calls of lba_grad_static that overlap on one GPU,
 * from several streams or threads, race; calls on one stream, or otherwise ordered, are fine.  The first call on
 * a device looks the memory's address up (no allocation, but a runtime query): make it before a stream capture
 * starts. */
int lba_grad_static(const float* G, const uint8_t* A, const uint8_t* B,
                    const uint32_t* of_mask, const int32_t* last_of,
                    float* dX, float* dW, int64_t M, int64_t N, int64_t K, int32_t ste, void* hip_stream);

/* Bytes of workspace lba_grad_ws needs for a shape (two brick maps: about M * N * K / 2^19 bytes; 0 for an empty
 * or invalid shape). */
size_t lba_grad_workspace_bytes(int64_t M, int64_t N, int64_t K);

/* Bytes of workspace from which lba_grad_ws / lba_grad_premapped combine every split sum of a call through the
 * workspace instead of atomic adds (see lba_grad_ws): lba_grad_workspace_bytes plus the slices of the larger of the
 * two products, a multiple of 256; equal to lba_grad_workspace_bytes where no sum is split; 0 for an empty or
 * invalid shape.  (ResNet-50 at batch 64: at most 38 MB for a layer.) */
size_t lba_grad_workspace_bytes_fast(int64_t M, int64_t N, int64_t K);

/* Static, human-readable text for a status code (never NULL). */
const char* lba_strerror(int code);

/* Which kernel a call would run, without running it (host only; needs no GPU).
 * The numeric result never depends on this choice; it is exposed for benchmarking reports. */
typedef struct {
    int32_t kernel;        /* 0: scaled-domain FP32-carrier kernel, 1: general kernel            */
    int32_t prod_mode;     /* kernel 0: 0 Q_prod is the identity, 1 flush only, 2 flush + clamp,
                              3 / 4 truncated mantissa (+ clamp), 5 / 6 nearest-even mantissa (+ clamp) */
    int32_t round;         /* rounding of Q_acc as executed                                       */
    int32_t tile_m, tile_n, tile_k;   /* workgroup tile                                           */
    int32_t thread_m, thread_n;       /* outputs per lane                                         */
    int32_t grid_x, grid_y;           /* workgroups launched                                      */
    int32_t valu_per_mac_x100;        /* kernel 0: full-rate VALU issue slots per MAC of the inner
                                         loop without the accumulator clamp, times 100 (a half-rate
                                         instruction counts as 2 slots); kernel 1: the budget of a plain
                                         FMAq step (10 floor, 12 nearest-even, 4 more with event bits), which
                                         is less than its loop issues */
    int32_t tail_blocks;              /* tail_blocks + mid_blocks > 0: mixed grid: grid_x counts, in this order,
                                         grid_x - mid_blocks - tail_blocks workgroups of tile_m x tile_n,
                                         mid_blocks workgroups of 48 x 64 (3 x 4 outputs per lane) on the rows
                                         after them and tail_blocks workgroups of 32 x 32 (2 x 2 per lane) on
                                         the last rows (of 32 x 16, 2 x 1 per lane, where the forward call's tail
                                         would otherwise leave most CUs idle); grid_y is 1                    */
    int32_t mid_blocks;
} lba_plan_info;

/* with_masks: 0 the forward call, 1 the recompute call with event planes, 2 lba_gemm_bwd_diff,
 * 3 lba_gemm_bwd with the overflow plane alone (uf_mask == NULL). */
int lba_plan_query(int64_t M, int64_t N, int64_t K, lba_qfmt qprod, lba_qfmt qacc,
                   int32_t order, int32_t with_masks, lba_plan_info* out);

/* The kernel the same call would launch, named as a profiler prints its template instantiation without the
 * namespace and the argument list (e.g. "lba_fast_mixed_kernel<32, 1, 0, 0>"), written to buf (NUL-terminated,
 * truncated to buf_len).  For benchmark reports that look up profiler records of the kernel that ran; host
 * only.  Returns LBA_OK, LBA_ERR_NULL or the status lba_plan_query would return. */
int lba_plan_kernel_name(int64_t M, int64_t N, int64_t K, lba_qfmt qprod, lba_qfmt qacc,
                         int32_t order, int32_t with_masks, char* buf, size_t buf_len);

/* lba_plan_query for the operand formats of lba_gemm_in (the biases are folded as that call folds them). */
int lba_plan_query_in(int64_t M, int64_t N, int64_t K, lba_infmt fmt_a, lba_infmt fmt_b,
                      lba_qfmt qprod, lba_qfmt qacc, int32_t order, int32_t with_masks, lba_plan_info* out);

/* lba_plan_kernel_name for the operand formats of lba_gemm_in / lba_gemm_bwd_in. */
int lba_plan_kernel_name_in(int64_t M, int64_t N, int64_t K, lba_infmt fmt_a, lba_infmt fmt_b,
                            lba_qfmt qprod, lba_qfmt qacc, int32_t order, int32_t with_masks, char* buf, size_t buf_len);

#ifdef __cplusplus
}
#endif
#endif /* LBA_H_ */
