// lba_internal.h -- host-side plan of one LBA GEMM call and the parameter block its kernel reads.
// Shared by the planner (plain C++, testable without a GPU) and the HIP translation unit.
#ifndef LBA_INTERNAL_H_
#define LBA_INTERNAL_H_

#include <stdint.h>

#include "lba.h"

namespace lba {

enum { KERNEL_FAST = 0, KERNEL_GEN = 1 };
enum { PM_IDENT = 0, PM_FLUSH = 1, PM_FLUSH_CLAMP = 2,
       PM_TRUNC = 3, PM_TRUNC_CLAMP = 4,     // + the product's mantissa truncated to Q_prod's M bits
       PM_RNE = 5, PM_RNE_CLAMP = 6 };       // + ... rounded to nearest-even (kernels with AMODE = 1 only)

// Uniform (scalar-register) parameters of a launch.  All thresholds are exact FP32 values.
struct KParams {
    const uint8_t* A;
    const uint8_t* B;
    float* C;
    uint32_t* of_mask;
    uint32_t* uf_mask;
    uint32_t* of_mask2;      // second-level planes of the chunked order (bit j%32 of word j/32, chunk j)
    uint32_t* uf_mask2;
    int32_t M, N, K;
    int32_t batch;           // grid z; member z reads A + z*stride_a, B + z*stride_b, writes C + z*stride_c
    int64_t stride_a, stride_b, stride_c;   // in elements (bytes for A and B, floats for C)
    int32_t ld_align;        // 16: every row start of A and B is 16-byte aligned; 1: any alignment
    int32_t c_vec;           // 1 if rows of C (and of the planes) can take 16-byte stores
    // operand decode: value(code) * 2^exp_a / 2^exp_b, folded into the lookup tables
    int32_t exp_a, exp_b;
    int32_t out_exp;         // C = S * 2^out_exp
    float kc;                // FAST with an explicit product: t = p * kc + S
    float fast_thresh;       // FAST: a k-tile needs no clamp if every |S| is below this at its start
    float fast_thresh4;      // FAST: same for four consecutive k-tiles
    int32_t dyn_bound;       // FAST: 1: the four-tile bound fails (R_OF within 128 maximal products of zero): also test, per
                             // k-tile, R_OF against 32 products of the largest operands actually staged
    float rof_grow1;         // FAST: R_OF divided by the growth nearest-even rounding can add over one k-tile (rounded down)
    // accumulator quantizer, in the kernel's (possibly scaled) domain
    uint32_t mask_a; uint32_t half_a; int32_t sh_a; float rof_a; float ruf_a;
    // product quantizer
    uint32_t mask_p; uint32_t half_p; int32_t sh_p; float rof_p; float ruf_p;
    // operand code formats as the kernels decode them (canonical bias 2^(E-1) - 1; the caller's bias
    // is folded into the quantizers and out_exp): {4, 3} takes the hardware FP8 conversion
    int32_t in_ea, in_ma, in_eb, in_mb;
    // implicit im2col (conv = 1): A is an NHWC activation tensor [n, cv_h, cv_w, cv_c]; row m of the GEMM is
    // output pixel (n, oh, ow) and k runs over (kh, kw, c), c fastest; taps outside the image read as code 0
    int32_t conv, cv_vec;    // cv_vec: cv_c % 16 == 0 and A 16-byte aligned (a 16-byte piece is one load)
    int32_t cv_h, cv_w, cv_c, cv_kw, cv_stride, cv_pad, cv_oh, cv_ow;
    uint64_t cv_magic_c, cv_magic_kw;   // ceil(2^40 / d): x / d == (x * magic) >> 40 for x < 2^24, d < 2^14
    // mixed grid (lba_fast_mixed_kernel): workgroups below mix_main take 64 x 64 tiles of the rows below
    // mix_m_main (mix_gx_main of them per tile column), the next mix_half take 48 x 64 tiles (3 x 4 outputs per lane) of the rows below
    // mix_m_half (mix_gx_half per tile column; the forward kernel only), the rest 32 x 32 tiles of the remaining rows
    int32_t mix_main, mix_gx_main, mix_gx_tail, mix_m_main;
    int32_t mix_half, mix_gx_half, mix_m_half;
    int32_t mix_tail16;      // the tail's tiles are 32 x 16 (forward kernels; set where the tail runs alone on the chip)
    // brick maps of the overflow plane as a by-product of the recompute call (lba_gemm_bwd_ws), else null: byte
    // ((k / 256) * map_rbx + m / 128) * map_sbx + n / 32 of map_dx and ((k / 256) * map_rbw + n / 128) * map_sbw + m / 32
    // of map_dw are set when a step of that brick overflows (the maps arrive zeroed)
    uint8_t* map_dx;
    uint8_t* map_dw;
    int32_t map_rbx, map_sbx, map_rbw, map_sbw;
    int32_t prod_round;      // GEN: product mantissa narrower than a product of two operands
    int32_t prod_rne;        // GEN: its rounding
    float diff_eps;          // DIFF plane (written through of_mask): the threshold eps2, exact
};

struct Plan {
    int kernel;              // KERNEL_FAST / KERNEL_GEN
    int prod_mode;           // PM_*
    int round;               // LBA_ROUND_*
    int events;              // 1: also write the event planes; 2: write the DIFF plane (through kp.of_mask)
    int order;               // LBA_ORDER_*
    int tm, tn, bk;          // outputs per lane (tm x tn), k-depth of a tile; tile = 16tm x 16tn
    int grid_x, grid_y;
    int valu_per_mac_x100;
    int mix_tail;            // > 0: mixed grid with that many 32 x 32 workgroups after kp.mix_main 64 x 64 ones
    int of_only;             // 1 (events == 1): only the overflow plane is asked for (no underflow tests)
    int uf_class;            // 1 (events == 1, underflow plane): an underflowed product is a denormal number (never zero): one class test
    int rne_odd;             // 1: nearest-even through two directed sums and round-to-odd (RND_RNE_ODD; 4 x 4 only)
    int kpar;                // > 0 (chunked order, forward): lba_kpar_kernel; 1: 32 x 32 outputs per workgroup and 4 chunks in flight,
                             // 3: 8 x 16 outputs and 16 chunks
    int amode;               // 1: A is read as im2col rows and / or an operand is not E4M3 (4 x 4 lane block only);
                             // 2: A is read as im2col rows, E4M3 operands, forward call (any lane block, mixed grids)
    KParams kp;
};

// What the planner needs to know about the operand formats (canonical biases).
struct InSpec {
    int ea, ma, eb, mb;      // exponent / mantissa bits of A's and B's codes
    int sig_bits;            // most significant bits a product can have: (ma + 1) + (mb + 1)
    int min_lsb;             // every product is a multiple of 2^min_lsb
    int ptop;                // every |product| < 2^(ptop + 1)
    double max_prod;         // largest |product|
    int delta;               // (bias_a - canonical) + (bias_b - canonical): folded into the quantizers
};
int make_in_spec(const lba_infmt& fa, const lba_infmt& fb, InSpec* out);   // LBA_OK or LBA_ERR_FORMAT
const InSpec& e4m3_spec();

// Validation shared by every entry point; returns an lba status code.
int validate_shapes(int64_t M, int64_t N, int64_t K);
int validate_fmt(const lba_qfmt& q);

// Builds the plan (pointers in kp are left null).  Returns an lba status code.
int make_plan(int64_t M, int64_t N, int64_t K, const lba_qfmt& qprod, const lba_qfmt& qacc,
              int order, int events, Plan* out, int64_t batch = 1, const InSpec* in = nullptr, bool conv = false);

// Gradient products: how many slices of the summation index s a launch of `blocks` workgroups (4 waves
// of 16 rows each) is cut into so that the chip has enough waves, and the slice length (a multiple of 4).
void plan_grad_split(int64_t blocks, int64_t S, int* split, int32_t* s_chunk);

}  // namespace lba
#endif
