// lba_plan.cpp -- argument validation and kernel selection for the LBA GEMM (host only, no HIP).
//
// The quantizer Q_{M,E,b} is the one of arXiv 2401.14110 Sec. 2.3; FMAq = Q_acc(Q_prod(x w) + s)
// is Sec. 3.  Two kernels implement one FMAq step, both on an FP32 carrier:
//
// FAST  works in a scaled domain where the accumulator's R_UF sits at 2^-126, the smallest FP32
//       normal, with FP32 denormals flushed: the hardware flush of the add IS Q_acc's underflow.
//       Operands are decoded as a * 2^exp_a, b * 2^exp_b.
//         PM_IDENT        t = fma(a', b', S)                 (Q_prod cannot change any product)
//         PM_FLUSH        p = a' * b'  in the domain where Q_prod's R_UF is 2^-126, so the
//                         multiply's flush is Q_prod's underflow; t = fma(p, kc, S) moves p into
//                         the accumulator's domain exactly (kc is a power of two)
//         PM_FLUSH_CLAMP  same, p clamped to +-R_OF of Q_prod in between
//       then mantissa rounding by bit manipulation and a clamp to +-R_OF of Q_acc.
//       Exactness: an E4M3 product has at most 8 significant bits, so a'*b' is exact; the fma
//       rounds the exact sum once to 24 bits.
//         floor:   the kernel runs with the FP32 rounding mode "toward zero"; truncating to 24
//                  bits and then to M+1 bits equals truncating the exact sum to M+1 bits.  Always
//                  exact, any M.
//         nearest: the fma rounds to nearest-even at 24 bits, then the bit trick rounds to M+1
//                  bits.  The double rounding is harmless iff the first rounding can never land
//                  exactly on a midpoint of the M+1-bit grid.  The first rounding is inexact only
//                  when the smaller operand's lowest bit is more than 23 places below the sum's
//                  leading bit; the larger operand then decides the neighbourhood, and if it lies
//                  ON the M+1-bit grid the sum stays within 2^(e-M-2) of a grid point provided
//                  the smaller operand has at most 22-M significant bits.  Hence the conditions
//                  checked in rne_fast_ok(): M <= 10; products on the accumulator grid (8 <= M+1),
//                  or else every inexact 24-bit sum beyond R_OF; a saturated product
//                  (M_prod+1 bits) within the same bit budget or impossible; and the flush
//                  decision near 2^-126 unaffected (no sum can sit within 2^-150 below 2^-126).
//       Everything else falls to GEN.
//
// GEN   works in the plain domain with every step explicit (product rounding, flush, clamp, add,
//       rounding, flush, clamp).  For nearest-even it adds twice, once rounding toward +inf and
//       once toward -inf: the smaller magnitude is the truncated sum and the two differ iff the
//       sum was inexact, which gives the sticky bit for a correct single rounding at any M.
//       It also produces the per-step event bits for lba_gemm_bwd.

#include <cmath>
#include <cstring>

#include <algorithm>

#include "lba_internal.h"

namespace lba {

static const int64_t kMaxK = 2147483647LL - 63;     // padded k stays below 2^31
// one workgroup of 256 lanes per 64 rows along grid x: a launch holds fewer than 2^32 lanes per grid
// dimension (larger grids are cut short without an error), i.e. at most 2^24 - 1 workgroups
static const int64_t kMaxM = ((1LL << 24) - 1) * 64;
static const int64_t kMaxN = 1LL << 21;

static inline int canon_bias(int E) { return (1 << (E - 1)) - 1; }

int make_in_spec(const lba_infmt& fa, const lba_infmt& fb, InSpec* out) {
    const lba_infmt* f[2] = {&fa, &fb};
    for (int i = 0; i < 2; ++i) {
        if (f[i]->exp_bits < 2 || f[i]->exp_bits > 5 || f[i]->man_bits != 7 - f[i]->exp_bits) return LBA_ERR_FORMAT;
        if (f[i]->bias < -32 || f[i]->bias > 32) return LBA_ERR_FORMAT;
    }
    InSpec s;
    s.ea = fa.exp_bits; s.ma = fa.man_bits; s.eb = fb.exp_bits; s.mb = fb.man_bits;
    s.sig_bits = s.ma + s.mb + 2;
    const int ba = canon_bias(s.ea), bb = canon_bias(s.eb);
    s.min_lsb = (1 - ba - s.ma) + (1 - bb - s.mb);                     // subnormal unit x subnormal unit
    const int ta = (1 << s.ea) - 1 - ba, tb = (1 << s.eb) - 1 - bb;    // top exponents
    s.ptop = ta + tb + 1;
    s.max_prod = std::ldexp(2.0 - std::ldexp(1.0, -s.ma), ta) * std::ldexp(2.0 - std::ldexp(1.0, -s.mb), tb);
    s.delta = (fa.bias - ba) + (fb.bias - bb);
    *out = s;
    return LBA_OK;
}

const InSpec& e4m3_spec() {                                  // 480 * 480 = 230400 < 2^18, multiples of 2^-18
    static const InSpec s = {4, 3, 4, 3, 8, -18, 17, 230400.0, 0};
    return s;
}

int validate_shapes(int64_t M, int64_t N, int64_t K) {
    if (M < 0 || N < 0 || K < 0) return LBA_ERR_SHAPE;
    if (M > kMaxM || K > kMaxK || N > kMaxN) return LBA_ERR_SHAPE;
    return LBA_OK;
}

int validate_fmt(const lba_qfmt& q) {
    if (q.man_bits < 1 || q.man_bits > 23) return LBA_ERR_FORMAT;
    if (q.exp_bits < 2 || q.exp_bits > 7) return LBA_ERR_FORMAT;
    const int r = q.round & ~LBA_NO_UNDERFLOW;
    if (r != LBA_ROUND_FLOOR && r != LBA_ROUND_RNE) return LBA_ERR_FORMAT;
    if (q.bias > 126) return LBA_ERR_FORMAT;
    if ((1 << q.exp_bits) - q.bias - 1 > 127) return LBA_ERR_FORMAT;
    return LBA_OK;
}

static inline int top_exp(const lba_qfmt& q) { return (1 << q.exp_bits) - q.bias - 1; }

static inline float rof_value(const lba_qfmt& q, int shift) {
    return (float)std::ldexp(2.0 - std::ldexp(1.0, -q.man_bits), top_exp(q) + shift);
}

static void fill_quant(const lba_qfmt& q, int shift, uint32_t* mask, uint32_t* half, int32_t* sh,
                       float* rof, float* ruf) {
    *sh = 23 - q.man_bits;
    *mask = (*sh == 0) ? 0xFFFFFFFFu : (0xFFFFFFFFu << *sh);
    *half = (*sh == 0) ? 0u : ((1u << (*sh - 1)) - 1u);
    *rof = rof_value(q, shift);
    *ruf = (float)std::ldexp(1.0, -q.bias + shift);
}

// Can Q_prod's underflow / overflow ever fire on a product of two E4M3 values?
static bool prod_flush_possible(const lba_qfmt& qp, const InSpec& in) { return qp.bias < -in.min_lsb; }   // R_UF above the smallest product
static bool prod_clamp_possible(const lba_qfmt& qp, const InSpec& in) {
    return std::ldexp(2.0 - std::ldexp(1.0, -qp.man_bits), top_exp(qp)) <= in.max_prod;
}

// Nearest-even in the scaled kernel rounds twice (FP32's 24 bits, then M+1 bits).  That equals one
// rounding unless the 24-bit result is inexact and lands on a midpoint of the (M+1)-bit grid.
// Let pb be the significant bits of a product after Q_prod (at most 8 for E4M3 operands).
//  * The sum is inexact because of low bits of the product only when the product is far below the
//    partial sum S (a grid point); it then stays within 2^(e-23+pb) of S and clear of every midpoint
//    (at least 2^(e-M-2) away) provided pb + M <= 20.
//  * It is inexact because of low bits of S only when S is far below the product.  If products lie
//    on the accumulator's grid (pb <= M+1) the same argument applies with the roles swapped.  Else a
//    product can itself be a midpoint and a tiny S must break the tie: such an S has its lowest bit at
//    or above l = max(min_lsb, -b - M) (every sum is a multiple of 2^min_lsb; S >= 2^-b has M+1
//    bits), so the sum is inexact only from 2^(24+l) on; when that is above R_OF the result saturates
//    whatever the rounding.
static bool rne_fast_ok(const lba_qfmt& qp, const lba_qfmt& qa, bool clamp, bool flush, bool nouf_a,
                        const InSpec& in) {
    if (qa.man_bits > 10) return false;
    int pb = in.sig_bits < qp.man_bits + 1 ? in.sig_bits : qp.man_bits + 1;
    if (clamp && qp.man_bits + 1 > pb) pb = qp.man_bits + 1;            // a saturated product has M_prod+1 bits
    if (pb + qa.man_bits > 20) return false;
    if (pb > qa.man_bits + 1) {
        const int low = nouf_a ? in.min_lsb : std::max(in.min_lsb, -qa.bias - qa.man_bits);
        if (24 + low < top_exp(qa) + 1) return false;
    }
    if (nouf_a) return true;                               // no flush threshold to disturb
    int bpe = flush ? qp.bias : -in.min_lsb;               // nonzero |p| >= 2^-bpe
    if (bpe - qa.bias >= 24) return false;                 // a product could hide below 2^-150
    return true;
}

// The round-to-odd variant (two directed sums per step) has no double rounding: it is exact whenever the
// second rounding keeps at most 22 bits, with the same condition at the flush threshold as above.
static bool rne_odd_ok(const lba_qfmt& qp, const lba_qfmt& qa, bool flush, bool nouf_a, const InSpec& in) {
    if (qa.man_bits > 21) return false;
    if (nouf_a) return true;
    const int bpe = flush ? qp.bias : -in.min_lsb;
    return bpe - qa.bias < 24;
}

#ifndef LBA_FAST_BK
#define LBA_FAST_BK 32
#endif

// Lane block (outputs per lane).  4 x 4 (64 x 64 per workgroup) was the fastest on every large GEMM
// measured (8 x 8, 8 x 4 and 4 x 8 lost to it through lower occupancy and coarser grids).  GEMMs
// with few outputs cannot keep two waves on every SIMD with 16 chains per lane: between 512 and 1024
// workgroups 2 x 4 measured 3-6 % faster; up to 256 workgroups of 64 x 64 a CU would hold one wave per SIMD,
// which issues at half rate, so those grids take 2 x 4 (129-256) or 2 x 2 (up to 128): 1.6-3 times faster.
// The choice never changes a result.
static void pick_tile(int64_t M, int64_t N, int64_t batch, int kernel, int events, int prod_mode, int amode, int rne_odd, int* tm, int* tn, int* bk) {
    *tm = 4; *tn = 4;
    *bk = (kernel == KERNEL_GEN || events) ? 32 : LBA_FAST_BK;
    if (kernel == KERNEL_FAST) {
        const int64_t blocks = ((M + 63) / 64) * ((N + 63) / 64) * (batch > 0 ? batch : 1);
        if (events) return;                                    // the recompute kernel is 4 x 4 only
        if (prod_mode == PM_TRUNC || prod_mode == PM_TRUNC_CLAMP || amode || rne_odd) return;   // built for 4 x 4 only
        // a single wave per SIMD issues at half rate (256 workgroups of 64 x 64 take as long as 512): small
        // grids are cut finer until every CU has two workgroups
        if (blocks <= 128) { *tm = 2; *tn = 2; }
        else if (blocks <= 384) *tm = 2;
        else if (blocks > 512 && blocks <= 1024) *tm = 2;
    }
}

// A launch of B equal workgroups on 256 CUs takes ceil(B / 256) rounds of one workgroup per CU (four
// run side by side, but they share the CU's issue slots); when the last round is mostly empty, the rows
// of that round are cut into 32 x 32 tiles instead (a quarter of the work each, at about 0.8 of the
// efficiency), which the launch then finishes in quarter rounds.  Used when the model says 3 % or more.
// Fills in a mixed grid: gx_main tile rows of 64 x 64 workgroups, then gx_half tile rows of 48 x 64 ones, then
// 32 x 32 workgroups on whatever rows are left.  False when the counts do not fit a launch.
static bool set_mixed_grid(int64_t M, int64_t N, int64_t gx_main, int64_t gx_half, Plan* p) {
    const int64_t gy = (N + 63) / 64;
    const int64_t m_main = gx_main * 64, m_half = m_main + gx_half * 48;
    if (gx_main < 0 || gx_half < 0 || m_half > M) return false;
    const int64_t gx_tail = m_half < M ? (M - m_half + 31) / 32 : 0;
    // The forward call's tail as 32 x 16 tiles: where the workgroups before it fill the chip's 1024 slots (four per CU)
    // a whole number of times (or there are none), so that the tail starts on an empty chip, and it has at most 128 workgroups of 32 x 32
    // (a lone wave per SIMD issues at half rate; twice the workgroups of half the size, still at most one per CU, take
    // less time: the 12544 x 256 x 2304 layer 451 -> 437 us; with two per CU, 200704 x 64 x 576, nothing is gained).
    const int64_t before = (gx_main + gx_half) * gy;
    const bool tail16 = p->events == 0 && before % 1024 == 0 && gx_tail > 0 && gx_tail * ((N + 31) / 32) <= 128;
    const int64_t gy_tail = tail16 ? (N + 15) / 16 : (N + 31) / 32, tail = gx_tail * gy_tail;
    p->kp.mix_tail16 = tail16 ? 1 : 0;
    const int64_t total = (gx_main + gx_half) * gy + tail;
    if (total > 2147483647LL || gx_half * gy + tail < 1) return false;
    p->mix_tail = (int)(gx_half * gy + tail);
    p->tm = 4; p->tn = 4;
    p->kp.mix_main = (int32_t)(gx_main * gy);
    p->kp.mix_gx_main = (int32_t)(gx_main > 0 ? gx_main : 1);
    p->kp.mix_m_main = (int32_t)m_main;
    p->kp.mix_half = (int32_t)(gx_half * gy);
    p->kp.mix_gx_half = (int32_t)(gx_half > 0 ? gx_half : 1);
    p->kp.mix_m_half = (int32_t)m_half;
    p->kp.mix_gx_tail = (int32_t)(gx_tail > 0 ? gx_tail : 1);
    p->grid_x = (int)total;
    p->grid_y = 1;
    return true;
}

static void plan_mixed_grid(int64_t M, int64_t N, int64_t batch, Plan* p) {
    p->mix_tail = 0;
    if (p->kernel != KERNEL_FAST || p->rne_odd || batch != 1) return;
    // other operand formats, rounded products: the forward call (lba_fast_in_mixed_kernel) and the recompute call's OF / UF
    // planes (lba_fast_bwd_in_mixed_kernel: floor, the product modes that have a scaled recompute kernel)
    if (p->amode == 1 && (p->events == 2 || (p->events == 1 && p->round != LBA_ROUND_FLOOR))) return;
    if (p->amode == 1 && p->events == 1 && p->prod_mode != PM_FLUSH && p->prod_mode != PM_FLUSH_CLAMP &&
        p->prod_mode != PM_TRUNC && p->prod_mode != PM_TRUNC_CLAMP) return;
    // the recompute call has the mixed grid under the sequential order, and for the DIFF plane under both
    if (p->events == 1 && p->order != LBA_ORDER_SEQ) return;
    if (p->amode != 1 && p->prod_mode != PM_IDENT && p->prod_mode != PM_FLUSH && p->prod_mode != PM_FLUSH_CLAMP) return;
    const int64_t gx = (M + 63) / 64, gy = (N + 63) / 64, blocks = gx * gy;
    // those kernels have the 4 x 4 lane block alone outside the mixed grid: a grid too small for it (a single wave per
    // SIMD issues at half rate) becomes 32 x 32 workgroups throughout
    if (p->amode == 1 && blocks <= 256 && set_mixed_grid(M, N, 0, 0, p)) return;
    // the smallest grids of the forward call (at most 128 workgroups of 32 x 32, e.g. a 64 x 1000 classifier layer): the
    // tail's 32 x 16 tiles throughout, twice the workgroups of the 2 x 2 lane block
    if (p->events == 0 && ((M + 31) / 32) * ((N + 31) / 32) <= 128 && set_mixed_grid(M, N, 0, 0, p)) return;
    if (blocks > 256 * 16) return;
    // Rounds of 48 x 64 workgroups (forward call only; measured on M sweeps at N = 256 and 512, whose rates depend on
    // blocks / 256 alone): a CU that holds three 64 x 64 workgroups, or one, issues well below one that holds four or
    // two, and a launch just above a whole number of rounds pays a nearly empty round.  Whole rounds of the
    // three-quarter tile put 2 or 4 equal workgroups on every CU where the 64 x 64 tile gives 1.5 or 3, and one such
    // round after the full rounds of 64 x 64 replaces a last round that would be 60-77 % full.
    const int64_t gy32 = (N + 31) / 32;
    if (p->events == 0 && blocks > 256 && gy <= 256) {
        const int64_t b = (M / 48) * gy / 256;                 // whole rounds of 48 x 64 workgroups
        if (b >= 1 && b <= 4) {
            const int64_t gx_half = b * 256 / gy;
            const int64_t rows_left = M - gx_half * 48;
            const int64_t nq = (rows_left + 31) / 32 * gy32;   // 32 x 32 workgroups after them
            const bool take = (b == 1 && blocks >= 282) || (b == 2 && nq <= 256) || (b == 3 && nq <= 256 && blocks >= 600) ||
                              (b == 4 && nq <= 256 && blocks >= 780);
            if (take && rows_left >= 0 && set_mixed_grid(M, N, 0, gx_half, p)) return;
        }
        const int64_t a = blocks / 256;                        // full rounds of 64 x 64, then one round of 48 x 64
        if (a >= 3 && a <= 8) {
            const int64_t gx_main = a * 256 / gy;
            const int64_t mids = (M - gx_main * 64) / 48;
            if (gx_main >= 1 && mids * gy >= 205 && mids * gy <= 256 && set_mixed_grid(M, N, gx_main, mids, p)) return;
        }
    }
    if (blocks <= 384) return;
    const int64_t rounds = blocks / 256;
    const int64_t gx_main = (rounds * 256) / gy;               // whole tile rows inside the full rounds
    if (gx_main < 1 || gx_main >= gx) return;
    const int64_t m_main = gx_main * 64;
    const int64_t gx_tail = (M - m_main + 31) / 32, gy_tail = (N + 31) / 32, tail = gx_tail * gy_tail;
    if (gx_main * gy + tail > 2147483647LL) return;
    double plain = (double)((blocks + 255) / 256);
    if (p->tm == 2 && p->tn == 4) plain = 0.5 * (double)((2 * blocks + 255) / 256) / 0.95;   // the 32 x 64 choice
    const double mixed = (double)(gx_main * gy) / 256.0 + (double)((tail + 255) / 256) * 0.25 / 0.8;
    if (mixed > 0.97 * plain) return;
    set_mixed_grid(M, N, gx_main, 0, p);
}

int make_plan(int64_t M, int64_t N, int64_t K, const lba_qfmt& qp_in, const lba_qfmt& qa_in,
              int order, int events, Plan* out, int64_t batch, const InSpec* in_spec, bool conv) {
    const InSpec& in = in_spec ? *in_spec : e4m3_spec();
    int rc = validate_shapes(M, N, K);
    if (rc != LBA_OK) return rc;
    if ((rc = validate_fmt(qp_in)) != LBA_OK) return rc;
    if ((rc = validate_fmt(qa_in)) != LBA_OK) return rc;
    // the no-underflow flag is split off; qp / qa below carry the plain rounding code
    lba_qfmt qp = qp_in, qa = qa_in;
    const bool nouf_p = (qp.round & LBA_NO_UNDERFLOW) != 0, nouf_a = (qa.round & LBA_NO_UNDERFLOW) != 0;
    qp.round &= ~LBA_NO_UNDERFLOW;
    qa.round &= ~LBA_NO_UNDERFLOW;
    if (order != LBA_ORDER_SEQ && order != LBA_ORDER_CHUNK16) return LBA_ERR_UNSUPPORTED;

    Plan p;
    std::memset(&p, 0, sizeof(p));
    p.events = events == 2 ? 2 : (events ? 1 : 0);
    p.of_only = events == 3 ? 1 : 0;
    p.order = order;
    p.round = qa.round;
    KParams& kp = p.kp;
    kp.M = (int32_t)M; kp.N = (int32_t)N; kp.K = (int32_t)K;

    kp.in_ea = in.ea; kp.in_ma = in.ma; kp.in_eb = in.eb; kp.in_mb = in.mb;
    const bool flush = prod_flush_possible(qp, in) && !nouf_p;
    const bool clamp = prod_clamp_possible(qp, in);
    const bool prod_round = qp.man_bits + 1 < in.sig_bits;   // Q_prod's mantissa is narrower than a product

    // effective biases: with R_UF at 2^(ptop+3) or above every product / every sum underflows anyway
    const int lowest = -(in.ptop + 3);
    const int bpe = !flush ? (qp.bias > -in.min_lsb ? qp.bias : -in.min_lsb) : (qp.bias < lowest ? lowest : qp.bias);
    const int bae = qa.bias < lowest ? lowest : qa.bias;
    // kernel domains: the product's R_UF at 2^-126 (or, when Q_prod cannot flush, the smallest
    // product 2^-18 at or above 2^-126); the accumulator's R_UF at 2^-126, or, with the
    // no-underflow flag, a fixed 2^-60 that keeps every sum (a multiple of 2^-18) a normal number
    const int c_p_dom = bpe - 126;
    const int c_a_dom = nouf_a ? -60 : bae - 126;

    // a narrower product mantissa is one bit mask (truncation) or bfe / add3 / and (nearest-even) on the
    // exact FP32 product (the recompute call: truncation only)
    bool fast = !prod_round || !events || (qp.round == LBA_ROUND_FLOOR && order == LBA_ORDER_SEQ);
    // the recompute call has a scaled-domain kernel when Q_prod can underflow (its product-underflow test is
    // the multiply's flush); nearest-even accumulators on E4M3 matrices whose products Q_prod does not round
    // (and only where rounding twice is exact, below); anything else takes the general kernel
    if (events && !flush) fast = false;
    if (events && qa.round != LBA_ROUND_FLOOR && (prod_round || conv || in.ea != 4 || in.eb != 4)) fast = false;
    bool rne_odd = false;
    if (fast && qa.round == LBA_ROUND_RNE && !rne_fast_ok(qp, qa, clamp, flush, nouf_a, in)) {
        // E4M3 matrices, Q_prod without mantissa rounding, forward call: the round-to-odd variant
        rne_odd = !events && !prod_round && !conv && in.ea == 4 && in.eb == 4 && rne_odd_ok(qp, qa, flush, nouf_a, in);
        if (!rne_odd) fast = false;
    }
    if (fast && (flush || clamp) && std::abs(c_a_dom - c_p_dom) > 120) fast = false;   // kc must be an FP32 normal
    // the fixed domain of the no-underflow flag must keep R_OF of Q_acc an FP32 normal there (a top exponent
    // below -66 would put it among the flushed denormals and every chain would clamp to 0)
    if (fast && nouf_a && top_exp(qa) + c_a_dom < -126) fast = false;
    // ... and every non-zero sum: sums are multiples of the products' unit, 2^min_lsb, or, where Q_prod can
    // saturate, of the unit of its R_OF; if even the smallest product saturates they are multiples of R_OF itself
    if (fast && nouf_a) {
        int low = in.min_lsb;
        if (clamp) low = (top_exp(qp) + 1 <= in.min_lsb) ? top_exp(qp) : std::min(in.min_lsb, top_exp(qp) - qp.man_bits);
        if (low + c_a_dom < -126) fast = false;
    }
    // the DIFF kernel also forms p * kc * 2^60 and S * 2^60
    if (fast && events == 2 && (std::abs(c_a_dom - c_p_dom) > 60 || top_exp(qa) + c_a_dom + 61 > 126)) fast = false;
    // the recompute kernel reads an accumulator underflow off a denormal sum: with S = 0 the sum is the product,
    // at least 2^-126 in its own domain, which must not fall below the smallest denormal in the accumulator's
    if (fast && events && events != 2 && c_p_dom - c_a_dom > 23) fast = false;
    // the DIFF plane's scaled-domain kernel: E4M3 operands, Q_prod without mantissa rounding
    if (events == 2 && (prod_round || nouf_a || conv || in.ea != 4 || in.eb != 4)) fast = false;

    if (fast) {
        p.kernel = KERNEL_FAST;
        p.prod_mode = !prod_round ? (clamp ? PM_FLUSH_CLAMP : (flush ? PM_FLUSH : PM_IDENT))
                      : qp.round == LBA_ROUND_FLOOR ? (clamp ? PM_TRUNC_CLAMP : PM_TRUNC)
                                                    : (clamp ? PM_RNE_CLAMP : PM_RNE);
        const int c_a = c_a_dom;
        const int c_p = (p.prod_mode == PM_IDENT) ? c_a : c_p_dom;
        kp.exp_a = c_p / 2;                                // split the product's scale over a and b
        kp.exp_b = c_p - kp.exp_a;
        kp.kc = (float)std::ldexp(1.0, c_a - c_p);
        kp.out_exp = -c_a;
        // recompute call with an underflow plane: where the smallest non-zero product, 2^(min_lsb + c_p) here, is an FP32
        // denormal number at worst (not below 2^-149, where the multiply would return zero), a product that underflows
        // Q_prod is one, and one class test finds it
        p.uf_class = (p.events == 1 && !p.of_only && flush && in.min_lsb + c_p >= -149) ? 1 : 0;
        fill_quant(qa, c_a, &kp.mask_a, &kp.half_a, &kp.sh_a, &kp.rof_a, &kp.ruf_a);
        fill_quant(qp, c_p, &kp.mask_p, &kp.half_p, &kp.sh_p, &kp.rof_p, &kp.ruf_p);
        // Issue slots per MAC of the clamp-free inner loop, in units of one full-rate VALU op
        // (v_mul_f32 / v_fma_f32 / v_and_b32 with register operands: 32 lanes per clock per SIMD).
        // v_med3_f32, v_bfe_u32 and v_add3_u32 issue at half that rate and count 2.
        int slots = (p.prod_mode == PM_IDENT) ? 2 : 3;           // [mul,] fma, and
        if (p.prod_mode == PM_FLUSH_CLAMP || p.prod_mode == PM_TRUNC_CLAMP || p.prod_mode == PM_RNE_CLAMP) slots += 2;   // med3 on the product
        if (prod_round) slots += (qp.round == LBA_ROUND_FLOOR) ? 1 : 5;   // and [, bfe, add3] on the product
        if (qa.round == LBA_ROUND_RNE) slots += (qa.man_bits == 7 && !rne_odd) ? 1 : 4;   // M = 7: cvt to bfloat16 replaces and; else bfe, add3
        if (rne_odd) slots += 4;                                  // second fma, bfe, bfi
        p.valu_per_mac_x100 = slots * 100;
        if (events) {
            // both planes, a k-tile that cannot overflow: mul, fma, and at full rate; zero test of the product, class
            // test of the sum, carry-in add at half rate; the operand tests (8 per 16 chains); nearest-even adds the
            // flushing multiply, bfe, add3.  (A tile that can overflow adds med3, a compare and a carry-in add: 6.)
            p.valu_per_mac_x100 = 1000 + (qa.round == LBA_ROUND_RNE ? 500 : 0);
            // an underflowed product found by its class (one half-rate test) instead of its zero test and the operands' tests
            if (p.uf_class) p.valu_per_mac_x100 -= 100;
            if (p.prod_mode == PM_FLUSH_CLAMP || p.prod_mode == PM_TRUNC_CLAMP) p.valu_per_mac_x100 += 200;
            if (p.prod_mode == PM_TRUNC || p.prod_mode == PM_TRUNC_CLAMP) p.valu_per_mac_x100 += 100;
        }
        if (events == 2)                                         // mul, fma, and, mul, max, min, mul, sub, cmp; med3, addc at half rate; nearest-even: bfe, add3
            p.valu_per_mac_x100 = 1300 + (p.prod_mode == PM_FLUSH_CLAMP ? 200 : 0) + (qa.round == LBA_ROUND_RNE ? 400 : 0);
        if (order == LBA_ORDER_CHUNK16)                          // add, and [, bfe, add3], zero per 16 steps
            p.valu_per_mac_x100 += (events == 2 ? 1300 : events ? 900 : (qa.round == LBA_ROUND_RNE ? 700 : 300)) / 16;
    } else {
        p.kernel = KERNEL_GEN;
        p.prod_mode = PM_FLUSH_CLAMP;
        kp.exp_a = 0; kp.exp_b = 0; kp.out_exp = 0; kp.kc = 1.0f;
        fill_quant(qa, 0, &kp.mask_a, &kp.half_a, &kp.sh_a, &kp.rof_a, &kp.ruf_a);
        fill_quant(qp, 0, &kp.mask_p, &kp.half_p, &kp.sh_p, &kp.rof_p, &kp.ruf_p);
        if (nouf_p) kp.ruf_p = 0.0f;                       // nothing is below it
        if (nouf_a) kp.ruf_a = 0.0f;
        kp.prod_round = prod_round ? 1 : 0;
        kp.prod_rne = (qp.round == LBA_ROUND_RNE) ? 1 : 0;
        // Priced at the budget of a straightforward FMAq step, not at what the compiled loop issues (18 to 60
        // VALU instructions per MAC, depending on the variant): exact multiply, two range checks on the product,
        // exact add, mantissa rounding, two range checks on the sum, decode = 10 slots for floor, 12 for
        // nearest-even; 4 more with event bits or the DIFF bit.  A long loop cannot raise its own score.
        p.valu_per_mac_x100 = (qa.round == LBA_ROUND_RNE ? 1200 : 1000) + (events ? 400 : 0);
    }
    p.amode = (conv || in.ea != 4 || in.eb != 4 || p.prod_mode == PM_RNE || p.prod_mode == PM_RNE_CLAMP ||
               (events && (p.prod_mode == PM_TRUNC || p.prod_mode == PM_TRUNC_CLAMP))) ? 1 : 0;
    // im2col rows of E4M3 codes, products that Q_prod does not round, the forward call or the recompute call for the
    // event planes under floor rounding and the sequential order: the kernels of the row-major case with the gather
    // in place of A's fetch, on the same tiles and grids
    if (conv && fast && batch == 1 && in.ea == 4 && in.eb == 4 &&
        (p.prod_mode == PM_IDENT || p.prod_mode == PM_FLUSH || p.prod_mode == PM_FLUSH_CLAMP) &&
        (!events || (p.events == 1 && qa.round == LBA_ROUND_FLOOR && order == LBA_ORDER_SEQ && p.prod_mode != PM_IDENT)))
        p.amode = 2;
    p.rne_odd = (fast && rne_odd) ? 1 : 0;
    pick_tile(M, N, batch, p.kernel, p.events, p.prod_mode, p.amode == 1, p.rne_odd, &p.tm, &p.tn, &p.bk);
    kp.batch = 1;
    kp.fast_thresh = -1.0f;
    kp.fast_thresh4 = -1.0f;
    if (p.kernel == KERNEL_FAST) {
        // |S| can grow by at most max|p| per step (and by the rounding, for nearest-even): below
        // this bound at the start of n k-tiles, no sum inside them reaches R_OF of Q_acc.
        const int c_a = -kp.out_exp;
        double pmax = in.max_prod;
        if (clamp) pmax = std::ldexp(2.0 - std::ldexp(1.0, -qp.man_bits), top_exp(qp));
        pmax = std::ldexp(pmax, c_a);
        for (int n = 1; n <= 4; n += 3) {
            const int steps = n * p.bk;
            double th = (double)kp.rof_a;
            if (qa.round == LBA_ROUND_RNE)
                th /= std::pow((1.0 + std::ldexp(1.0, -qa.man_bits - 1)) * (1.0 + std::ldexp(1.0, -24)), steps);
            th -= (double)steps * pmax;
            float thf = (float)th;
            if ((double)thf > th) thf = std::nextafterf(thf, -INFINITY);
            if (th > 0.0 && thf > 0.0f) (n == 1 ? kp.fast_thresh : kp.fast_thresh4) = thf;
        }
        // the bound that follows the data (kernels for E4M3 matrices only): wanted where the fixed one is weak
        double g1 = (double)kp.rof_a;
        if (qa.round == LBA_ROUND_RNE)
            g1 /= std::pow((1.0 + std::ldexp(1.0, -qa.man_bits - 1)) * (1.0 + std::ldexp(1.0, -24)), p.bk);
        float g1f = (float)g1;
        if ((double)g1f > g1) g1f = std::nextafterf(g1f, -INFINITY);
        kp.rof_grow1 = g1f;
        // (floor only: under nearest-even the growth allowance eats most of the margin, and the sweep of 4096^3 formats
        // measured no gain there)
        kp.dyn_bound = (p.amode != 1 && !p.rne_odd && qa.round == LBA_ROUND_FLOOR && kp.fast_thresh4 <= 0.0f) ? 1 : 0;
    }
    const int64_t bm = 16 * p.tm, bn = 16 * p.tn;
    p.grid_x = (int)((M + bm - 1) / bm);
    p.grid_y = (int)((N + bn - 1) / bn);
    // Chunked order, forward call, fewer than 512 workgroups even of 32 x 32 outputs (less than two waves on every
    // SIMD whatever the lane block): the chunks of an output are independent first-level chains, so a workgroup
    // takes 8 x 16 outputs and runs 16 chunks of them side by side (lba_kpar_kernel); chains shorter than 128 steps
    // take 32 x 32 outputs and 4 chunks.  Measured: 64 x 1000 x 2048 1.4 -> 6.4e12 MAC/s, 256 x 256 x 4096
    // 1.5 -> 7.3e12; from 512 workgroups of 32 x 32 on it no longer pays.
    p.kpar = 0;
    if (p.kernel == KERNEL_FAST && order == LBA_ORDER_CHUNK16 && !events && !p.amode && !p.rne_odd && batch == 1 && K > 16 &&
        (p.prod_mode == PM_IDENT || p.prod_mode == PM_FLUSH || p.prod_mode == PM_FLUSH_CLAMP)) {
        const int64_t b32 = ((M + 31) / 32) * ((N + 31) / 32);
        if (b32 < 512 && (N + 15) / 16 <= 65535) {
            p.kpar = K < 128 ? 1 : 3;
            const int64_t tm = p.kpar == 1 ? 32 : 8, tn = p.kpar == 1 ? 32 : 16;
            p.tm = p.kpar == 3 ? 2 : 4; p.tn = 4;
            p.grid_x = (int)((M + tm - 1) / tm);
            p.grid_y = (int)((N + tn - 1) / tn);
        }
    }
    if (p.kpar == 0) plan_mixed_grid(M, N, batch, &p);
    *out = p;
    return LBA_OK;
}

// 256 CUs x 4 SIMDs x 4 waves want about 4096 waves = 1024 workgroups; a slice keeps at least 64 values
// of s so that the atomic adds stay a small fraction of the work.
void plan_grad_split(int64_t blocks, int64_t S, int* split, int32_t* s_chunk) {
    int64_t want = blocks > 0 ? (1024 + blocks - 1) / blocks : 1;
    const int64_t most = S > 64 ? S / 64 : 1;
    if (want > most) want = most;
    if (want > 65535) want = 65535;
    if (want < 1) want = 1;
    int64_t chunk = (S + want - 1) / want;
    chunk = (chunk + 3) / 4 * 4;
    if (chunk < 4) chunk = 4;
    *s_chunk = (int32_t)chunk;
    *split = (int)((S + chunk - 1) / chunk);
    if (*split < 1) *split = 1;
}

}  // namespace lba
