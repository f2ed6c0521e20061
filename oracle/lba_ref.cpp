// lba_ref.cpp -- CPU oracle for the simulated low-bit-width-accumulator (LBA) matrix product.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, exact definition that the HIP library
// is checked against.  It shares no code with the HIP path and must never be called from it:
// only the test-suite, the smoke check and the benchmark's CPU-baseline leg may load it.
//
// What it computes (paper arXiv 2401.14110):
//   * the floating-point quantizer Q_{M,E,b} of Sec. 2.3, Eq. (floating-point quantization):
//       R_OF = 2^(2^E-b-1) * (2 - 2^-M),  R_UF = 2^-b
//       |x| >= R_OF -> sign(x) * R_OF          (saturation, never inf)
//       |x| <  R_UF -> 0                       (flush; tested on the un-rounded |x|)
//       else sign(x) * 2^e * (1 + m),  e = floor(log2|x|),  m = 2^-M Round(2^M (|x| 2^-e - 1))
//     Round is "floor" (truncate the magnitude; Sec. 3, "floor ... via bit-mask") or
//     round-to-nearest-even (the generic Round of the equation).
//     With the no-underflow flag (the first stage of the paper's fine-tuning runs FMAq "excluding
//     underflow events", Sec. 3; Fig. 2b) the second case is dropped: values below R_UF keep their
//     M-bit mantissa, as if the exponent range had no lower end.
//   * FMAq(x, w, s) = Q_acc(Q_prod(x*w) + s), Sec. 3, Eq. (fmaq); x*w and the sum are EXACT reals,
//     only the two quantizers round.
//   * the sequential recursion S_0 = 0, S_{i+1} = FMAq(x_i, w_i, S_i), y = S_K over all K products
//     (App. D, Eq. (fma_rec)/(FMA_expanded); all K products are accumulated, see the readings
//     listed in the design notes), for Y = X W^T (App. A): C[m,n] = chain over A[m,:], B[n,:].
//   * chunked accumulation (Sec. 3 "chunk size of 16", App. D last paragraph, Fig. 1 right):
//     ceil(K/16) first-level chains of <= 16 products each started from 0, then a second-level
//     sequential chain T_0 = 0, T_{j+1} = Q_acc(T_j + c_j) over the chunk results in chunk order.
//   * per-step event bits for the fine-grained gradient estimators (Sec. 4, App. D, STE^OF):
//       OF_k = [ |Q_prod(x_k w_k) + S_k| >= R_OF^acc ]
//       UF_k = [ x_k w_k != 0 and Q_prod(x_k w_k) == 0 ]  or  [ t_k != 0 and |t_k| < R_UF^acc ]
//     and for STE^DIFF (Sec. 4 "Immediate / DIFF", App. D): with z = FMAq(x_k, w_k, S_k),
//       STE^DIFF_k = [ |z - S_k| / (|x_k w_k| + eps1) > eps2 ]
//     read with eps1 -> 0+ (the paper adds it only to keep the denominator valid: a zero product
//     gives the ratio 0), i.e. STE^DIFF_k = [ |z - S_k| > eps2 * |x_k w_k| ] over exact reals, with
//     x_k w_k the un-quantized product.  The plane holds DIFF_k = 1 - STE^DIFF_k (1 = gradient
//     blocked, the polarity of OF_k).  eps2 is a parameter of the call; eps2 = 0 is the "no change"
//     plane [ z == S_k ].
//
// Inputs are OCP FP8 E4M3 codes (1 sign, 4 exponent, 3 mantissa bits, exponent bias 7, no inf):
//   e == 0: (-1)^s * m * 2^-9 ;  e > 0: (-1)^s * (8+m) * 2^(e-10).  The two NaN codes (0x7f, 0xff)
//   are read as the bit pattern's normal number (+-480) so that behaviour is defined.
// The *_in entry points take any 8-bit code format "1 sign, E exponent, M = 7 - E mantissa bits,
// integer exponent bias" per operand (the paper's weights and activations are M4E3 with a per-tensor
// "flex" bias, Sec. 3.1): e == 0: (-1)^s * m * 2^(1-bias-M) ; e > 0: (-1)^s * (2^M + m) * 2^(e-bias-M);
// every code is finite.  E4M3 above is (E, M, bias) = (4, 3, 7).
//
// Exactness: every quantity is an integer multiple of 2^L for one call-wide L, held as an exact
// unsigned integer magnitude plus a sign.  The integer type is chosen from the bit span the two
// formats can reach: unsigned __int128 when it fits in 126 bits, else a 320-bit integer.
// No floating-point arithmetic is used anywhere on the numeric path.
//
// Build: clang++ -O2 -std=c++17 -shared -fPIC (uses the _BitInt extension for the wide carrier).

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <thread>
#include <vector>

namespace {

typedef unsigned __int128 u128;
typedef unsigned _BitInt(320) u320;

enum { ROUND_FLOOR = 0, ROUND_RNE = 1, FLAG_NO_UNDERFLOW = 0x100 };
enum { ORDER_SEQ = 0, ORDER_CHUNK16 = 1 };
enum { REF_OK = 0, REF_ERR_NULL = 1, REF_ERR_SHAPE = 2, REF_ERR_FORMAT = 3, REF_ERR_UNSUPPORTED = 4 };
enum { EV_OF = 1, EV_UF = 2, EV_DIFF = 4 };

struct Fmt { int32_t E, M, b, round; };

bool fmt_ok(const Fmt& f) {
    if (f.M < 1 || f.M > 23) return false;
    if (f.E < 2 || f.E > 7) return false;
    const int r = f.round & ~FLAG_NO_UNDERFLOW;
    if (r != ROUND_FLOOR && r != ROUND_RNE) return false;
    if (f.b > 126) return false;                       // R_UF = 2^-b must be an FP32 normal
    if ((1 << f.E) - f.b - 1 > 127) return false;      // top exponent must be an FP32 exponent
    return true;
}
inline int top_exp(const Fmt& f) { return (1 << f.E) - f.b - 1; }

// E4M3 code -> (negative?, integer significand, exponent of the significand's unit bit)
struct Dec { bool neg; int sig; int lsb; };
inline Dec decode_e4m3(uint8_t c) {
    Dec d;
    d.neg = (c >> 7) != 0;
    int e = (c >> 3) & 15, m = c & 7;
    if (e == 0) { d.sig = m; d.lsb = -9; }
    else        { d.sig = 8 + m; d.lsb = e - 10; }
    return d;
}

// Operand code format of the *_in entry points: 1 sign bit, E exponent bits, M = 7 - E mantissa bits.
struct InFmt { int32_t E, M, bias; };
const InFmt kE4M3 = {4, 3, 7};
bool infmt_ok(const InFmt& f) {
    return f.E >= 2 && f.E <= 5 && f.M == 7 - f.E && f.bias >= -32 && f.bias <= 32;
}
inline Dec decode_in(uint8_t c, const InFmt& f) {
    Dec d;
    d.neg = (c >> 7) != 0;
    int e = (c >> f.M) & ((1 << f.E) - 1), m = c & ((1 << f.M) - 1);
    if (e == 0) { d.sig = m; d.lsb = 1 - f.bias - f.M; }
    else        { d.sig = (1 << f.M) + m; d.lsb = e - f.bias - f.M; }
    return d;
}
inline int in_min_lsb(const InFmt& f) { return 1 - f.bias - f.M; }                 // unit of the subnormals
inline int in_top_exp(const InFmt& f) { return (1 << f.E) - 1 - f.bias; }          // largest value < 2^(top+1)

template <class T> inline int msb_index(T x) {        // index of the highest set bit, x != 0
    int i = -1;
    while (x != 0) { x >>= 1; ++i; }
    return i;
}
template <> inline int msb_index<u128>(u128 x) {
    uint64_t hi = (uint64_t)(x >> 64), lo = (uint64_t)x;
    return hi ? 127 - __builtin_clzll(hi) : 63 - __builtin_clzll(lo);
}

// One quantizer bound to the call-wide unit 2^L: all thresholds as integers in that unit.
template <class T> struct Quant {
    int L, M, round;
    bool no_uf;
    T rof, ruf;
    void init(const Fmt& f, int L_) {
        L = L_; M = f.M; round = f.round & ~FLAG_NO_UNDERFLOW;
        no_uf = (f.round & FLAG_NO_UNDERFLOW) != 0;
        ruf = (T)1 << (-f.b - L);
        rof = (((T)1 << (f.M + 1)) - 1) << (top_exp(f) - f.M - L);
    }
    // magnitude in, magnitude out; *ev receives EV_OF / EV_UF when those cases fire
    inline T apply(T x, int* ev) const {
        if (x == 0) return x;
        if (x >= rof) { *ev |= EV_OF; return rof; }
        if (x < ruf && !no_uf) { *ev |= EV_UF; return 0; }
        int drop = msb_index(x) - M;                   // bits below the M-bit mantissa
        if (drop <= 0) return x;
        T q = x >> drop;
        if (round == ROUND_RNE) {
            T rem = x - (q << drop);
            T half = (T)1 << (drop - 1);
            if (rem > half || (rem == half && (q & 1) != 0)) q += 1;
        }
        return q << drop;                              // a mantissa carry lands on 2^(e+1)
    }
};

template <class T> struct SVal { bool neg; T mag; };   // sign-magnitude exact value, unit 2^L

template <class T> inline SVal<T> add_exact(SVal<T> a, SVal<T> b) {
    SVal<T> r;
    if (a.neg == b.neg) { r.neg = a.neg; r.mag = a.mag + b.mag; }
    else if (a.mag >= b.mag) { r.neg = a.neg; r.mag = a.mag - b.mag; }
    else { r.neg = b.neg; r.mag = b.mag - a.mag; }
    if (r.mag == 0) r.neg = false;
    return r;
}

template <class T> inline float to_float(SVal<T> v, int L) {
    if (v.mag == 0) return 0.0f;                       // canonical +0
    T m = v.mag; int e = L;
    while ((m & 1) == 0) { m >>= 1; ++e; }
    float f = std::ldexp((float)(uint64_t)m, e);       // m < 2^24 for every format allowed
    return v.neg ? -f : f;
}

// eps2 of STE^DIFF as an exact dyadic number m * 2^e (m = 0: the "no change" limit)
struct DiffEps { bool on; uint64_t m; int e; };
const DiffEps kNoDiff = {false, 0, 0};

template <class T> struct Chain {
    Quant<T> qp, qa;
    int L;
    DiffEps eps = kNoDiff;
    Dec ta[256], tb[256];                              // decoded operand codes
    void set_inputs(const InFmt& fa, const InFmt& fb) {
        for (int c = 0; c < 256; ++c) { ta[c] = decode_in((uint8_t)c, fa); tb[c] = decode_in((uint8_t)c, fb); }
    }
    // one FMAq step: S <- Q_acc(Q_prod(a*b) + S); returns the event bits of this step
    inline int step(SVal<T>& S, uint8_t ca, uint8_t cb) const {
        Dec a = ta[ca], b = tb[cb];
        int ev_p = 0, ev_a = 0, ev = 0;
        SVal<T> p;
        p.mag = (T)(uint32_t)(a.sig * b.sig) << (a.lsb + b.lsb - L);
        p.neg = a.neg != b.neg;
        bool prod_nonzero = p.mag != 0;
        p.mag = qp.apply(p.mag, &ev_p);
        if (p.mag == 0) p.neg = false;
        if (prod_nonzero && p.mag == 0) ev |= EV_UF;   // product underflow
        T raw = (T)(uint32_t)(a.sig * b.sig) << (a.lsb + b.lsb - L);   // |x w|, before Q_prod
        SVal<T> S_old = S;
        SVal<T> t = add_exact(p, S);
        S.mag = qa.apply(t.mag, &ev_a);
        S.neg = (S.mag != 0) && t.neg;
        ev |= ev_a;                                    // accumulator overflow / underflow
        if (eps.on) {
            // STE^DIFF = [ |z - S_old| > eps2 |x w| ]; both sides scaled to integers of one unit
            SVal<T> minus_old = S_old;
            if (minus_old.mag != 0) minus_old.neg = !minus_old.neg;
            T d = add_exact(S, minus_old).mag;
            T rhs = raw * (T)eps.m;                    // raw has at most 12 bits, eps.m at most 53
            if (eps.e >= 0) rhs <<= eps.e; else d <<= -eps.e;
            if (!(d > rhs)) ev |= EV_DIFF;
        }
        return ev;
    }
    // second-level step of chunked accumulation: T <- Q_acc(T + c)
    inline int step2(SVal<T>& Tacc, SVal<T> c) const {
        int ev = 0;
        SVal<T> t = add_exact(c, Tacc);
        Tacc.mag = qa.apply(t.mag, &ev);
        Tacc.neg = (Tacc.mag != 0) && t.neg;
        return ev;
    }
};

inline void set_bit(uint32_t* plane, int64_t M, int64_t N, int64_t m, int64_t n, int64_t k) {
    plane[((k >> 5) * M + m) * N + n] |= 1u << (k & 31);
}

template <class T>
void gemm_rows(const Chain<T>& ch, const uint8_t* A, const uint8_t* B, float* C,
               uint32_t* of_mask, uint32_t* uf_mask, uint32_t* of2_mask, uint32_t* uf2_mask, uint32_t* diff_mask,
               int64_t M, int64_t N, int64_t K, int order, int64_t m_lo, int64_t m_hi) {
    for (int64_t m = m_lo; m < m_hi; ++m) {
        const uint8_t* a = A + m * K;
        for (int64_t n = 0; n < N; ++n) {
            const uint8_t* b = B + n * K;
            SVal<T> S = {false, 0};
            if (order == ORDER_SEQ) {
                for (int64_t k = 0; k < K; ++k) {
                    int ev = ch.step(S, a[k], b[k]);
                    if (of_mask && (ev & EV_OF)) set_bit(of_mask, M, N, m, n, k);
                    if (uf_mask && (ev & EV_UF)) set_bit(uf_mask, M, N, m, n, k);
                    if (diff_mask && (ev & EV_DIFF)) set_bit(diff_mask, M, N, m, n, k);
                }
            } else {
                SVal<T> Tacc = {false, 0};
                for (int64_t k0 = 0, j = 0; k0 < K; k0 += 16, ++j) {
                    S = {false, 0};
                    int64_t k1 = std::min<int64_t>(k0 + 16, K);
                    for (int64_t k = k0; k < k1; ++k) {
                        int ev = ch.step(S, a[k], b[k]);
                        if (of_mask && (ev & EV_OF)) set_bit(of_mask, M, N, m, n, k);
                        if (uf_mask && (ev & EV_UF)) set_bit(uf_mask, M, N, m, n, k);
                        if (diff_mask && (ev & EV_DIFF)) set_bit(diff_mask, M, N, m, n, k);
                    }
                    int ev2 = ch.step2(Tacc, S);
                    if (of2_mask && (ev2 & EV_OF)) set_bit(of2_mask, M, N, m, n, j);
                    if (uf2_mask && (ev2 & EV_UF)) set_bit(uf2_mask, M, N, m, n, j);
                }
                S = Tacc;
            }
            if (C) C[m * N + n] = to_float(S, ch.L);
        }
    }
}

// Smallest unit exponent and bit span needed by a pair of formats.
void span_of(const Fmt& qp, const Fmt& qa, int* L, int* bits, const InFmt& ia = kE4M3, const InFmt& ib = kE4M3) {
    int l = in_min_lsb(ia) + in_min_lsb(ib);           // unit of the smallest product (E4M3: (2^-9)^2)
    l = std::min(l, -qp.b - qp.M);
    l = std::min(l, -qa.b - qa.M);
    int ptop = in_top_exp(ia) + in_top_exp(ib) + 1;    // every product is below 2^(ptop+1) (E4M3: 480*480 < 2^18)
    int top = std::max(std::max(top_exp(qp), top_exp(qa)), ptop);
    *L = l;
    *bits = (top + 1) + 1 - l + 1;                     // a sum of two such values, plus one spare
}

template <class T>
int run_gemm(const uint8_t* A, const uint8_t* B, float* C, uint32_t* of_mask, uint32_t* uf_mask,
             uint32_t* of2_mask, uint32_t* uf2_mask,
             int64_t M, int64_t N, int64_t K, const Fmt& qp, const Fmt& qa, int order, int L,
             int nthreads, const InFmt& ia, const InFmt& ib, uint32_t* diff_mask, DiffEps eps) {
    Chain<T> ch;
    ch.L = L;
    ch.eps = eps;
    ch.qp.init(qp, L);
    ch.qa.init(qa, L);
    ch.set_inputs(ia, ib);
    int64_t W = (K + 31) / 32;
    if (of_mask) std::memset(of_mask, 0, sizeof(uint32_t) * (size_t)(W * M * N));
    if (uf_mask) std::memset(uf_mask, 0, sizeof(uint32_t) * (size_t)(W * M * N));
    if (diff_mask) std::memset(diff_mask, 0, sizeof(uint32_t) * (size_t)(W * M * N));
    int64_t W2 = ((K + 15) / 16 + 31) / 32;
    if (of2_mask) std::memset(of2_mask, 0, sizeof(uint32_t) * (size_t)(W2 * M * N));
    if (uf2_mask) std::memset(uf2_mask, 0, sizeof(uint32_t) * (size_t)(W2 * M * N));
    if (M == 0 || N == 0) return REF_OK;
    int nt = std::max(1, nthreads);
    nt = (int)std::min<int64_t>(nt, M);
    if (nt == 1) {
        gemm_rows<T>(ch, A, B, C, of_mask, uf_mask, of2_mask, uf2_mask, diff_mask, M, N, K, order, 0, M);
        return REF_OK;
    }
    // rows are split in contiguous slabs; two threads never touch the same output or mask word
    std::vector<std::thread> pool;
    for (int t = 0; t < nt; ++t) {
        int64_t lo = M * t / nt, hi = M * (t + 1) / nt;
        pool.emplace_back([=, &ch]() {
            gemm_rows<T>(ch, A, B, C, of_mask, uf_mask, of2_mask, uf2_mask, diff_mask, M, N, K, order, lo, hi);
        });
    }
    for (auto& th : pool) th.join();
    return REF_OK;
}

int gemm_entry(const uint8_t* A, const uint8_t* B, float* C, uint32_t* of_mask, uint32_t* uf_mask,
               uint32_t* of2_mask, uint32_t* uf2_mask,
               int64_t M, int64_t N, int64_t K, Fmt qp, Fmt qa, int order, int nthreads,
               InFmt ia = kE4M3, InFmt ib = kE4M3, uint32_t* diff_mask = nullptr, DiffEps eps = kNoDiff) {
    if (M < 0 || N < 0 || K < 0) return REF_ERR_SHAPE;
    if (!fmt_ok(qp) || !fmt_ok(qa) || !infmt_ok(ia) || !infmt_ok(ib)) return REF_ERR_FORMAT;
    if (order != ORDER_SEQ && order != ORDER_CHUNK16) return REF_ERR_UNSUPPORTED;
    if (M * N > 0 && ((K > 0 && (!A || !B)))) return REF_ERR_NULL;
    int L, bits;
    span_of(qp, qa, &L, &bits, ia, ib);
    if (eps.on) bits += 54 + std::abs(eps.e);          // room for the scaled sides of the DIFF comparison
    if (bits > 318) return REF_ERR_FORMAT;
    if (bits <= 126)
        return run_gemm<u128>(A, B, C, of_mask, uf_mask, of2_mask, uf2_mask, M, N, K, qp, qa, order, L, nthreads, ia, ib, diff_mask, eps);
    return run_gemm<u320>(A, B, C, of_mask, uf_mask, of2_mask, uf2_mask, M, N, K, qp, qa, order, L, nthreads, ia, ib, diff_mask, eps);
}

}  // namespace

extern "C" {

typedef struct { int32_t exp_bits, man_bits, bias, round; } lba_ref_qfmt;

static Fmt cvt(lba_ref_qfmt q) { Fmt f = {q.exp_bits, q.man_bits, q.bias, q.round}; return f; }

// C[m,n] = LBA chain over A[m,:], B[n,:]; host pointers; A [M,K], B [N,K] E4M3 codes, C [M,N] f32.
int lba_ref_gemm(const uint8_t* A, const uint8_t* B, float* C, int64_t M, int64_t N, int64_t K,
                 lba_ref_qfmt qprod, lba_ref_qfmt qacc, int32_t order, int32_t nthreads) {
    if (M * N > 0 && !C) return REF_ERR_NULL;
    return gemm_entry(A, B, C, nullptr, nullptr, nullptr, nullptr, M, N, K, cvt(qprod), cvt(qacc), order, nthreads);
}

// Same chain, also writing the event bit-planes.  Plane layout: word index ((k/32)*M + m)*N + n,
// bit k%32; tail bits zero.  For the chunked order, of2/uf2 (nullable) receive the second-level
// events with the chunk index in place of k.
int lba_ref_gemm_bwd(const uint8_t* A, const uint8_t* B, float* C, uint32_t* of_mask, uint32_t* uf_mask,
                     uint32_t* of2_mask, uint32_t* uf2_mask,
                     int64_t M, int64_t N, int64_t K,
                     lba_ref_qfmt qprod, lba_ref_qfmt qacc, int32_t order, int32_t nthreads) {
    return gemm_entry(A, B, C, of_mask, uf_mask, of2_mask, uf2_mask, M, N, K, cvt(qprod), cvt(qacc), order, nthreads);
}

typedef struct { int32_t exp_bits, man_bits, bias; } lba_ref_infmt;
static InFmt cvt_in(lba_ref_infmt f) { InFmt r = {f.exp_bits, f.man_bits, f.bias}; return r; }

// eps2 >= 0 as an exact dyadic number (any finite double is one, with an odd mantissa below 2^53)
static bool parse_eps(double eps2, DiffEps* eps) {
    if (!(eps2 >= 0.0) || std::isinf(eps2)) return false;
    eps->on = true; eps->m = 0; eps->e = 0;
    if (eps2 > 0.0) {
        int e2;
        double fr = std::frexp(eps2, &e2);
        uint64_t mant = (uint64_t)std::ldexp(fr, 53);
        int e = e2 - 53;
        while ((mant & 1) == 0) { mant >>= 1; ++e; }
        eps->m = mant; eps->e = e;
    }
    return true;
}

// The DIFF plane (1 - STE^DIFF per step, first-level steps under either order) for a threshold
// eps2 >= 0 given as a double; its exact value is used.
int lba_ref_gemm_diff(const uint8_t* A, const uint8_t* B, float* C, uint32_t* diff_mask,
                      int64_t M, int64_t N, int64_t K,
                      lba_ref_qfmt qprod, lba_ref_qfmt qacc, int32_t order, double eps2, int32_t nthreads) {
    if (!diff_mask && M * N * K > 0) return REF_ERR_NULL;
    DiffEps eps;
    if (!parse_eps(eps2, &eps)) return REF_ERR_FORMAT;
    return gemm_entry(A, B, C, nullptr, nullptr, nullptr, nullptr, M, N, K, cvt(qprod), cvt(qacc), order, nthreads,
                      kE4M3, kE4M3, diff_mask, eps);
}

// ... for operands in any 8-bit sign-exponent-mantissa code format
int lba_ref_gemm_diff_in(const uint8_t* A, const uint8_t* B, float* C, uint32_t* diff_mask,
                         int64_t M, int64_t N, int64_t K, lba_ref_infmt fmt_a, lba_ref_infmt fmt_b,
                         lba_ref_qfmt qprod, lba_ref_qfmt qacc, int32_t order, double eps2, int32_t nthreads) {
    if (!diff_mask && M * N * K > 0) return REF_ERR_NULL;
    DiffEps eps;
    if (!parse_eps(eps2, &eps)) return REF_ERR_FORMAT;
    return gemm_entry(A, B, C, nullptr, nullptr, nullptr, nullptr, M, N, K, cvt(qprod), cvt(qacc), order, nthreads,
                      cvt_in(fmt_a), cvt_in(fmt_b), diff_mask, eps);
}


// lba_ref_gemm / lba_ref_gemm_bwd for operands in any 8-bit sign-exponent-mantissa code format.
int lba_ref_gemm_in(const uint8_t* A, const uint8_t* B, float* C, uint32_t* of_mask, uint32_t* uf_mask,
                    int64_t M, int64_t N, int64_t K, lba_ref_infmt fmt_a, lba_ref_infmt fmt_b,
                    lba_ref_qfmt qprod, lba_ref_qfmt qacc, int32_t order, int32_t nthreads) {
    return gemm_entry(A, B, C, of_mask, uf_mask, nullptr, nullptr, M, N, K, cvt(qprod), cvt(qacc), order, nthreads,
                      cvt_in(fmt_a), cvt_in(fmt_b));
}

// Value of a code of such a format as a double (exact); NaN for an invalid format.
double lba_ref_decode_in(uint8_t code, lba_ref_infmt f) {
    InFmt g = cvt_in(f);
    if (!infmt_ok(g)) return std::nan("");
    Dec d = decode_in(code, g);
    double v = std::ldexp((double)d.sig, d.lsb);
    return d.neg ? -v : v;
}

// Value of an E4M3 code as a double (exact).
double lba_ref_decode(uint8_t code) {
    Dec d = decode_e4m3(code);
    double v = std::ldexp((double)d.sig, d.lsb);
    return d.neg ? -v : v;
}

// Q(x) for a double x (every finite double is an exact dyadic rational, so this is exact).
// *events receives EV_OF (1) / EV_UF (2).  Returns an error code.
int lba_ref_quantize(double x, lba_ref_qfmt q, double* out, int32_t* events) {
    Fmt f = cvt(q);
    if (!fmt_ok(f) || !out) return REF_ERR_FORMAT;
    int ev = 0;
    if (events) *events = 0;
    if (x == 0.0 || x != x) { *out = 0.0; return (x != x) ? REF_ERR_UNSUPPORTED : REF_OK; }
    bool neg = std::signbit(x);
    double ax = std::fabs(x);
    int top = top_exp(f);
    double rof = std::ldexp(2.0 - std::ldexp(1.0, -f.M), top);
    double res;
    if (std::isinf(ax) || ax >= std::ldexp(1.0, top + 2)) { res = rof; ev = EV_OF; }   // far above R_OF
    else if (ax < std::ldexp(1.0, -f.b - 2) && !(f.round & FLAG_NO_UNDERFLOW)) { res = 0.0; ev = EV_UF; }   // far below R_UF
    else {
        int e2;
        double fr = std::frexp(ax, &e2);               // ax = fr * 2^e2, fr in [0.5, 1)
        uint64_t mant = (uint64_t)std::ldexp(fr, 53);  // exact 53-bit integer
        int lsb = e2 - 53;
        int L = std::min(lsb, -f.b - f.M);
        if (top + 2 - L > 300) return REF_ERR_UNSUPPORTED;   // beyond the 320-bit carrier (no-underflow flag, tiny x)
        Quant<u320> qq; qq.init(f, L);
        u320 mag = (u320)mant << (lsb - L);
        mag = qq.apply(mag, &ev);
        // back to double: at most M+1 significant bits
        if (mag == 0) res = 0.0;
        else {
            int e = L;
            while ((mag & 1) == 0) { mag >>= 1; ++e; }
            res = std::ldexp((double)(uint64_t)mag, e);
        }
    }
    if (events) *events = ev;
    *out = (res == 0.0) ? 0.0 : (neg ? -res : res);
    return REF_OK;
}

// One FMAq step on E4M3 codes a, b and an accumulator value s (must be a Q_acc value or 0).
int lba_ref_fmaq(uint8_t a, uint8_t b, double s, lba_ref_qfmt qprod, lba_ref_qfmt qacc,
                 double* out, int32_t* events) {
    Fmt fp = cvt(qprod), fa = cvt(qacc);
    if (!fmt_ok(fp) || !fmt_ok(fa) || !out) return REF_ERR_FORMAT;
    int L, bits;
    span_of(fp, fa, &L, &bits);
    Chain<u320> ch; ch.L = L; ch.qp.init(fp, L); ch.qa.init(fa, L); ch.set_inputs(kE4M3, kE4M3);
    SVal<u320> S = {false, 0};
    if (s != 0.0) {
        int e2; double fr = std::frexp(std::fabs(s), &e2);
        uint64_t mant = (uint64_t)std::ldexp(fr, 53);
        int lsb = e2 - 53;
        while ((mant & 1) == 0) { mant >>= 1; ++lsb; }
        if (lsb < L) return REF_ERR_UNSUPPORTED;       // s is not a value of this accumulator grid
        S.mag = (u320)mant << (lsb - L);
        S.neg = s < 0;
    }
    int ev = ch.step(S, a, b);
    if (events) *events = ev;
    double r = 0.0;
    if (S.mag != 0) {
        int e = L; u320 m = S.mag;
        while ((m & 1) == 0) { m >>= 1; ++e; }
        r = std::ldexp((double)(uint64_t)m, e);
        if (S.neg) r = -r;
    }
    *out = r;
    return REF_OK;
}

// Which integer carrier a format pair needs: 128 or 320 (bits); 0 on a format error.
int lba_ref_carrier_bits(lba_ref_qfmt qprod, lba_ref_qfmt qacc) {
    Fmt fp = cvt(qprod), fa = cvt(qacc);
    if (!fmt_ok(fp) || !fmt_ok(fa)) return 0;
    int L, bits;
    span_of(fp, fa, &L, &bits);
    return bits <= 126 ? 128 : 320;
}

}  // extern "C"
