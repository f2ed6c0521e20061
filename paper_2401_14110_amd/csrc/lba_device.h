// lba_device.h -- gfx950 device code (kernel templates) of the simulated low-bit-width-accumulator GEMM.
//
// One FMAq step is  S <- Q_acc(Q_prod(a*b) + S)  (arXiv 2401.14110, Sec. 3) with the quantizer of
// Sec. 2.3; each output element C[m,n] is the K-long sequential chain of App. D.  The chain is a
// strict dependency in k, so parallelism is over outputs only: every lane owns a TM x TN block of
// independent chains held in registers, a 256-lane workgroup owns a (16 TM) x (16 TN) tile of C,
// and k advances in lock-step through tiles of A and B staged in LDS.
//
// Data path per k-tile (depth BK):
//   global: each lane fetches 16 contiguous bytes (one row, 16 k) of A and/or B   [coalescing is
//           irrelevant here: < 0.1 byte per MAC]
//   decode: E4M3 bytes -> FP32 with the hardware FP8 conversion times a power-of-two scale (other code
//           formats through an exact FP16 image, or arithmetically); the general kernel uses a 256-entry
//           LDS table of value(code) * 2^exp; operands arrive pre-scaled into the kernel's domain
//   LDS:    tiles are stored k-major ([k][row], row contiguous) so that a lane reads its 4 / 8
//           operand values of one k with one / two 16-byte reads, without bank conflicts
//   VALU:   TM*TN chains advance by one step; all FP32 ops are exact or a single rounding
//           (see lba_plan.cpp for the argument)
// Two LDS stages; the next tile's global loads are in flight while the current one is consumed.
//
// The wave's FP mode is changed with s_setreg (rounding mode) and the translation unit is built
// with FP32 denormals flushed.

#ifndef LBA_DEVICE_H_
#define LBA_DEVICE_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lba_internal.h"

namespace lba {

// ---------------------------------------------------------------------------------------------
// wave FP mode
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void set_round_nearest() { asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 0, 2), 0\n\ts_nop 1" ::: "memory"); }
__device__ __forceinline__ void set_round_pinf()    { asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 0, 2), 1\n\ts_nop 1" ::: "memory"); }
__device__ __forceinline__ void set_round_ninf()    { asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 0, 2), 2\n\ts_nop 1" ::: "memory"); }
__device__ __forceinline__ void set_round_zero()    { asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 0, 2), 3\n\ts_nop 1" ::: "memory"); }
// the same two without the memory clobber, for inner loops whose mode-dependent operations are all
// volatile assembly themselves (volatile statements keep their order; loads may still move across)
__device__ __forceinline__ void set_round_nearest_nm() { asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 0, 2), 0\n\ts_nop 1"); }
__device__ __forceinline__ void set_round_pinf_nm() { asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 0, 2), 1\n\ts_nop 1"); }
__device__ __forceinline__ void set_round_ninf_nm() { asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 0, 2), 2\n\ts_nop 1"); }
__device__ __forceinline__ void set_round_zero_nm() { asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 0, 2), 3\n\ts_nop 1"); }
__device__ __forceinline__ void set_flush_f32()     { asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 4, 2), 0\n\ts_nop 1" ::: "memory"); }

// FP16 denormals on (MODE[7:6] = 3): the staging decodes 8-bit codes through an exact FP16 image
__device__ __forceinline__ void set_denorm_f16()    { asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 6, 2), 3\n\ts_nop 1" ::: "memory"); }

__device__ __forceinline__ float med3(float x, float lo, float hi) { return __builtin_amdgcn_fmed3f(x, lo, hi); }

// ---------------------------------------------------------------------------------------------
// operand decode table: E4M3 code -> value * 2^e as an exact FP32 (Sec. "inputs" of lba.h)
// ---------------------------------------------------------------------------------------------
// (E exponent bits, M mantissa bits, bias 2^(E-1) - 1; E = 4, M = 3 is E4M3)
__device__ __forceinline__ float decode_entry(int code, int e, int E, int M) {
    const int ex = (code >> M) & ((1 << E) - 1), m = code & ((1 << M) - 1);
    const int bias = (1 << (E - 1)) - 1;
    const int sig = ex ? ((1 << M) + m) : m;
    const int lsb = (ex ? ex : 1) - bias - M;
    const float v = __builtin_ldexpf((float)sig, lsb + e);
    return (code & 0x80) ? -v : v;
}

// ---------------------------------------------------------------------------------------------
// FMAq step policies
// ---------------------------------------------------------------------------------------------
// Mantissa rounding of an FP32 word to the top (23 - sh) mantissa bits, nearest-even, for a word
// that is already the exact value or a harmless first rounding of it.
__device__ __forceinline__ uint32_t rne_bits(uint32_t u, uint32_t half, int sh, uint32_t mask) {
    return (u + half + ((u >> sh) & 1u)) & mask;
}

// Internal rounding code of the fast kernel: nearest-even to 8 significant bits (M = 7) done by
// the hardware float -> bfloat16 conversion, whose packed result with a zero low half is the FP32
// word of the rounded value.  Same function as the bfe/add3/and sequence, in one instruction.
enum { RND_RNE_BF16 = 2 };
// Internal rounding code: nearest-even that is exact for every M <= 21.  The exact sum is formed twice,
// rounded toward +inf and toward -inf (the wave's mode is switched once per k-step for all chains of a
// lane); the two results are equal iff the sum is exact and otherwise neighbours, and the one whose last
// bit is 1 is the sum rounded to odd at 24 bits.  Nearest-even at M + 1 <= 22 bits of that word equals
// nearest-even of the exact sum (the odd last bit keeps an inexact sum off every midpoint and on its side).
enum { RND_RNE_ODD = 3 };

// of two words that are equal or neighbours: the one with the odd last bit
__device__ __forceinline__ float odd_of(float up, float un) {
    const uint32_t u = __float_as_uint(up), n = __float_as_uint(un);
    const uint32_t pick = (uint32_t)(((int32_t)(u << 31)) >> 31);               // all ones iff up is odd
    return __uint_as_float((u & pick) | (n & ~pick));
}

__device__ __forceinline__ float rne_to_8_bits(float t) {
    typedef float v2f __attribute__((ext_vector_type(2)));
    typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
    const v2f v = {0.0f, t};
    return __uint_as_float(__builtin_bit_cast(uint32_t, __builtin_convertvector(v, v2bf)));
}

// Per-wave constants of the fast kernel, forced into vector registers: on gfx950 the simple
// FP32 / bitwise VALU ops issue at twice the rate when all their operands are VGPRs.
struct FastConst {
    float kc, rof, rofp;
    uint32_t mask, half, maskp, halfp;
    int sh, shp;
};

// One k-step for a GROUP of NCH independent chains, written phase by phase (all products, then
// all adds, then all roundings) so that consecutive instructions never depend on each other.
// CLAMP = false is used for k-tiles in which no chain can reach R_OF (see lba_fast_kernel).
template <int PM, int RND, bool CLAMP, int I0, int NI, int TM, int NJ>
__device__ __forceinline__ void fast_group(float (&accf)[TM][NJ], const float (&af)[TM], const float (&b)[NJ],
                                           const FastConst& c) {
    float (*acc)[NJ] = &accf[I0];
    const float* a = &af[I0];
    if (PM == PM_IDENT && RND == RND_RNE_ODD) {
        float up[NI][NJ], un[NI][NJ];
        set_round_pinf_nm();
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(up[i][j]) : "v"(a[i]), "v"(b[j]), "v"(acc[i][j]));
        set_round_ninf_nm();
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(un[i][j]) : "v"(a[i]), "v"(b[j]), "v"(acc[i][j]));
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) acc[i][j] = odd_of(up[i][j], un[i][j]);
    } else if (PM == PM_IDENT) {
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) acc[i][j] = __builtin_fmaf(a[i], b[j], acc[i][j]);
    } else {
        float q[NI][NJ];
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) q[i][j] = a[i] * b[j];        // exact; flushed below Q_prod's R_UF
        __builtin_amdgcn_sched_barrier(0);
        if (PM == PM_TRUNC || PM == PM_TRUNC_CLAMP) {                   // Q_prod's mantissa, by truncation
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j) q[i][j] = __uint_as_float(__float_as_uint(q[i][j]) & c.maskp);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (PM == PM_RNE || PM == PM_RNE_CLAMP) {
            // the product is exact in FP32, so this is Q_prod's one nearest-even rounding (a carry moves
            // to the next binade by itself); the flush above was decided on the unrounded product
            uint32_t l[NI][NJ];
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j) l[i][j] = (__float_as_uint(q[i][j]) >> c.shp) & 1u;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j) q[i][j] = __uint_as_float((__float_as_uint(q[i][j]) + c.halfp + l[i][j]) & c.maskp);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (PM == PM_FLUSH_CLAMP || PM == PM_TRUNC_CLAMP || PM == PM_RNE_CLAMP) {
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j) q[i][j] = med3(q[i][j], -c.rofp, c.rofp);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (RND == RND_RNE_ODD) {
            float up[NI][NJ], un[NI][NJ];
            set_round_pinf_nm();
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j) asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(up[i][j]) : "v"(q[i][j]), "v"(c.kc), "v"(acc[i][j]));
            set_round_ninf_nm();
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j) asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(un[i][j]) : "v"(q[i][j]), "v"(c.kc), "v"(acc[i][j]));
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j) acc[i][j] = odd_of(up[i][j], un[i][j]);
        } else {
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j) acc[i][j] = __builtin_fmaf(q[i][j], c.kc, acc[i][j]);   // one rounding of the exact sum
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    if (RND == RND_RNE_BF16) {
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) acc[i][j] = rne_to_8_bits(acc[i][j]);
    } else {
        if (RND == LBA_ROUND_RNE || RND == RND_RNE_ODD) {
            uint32_t l[NI][NJ];
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j) l[i][j] = (__float_as_uint(acc[i][j]) >> c.sh) & 1u;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j) acc[i][j] = __uint_as_float(__float_as_uint(acc[i][j]) + c.half + l[i][j]);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) acc[i][j] = __uint_as_float(__float_as_uint(acc[i][j]) & c.mask);
    }
    if (CLAMP) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j) acc[i][j] = med3(acc[i][j], -c.rof, c.rof);
    }
    __builtin_amdgcn_sched_barrier(0);
}

// General step: plain domain, every sub-step explicit.  EVENTS adds the two event bits.
struct GenOut { float S; uint32_t of; uint32_t uf; };

template <int RND>
__device__ __forceinline__ float gen_product(float a, float b, const KParams& p, uint32_t* uf1) {
    float pr = a * b;                                          // exact
    uint32_t u = __float_as_uint(pr);
    if (p.prod_round) {
        if (p.prod_rne) u = rne_bits(u, p.half_p, p.sh_p, p.mask_p);   // input exact: one rounding
        else u &= p.mask_p;
    }
    float q = __uint_as_float(u);
    const bool fl = __builtin_fabsf(pr) < p.ruf_p;             // decided on the un-rounded product
    *uf1 = (fl && pr != 0.0f) ? 1u : 0u;
    q = fl ? 0.0f : q;
    return med3(q, -p.rof_p, p.rof_p);
}

// Accumulator quantizer from the truncated sum's word uz (sign-magnitude, exact decisions) and
// the sticky bit.
__device__ __forceinline__ float gen_acc_rne(uint32_t uz, uint32_t sticky, const KParams& p,
                                             uint32_t* of, bool* small) {
    const uint32_t mag = uz & 0x7FFFFFFFu;
    const uint32_t sign = uz & 0x80000000u;
    const uint32_t rofb = __float_as_uint(p.rof_a), rufb = __float_as_uint(p.ruf_a);
    *of = mag >= rofb ? 1u : 0u;
    *small = mag < rufb;
    const int s1 = p.sh_a + 1;
    uint32_t w = (mag << 1) | sticky;                          // one more bit of precision
    const uint32_t lowmask = (1u << s1) - 1u;
    w = (w + (lowmask >> 1) + ((w >> s1) & 1u)) & ~lowmask;
    uint32_t r = sign | (w >> 1);
    r = *of ? (sign | rofb) : r;
    r = *small ? 0u : r;
    return __uint_as_float(r);
}

// ---------------------------------------------------------------------------------------------
// tile kernel
// ---------------------------------------------------------------------------------------------
template <int ROWS, int BK>
struct Stage {
    static constexpr int kChunks = ROWS * BK / 16;                         // 16-byte pieces per tile
    static constexpr int kPerLane = (kChunks + 255) / 256;
    static_assert(ROWS == 48 || (ROWS & (ROWS - 1)) == 0, "tile rows: a power of two, or 48");
    // k-major LDS tile: floats per k.  A 48-row tile (3 rows per lane) keeps the 64-row pitch, each lane's three
    // rows in the first three of its four slots, so that a lane still reads its operands with one 16-byte read.
    static constexpr int kPitch = ROWS == 48 ? 64 : ROWS;
    static __device__ __forceinline__ int slot(int row) { return ROWS == 48 ? row + row / 3 : row; }
    // lanes that take B's pieces: the highest-numbered ones, so that A and B share the work
    static constexpr int kTailShift = kChunks < 256 ? 256 - kChunks : 0;
};

// Fetch this lane's 16-byte pieces of one operand tile into registers (zero outside the matrix).
// ld_align == 16: every piece is 16-byte aligned and wholly inside its row (K % 16 == 0).
// Otherwise: five 4-byte-aligned loads cover the piece at any byte offset and are funnel-shifted
// into place.  Each load address is clamped to the aligned word holding the last valid byte, so
// every word read contains at least one byte of the matrix (it cannot cross into another page).
template <int ROWS, int BK>
__device__ __forceinline__ void fetch_tile(const uint8_t* __restrict__ G, int rows, int K, int r0, int k0,
                                           int ld_align, int tid, uint4 (&regs)[Stage<ROWS, BK>::kPerLane]) {
#pragma unroll
    for (int i = 0; i < Stage<ROWS, BK>::kPerLane; ++i) {
        const int c = tid + i * 256;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (c >= 0 && c < Stage<ROWS, BK>::kChunks) {
            const int row = c % ROWS;                                       // division by a constant
            const int kq = c / ROWS;
            const int r = r0 + row, k = k0 + kq * 16;
            if (r < rows && k < K) {
                const uint8_t* src = G + (int64_t)r * K + k;
                if (ld_align == 16) {
                    v = *reinterpret_cast<const uint4*>(src);
                } else {
                    const int nvalid = (K - k) < 16 ? (K - k) : 16;         // bytes of this piece inside the row
                    const uintptr_t a0 = reinterpret_cast<uintptr_t>(src);
                    const uintptr_t first = a0 & ~(uintptr_t)3;
                    const uintptr_t last = (a0 + (uintptr_t)(nvalid - 1)) & ~(uintptr_t)3;
                    uint32_t d[5];
#pragma unroll
                    for (int j = 0; j < 5; ++j) {
                        uintptr_t a = first + 4u * j;
                        a = a < last ? a : last;
                        d[j] = *reinterpret_cast<const uint32_t*>(a);
                    }
                    const uint32_t sh = (uint32_t)(a0 & 3u) * 8u;
                    uint32_t w[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        w[j] = __builtin_amdgcn_alignbit(d[j + 1], d[j], sh);   // ({d[j+1], d[j]} >> sh)[31:0]
                        const int nb = nvalid - 4 * j;                      // valid bytes in this word
                        const uint32_t keep = nb >= 4 ? 0xFFFFFFFFu : (nb <= 0 ? 0u : ((1u << (8 * nb)) - 1u));
                        w[j] &= keep;
                    }
                    v = make_uint4(w[0], w[1], w[2], w[3]);
                }
            }
        }
        regs[i] = v;
    }
}

// Implicit im2col: the same pieces gathered from an NHWC activation tensor.  Row r is output pixel
// (n, oh, ow); byte k of the row is X[n, oh*stride - pad + kh, ow*stride - pad + kw, c] with
// k = (kh * KW + kw) * C + c, or code 0 (the value +0) outside the image.  With C % 16 == 0 a 16-byte
// piece lies inside one tap and is one aligned load; otherwise its bytes are gathered one by one.
__device__ __forceinline__ uint32_t div_magic(uint32_t x, uint64_t magic) { return (uint32_t)(((uint64_t)x * magic) >> 40); }

template <int ROWS, int BK>
__device__ __forceinline__ void fetch_tile_conv(const uint8_t* __restrict__ X, const KParams& p, int r0, int k0,
                                                int tid, uint4 (&regs)[Stage<ROWS, BK>::kPerLane]) {
#pragma unroll
    for (int i = 0; i < Stage<ROWS, BK>::kPerLane; ++i) {
        const int c = tid + i * 256;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (c >= 0 && c < Stage<ROWS, BK>::kChunks) {
            const int row = c % ROWS;
            const int kq = c / ROWS;
            const int r = r0 + row, k = k0 + kq * 16;
            if (r < p.M && k < p.K) {
                const int ow = r % p.cv_ow, t = r / p.cv_ow;            // the lane's row never changes: hoisted
                const int oh = t % p.cv_oh, n = t / p.cv_oh;
                const int ih0 = oh * p.cv_stride - p.cv_pad, iw0 = ow * p.cv_stride - p.cv_pad;
                const int64_t img = (int64_t)n * p.cv_h;
                if (p.cv_vec) {
                    const int tap = (int)div_magic((uint32_t)k, p.cv_magic_c), ch = k - tap * p.cv_c;
                    const int kh = (int)div_magic((uint32_t)tap, p.cv_magic_kw), kw = tap - kh * p.cv_kw;
                    const int ih = ih0 + kh, iw = iw0 + kw;
                    if (ih >= 0 && ih < p.cv_h && iw >= 0 && iw < p.cv_w)
                        v = *reinterpret_cast<const uint4*>(X + ((img + ih) * p.cv_w + iw) * p.cv_c + ch);
                } else {
                    uint32_t w[4] = {0u, 0u, 0u, 0u};
                    for (int j = 0; j < 16; ++j) {
                        const int kk = k + j;
                        if (kk < p.K) {
                            const int tap = (int)div_magic((uint32_t)kk, p.cv_magic_c), ch = kk - tap * p.cv_c;
                            const int kh = (int)div_magic((uint32_t)tap, p.cv_magic_kw), kw = tap - kh * p.cv_kw;
                            const int ih = ih0 + kh, iw = iw0 + kw;
                            if (ih >= 0 && ih < p.cv_h && iw >= 0 && iw < p.cv_w)
                                w[j >> 2] |= (uint32_t)X[((img + ih) * p.cv_w + iw) * p.cv_c + ch] << (8 * (j & 3));
                        }
                    }
                    v = make_uint4(w[0], w[1], w[2], w[3]);
                }
            }
        }
        regs[i] = v;
    }
}

// A's pieces: a row-major matrix, or an activation tensor read as im2col rows.
template <int ROWS, int BK>
__device__ __forceinline__ void fetch_tile_a(const uint8_t* __restrict__ A, const KParams& p, int r0, int k0,
                                             int tid, uint4 (&regs)[Stage<ROWS, BK>::kPerLane]) {
    if (p.conv) fetch_tile_conv<ROWS, BK>(A, p, r0, k0, tid, regs);     // uniform
    else        fetch_tile<ROWS, BK>(A, p.M, p.K, r0, k0, p.ld_align, tid, regs);
}

// The same gather with the part that depends on the lane's row alone taken out of the k loop (kernels that read
// im2col rows of E4M3 codes: AMODE 2).  With k-tiles of 32 a lane fetches one 16-byte piece per tile, always of the
// same row: ConvLane keeps that row's image and the input coordinates of tap (0, 0).  The load of a piece is
// unconditional (a piece outside the image or the matrix reads the first bytes of an image and is zeroed afterwards),
// so that it can be scheduled like the loads of a row-major matrix.
struct ConvLane {
    const uint8_t* img;      // X + n * H * W * C
    int ih0, iw0;            // input row / column of tap (0, 0)
    int kq16;                // the lane's k offset inside a tile
    bool ok;                 // the lane has a piece and its row is inside the matrix
};

template <int ROWS, int BK>
__device__ __forceinline__ ConvLane conv_lane(const uint8_t* __restrict__ X, const KParams& p, int r0, int tid) {
    static_assert(Stage<ROWS, BK>::kPerLane == 1, "one piece per lane and tile");
    ConvLane L;
    const int c = tid;
    const int row = c % ROWS, kq = c / ROWS;
    const int r = r0 + row;
    L.ok = c >= 0 && c < Stage<ROWS, BK>::kChunks && r < p.M;
    const int rr = L.ok ? r : 0;
    const int ow = rr % p.cv_ow, t = rr / p.cv_ow;
    const int oh = t % p.cv_oh, n = t / p.cv_oh;
    L.ih0 = oh * p.cv_stride - p.cv_pad;
    L.iw0 = ow * p.cv_stride - p.cv_pad;
    L.img = X + (int64_t)n * p.cv_h * p.cv_w * p.cv_c;
    L.kq16 = kq * 16;
    return L;
}

template <int ROWS, int BK>
__device__ __forceinline__ void fetch_tile_conv_lane(const ConvLane& L, const KParams& p, int k0,
                                                     uint4 (&regs)[Stage<ROWS, BK>::kPerLane]) {
    const int k = k0 + L.kq16;
    const int tap = (int)div_magic((uint32_t)k, p.cv_magic_c);
    int ch = k - tap * p.cv_c;
    int kh = (int)div_magic((uint32_t)tap, p.cv_magic_kw), kw = tap - kh * p.cv_kw;
    if (p.cv_vec) {                                            // uniform
        const int ih = L.ih0 + kh, iw = L.iw0 + kw;
        const bool in = L.ok && k < p.K && (unsigned)ih < (unsigned)p.cv_h && (unsigned)iw < (unsigned)p.cv_w;
        const int64_t off = in ? ((int64_t)ih * p.cv_w + iw) * p.cv_c + ch : 0;   // (an image holds 16 bytes or more)
        const uint4 v = *reinterpret_cast<const uint4*>(L.img + off);
        regs[0] = in ? v : make_uint4(0u, 0u, 0u, 0u);
    } else {
        uint32_t w[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {                          // four independent byte loads per word
            uint32_t b[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {                      // (kh, kw, ch) step along with k
                const int ih = L.ih0 + kh, iw = L.iw0 + kw;
                const bool in = L.ok && k + 4 * q + j < p.K && (unsigned)ih < (unsigned)p.cv_h && (unsigned)iw < (unsigned)p.cv_w;
                const int64_t off = in ? ((int64_t)ih * p.cv_w + iw) * p.cv_c + ch : 0;
                const uint32_t v = L.img[off];
                b[j] = in ? v : 0u;
                if (++ch == p.cv_c) { ch = 0; if (++kw == p.cv_kw) { kw = 0; ++kh; } }
            }
            w[q] = b[0] | (b[1] << 8) | (b[2] << 16) | (b[3] << 24);
        }
        regs[0] = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// Decode the fetched pieces through the table and store them k-major into one LDS stage.
template <int ROWS, int BK>
__device__ __forceinline__ void store_tile(float* __restrict__ dst /* [BK][ROWS] */, const float* __restrict__ lut,
                                           int tid, const uint4 (&regs)[Stage<ROWS, BK>::kPerLane]) {
#pragma unroll
    for (int i = 0; i < Stage<ROWS, BK>::kPerLane; ++i) {
        const int c = tid + i * 256;
        if (c >= 0 && c < Stage<ROWS, BK>::kChunks) {
            const int row = Stage<ROWS, BK>::slot(c % ROWS);
            const int kq = c / ROWS;
            const uint32_t w[4] = {regs[i].x, regs[i].y, regs[i].z, regs[i].w};
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const uint32_t code = (w[j >> 2] >> (8 * (j & 3))) & 0xFFu;
                dst[(kq * 16 + j) * Stage<ROWS, BK>::kPitch + row] = lut[code];
            }
        }
    }
}

// Same, decoding with the hardware FP8 conversion (gfx950 decodes OCP E4M3) and one exact
// multiply by the power-of-two scale.  The two NaN codes, which the conversion would turn into NaN,
// are patched to +-480 * scale on a rarely taken path so that every code has a defined value.
// Codes of another format with E < 4 go through FP16: sign | (e << 10) | (m << (10 - M)) is the FP16 number
// value(code) * 2^(bias - 15), subnormals included, so the hardware FP16 -> FP32 conversion and one exact
// multiply by 2^(15 - bias + scale_exp) decode it.  E = 5 would put e = 31 on FP16's inf / NaN codes and is
// decoded arithmetically (integer significand times a power of two).
// PAD: floats inserted after every 16 k (the K-parallel kernel reads several 16-k pieces at once and keeps them
// on different banks that way).
// lane_max (E4M3 path only): if not null, raised to the largest magnitude this lane stored.
template <int ROWS, int BK, int PAD = 0>
__device__ __forceinline__ void store_tile_cvt(float* __restrict__ dst /* [BK][ROWS] */, float scale,
                                               int tid, const uint4 (&regs)[Stage<ROWS, BK>::kPerLane],
                                               int E = 4, int M = 3, int scale_exp = 0, float* lane_max = nullptr) {
    typedef float v2f __attribute__((ext_vector_type(2)));
    if (E != 4) {                                              // uniform
#pragma unroll
        for (int i = 0; i < Stage<ROWS, BK>::kPerLane; ++i) {
            const int c = tid + i * 256;
            if (c >= 0 && c < Stage<ROWS, BK>::kChunks) {
                const int row = Stage<ROWS, BK>::slot(c % ROWS);
                const int kq = c / ROWS;
                const uint32_t w[4] = {regs[i].x, regs[i].y, regs[i].z, regs[i].w};
                const float sc16 = __builtin_ldexpf(1.0f, 15 - ((1 << (E - 1)) - 1) + scale_exp);
                const int up = 10 - M;
                if (E < 4) {
#pragma unroll
                    for (int j = 0; j < 16; ++j) {
                        const uint32_t code = (w[j >> 2] >> (8 * (j & 3))) & 0xFFu;
                        const uint16_t h = (uint16_t)(((code & 0x80u) << 8) | ((code & 0x7Fu) << up));
                        dst[(kq * 16 + j) * Stage<ROWS, BK>::kPitch + row + kq * PAD] = (float)__builtin_bit_cast(_Float16, h) * sc16;
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 16; ++j) {
                        const int code = (int)((w[j >> 2] >> (8 * (j & 3))) & 0xFFu);
                        dst[(kq * 16 + j) * Stage<ROWS, BK>::kPitch + row + kq * PAD] = decode_entry(code, scale_exp, E, M);
                    }
                }
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < Stage<ROWS, BK>::kPerLane; ++i) {
        const int c = tid + i * 256;
        if (c >= 0 && c < Stage<ROWS, BK>::kChunks) {
            const int row = Stage<ROWS, BK>::slot(c % ROWS);
            const int kq = c / ROWS;
            const uint32_t w[4] = {regs[i].x, regs[i].y, regs[i].z, regs[i].w};
            float f[16];
            uint32_t nan_any = 0u;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const v2f lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[d], false);
                const v2f hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[d], true);
                f[4 * d + 0] = lo.x * scale; f[4 * d + 1] = lo.y * scale;
                f[4 * d + 2] = hi.x * scale; f[4 * d + 3] = hi.y * scale;
                nan_any |= ((w[d] & 0x7F7F7F7Fu) + 0x01010101u) & 0x80808080u;   // a byte with low 7 bits all set
            }
            if (nan_any) {
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const uint32_t code = (w[j >> 2] >> (8 * (j & 3))) & 0xFFu;
                    if ((code & 0x7Fu) == 0x7Fu) f[j] = (code & 0x80u) ? -480.0f * scale : 480.0f * scale;
                }
            }
#pragma unroll
            for (int j = 0; j < 16; ++j) dst[(kq * 16 + j) * Stage<ROWS, BK>::kPitch + row + kq * PAD] = f[j];
            if (lane_max) {
                float m = *lane_max;
#pragma unroll
                for (int j = 0; j < 16; j += 2) m = __builtin_fmaxf(m, __builtin_fmaxf(__builtin_fabsf(f[j]), __builtin_fabsf(f[j + 1])));
                *lane_max = m;
            }
        }
    }
}

// Largest magnitudes of the operand tiles a workgroup has just staged, for a bound on the tile's products that
// follows the data: every lane hands in the largest magnitude it stored (0 if it stored nothing); lanes 0..127
// stage A, lanes 128..255 stage B.  slot: 4 floats of LDS, published by the next barrier.
__device__ __forceinline__ void publish_tile_max(float* slot, float lane_max, int tid) {
    float m = lane_max;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = __builtin_fmaxf(m, __shfl_xor(m, o, 64));
    if ((tid & 63) == 0) slot[tid >> 6] = m;
}

// R_OF (shrunk by the growth of nearest-even rounding over the tile) minus 32 products of the largest operands
// of the tile: sums that start the tile below it cannot reach R_OF inside it.  The factor covers the roundings
// of this expression itself.
__device__ __forceinline__ float tile_threshold(const float* slot, float rof_grow1, float kc) {
    const float amax = __builtin_fmaxf(slot[0], slot[1]), bmax = __builtin_fmaxf(slot[2], slot[3]);
    return rof_grow1 - 32.0f * 1.001f * (amax * bmax) * kc;
}

// Reads the TM + TN operand values of one k from an LDS stage (TM in {2, 3, 4}, TN in {1, 2, 4}): the lane's
// rows ty*TM .. and columns tx*TN .. are contiguous in the k-major tiles (BM, BN: floats per k; three rows
// per lane sit in slots of four, see Stage).
template <int TM, int TN, int BM, int BN>
__device__ __forceinline__ void read_operands(const float* As, const float* Bs, int k, int tx, int ty,
                                              float (&a)[TM], float (&b)[TN]) {
    static_assert((TM == 2 || TM == 3 || TM == 4) && (TN == 1 || TN == 2 || TN == 4), "lane block");
    if (TM == 4) {
        const float4 v = *reinterpret_cast<const float4*>(As + k * BM + ty * 4);
        a[0] = v.x; a[1] = v.y; a[TM - 2] = v.z; a[TM - 1] = v.w;
    } else if (TM == 3) {
        const float4 v = *reinterpret_cast<const float4*>(As + k * BM + ty * 4);
        a[0] = v.x; a[1] = v.y; a[TM - 1] = v.z;
    } else {
        const float2 v = *reinterpret_cast<const float2*>(As + k * BM + ty * 2);
        a[0] = v.x; a[1] = v.y;
    }
    if (TN == 4) {
        const float4 w = *reinterpret_cast<const float4*>(Bs + k * BN + tx * 4);
        b[0] = w.x; b[1] = w.y; b[TN - 2] = w.z; b[TN - 1] = w.w;
    } else if (TN == 2) {
        const float2 w = *reinterpret_cast<const float2*>(Bs + k * BN + tx * 2);
        b[0] = w.x; b[TN - 1] = w.y;
    } else {
        b[0] = Bs[k * BN + tx];
    }
}

// Second level of the chunked order (Sec. 3, Fig. 1 right): T <- Q_acc(T + S), then S <- 0,
// for all chains of the lane, phase by phase.  T and S are both values of Q_acc's grid, so the
// same one-rounding argument as for a product step applies.
template <int RND, bool CLAMP, int TM, int TN>
__device__ __forceinline__ void fast_level2(float (&top)[TM][TN], float (&acc)[TM][TN], const FastConst& c) {
    if (RND == RND_RNE_ODD) {
        float up[TM][TN], un[TM][TN];
        set_round_pinf_nm();
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) asm volatile("v_add_f32 %0, %1, %2" : "=v"(up[i][j]) : "v"(top[i][j]), "v"(acc[i][j]));
        set_round_ninf_nm();
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) asm volatile("v_add_f32 %0, %1, %2" : "=v"(un[i][j]) : "v"(top[i][j]), "v"(acc[i][j]));
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) top[i][j] = odd_of(up[i][j], un[i][j]);
    } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) top[i][j] = top[i][j] + acc[i][j];
    }
    __builtin_amdgcn_sched_barrier(0);
    if (RND == RND_RNE_BF16) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) { top[i][j] = rne_to_8_bits(top[i][j]); acc[i][j] = 0.0f; }
    } else {
        if (RND == LBA_ROUND_RNE || RND == RND_RNE_ODD) {
            uint32_t l[TM][TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) l[i][j] = (__float_as_uint(top[i][j]) >> c.sh) & 1u;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) top[i][j] = __uint_as_float(__float_as_uint(top[i][j]) + c.half + l[i][j]);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                top[i][j] = __uint_as_float(__float_as_uint(top[i][j]) & c.mask);
                acc[i][j] = 0.0f;
            }
    }
    if (CLAMP) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) top[i][j] = med3(top[i][j], -c.rof, c.rof);
    }
    __builtin_amdgcn_sched_barrier(0);
}

// All chains of the lane advance by one k.
template <int PM, int RND, bool CLAMP, int TM, int TN>
__device__ __forceinline__ void fast_kstep(float (&acc)[TM][TN], const float (&a)[TM], const float (&b)[TN],
                                           const FastConst& c) {
    fast_group<PM, RND, CLAMP, 0, TM, TM, TN>(acc, a, b, c);
}

// One k-tile from LDS, fully unrolled; operands are read one k ahead of their use (four with the 2 x 2 block).  With the
// chunked order every 16th step is followed by the second-level step (tiles start at multiples
// of 16, so chunk boundaries are compile-time positions).
template <int PM, int RND, int ORDER, bool CLAMP, int TM, int TN, int BK, int BM, int BN>
__device__ __forceinline__ void fast_tile(float (&acc)[TM][TN], float (&top)[TM][TN], const float* As, const float* Bs,
                                          int tx, int ty, const FastConst& c) {
    if constexpr (TM * TN <= 4) {
        // The 2 x 2 block runs where a CU holds one workgroup (see fast_stage_depth): its 12 instructions per step do
        // not cover an LDS round trip, so it reads four steps ahead.
        constexpr int AHEAD = 4, SLOTS = AHEAD + 1;
        float a[SLOTS][TM], b[SLOTS][TN];
#pragma unroll
        for (int k = 0; k < AHEAD; ++k) read_operands<TM, TN, BM, BN>(As, Bs, k, tx, ty, a[k], b[k]);
#pragma unroll
        for (int k = 0; k < BK; ++k) {
            if (k + AHEAD < BK) read_operands<TM, TN, BM, BN>(As, Bs, k + AHEAD, tx, ty, a[(k + AHEAD) % SLOTS], b[(k + AHEAD) % SLOTS]);
            fast_kstep<PM, RND, CLAMP, TM, TN>(acc, a[k % SLOTS], b[k % SLOTS], c);
            if (ORDER == LBA_ORDER_CHUNK16 && ((k + 1) & 15) == 0) fast_level2<RND, CLAMP, TM, TN>(top, acc, c);
        }
    } else {
        float a0[TM], b0[TN], a1[TM], b1[TN];
        read_operands<TM, TN, BM, BN>(As, Bs, 0, tx, ty, a0, b0);
#pragma unroll
        for (int k = 0; k < BK; k += 2) {
            read_operands<TM, TN, BM, BN>(As, Bs, k + 1, tx, ty, a1, b1);
            fast_kstep<PM, RND, CLAMP, TM, TN>(acc, a0, b0, c);
            if (k + 2 < BK) read_operands<TM, TN, BM, BN>(As, Bs, k + 2, tx, ty, a0, b0);
            fast_kstep<PM, RND, CLAMP, TM, TN>(acc, a1, b1, c);
            if (ORDER == LBA_ORDER_CHUNK16 && ((k + 2) & 15) == 0) fast_level2<RND, CLAMP, TM, TN>(top, acc, c);
        }
    }
}

// k-steps that a workgroup fetches and stages at a time.  The 2 x 2 lane block runs where a CU holds one workgroup
// (small grids; the 32 x 32 tail of a mixed grid once the larger workgroups have finished): 32 steps of its 12
// instructions take 0.7 us, the next tile's global loads 1.5 us, and nothing else on the CU covers the difference,
// so it fetches 64 steps at a time (the same 32 KB of LDS as the two 64 x 64 stages of the larger blocks).  The
// tile logic (clamp-free tiles, their bounds) stays per BK steps.
__host__ __device__ constexpr int fast_stage_depth(int TM, int TN, int BK) { return TM * TN <= 4 ? 2 * BK : BK; }

#ifndef LBA_FAST_MIN_WAVES
#define LBA_FAST_MIN_WAVES 4        // waves per SIMD the register allocation must allow
#endif

// AMODE 0: A is a row-major matrix of E4M3 codes and so is B (the default; no other case costs it anything).
// AMODE 1: A may be an activation tensor read as im2col rows and either operand may use another code format.
// AMODE 2: A is an activation tensor of E4M3 codes read as im2col rows, B a matrix of E4M3 codes: AMODE 0 with
//          the gather of fetch_tile_conv_lane in place of A's row-major fetch.
// The work of one workgroup: the (16 TM) x (16 TN) tile of C at (m0, n0); smem holds two stages.
template <int TM, int TN, int BK, int PM, int RND, int ORDER, int AMODE>
__device__ __forceinline__ void fast_body(const KParams& p, float* __restrict__ smem, int m0, int n0) {
    static_assert(BK % 16 == 0, "chunk boundaries must fall on fixed positions of a k-tile");
    constexpr int BM = 16 * TM, BN = 16 * TN;
    constexpr int BKS = fast_stage_depth(TM, TN, BK);          // k-steps fetched and staged at a time
    constexpr int BMP = Stage<BM, BKS>::kPitch;               // floats per k of the A tile in LDS
    constexpr int STAGE = BKS * (BMP + BN);

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int tidb = tid - Stage<BN, BKS>::kTailShift;      // B's pieces go to the last lanes
    // batch member blockIdx.z (strides are 0 for a single GEMM)
    const uint8_t* pA = p.A + (int64_t)blockIdx.z * p.stride_a;
    const uint8_t* pB = p.B + (int64_t)blockIdx.z * p.stride_b;
    float* pC = p.C ? p.C + (int64_t)blockIdx.z * p.stride_c : nullptr;

    const float sc_a = __builtin_ldexpf(1.0f, p.exp_a), sc_b = __builtin_ldexpf(1.0f, p.exp_b);
    set_flush_f32();
    if (AMODE == 1) set_denorm_f16();
    if (RND == LBA_ROUND_FLOOR) set_round_zero();

    FastConst c;
    c.kc = p.kc; c.rof = p.rof_a; c.rofp = p.rof_p; c.mask = p.mask_a; c.half = p.half_a; c.sh = p.sh_a; c.maskp = p.mask_p; c.halfp = p.half_p; c.shp = p.sh_p;
    float thresh = p.fast_thresh, thresh4 = p.fast_thresh4;
    int safe_tiles = 0;
    asm volatile("" : "+v"(c.kc), "+v"(c.rof), "+v"(c.rofp), "+v"(c.mask), "+v"(c.half), "+v"(c.maskp), "+v"(c.halfp), "+v"(thresh), "+v"(thresh4));

    float acc[TM][TN], top[TM][TN];                            // top: second-level sums (chunked order only)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) { acc[i][j] = 0.0f; top[i][j] = 0.0f; }

    uint4 ra[Stage<BM, BKS>::kPerLane], rb[Stage<BN, BKS>::kPerLane];
    const int ntiles = (p.K + BKS - 1) / BKS;                  // K > 0 here; division by a constant

    // Formats whose R_OF is within a few maximal products of zero (the planner's flag: the fixed bounds below fail
    // for four tiles at once) also get a bound per tile from the operands actually staged.
    __shared__ float tile_max[2][4];
    const bool dyn = AMODE != 1 && p.dyn_bound != 0;           // uniform
    auto stage_tiles = [&](float* Ad, int st) {
        if (dyn) {
            float lm = 0.0f;
            store_tile_cvt<BM, BKS>(Ad, sc_a, tid, ra, 4, 3, 0, &lm);
            store_tile_cvt<BN, BKS>(Ad + BKS * BMP, sc_b, tidb, rb, 4, 3, 0, &lm);
            publish_tile_max(tile_max[st], lm, tid);
        } else {
            store_tile_cvt<BM, BKS>(Ad, sc_a, tid, ra, AMODE == 1 ? p.in_ea : 4, p.in_ma, p.exp_a);
            store_tile_cvt<BN, BKS>(Ad + BKS * BMP, sc_b, tidb, rb, AMODE == 1 ? p.in_eb : 4, p.in_mb, p.exp_b);
        }
    };
    ConvLane cl;
    if (AMODE == 2) cl = conv_lane<BM, BKS>(pA, p, m0, tid);
    auto fetch_a = [&](int k0) {
        if (AMODE == 2)      fetch_tile_conv_lane<BM, BKS>(cl, p, k0, ra);
        else if (AMODE == 1) fetch_tile_a<BM, BKS>(pA, p, m0, k0, tid, ra);
        else                 fetch_tile<BM, BKS>(pA, p.M, p.K, m0, k0, p.ld_align, tid, ra);
    };
    fetch_a(0);
    fetch_tile<BN, BKS>(pB, p.N, p.K, n0, 0, p.ld_align, tidb, rb);
    stage_tiles(smem, 0);
    __syncthreads();

    for (int t = 0; t < ntiles; ++t) {
        const float* As0 = smem + (t & 1) * STAGE;
        const float* Bs0 = As0 + BKS * BMP;
        const bool more = (t + 1) < ntiles;
        if (more) {
            fetch_a((t + 1) * BKS);
            fetch_tile<BN, BKS>(pB, p.N, p.K, n0, (t + 1) * BKS, p.ld_align, tidb, rb);
        }
        for (int part = 0; part < BKS / BK; ++part) {              // the planner's bounds are per BK steps
        const float* As = As0 + part * BK * BMP;
        const float* Bs = Bs0 + part * BK * BN;
        // (Chunked order: the test is on the second-level sums; a first-level sum starts from 0 and
        // is covered by the same bound.)
        // If every chain of the wave starts a tile below R_OF - n * BK * max|p| (scaled down further
        // for nearest-even), no sum inside the next n tiles can reach R_OF: the clamp is a no-op there
        // and a clamp-free copy of the loop runs.  The test is per wave (uniform branch) and is made
        // for n = 4 and n = 1; after a successful n = 4 test the next three tiles are not tested.
        if (safe_tiles == 0) {
            float mx = 0.0f;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; j += 2) {
                    constexpr int J1 = TN > 1 ? 1 : 0;             // the pair's second column (the same one when TN = 1)
                    mx = (ORDER == LBA_ORDER_CHUNK16)
                             ? __builtin_fmaxf(mx, __builtin_fmaxf(__builtin_fabsf(top[i][j]), __builtin_fabsf(top[i][j + J1])))
                             : __builtin_fmaxf(mx, __builtin_fmaxf(__builtin_fabsf(acc[i][j]), __builtin_fabsf(acc[i][j + J1])));
                }
            safe_tiles = __all(mx < thresh4) ? 4 : (__all(mx < thresh) ? 1 : 0);
            if (dyn && safe_tiles == 0 && __all(mx < tile_threshold(tile_max[t & 1], p.rof_grow1, c.kc))) safe_tiles = 1;
        }
        if (safe_tiles > 0) {
            --safe_tiles;
            fast_tile<PM, RND, ORDER, false, TM, TN, BK, BMP, BN>(acc, top, As, Bs, tx, ty, c);
        } else {
            fast_tile<PM, RND, ORDER, true, TM, TN, BK, BMP, BN>(acc, top, As, Bs, tx, ty, c);
        }
        }
        if (more) stage_tiles(smem + ((t + 1) & 1) * STAGE, (t + 1) & 1);
        __syncthreads();
    }
    if (RND == LBA_ROUND_FLOOR || RND == RND_RNE_ODD) set_round_nearest();

    // C = S * 2^out_exp, zero written as +0
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = m0 + ty * TM + i;
        if (m >= p.M) continue;
        const int n = n0 + tx * TN;
        float v[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const float s = (ORDER == LBA_ORDER_CHUNK16) ? top[i][j] : acc[i][j];
            v[j] = (s == 0.0f) ? 0.0f : __builtin_ldexpf(s, p.out_exp);
        }
        float* dst = pC + (int64_t)m * p.N + n;
        if (TN == 4 && p.c_vec && n + 3 < p.N) {
            *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[TN - 2], v[TN - 1]);
        } else if (TN == 2 && p.c_vec && n + 1 < p.N) {
            *reinterpret_cast<float2*>(dst) = make_float2(v[0], v[1]);
        } else {
#pragma unroll
            for (int j = 0; j < TN; ++j)
                if (n + j < p.N) dst[j] = v[j];
        }
    }
}

// Stores the 16 event words of a lane for plane word `word` (one word per chain): wof / wuf hold the
// bits shifted in first-highest, `nbits` of them since the last store; bit 0 of the stored word is the
// first of them and bits at or above `valid` are cleared.  The registers are zeroed.
template <int TM, int TN>
__device__ __forceinline__ void store_event_words(uint32_t* of_plane, uint32_t* uf_plane, int word, int nbits, int valid,
                                                  uint32_t (&wof)[TM][TN], uint32_t (&wuf)[TM][TN],
                                                  int m0, int n0, int tx, int ty, const KParams& p) {
    static_assert(TN == 4 || TN == 2, "4 or 2 outputs per lane along n");
    const uint32_t vmask = valid >= 32 ? 0xFFFFFFFFu : ((1u << valid) - 1u);
    const int up = 32 - nbits;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = m0 + ty * TM + i;
        if (m < p.M) {
            const int n = n0 + tx * TN;
            const int64_t off = ((int64_t)word * p.M + m) * p.N + n;
            uint32_t o[TN], u[TN];
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                o[j] = __builtin_bitreverse32(wof[i][j] << up) & vmask;
                u[j] = __builtin_bitreverse32(wuf[i][j] << up) & vmask;
            }
            // written once and not read again by this call: non-temporal stores, so that the plane (one word per 32
            // MACs, more bytes than A, B and C together) does not push the operand tiles out of L2
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
            if (p.c_vec && n + TN - 1 < p.N) {                 // N % 4 == 0 and aligned planes: 16- or 8-byte stores
                if (TN == 4) {
                    if (of_plane) __builtin_nontemporal_store(u32x4{o[0], o[1], o[TN - 2], o[TN - 1]}, reinterpret_cast<u32x4*>(of_plane + off));
                    if (uf_plane) __builtin_nontemporal_store(u32x4{u[0], u[1], u[TN - 2], u[TN - 1]}, reinterpret_cast<u32x4*>(uf_plane + off));
                } else {
                    if (of_plane) __builtin_nontemporal_store(u32x2{o[0], o[1]}, reinterpret_cast<u32x2*>(of_plane + off));
                    if (uf_plane) __builtin_nontemporal_store(u32x2{u[0], u[1]}, reinterpret_cast<u32x2*>(uf_plane + off));
                }
            } else {
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    if (n + j < p.N) {
                        if (of_plane) __builtin_nontemporal_store(o[j], of_plane + off + j);
                        if (uf_plane) __builtin_nontemporal_store(u[j], uf_plane + off + j);
                    }
            }
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) { wof[i][j] = 0u; wuf[i][j] = 0u; }
    }
}

template <int TM, int TN, int BK, int PM, int RND, int ORDER, int AMODE = 0>
__global__ void __launch_bounds__(256, LBA_FAST_MIN_WAVES) lba_fast_kernel(const KParams p) {
    __shared__ __attribute__((aligned(16))) float smem[2 * fast_stage_depth(TM, TN, BK) * 16 * (TM + TN)];
    fast_body<TM, TN, BK, PM, RND, ORDER, AMODE>(p, smem, blockIdx.x * 16 * TM, blockIdx.y * 16 * TN);
}

// Mixed grid for launches that would leave the last round of 64 x 64 workgroups half empty, or a CU with an odd
// number of workgroups: the first mix_main workgroups (rows below mix_m_main) take 64 x 64 tiles with 4 x 4 outputs
// per lane, the next mix_half (rows below mix_m_half) 48 x 64 tiles with 3 x 4 per lane, three quarters of the work
// each, and the rest covers the remaining rows with 32 x 32 tiles (2 x 2 per lane), a quarter of the work each, so
// that the tail of the launch is cut four times finer.  Workgroups are numbered rows-first in every region.
// mix_tail16: the tail takes 32 x 16 tiles (2 x 1 per lane) instead.  The planner sets it where the tail starts on
// an empty chip (the workgroups before it fill every slot a whole number of times) and its workgroups, doubled,
// are still at most one per CU: a lone 2 x 2 wave issues its 15 instructions per step (12 arithmetic, two LDS
// reads, a wait) at 4 to 5 cycles each, twice as many waves issue 9.  Elsewhere the narrower tile would only read
// more from LDS per MAC.
// b: the workgroup's number in the launch.
template <int BK, int PM, int RND, int ORDER, int AMODE>
__device__ __forceinline__ void fast_mixed_body(const KParams& p, float* smem, const int b) {
    if (b < p.mix_main) {                                      // uniform
        const int by = b / p.mix_gx_main, bx = b - by * p.mix_gx_main;
        fast_body<4, 4, BK, PM, RND, ORDER, AMODE>(p, smem, bx * 64, by * 64);
    } else if (b < p.mix_main + p.mix_half) {
        const int t = b - p.mix_main;
        const int by = t / p.mix_gx_half, bx = t - by * p.mix_gx_half;
        fast_body<3, 4, BK, PM, RND, ORDER, AMODE>(p, smem, p.mix_m_main + bx * 48, by * 64);
    } else {
        const int t = b - p.mix_main - p.mix_half;
        const int by = t / p.mix_gx_tail, bx = t - by * p.mix_gx_tail;
        if (p.mix_tail16) fast_body<2, 1, BK, PM, RND, ORDER, AMODE>(p, smem, p.mix_m_half + bx * 32, by * 16);   // uniform
        else              fast_body<2, 2, BK, PM, RND, ORDER, AMODE>(p, smem, p.mix_m_half + bx * 32, by * 32);
    }
}

template <int BK, int PM, int RND, int ORDER>
__global__ void __launch_bounds__(256, LBA_FAST_MIN_WAVES) lba_fast_mixed_kernel(const KParams p) {
    __shared__ __attribute__((aligned(16))) float smem[2 * BK * 16 * 8];
    fast_mixed_body<BK, PM, RND, ORDER, 0>(p, smem, blockIdx.x);
}

// The same with A read as im2col rows of an NHWC tensor (AMODE 2).
template <int BK, int PM, int RND, int ORDER>
__global__ void __launch_bounds__(256, LBA_FAST_MIN_WAVES) lba_fast_conv_mixed_kernel(const KParams p) {
    __shared__ __attribute__((aligned(16))) float smem[2 * BK * 16 * 8];
    fast_mixed_body<BK, PM, RND, ORDER, 2>(p, smem, blockIdx.x);
}

// The same for other operand formats and / or im2col rows whose products Q_prod rounds (AMODE 1).
template <int BK, int PM, int RND, int ORDER>
__global__ void __launch_bounds__(256, LBA_FAST_MIN_WAVES) lba_fast_in_mixed_kernel(const KParams p) {
    __shared__ __attribute__((aligned(16))) float smem[2 * BK * 16 * 8];
    fast_mixed_body<BK, PM, RND, ORDER, 1>(p, smem, blockIdx.x);
}

// ---------------------------------------------------------------------------------------------
// K-parallel kernel for the chunked order (forward call, launches with too few outputs to fill the chip)
// ---------------------------------------------------------------------------------------------
// Under the chunked order (Sec. 3, Fig. 1 right) the chunks of 16 products are independent chains from 0; only
// the second level, T <- Q_acc(T + chunk sum) over the chunks in order, is sequential.  When a product has too
// few outputs for one lane per 4 x 4 block of them to fill the chip, a workgroup takes a small tile of outputs and
// runs CF = 4 * CPW chunks of it side by side: wave w and, inside a wave, lane group cw own chunk w * CPW + cw of
// the current k-tile (16 * CF steps deep); every lane still advances TM x TN chains.  After the 16 steps the chunk
// sums go through LDS to the lanes that own the outputs' second-level sums, which add them in chunk order.
// The result is the chunked order's, bit for bit: the first level is the same chain per chunk, the second level
// the same ordered chain.
//   CPW = 1: 64 lane blocks of 4 x 4 per wave, tile 32 x 32, 4 chunks in flight (k-tile 64)
//   CPW = 4: 16 lane blocks of 2 x 4 per wave, tile 8 x 16, 16 chunks in flight (k-tile 256)
// One LDS stage (the next tile's global loads are in flight during the steps and are decoded into LDS while the
// second level runs), two barriers per k-tile.
template <int RND>
__device__ __forceinline__ float level2_scalar(float T, float cs, const FastConst& c) {
    float u = T + cs;                                          // both on Q_acc's grid: one rounding of the exact sum
    if (RND == RND_RNE_BF16) {
        u = rne_to_8_bits(u);
    } else {
        uint32_t w = __float_as_uint(u);
        if (RND == LBA_ROUND_RNE) w = w + c.half + ((w >> c.sh) & 1u);
        u = __uint_as_float(w & c.mask);
    }
    return med3(u, -c.rof, c.rof);
}

template <int TM, int TN, int CPW, int PM, int RND>
__global__ void __launch_bounds__(256, (CPW == 4 && TM == 4) ? 3 : 4) lba_kpar_kernel(const KParams p) {
    constexpr int SUB = 64 / CPW;                              // lane blocks per wave
    constexpr int SX = CPW == 1 ? 8 : 4, SY = SUB / SX;        // ... arranged SY x SX
    constexpr int BM = SY * TM, BN = SX * TN;                  // outputs of the workgroup
    constexpr int CF = 4 * CPW, BKT = 16 * CF;                 // chunks in flight, depth of a k-tile
    constexpr int PAD_A = CPW == 1 ? 0 : (BM >= 16 ? 16 : 8), PAD_B = CPW == 1 ? 0 : 16;
    constexpr int A_FLOATS = BKT * BM + CF * PAD_A, B_FLOATS = BKT * BN + CF * PAD_B;
    constexpr int OUT = BM * BN, OPL = (OUT + 255) / 256;      // outputs, second-level sums per lane
    __shared__ __attribute__((aligned(16))) float smem[A_FLOATS + B_FLOATS + CF * OUT];
    float* As = smem;
    float* Bs = smem + A_FLOATS;
    float* xs = Bs + B_FLOATS;                                 // [chunk][output]

    const int tid = threadIdx.x;
    const int wave = tid >> 6, l = tid & 63;
    const int cw = l / SUB, st = l % SUB;
    const int ty = st / SX, tx = st % SX;
    const int chunk = wave * CPW + cw;                         // this lane's chunk of a k-tile
    const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
    const int tidb = tid - Stage<BN, BKT>::kTailShift;

    const float sc_a = __builtin_ldexpf(1.0f, p.exp_a), sc_b = __builtin_ldexpf(1.0f, p.exp_b);
    set_flush_f32();
    if (RND == LBA_ROUND_FLOOR) set_round_zero();

    FastConst c;
    c.kc = p.kc; c.rof = p.rof_a; c.rofp = p.rof_p; c.mask = p.mask_a; c.half = p.half_a; c.sh = p.sh_a; c.maskp = p.mask_p; c.halfp = p.half_p; c.shp = p.sh_p;
    asm volatile("" : "+v"(c.kc), "+v"(c.rof), "+v"(c.rofp), "+v"(c.mask), "+v"(c.half), "+v"(c.maskp), "+v"(c.halfp));
    // a first-level sum starts from 0 and takes 16 steps: if 32 steps from 0 cannot reach R_OF (the bound the other
    // kernels test per k-tile), the clamp is a no-op
    const bool noclamp = p.fast_thresh > 0.0f;                 // uniform

    float T[OPL];
#pragma unroll
    for (int r = 0; r < OPL; ++r) T[r] = 0.0f;

    // two register sets for operand pieces in flight: the loads of tile t + 2 are issued at the start of tile t and
    // decoded into LDS during tile t + 1, so that a whole tile period covers their latency (a k-tile of this kernel
    // is short: 16 steps)
    uint4 ra0[Stage<BM, BKT>::kPerLane], rb0[Stage<BN, BKT>::kPerLane], ra1[Stage<BM, BKT>::kPerLane], rb1[Stage<BN, BKT>::kPerLane];
    const int ntiles = (p.K + BKT - 1) / BKT;

    fetch_tile<BM, BKT>(p.A, p.M, p.K, m0, 0, p.ld_align, tid, ra0);
    fetch_tile<BN, BKT>(p.B, p.N, p.K, n0, 0, p.ld_align, tidb, rb0);
    if (ntiles > 1) {
        fetch_tile<BM, BKT>(p.A, p.M, p.K, m0, BKT, p.ld_align, tid, ra1);
        fetch_tile<BN, BKT>(p.B, p.N, p.K, n0, BKT, p.ld_align, tidb, rb1);
    }
    store_tile_cvt<BM, BKT, PAD_A>(As, sc_a, tid, ra0);
    store_tile_cvt<BN, BKT, PAD_B>(Bs, sc_b, tidb, rb0);
    __syncthreads();

    const float* Ac = As + chunk * PAD_A;
    const float* Bc = Bs + chunk * PAD_B;
    // one k-tile: `next` holds the pieces of tile t + 1 (to be decoded into LDS), `free` takes those of tile t + 2
    auto tile = [&](int t, uint4 (&next_a)[Stage<BM, BKT>::kPerLane], uint4 (&next_b)[Stage<BN, BKT>::kPerLane],
                    uint4 (&free_a)[Stage<BM, BKT>::kPerLane], uint4 (&free_b)[Stage<BN, BKT>::kPerLane]) {
        const bool more = (t + 1) < ntiles;
        // first level: this lane's chunk, 16 steps from 0 (a chunk beyond K reads zeros and sums to 0)
        float acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = 0.0f;
        if (noclamp) {
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                float a[TM], b[TN];
                read_operands<TM, TN, BM, BN>(Ac, Bc, chunk * 16 + s, tx, ty, a, b);
                fast_group<PM, RND, false, 0, TM, TM, TN>(acc, a, b, c);
            }
        } else {
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                float a[TM], b[TN];
                read_operands<TM, TN, BM, BN>(Ac, Bc, chunk * 16 + s, tx, ty, a, b);
                fast_group<PM, RND, true, 0, TM, TM, TN>(acc, a, b, c);
            }
        }
        // chunk sums to the owners of the outputs
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            float* dst = xs + chunk * OUT + (ty * TM + i) * BN + tx * TN;
            if (TN == 4) *reinterpret_cast<float4*>(dst) = make_float4(acc[i][0], acc[i][1], acc[i][TN - 2], acc[i][TN - 1]);
            else         *reinterpret_cast<float2*>(dst) = make_float2(acc[i][0], acc[i][1]);
        }
        __syncthreads();                                       // chunk sums visible; every lane is done with the operand tiles
        if (more) {
            store_tile_cvt<BM, BKT, PAD_A>(As, sc_a, tid, next_a);
            store_tile_cvt<BN, BKT, PAD_B>(Bs, sc_b, tidb, next_b);
        }
        if (t + 3 < ntiles) {                                  // `next` is free again: tile t + 3 (tile t + 2 is in `free`)
            fetch_tile<BM, BKT>(p.A, p.M, p.K, m0, (t + 3) * BKT, p.ld_align, tid, next_a);
            fetch_tile<BN, BKT>(p.B, p.N, p.K, n0, (t + 3) * BKT, p.ld_align, tidb, next_b);
        }
        (void)free_a; (void)free_b;
        // second level, in chunk order (Sec. 3: no Q_prod here); the owners are the last lanes of the workgroup (the
        // first ones have more operand pieces to decode)
#pragma unroll
        for (int r = 0; r < OPL; ++r) {
            const int o = OUT >= 256 ? tid + 256 * r : tid - (256 - OUT);
            if (OUT >= 256 || o >= 0) {
#pragma unroll
                for (int cc = 0; cc < CF; ++cc) T[r] = level2_scalar<RND>(T[r], xs[cc * OUT + o], c);
            }
        }
        __syncthreads();                                       // next operand tiles visible; chunk sums consumed
    };
    // at the start of tile t: set 1 holds tile t + 1 (t even) / set 0 (t odd); tile 2 goes to set 0 once it is decoded
    if (ntiles > 2) {
        // set 0 was decoded above: reuse it for tile 2 right away
        fetch_tile<BM, BKT>(p.A, p.M, p.K, m0, 2 * BKT, p.ld_align, tid, ra0);
        fetch_tile<BN, BKT>(p.B, p.N, p.K, n0, 2 * BKT, p.ld_align, tidb, rb0);
    }
    for (int t = 0; t < ntiles; t += 2) {
        tile(t, ra1, rb1, ra0, rb0);
        if (t + 1 < ntiles) tile(t + 1, ra0, rb0, ra1, rb1);
    }
    if (RND == LBA_ROUND_FLOOR) set_round_nearest();

#pragma unroll
    for (int r = 0; r < OPL; ++r) {
        const int o = OUT >= 256 ? tid + 256 * r : tid - (256 - OUT);
        if (OUT >= 256 || o >= 0) {
            const int m = m0 + o / BN, n = n0 + o % BN;
            if (m < p.M && n < p.N) p.C[(int64_t)m * p.N + n] = (T[r] == 0.0f) ? 0.0f : __builtin_ldexpf(T[r], p.out_exp);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// fast recompute kernel: forward chain + event planes (Q_prod can flush; floor or nearest-even)
// ---------------------------------------------------------------------------------------------
// Same scaled domain as lba_fast_kernel.  The wave runs with FP32 denormals flushed on INPUT but kept on OUTPUT
// (MODE.FP_DENORM = 2): a sum below the accumulator's R_UF (2^-126 here) comes out of the fused multiply-add as a
// denormal number, which is exactly the accumulator-underflow event (t != 0 and |t| < R_UF: an exact zero sum is
// not a denormal), and the next instruction that reads it takes it as zero, which is the flush.  Every non-zero
// sum below 2^-126 is representable there: with S != 0 a sum of an (M+1)-bit and a product's <= 12-bit value is
// zero or at least 2^-126-23 in magnitude, and with S = 0 it is the product itself, at least 2^-126 in the
// product's domain, i.e. 2^(c_a - c_p - 126) here (the planner admits c_p - c_a <= 23).
//   OF_k  <=>  |t| >= R_OF.  Floor: the clamped, truncated sum has magnitude exactly R_OF.  Nearest-even: decided
//         on a second sum rounded toward zero (a sum just below R_OF may round up to it without being an overflow).
//   product underflow  <=>  the product reads as zero although both operands are non-zero (UF = 1), or, where the
//         smallest non-zero product is at least 2^-149 here (the planner's test; UF = 2), the product is a denormal
//         number: it underflowed, was kept by the multiply, and reads as zero from then on.  One class test per step
//         instead of a compare, two scalar ands and the operands' own tests: the sweep's recompute 57.7 -> 45 ms.
//   accumulator underflow  <=>  the sum is a denormal number
// Nearest-even: the sum is rounded once to 24 bits and then to M+1 bits by bit manipulation (the planner admits
// the formats for which that equals one rounding); a denormal sum is flushed by one multiply by 1 first.
// One 32-bit word per chain and k-tile: bits are shifted in (first k highest) and reversed at the end.
// A k-tile that starts with every |S| of the wave below R_OF - BK * max|p| cannot overflow: it skips the clamp
// and the overflow test (its OF words are zero), and with no underflow plane asked for it is the forward tile.
// Chunked order: after the 16th step of a chunk the chunk sum S joins the second-level sum,
// T <- Q_acc(T + S) with its own two event bits, and S restarts from 0; the test above is made on T.
__device__ __forceinline__ void set_denorm_out_f32() { asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 4, 2), 2\n\ts_nop 1" ::: "memory"); }

// lane mask of the lanes whose word is a denormal number (the bit pattern is tested, whatever the wave's mode)
__device__ __forceinline__ uint64_t ballot_denormal(float x, uint32_t cls) {
    uint64_t m;
    asm("v_cmp_class_f32 %0, %1, %2" : "=s"(m) : "v"(x), "v"(cls));
    return m;
}

struct BwdConst {
    float kc, rof, rofp, one;
    uint32_t mask, maskp, half, cls;
    int sh;
};

// nearest-even at M+1 bits of a 24-bit sum that may be a denormal number (flushed first: one multiply by 1)
// (FLUSHED: the wave flushes denormal results itself, nothing to do)
__device__ __forceinline__ float bwd_round(float td, const BwdConst& c, int RND, bool FLUSHED) {
    if (RND == LBA_ROUND_FLOOR) return __uint_as_float(__float_as_uint(td) & c.mask);
    float tf = td;
    if (!FLUSHED) asm("v_mul_f32 %0, %1, %2" : "=v"(tf) : "v"(td), "v"(c.one));
    const uint32_t u = __float_as_uint(tf);
    return __uint_as_float((u + c.half + ((u >> c.sh) & 1u)) & c.mask);
}

// One k-tile with event bits.  QUIET: no sum of the tile can reach R_OF (no clamp, no overflow test).
template <int TM, int TN, int PM, int RND, int ORDER, int UF, bool QUIET, int BM, int BN>
__device__ __forceinline__ void bwd_tile(float (&acc)[TM][TN], float (&top)[TM][TN], uint32_t (&wof)[TM][TN], uint32_t (&wuf)[TM][TN],
                                         uint32_t (&wof2)[TM][TN], uint32_t (&wuf2)[TM][TN], const float* As, const float* Bs,
                                         int tx, int ty, const BwdConst& c) {
    constexpr bool DIRECTED = (RND != LBA_ROUND_FLOOR) && !QUIET;      // a second, toward-zero sum decides the overflow
#pragma unroll 4
    for (int k = 0; k < 32; ++k) {
        float a[TM], b[TN];
        read_operands<TM, TN, BM, BN>(As, Bs, k, tx, ty, a, b);
        // all tests produce 64-bit lane masks; the event logic runs on the scalar unit
        uint64_t nza[TM], nzb[TN];
        if (UF == 1) {
#pragma unroll
            for (int i = 0; i < TM; ++i) nza[i] = __builtin_amdgcn_ballot_w64(a[i] != 0.0f);
#pragma unroll
            for (int j = 0; j < TN; ++j) nzb[j] = __builtin_amdgcn_ballot_w64(b[j] != 0.0f);
        }
        // the chains advance in groups of NI rows (8 chains for the 4 x 4 lane block): enough independent work per
        // phase, half the temporaries
        constexpr int NI = TM >= 2 ? 2 : 1;
#pragma unroll
        for (int i0 = 0; i0 < TM; i0 += NI) {
            float q[NI][TN], td[NI][TN], tz[NI][TN];
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) q[i][j] = a[i0 + i] * b[j];   // below Q_prod's R_UF: a denormal, read as zero from here on
            uint64_t qden[NI][TN];                                         // UF == 2: the product itself says that it underflowed
            if (UF == 2) {
#pragma unroll
                for (int i = 0; i < NI; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) qden[i][j] = ballot_denormal(q[i][j], c.cls);
            }
            if (PM == PM_TRUNC || PM == PM_TRUNC_CLAMP) {                  // Q_prod's mantissa, by truncation
#pragma unroll
                for (int i = 0; i < NI; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) q[i][j] = __uint_as_float(__float_as_uint(q[i][j]) & c.maskp);
            }
            if (PM == PM_FLUSH_CLAMP || PM == PM_TRUNC_CLAMP) {
#pragma unroll
                for (int i = 0; i < NI; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) q[i][j] = med3(q[i][j], -c.rofp, c.rofp);
            }
            if (DIRECTED) {
                set_round_zero_nm();
#pragma unroll
                for (int i = 0; i < NI; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(tz[i][j]) : "v"(q[i][j]), "v"(c.kc), "v"(acc[i0 + i][j]));
                set_round_nearest_nm();
#pragma unroll
                for (int i = 0; i < NI; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(td[i][j]) : "v"(q[i][j]), "v"(c.kc), "v"(acc[i0 + i][j]));
            } else {
                // the wave's rounding mode never changes in this copy of the loop: toward zero (floor) or nearest
#pragma unroll
                for (int i = 0; i < NI; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) asm("v_fma_f32 %0, %1, %2, %3" : "=v"(td[i][j]) : "v"(q[i][j]), "v"(c.kc), "v"(acc[i0 + i][j]));
            }
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    uint64_t uf = 0;
                    if (UF == 2) {
                        uf = qden[i][j] | ballot_denormal(td[i][j], c.cls);
                    } else if (UF) {
                        const uint64_t zq = __builtin_amdgcn_ballot_w64(q[i][j] == 0.0f);
                        uf = (zq & nza[i0 + i] & nzb[j]) | ballot_denormal(td[i][j], c.cls);
                    }
                    float tsum = bwd_round(td[i][j], c, RND, !UF);
                    if (!QUIET) {
                        tsum = med3(tsum, -c.rof, c.rof);
                        const uint64_t of = DIRECTED ? __builtin_amdgcn_ballot_w64(__builtin_fabsf(tz[i][j]) >= c.rof)
                                                     : __builtin_amdgcn_ballot_w64(__builtin_fabsf(tsum) == c.rof);
                        // word <- 2 * word + (this lane's bit of the mask): add with the mask as carry-in
                        asm volatile("v_addc_co_u32 %0, vcc, %0, %0, %1" : "+v"(wof[i0 + i][j]) : "s"(of) : "vcc");
                    }
                    if (UF) asm volatile("v_addc_co_u32 %0, vcc, %0, %0, %1" : "+v"(wuf[i0 + i][j]) : "s"(uf) : "vcc");
                    acc[i0 + i][j] = tsum;
                }
        }
        if (ORDER == LBA_ORDER_CHUNK16 && (k & 15) == 15) {
            float ud[TM][TN], uz[TM][TN];
            if (DIRECTED) {
                set_round_zero_nm();
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) asm volatile("v_add_f32 %0, %1, %2" : "=v"(uz[i][j]) : "v"(top[i][j]), "v"(acc[i][j]));
                set_round_nearest_nm();
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) asm volatile("v_add_f32 %0, %1, %2" : "=v"(ud[i][j]) : "v"(top[i][j]), "v"(acc[i][j]));
            } else {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) asm("v_add_f32 %0, %1, %2" : "=v"(ud[i][j]) : "v"(top[i][j]), "v"(acc[i][j]));
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    float u = bwd_round(ud[i][j], c, RND, !UF);
                    if (!QUIET) {
                        u = med3(u, -c.rof, c.rof);
                        const uint64_t of = DIRECTED ? __builtin_amdgcn_ballot_w64(__builtin_fabsf(uz[i][j]) >= c.rof)
                                                     : __builtin_amdgcn_ballot_w64(__builtin_fabsf(u) == c.rof);
                        asm volatile("v_addc_co_u32 %0, vcc, %0, %0, %1" : "+v"(wof2[i][j]) : "s"(of) : "vcc");
                    } else {
                        wof2[i][j] <<= 1;                                   // the chunk's (zero) bit
                    }
                    if (UF) {
                        const uint64_t uf = ballot_denormal(ud[i][j], c.cls);
                        asm volatile("v_addc_co_u32 %0, vcc, %0, %0, %1" : "+v"(wuf2[i][j]) : "s"(uf) : "vcc");
                    }
                    top[i][j] = u;
                    acc[i][j] = 0.0f;
                }
        }
    }
}

// Brick maps of the overflow plane as a by-product of the recompute (the gradient side's split of the immediate
// estimator): a brick is 128 rows x 32 s x 256 k of a gradient product (dX: rows m, s = n; dW: rows n, s = m) and its
// byte is set when one of its steps overflows.  Called after a k-tile that was not provably quiet, before its words
// are stored: wof holds the tile's bits, first step highest; `valid` steps of the tile lie below K.  A wave's
// outputs are 4 TM rows (inside one group of 32 rows) by 16 TN columns (one group of 32 columns, or two when
// TN = 4: lanes with tx < 8 and the others); tiles start at multiples of 16 TM and 16 TN, so no brick is straddled.
template <int TM, int TN>
__device__ __forceinline__ void mark_bricks(const uint32_t (&wof)[TM][TN], int m0, int n0, int t, int valid, int tx, int ty,
                                            const KParams& p) {
    uint32_t any = 0u;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
            if (m0 + ty * TM + i < p.M && n0 + tx * TN + j < p.N) any |= wof[i][j];
    if (valid < 32) any &= ~((1u << (32 - valid)) - 1u);       // steps at and beyond K
    const uint64_t dirty = __builtin_amdgcn_ballot_w64(any != 0u);
    if (dirty == 0) return;                                    // uniform; the usual case
    if ((threadIdx.x & 63) == 0) {                             // this lane's first row is the wave's (tx = 0)
        const int64_t kb = t >> 3;
        const int m = m0 + ty * TM;
        uint8_t* bw = p.map_dw + (kb * p.map_rbw + (n0 >> 7)) * p.map_sbw + (m >> 5);
        if (!*bw) *bw = 1;                                     // racing stores write the same value
        uint8_t* bx = p.map_dx + (kb * p.map_rbx + (m >> 7)) * p.map_sbx + (n0 >> 5);
        const uint64_t low = TN == 4 ? 0x00FF00FF00FF00FFull : ~0ull;   // lanes whose columns lie in the first group
        if ((dirty & low) && !*bx) *bx = 1;
        if (TN == 4 && (dirty & ~low) && !bx[1]) bx[1] = 1;
    }
}

template <int TM, int TN, int PM, int RND, int ORDER, int UF, int AMODE>
__device__ __forceinline__ void fast_bwd_body(const KParams& p, float* smem, const int m0, const int n0) {
    constexpr int BK = 32, BM = 16 * TM, BN = 16 * TN;
    constexpr int STAGE = BK * (BM + BN);

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int tidb = tid - Stage<BN, BK>::kTailShift;
    // batch member blockIdx.z (strides are 0 for a single GEMM)
    const uint8_t* pA = p.A + (int64_t)blockIdx.z * p.stride_a;
    const uint8_t* pB = p.B + (int64_t)blockIdx.z * p.stride_b;
    float* pC = p.C ? p.C + (int64_t)blockIdx.z * p.stride_c : nullptr;

    const float sc_a = __builtin_ldexpf(1.0f, p.exp_a), sc_b = __builtin_ldexpf(1.0f, p.exp_b);
    if (UF) set_denorm_out_f32();                              // without an underflow plane: plain flushing, as the forward kernel
    else    set_flush_f32();
    if (AMODE == 1) set_denorm_f16();
    if (RND == LBA_ROUND_FLOOR) set_round_zero();

    BwdConst c;
    c.kc = p.kc; c.rof = p.rof_a; c.rofp = p.rof_p; c.one = 1.0f; c.mask = p.mask_a; c.maskp = p.mask_p; c.half = p.half_a;
    c.cls = 0x90u;                                             // -denormal | +denormal
    c.sh = p.sh_a;
    asm volatile("" : "+v"(c.kc), "+v"(c.rof), "+v"(c.rofp), "+v"(c.one), "+v"(c.mask), "+v"(c.maskp), "+v"(c.half), "+v"(c.cls));
    FastConst fc;
    fc.kc = c.kc; fc.rof = c.rof; fc.rofp = c.rofp; fc.mask = c.mask; fc.half = c.half; fc.sh = p.sh_a; fc.maskp = c.maskp; fc.halfp = p.half_p; fc.shp = p.sh_p;
    float thresh = p.fast_thresh;
    asm volatile("" : "+v"(thresh));

    float acc[TM][TN], top[TM][TN];
    uint32_t wof[TM][TN], wuf[TM][TN], wof2[TM][TN], wuf2[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            acc[i][j] = 0.0f; wof[i][j] = 0u; wuf[i][j] = 0u;
            top[i][j] = 0.0f; wof2[i][j] = 0u; wuf2[i][j] = 0u;
        }

    uint4 ra[Stage<BM, BK>::kPerLane], rb[Stage<BN, BK>::kPerLane];
    const int ntiles = (p.K + BK - 1) / BK;

    // (the bound per tile from the operands actually staged: see fast_body)
    __shared__ float tile_max[2][4];
    const bool dyn = AMODE != 1 && p.dyn_bound != 0;           // uniform
    auto stage_tiles = [&](float* Ad, int st) {
        if (dyn) {
            float lm = 0.0f;
            store_tile_cvt<BM, BK>(Ad, sc_a, tid, ra, 4, 3, 0, &lm);
            store_tile_cvt<BN, BK>(Ad + BK * BM, sc_b, tidb, rb, 4, 3, 0, &lm);
            publish_tile_max(tile_max[st], lm, tid);
        } else {
            store_tile_cvt<BM, BK>(Ad, sc_a, tid, ra, AMODE == 1 ? p.in_ea : 4, p.in_ma, p.exp_a);
            store_tile_cvt<BN, BK>(Ad + BK * BM, sc_b, tidb, rb, AMODE == 1 ? p.in_eb : 4, p.in_mb, p.exp_b);
        }
    };
    ConvLane cl;
    if (AMODE == 2) cl = conv_lane<BM, BK>(pA, p, m0, tid);
    auto fetch_a = [&](int k0) {
        if (AMODE == 2)      fetch_tile_conv_lane<BM, BK>(cl, p, k0, ra);
        else if (AMODE == 1) fetch_tile_a<BM, BK>(pA, p, m0, k0, tid, ra);
        else                 fetch_tile<BM, BK>(pA, p.M, p.K, m0, k0, p.ld_align, tid, ra);
    };
    fetch_a(0);
    fetch_tile<BN, BK>(pB, p.N, p.K, n0, 0, p.ld_align, tidb, rb);
    stage_tiles(smem, 0);
    __syncthreads();

    for (int t = 0; t < ntiles; ++t) {
        const float* As = smem + (t & 1) * STAGE;
        const float* Bs = As + BK * BM;
        const bool more = (t + 1) < ntiles;
        if (more) {
            fetch_a((t + 1) * BK);
            fetch_tile<BN, BK>(pB, p.N, p.K, n0, (t + 1) * BK, p.ld_align, tidb, rb);
        }
        // no sum of this tile can reach R_OF (chunked order: the test is on the second-level sums; a first-level
        // sum starts from 0 and is covered by the same bound)
        float mx = 0.0f;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; j += 2)
                mx = (ORDER == LBA_ORDER_CHUNK16)
                         ? __builtin_fmaxf(mx, __builtin_fmaxf(__builtin_fabsf(top[i][j]), __builtin_fabsf(top[i][j + 1])))
                         : __builtin_fmaxf(mx, __builtin_fmaxf(__builtin_fabsf(acc[i][j]), __builtin_fabsf(acc[i][j + 1])));
        const bool quiet = __all(mx < thresh) || (dyn && __all(mx < tile_threshold(tile_max[t & 1], p.rof_grow1, c.kc)));
        if (quiet && !UF) {
            constexpr int FRND = RND == LBA_ROUND_FLOOR ? LBA_ROUND_FLOOR : LBA_ROUND_RNE;
            fast_tile<PM, FRND, ORDER, false, TM, TN, BK, BM, BN>(acc, top, As, Bs, tx, ty, fc);
            if (ORDER == LBA_ORDER_CHUNK16) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) wof2[i][j] <<= 2;         // the two chunks' (zero) bits
            }
        } else if (quiet) {
            bwd_tile<TM, TN, PM, RND, ORDER, UF, true, BM, BN>(acc, top, wof, wuf, wof2, wuf2, As, Bs, tx, ty, c);
        } else {
            bwd_tile<TM, TN, PM, RND, ORDER, UF, false, BM, BN>(acc, top, wof, wuf, wof2, wuf2, As, Bs, tx, ty, c);
            if (ORDER == LBA_ORDER_SEQ && p.map_dx) mark_bricks<TM, TN>(wof, m0, n0, t, p.K - t * BK, tx, ty, p);
        }
        store_event_words(p.of_mask, UF ? p.uf_mask : nullptr, t, 32, p.K - t * BK, wof, wuf, m0, n0, tx, ty, p);
        if (ORDER == LBA_ORDER_CHUNK16 && ((t & 15) == 15 || !more)) {
            // two chunks per k-tile: a second-level word is complete after 16 tiles
            const int chunks = (p.K + 15) >> 4;
            store_event_words(p.of_mask2, UF ? p.uf_mask2 : nullptr, t >> 4, 2 * ((t & 15) + 1), chunks - 32 * (t >> 4),
                              wof2, wuf2, m0, n0, tx, ty, p);
        }
        if (more) stage_tiles(smem + ((t + 1) & 1) * STAGE, (t + 1) & 1);
        __syncthreads();
    }
    if (RND == LBA_ROUND_FLOOR) set_round_nearest();
    set_flush_f32();

    if (pC) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int m = m0 + ty * TM + i;
            if (m >= p.M) continue;
            const int n = n0 + tx * TN;
            float v[TN];
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const float s = (ORDER == LBA_ORDER_CHUNK16) ? top[i][j] : acc[i][j];
                v[j] = (s == 0.0f) ? 0.0f : __builtin_ldexpf(s, p.out_exp);   // a denormal sum reads as zero here
            }
            float* dst = pC + (int64_t)m * p.N + n;
            if (p.c_vec && n + TN - 1 < p.N) {
                if (TN == 4) *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[TN - 2], v[TN - 1]);
                else         *reinterpret_cast<float2*>(dst) = make_float2(v[0], v[1]);
            } else {
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    if (n + j < p.N) dst[j] = v[j];
            }
        }
    }
}

template <int PM, int RND, int ORDER, int UF, int AMODE = 0>
__global__ void __launch_bounds__(256, ORDER == LBA_ORDER_CHUNK16 ? 2 : 4) lba_fast_bwd_kernel(const KParams p) {
    __shared__ __attribute__((aligned(16))) float smem[2 * 32 * 128];
    fast_bwd_body<4, 4, PM, RND, ORDER, UF, AMODE>(p, smem, blockIdx.x * 64, blockIdx.y * 64);
}

// The sequential order on E4M3 matrices on the mixed grid of lba_fast_mixed_kernel: 64 x 64 workgroups for the
// full rounds, 32 x 32 ones on the last rows.
template <int PM, int RND, int UF, int AMODE>
__device__ __forceinline__ void fast_bwd_mixed_body(const KParams& p, float* smem, const int b) {
    if (b < p.mix_main) {                                      // uniform
        const int by = b / p.mix_gx_main, bx = b - by * p.mix_gx_main;
        fast_bwd_body<4, 4, PM, RND, LBA_ORDER_SEQ, UF, AMODE>(p, smem, bx * 64, by * 64);
    } else {
        const int t = b - p.mix_main;
        const int by = t / p.mix_gx_tail, bx = t - by * p.mix_gx_tail;
        fast_bwd_body<2, 2, PM, RND, LBA_ORDER_SEQ, UF, AMODE>(p, smem, p.mix_m_main + bx * 32, by * 32);
    }
}

template <int PM, int RND, int UF>
__global__ void __launch_bounds__(256, 4) lba_fast_bwd_mixed_kernel(const KParams p) {
    __shared__ __attribute__((aligned(16))) float smem[2 * 32 * 128];
    fast_bwd_mixed_body<PM, RND, UF, 0>(p, smem, blockIdx.x);
}

// The same with A read as im2col rows of an NHWC tensor (AMODE 2).
template <int PM, int RND, int UF>
__global__ void __launch_bounds__(256, 4) lba_fast_bwd_conv_mixed_kernel(const KParams p) {
    __shared__ __attribute__((aligned(16))) float smem[2 * 32 * 128];
    fast_bwd_mixed_body<PM, RND, UF, 2>(p, smem, blockIdx.x);
}

// The same for other operand formats and truncated products (AMODE 1: the operands decoded with their run-time formats).
template <int PM, int RND, int UF>
__global__ void __launch_bounds__(256, 4) lba_fast_bwd_in_mixed_kernel(const KParams p) {
    __shared__ __attribute__((aligned(16))) float smem[2 * 32 * 128];
    fast_bwd_mixed_body<PM, RND, UF, 1>(p, smem, blockIdx.x);
}

// Recompute call for the DIFF plane (Sec. 4 "Immediate / DIFF", App. D, eps1 -> 0+) in the scaled domain:
// floor or (where rounding twice is exact) nearest-even rounding, E4M3 operands, Q_prod without mantissa rounding, flush kept.  Per step:
//   DIFF = [ |S' - S| <= eps2 * |x w| ],  both sides formed 2^60 above the accumulator's domain, where
// neither can be flushed; eps2 * |x w| has at most 12 + 8 significant bits (exact).  A product that Q_prod
// flushes leaves S' = S, so the flushed multiply (zero) gives the right bit too.
// The magnitude max(S', S) - min(S', S) is subtracted in the toward +inf mode: the right-hand side is a
// representable number, so the rounded-up difference exceeds it exactly when the exact one does, whatever
// the accumulator's width.  The mode-dependent operations of a step (product, sum, subtraction) are
// volatile assembly, which keeps them on their side of the two mode writes; everything else is exact.
// Writes the plane through p.of_mask.
template <int TM, int TN, int PM, int RND, int ORDER>
__device__ __forceinline__ void fast_diff_body(const KParams& p, float* smem, const int m0, const int n0) {
    constexpr int BK = 32, BM = 16 * TM, BN = 16 * TN;
    constexpr int STAGE = BK * (BM + BN);

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int tidb = tid - Stage<BN, BK>::kTailShift;
    const uint8_t* pA = p.A + (int64_t)blockIdx.z * p.stride_a;
    const uint8_t* pB = p.B + (int64_t)blockIdx.z * p.stride_b;
    float* pC = p.C ? p.C + (int64_t)blockIdx.z * p.stride_c : nullptr;

    const float sc_a = __builtin_ldexpf(1.0f, p.exp_a), sc_b = __builtin_ldexpf(1.0f, p.exp_b);
    set_flush_f32();
    if (RND == LBA_ROUND_FLOOR) set_round_zero();

    float kc = p.kc, rof = p.rof_a, rofp = p.rof_p, up = 0x1p60f, ce = p.kc * 0x1p60f * p.diff_eps;
    uint32_t mask = p.mask_a, half = p.half_a;
    const int sh = p.sh_a;
    asm volatile("" : "+v"(kc), "+v"(rof), "+v"(rofp), "+v"(mask), "+v"(half), "+v"(up), "+v"(ce));
    // mantissa rounding of a sum: a bit mask under the toward-zero mode (floor); nearest-even of the 24-bit
    // nearest-even sum by bit manipulation (the planner admits the formats for which that is one rounding)
    auto round_sum = [&](float t) -> float {
        const uint32_t u = __float_as_uint(t);
        if (RND == LBA_ROUND_FLOOR) return __uint_as_float(u & mask);
        return __uint_as_float((u + half + ((u >> sh) & 1u)) & mask);
    };

    float acc[TM][TN], accu[TM][TN], top[TM][TN];              // accu = acc * 2^60
    uint32_t wdf[TM][TN], unused[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) { acc[i][j] = 0.0f; accu[i][j] = 0.0f; top[i][j] = 0.0f; wdf[i][j] = 0u; unused[i][j] = 0u; }

    uint4 ra[Stage<BM, BK>::kPerLane], rb[Stage<BN, BK>::kPerLane];
    const int ntiles = (p.K + BK - 1) / BK;

    fetch_tile<BM, BK>(pA, p.M, p.K, m0, 0, p.ld_align, tid, ra);
    fetch_tile<BN, BK>(pB, p.N, p.K, n0, 0, p.ld_align, tidb, rb);
    store_tile_cvt<BM, BK>(smem, sc_a, tid, ra, 4, 3, p.exp_a);
    store_tile_cvt<BN, BK>(smem + BK * BM, sc_b, tidb, rb, 4, 3, p.exp_b);
    __syncthreads();

    for (int t = 0; t < ntiles; ++t) {
        const float* As = smem + (t & 1) * STAGE;
        const float* Bs = As + BK * BM;
        const bool more = (t + 1) < ntiles;
        if (more) {
            fetch_tile<BM, BK>(pA, p.M, p.K, m0, (t + 1) * BK, p.ld_align, tid, ra);
            fetch_tile<BN, BK>(pB, p.N, p.K, n0, (t + 1) * BK, p.ld_align, tidb, rb);
        }
#pragma unroll 4
        for (int k = 0; k < BK; ++k) {
            float a[TM], b[TN];
            read_operands<TM, TN, BM, BN>(As, Bs, k, tx, ty, a, b);
            {
                float hi[TM][TN], lo[TM][TN], rhs[TM][TN];
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {                          // the wave's own mode: toward zero, or nearest
                        float q0, tsum;
                        asm volatile("v_mul_f32 %0, %1, %2" : "=v"(q0) : "v"(a[i]), "v"(b[j]));
                        const float q = (PM == PM_FLUSH_CLAMP) ? med3(q0, -rofp, rofp) : q0;
                        asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(tsum) : "v"(q), "v"(kc), "v"(acc[i][j]));
                        tsum = round_sum(tsum);
                        tsum = med3(tsum, -rof, rof);
                        const float su = tsum * up;                         // exact
                        hi[i][j] = __builtin_fmaxf(su, accu[i][j]);
                        lo[i][j] = __builtin_fminf(su, accu[i][j]);
                        rhs[i][j] = __builtin_fabsf(q0) * ce;               // exact
                        acc[i][j] = tsum;
                        accu[i][j] = su;
                    }
                set_round_pinf_nm();
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        asm volatile("v_sub_f32 %0, %1, %2" : "=v"(hi[i][j]) : "v"(hi[i][j]), "v"(lo[i][j]));
                if (RND == LBA_ROUND_FLOOR) set_round_zero_nm(); else set_round_nearest_nm();
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const uint64_t blocked = __builtin_amdgcn_ballot_w64(!(hi[i][j] > rhs[i][j]));
                        asm volatile("v_addc_co_u32 %0, vcc, %0, %0, %1" : "+v"(wdf[i][j]) : "s"(blocked) : "vcc");
                    }
            }
            if (ORDER == LBA_ORDER_CHUNK16 && (k & 15) == 15) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        float u;
                        asm volatile("v_add_f32 %0, %1, %2" : "=v"(u) : "v"(top[i][j]), "v"(acc[i][j]));   // stays in the part that runs in the wave's own mode
                        u = round_sum(u);
                        top[i][j] = med3(u, -rof, rof);
                        acc[i][j] = 0.0f;
                        accu[i][j] = 0.0f;
                    }
            }
        }
        store_event_words(p.of_mask, nullptr, t, 32, p.K - t * BK, wdf, unused, m0, n0, tx, ty, p);
        if (more) {
            float* Ad = smem + ((t + 1) & 1) * STAGE;
            store_tile_cvt<BM, BK>(Ad, sc_a, tid, ra, 4, 3, p.exp_a);
            store_tile_cvt<BN, BK>(Ad + BK * BM, sc_b, tidb, rb, 4, 3, p.exp_b);
        }
        __syncthreads();
    }
    if (RND == LBA_ROUND_FLOOR) set_round_nearest();

    if (pC) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int m = m0 + ty * TM + i;
            if (m >= p.M) continue;
            const int n = n0 + tx * TN;
            float v[TN];
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const float s = (ORDER == LBA_ORDER_CHUNK16) ? top[i][j] : acc[i][j];
                v[j] = (s == 0.0f) ? 0.0f : __builtin_ldexpf(s, p.out_exp);
            }
            float* dst = pC + (int64_t)m * p.N + n;
            if (p.c_vec && n + TN - 1 < p.N) {
                if (TN == 4) *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[TN - 2], v[TN - 1]);
                else         *reinterpret_cast<float2*>(dst) = make_float2(v[0], v[1]);
            } else {
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    if (n + j < p.N) dst[j] = v[j];
            }
        }
    }
}

template <int PM, int RND, int ORDER>
__global__ void __launch_bounds__(256, 3) lba_fast_diff_kernel(const KParams p) {
    __shared__ __attribute__((aligned(16))) float smem[2 * 32 * 128];
    fast_diff_body<4, 4, PM, RND, ORDER>(p, smem, blockIdx.x * 64, blockIdx.y * 64);
}

// The same on the mixed grid of lba_fast_mixed_kernel: 64 x 64 workgroups for the full rounds, 32 x 32 ones on the
// last rows of the launch.
template <int PM, int RND, int ORDER>
__global__ void __launch_bounds__(256, 3) lba_fast_diff_mixed_kernel(const KParams p) {
    __shared__ __attribute__((aligned(16))) float smem[2 * 32 * 128];
    const int b = blockIdx.x;
    if (b < p.mix_main) {                                      // uniform
        const int by = b / p.mix_gx_main, bx = b - by * p.mix_gx_main;
        fast_diff_body<4, 4, PM, RND, ORDER>(p, smem, bx * 64, by * 64);
    } else {
        const int t = b - p.mix_main;
        const int by = t / p.mix_gx_tail, bx = t - by * p.mix_gx_tail;
        fast_diff_body<2, 2, PM, RND, ORDER>(p, smem, p.mix_m_main + bx * 32, by * 32);
    }
}

// dst <- Q_acc(add + dst) for the 16 chains of a lane, with exact decisions.
// Floor: one toward-zero add (the kernel runs in that mode).  Nearest-even: the add is done twice,
// toward +inf and toward -inf; the smaller magnitude is the truncated sum and the two differ iff the
// sum was inexact (the sticky bit).  With EVENTS, one OF and one UF bit per chain are shifted into
// wof / wuf (uf1 = product-underflow flags of this step).
template <int RND, bool EVENTS, bool MODESW = false>
__device__ __forceinline__ void gen_qadd_all(float (&dst)[4][4], const float (&add)[4][4], const KParams& p,
                                             uint32_t rofb, uint32_t rufb, const uint32_t (&uf1)[4][4],
                                             uint32_t (&wof)[4][4], uint32_t (&wuf)[4][4]) {
    constexpr int TM = 4, TN = 4;
    if (RND == LBA_ROUND_FLOOR) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const float S = dst[i][j];
                float tz;                                                   // toward zero: truncated exact sum
                if (MODESW) asm volatile("v_add_f32 %0, %1, %2" : "=v"(tz) : "v"(add[i][j]), "v"(S));   // ordered after the mode write
                else tz = add[i][j] + S;
                const uint32_t uz = __float_as_uint(tz);
                const uint32_t mag = uz & 0x7FFFFFFFu;
                const bool of = mag >= rofb, small = mag < rufb;
                uint32_t r = uz & p.mask_a;
                r = of ? ((uz & 0x80000000u) | rofb) : r;
                r = small ? 0u : r;
                dst[i][j] = __uint_as_float(r);
                if (EVENTS) {
                    const bool nz = add[i][j] != -S;                        // exact sum is not zero
                    wof[i][j] = (wof[i][j] << 1) | (of ? 1u : 0u);
                    wuf[i][j] = (wuf[i][j] << 1) | ((uf1[i][j] || (small && nz)) ? 1u : 0u);
                }
            }
    } else {
        float tp[TM][TN], tn[TM][TN], tr[TM][TN];
        if (p.sh_a == 0) {
            // M = 23: the 24-bit nearest-even sum is the mantissa rounding itself; the two
            // directed sums below still give the exact over/underflow decisions
            set_round_nearest();
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    asm volatile("v_add_f32 %0, %1, %2" : "=v"(tr[i][j]) : "v"(add[i][j]), "v"(dst[i][j]));
        }
        set_round_pinf();
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                asm volatile("v_add_f32 %0, %1, %2" : "=v"(tp[i][j]) : "v"(add[i][j]), "v"(dst[i][j]));
        set_round_ninf();
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                asm volatile("v_add_f32 %0, %1, %2" : "=v"(tn[i][j]) : "v"(add[i][j]), "v"(dst[i][j]));
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const float S = dst[i][j];
                const uint32_t up = __float_as_uint(tp[i][j]), un = __float_as_uint(tn[i][j]);
                const uint32_t sticky = (up ^ un) & 1u;                     // the two differ iff inexact
                const uint32_t uz = up < un ? up : un;                      // smaller magnitude (same sign)
                uint32_t of; bool small;
                float r = gen_acc_rne(uz, sticky, p, &of, &small);
                if (p.sh_a == 0) {
                    const uint32_t sign = uz & 0x80000000u;
                    uint32_t w = __float_as_uint(tr[i][j]);
                    w = of ? (sign | rofb) : w;
                    w = small ? 0u : w;
                    r = __uint_as_float(w);
                }
                dst[i][j] = r;
                if (EVENTS) {
                    const bool nz = add[i][j] != -S;
                    wof[i][j] = (wof[i][j] << 1) | of;
                    wuf[i][j] = (wuf[i][j] << 1) | ((uf1[i][j] || (small && nz)) ? 1u : 0u);
                }
            }
    }
}

// DIFF bits of one step for the 16 chains of a lane (Sec. 4 "Immediate / DIFF", App. D with eps1 -> 0+):
// wdf <- 2 * wdf + [ |S_new - S_old| <= eps2 * |x w| ].  The right-hand side is exact in FP32 (a product of
// two operands has at most 12 significant bits and eps2 at most 12); the difference is formed as
// max - min >= 0 rounded toward +inf, which exceeds a representable number iff the exact difference does.
// Both are FP32 normals or 0: sums of E4M3 products are multiples of 2^-18.  Leaves the rounding mode at
// +inf (FLOOR: back at toward-zero).
template <int RND>
__device__ __forceinline__ void gen_diff_all(const float (&s_old)[4][4], const float (&s_new)[4][4],
                                             const float (&a)[4], const float (&b)[4], float eps2,
                                             uint32_t (&wdf)[4][4]) {
    set_round_pinf();
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float hi = __builtin_fmaxf(s_old[i][j], s_new[i][j]);
            const float lo = __builtin_fminf(s_old[i][j], s_new[i][j]);
            float d;
            asm volatile("v_sub_f32 %0, %1, %2" : "=v"(d) : "v"(hi), "v"(lo));
            const float rhs = __builtin_fabsf(a[i] * b[j]) * eps2;
            wdf[i][j] = (wdf[i][j] << 1) | (d > rhs ? 0u : 1u);
        }
    if (RND == LBA_ROUND_FLOOR) set_round_zero();
}

// General kernel: 4 x 4 outputs per lane, 64 x 64 tile, BK = 32 (one event word per tile).
// DIFF (with EVENTS = false): writes the DIFF plane of the first-level steps through p.of_mask.
template <int RND, bool EVENTS, int ORDER, bool DIFF = false>
__global__ void __launch_bounds__(256) lba_gen_kernel(const KParams p) {
    constexpr int TM = 4, TN = 4, BK = 32, BM = 64, BN = 64;
    constexpr int STAGE = BK * (BM + BN);
    __shared__ __attribute__((aligned(16))) float smem[2 * STAGE];
    __shared__ float lut_a[256];
    __shared__ float lut_b[256];

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
    // batch member blockIdx.z (strides are 0 for a single GEMM)
    const uint8_t* pA = p.A + (int64_t)blockIdx.z * p.stride_a;
    const uint8_t* pB = p.B + (int64_t)blockIdx.z * p.stride_b;
    float* pC = p.C ? p.C + (int64_t)blockIdx.z * p.stride_c : nullptr;

    lut_a[tid] = decode_entry(tid, p.exp_a, p.in_ea, p.in_ma);
    lut_b[tid] = decode_entry(tid, p.exp_b, p.in_eb, p.in_mb);
    set_flush_f32();
    if (RND == LBA_ROUND_FLOOR) set_round_zero();

    float acc[TM][TN], top[TM][TN];                            // top: second-level sums (chunked order only)
    uint32_t wof[TM][TN], wuf[TM][TN], wof2[TM][TN], wuf2[TM][TN], no_uf1[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            acc[i][j] = 0.0f; top[i][j] = 0.0f; wof[i][j] = 0u; wuf[i][j] = 0u;
            wof2[i][j] = 0u; wuf2[i][j] = 0u; no_uf1[i][j] = 0u;
        }

    uint4 ra[Stage<BM, BK>::kPerLane], rb[Stage<BN, BK>::kPerLane];
    const int ntiles = (p.K + BK - 1) / BK;
    const uint32_t rofb = __float_as_uint(p.rof_a), rufb = __float_as_uint(p.ruf_a);

    fetch_tile_a<BM, BK>(pA, p, m0, 0, tid, ra);
    fetch_tile<BN, BK>(pB, p.N, p.K, n0, 0, p.ld_align, tid, rb);
    __syncthreads();
    store_tile<BM, BK>(smem, lut_a, tid, ra);
    store_tile<BN, BK>(smem + BK * BM, lut_b, tid, rb);
    __syncthreads();

    for (int t = 0; t < ntiles; ++t) {
        const float* As = smem + (t & 1) * STAGE;
        const float* Bs = As + BK * BM;
        const bool more = (t + 1) < ntiles;
        if (more) {
            fetch_tile_a<BM, BK>(pA, p, m0, (t + 1) * BK, tid, ra);
            fetch_tile<BN, BK>(pB, p.N, p.K, n0, (t + 1) * BK, p.ld_align, tid, rb);
        }
#pragma unroll 2
        for (int k = 0; k < BK; ++k) {
            const float4 av = *reinterpret_cast<const float4*>(As + k * BM + ty * 4);
            const float4 bv = *reinterpret_cast<const float4*>(Bs + k * BN + tx * 4);
            const float a[4] = {av.x, av.y, av.z, av.w};
            const float b[4] = {bv.x, bv.y, bv.z, bv.w};
            float pq[TM][TN];
            uint32_t uf1[TM][TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) pq[i][j] = gen_product<RND>(a[i], b[j], p, &uf1[i][j]);

            float s_old[TM][TN];
            if (DIFF) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) s_old[i][j] = acc[i][j];
            }
            gen_qadd_all<RND, EVENTS, DIFF>(acc, pq, p, rofb, rufb, uf1, wof, wuf);
            if (DIFF) gen_diff_all<RND>(s_old, acc, a, b, p.diff_eps, wof);
            if (ORDER == LBA_ORDER_CHUNK16 && (k & 15) == 15) {
                // second level (Sec. 3, Fig. 1 right): T <- Q_acc(T + S), S <- 0
                gen_qadd_all<RND, EVENTS, DIFF>(top, acc, p, rofb, rufb, no_uf1, wof2, wuf2);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) acc[i][j] = 0.0f;
            }
        }
        if (DIFF) store_event_words(p.of_mask, nullptr, t, 32, p.K - t * BK, wof, wuf, m0, n0, tx, ty, p);
        if (EVENTS) {
            store_event_words(p.of_mask, p.uf_mask, t, 32, p.K - t * BK, wof, wuf, m0, n0, tx, ty, p);
            if (ORDER == LBA_ORDER_CHUNK16 && ((t & 15) == 15 || !more)) {
                const int chunks = (p.K + 15) >> 4;
                store_event_words(p.of_mask2, p.uf_mask2, t >> 4, 2 * ((t & 15) + 1), chunks - 32 * (t >> 4),
                                  wof2, wuf2, m0, n0, tx, ty, p);
            }
        }
        if (more) {
            float* Ad = smem + ((t + 1) & 1) * STAGE;
            store_tile<BM, BK>(Ad, lut_a, tid, ra);
            store_tile<BN, BK>(Ad + BK * BM, lut_b, tid, rb);
        }
        __syncthreads();
    }
    set_round_nearest();

    if (pC) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int m = m0 + ty * 4 + i;
            if (m >= p.M) continue;
            const int n = n0 + tx * 4;
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float r = (ORDER == LBA_ORDER_CHUNK16) ? top[i][j] : acc[i][j];
                v[j] = (r == 0.0f) ? 0.0f : __builtin_ldexpf(r, p.out_exp);     // out_exp: the operand biases' scale
            }
            float* dst = pC + (int64_t)m * p.N + n;
            if (p.c_vec && n + 3 < p.N) {
                *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (n + j < p.N) dst[j] = v[j];
            }
        }
    }
}

}  // namespace lba
#endif
