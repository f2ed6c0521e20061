// lba_grad.hip -- the gradient side of the LBA product for gfx950: the last-overflow post-pass and
// the coefficient-masked gradient products of the fine-grained straight-through estimators
// (Sec. 4 and App. D of the paper).
//
//   dX[m, k] = sum_n g[m, n] * value(B[n, k]) * c[m, n, k]
//   dW[n, k] = sum_m g[m, n] * value(A[m, k]) * c[m, n, k]
//
// with c in {0, 1}: 1 (identity), 1 - OF_k (immediate / OF) or [k > last overflow of (m, n)]
// (recursive / OF under the sequential order).  Both products are the same kernel:
//
//   out[r, k] = sum_s g(r, s) * value(V[s, k]) * c(r, s, k)        dX: r = m, s = n, V = B
//                                                                  dW: r = n, s = m, V = A
//
// Mapping.  The 64 lanes of a wave are 64 consecutive k; a wave owns 16 rows r (16 accumulators per
// lane) and walks over s.  For one (r, s) everything but V is uniform across the wave: g(r, s) is one
// scalar, and the 64 coefficient bits of k0 .. k0+63 are exactly two words of the plane, i.e. a
// 64-bit lane mask.  They are fetched with scalar loads and the multiply-add runs with that mask as
// the wave's execution mask: one VALU instruction per 64 coefficient-masked MACs, no per-lane bit
// extraction.  The recursive estimator compares the lane's k with the scalar last-overflow index.
// Reductions over s never cross lanes.  When the launch would have too few waves, s is split over
// grid z and the partial sums are combined with floating-point atomic adds (the output is zeroed
// first): the summation order is then not fixed, results agree to FP32 rounding.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "lba.h"
#include "lba_internal.h"
#include "lba_launch.h"

namespace lba {

// lba_grad_mfma.hip: the identity estimator as a dense contraction on the matrix cores
bool grad_dense_ok(const float* G, const uint8_t* V, const int32_t* last_of, int64_t M, int64_t N, int64_t K);
int run_grad_dense(bool dx, const float* G, const uint8_t* V, const int32_t* last_of, float* out,
                   int64_t M, int64_t N, int64_t K, hipStream_t st, const uint8_t* bricks = nullptr,
                   float* partials = nullptr, size_t partial_bytes = 0);
size_t grad_dense_partial_bytes(int64_t M, int64_t N, int64_t K);

// Sizes of one launch; the pointers are separate kernel arguments so that they can be declared
// non-aliasing, which is what lets the compiler fetch the wave-uniform values with scalar loads.
struct GradDims {
    int32_t R, S, K;
    int32_t stride_r, stride_s;   // element (r, s) of G / last_of / one plane word-slab: r*stride_r + s*stride_s
    int64_t slab;              // M*N: distance between consecutive 32-k word slabs of the plane
    int32_t s_chunk;           // s values per grid z
    int32_t atomic;            // 1: gridDim.z > 1, combine with atomic adds
    int32_t vec_ok;            // 1: G, the plane and last_of are 16-byte aligned and N % 4 == 0 (wide scalar loads)
    uint32_t plane_xor;        // 0xFFFFFFFF: the plane holds OF bits (c = 1 - bit); 0: it holds the coefficients
    int32_t v16;               // 1: rows of codes are 16-byte aligned (V % 16 == 0, K % 16 == 0)
    // brick map (immediate estimator with a workspace): byte ((k / 256) * brick_rb + r / 128) * brick_sb + s / 32 is
    // non-zero where some coefficient of that brick is 0; this kernel then takes those bricks only (the matrix-core
    // kernel adds the others).  NULL: every brick.
    const uint8_t* bricks;
    int32_t brick_rb, brick_sb;
};

__device__ __forceinline__ float decode_e4m3(uint32_t code) {
    float v = __builtin_amdgcn_cvt_f32_fp8((int)code, 0);
    if ((code & 0x7Fu) == 0x7Fu) v = (code & 0x80u) ? -480.0f : 480.0f;   // the two NaN codes
    return v;
}

// acc += g[u] * v[u] on the lanes whose coefficient bit is set, u = 0..3: the two plane words
// (k0..k0+31 and k0+32..k0+63), xor-ed with `flip` (all ones for an OF plane, whose complement is the
// coefficient), are written straight into the execution mask.  The mask is saved and restored inside
// the statement, so the surrounding code never sees it changed.
__device__ __forceinline__ void masked_fmac4(float& acc, const uint32_t (&lo)[4], const uint32_t (&hi)[4],
                                             const float (&g)[4], const float (&v)[4], uint32_t flip) {
    uint64_t save;
    asm volatile(
        "s_mov_b64 %[sv], exec\n\t"
        "s_xor_b32 exec_lo, %[l0], %[f]\n\ts_xor_b32 exec_hi, %[h0], %[f]\n\tv_fmac_f32 %[a], %[g0], %[v0]\n\t"
        "s_xor_b32 exec_lo, %[l1], %[f]\n\ts_xor_b32 exec_hi, %[h1], %[f]\n\tv_fmac_f32 %[a], %[g1], %[v1]\n\t"
        "s_xor_b32 exec_lo, %[l2], %[f]\n\ts_xor_b32 exec_hi, %[h2], %[f]\n\tv_fmac_f32 %[a], %[g2], %[v2]\n\t"
        "s_xor_b32 exec_lo, %[l3], %[f]\n\ts_xor_b32 exec_hi, %[h3], %[f]\n\tv_fmac_f32 %[a], %[g3], %[v3]\n\t"
        "s_mov_b64 exec, %[sv]"
        : [a] "+v"(acc), [sv] "=&s"(save)
        : [l0] "s"(lo[0]), [h0] "s"(hi[0]), [g0] "s"(g[0]), [v0] "v"(v[0]),
          [l1] "s"(lo[1]), [h1] "s"(hi[1]), [g1] "s"(g[1]), [v1] "v"(v[1]),
          [l2] "s"(lo[2]), [h2] "s"(hi[2]), [g2] "s"(g[2]), [v2] "v"(v[2]),
          [l3] "s"(lo[3]), [h3] "s"(hi[3]), [g3] "s"(g[3]), [v3] "v"(v[3]), [f] "s"(flip)
        : "scc");
}

// acc += g[u] * v[u] on the lanes whose k exceeds last[u] (recursive estimator).  The four compares run
// under the full mask first; each result is a lane mask in a scalar register pair.
__device__ __forceinline__ void recursive_fmac4(float& acc, int k, const int32_t (&last)[4],
                                                const float (&g)[4], const float (&v)[4]) {
    uint64_t save, m0, m1, m2, m3;
    asm volatile(
        "v_cmp_gt_i32_e64 %[m0], %[k], %[t0]\n\t"
        "v_cmp_gt_i32_e64 %[m1], %[k], %[t1]\n\t"
        "v_cmp_gt_i32_e64 %[m2], %[k], %[t2]\n\t"
        "v_cmp_gt_i32_e64 %[m3], %[k], %[t3]\n\t"
        "s_mov_b64 %[sv], exec\n\t"
        "s_mov_b64 exec, %[m0]\n\tv_fmac_f32 %[a], %[g0], %[v0]\n\t"
        "s_mov_b64 exec, %[m1]\n\tv_fmac_f32 %[a], %[g1], %[v1]\n\t"
        "s_mov_b64 exec, %[m2]\n\tv_fmac_f32 %[a], %[g2], %[v2]\n\t"
        "s_mov_b64 exec, %[m3]\n\tv_fmac_f32 %[a], %[g3], %[v3]\n\t"
        "s_mov_b64 exec, %[sv]"
        : [a] "+v"(acc), [sv] "=&s"(save), [m0] "=&s"(m0), [m1] "=&s"(m1), [m2] "=&s"(m2), [m3] "=&s"(m3)
        : [k] "v"(k), [t0] "s"(last[0]), [t1] "s"(last[1]), [t2] "s"(last[2]), [t3] "s"(last[3]),
          [g0] "s"(g[0]), [g1] "s"(g[1]), [g2] "s"(g[2]), [g3] "s"(g[3]),
          [v0] "v"(v[0]), [v1] "v"(v[1]), [v2] "v"(v[2]), [v3] "v"(v[3]));
}

// The 4 x 4 block (rows ib..ib+3 of the wave, s..s+3) of scalars and the masked multiply-adds on it.
// FAST: all 16 elements exist and the four 16-byte groups along the contiguous index are aligned, so
// each is one wide scalar load; otherwise indices are clamped and g is zeroed outside the range.
// S_CONTIG: element (r, s) is contiguous along s (dX) or along r (dW).  Element offsets fit 32 bits.
// Where the plane has no second word slab (the last 64 k with K % 64 <= 32) P1 aliases P0: lanes 32..63
// then hold k >= K, whose operand value is 0 and whose sums are never stored.
template <int MODE, bool S_CONTIG, bool FAST>
__device__ __forceinline__ void grad_block(float (&acc)[16], int ib, int r0, int s, int s_end, int k,
                                           const float (&v)[4], const float* __restrict__ G,
                                           const uint32_t* __restrict__ P0, const uint32_t* __restrict__ P1,
                                           const int32_t* __restrict__ L, const GradDims& d) {
    uint32_t lo[4][4], hi[4][4];
    int32_t last[4][4];
    float g[4][4];
    if (FAST) {
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const uint32_t off = S_CONTIG ? (uint32_t)(r0 + ib + a) * (uint32_t)d.stride_r + (uint32_t)s
                                          : (uint32_t)(s + a) * (uint32_t)d.stride_s + (uint32_t)(r0 + ib);
            const float4 gv = *reinterpret_cast<const float4*>(G + off);
            const float ga[4] = {gv.x, gv.y, gv.z, gv.w};
            uint32_t la[4] = {0u, 0u, 0u, 0u}, ha[4] = {0u, 0u, 0u, 0u};
            int32_t ta[4] = {0, 0, 0, 0};
            if (MODE == LBA_STE_IMMEDIATE_OF) {
                const uint4 lv = *reinterpret_cast<const uint4*>(P0 + off);
                const uint4 hv = *reinterpret_cast<const uint4*>(P1 + off);
                la[0] = lv.x; la[1] = lv.y; la[2] = lv.z; la[3] = lv.w;
                ha[0] = hv.x; ha[1] = hv.y; ha[2] = hv.z; ha[3] = hv.w;
            }
            if (MODE == LBA_STE_RECURSIVE_OF) {
                const int4 tv = *reinterpret_cast<const int4*>(L + off);
                ta[0] = tv.x; ta[1] = tv.y; ta[2] = tv.z; ta[3] = tv.w;
            }
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int i = S_CONTIG ? a : b, u = S_CONTIG ? b : a;
                g[i][u] = ga[b]; lo[i][u] = la[b]; hi[i][u] = ha[b]; last[i][u] = ta[b];
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const bool in = (r0 + ib + i < d.R) && (s + u < s_end);
                const uint32_t off = (uint32_t)min(r0 + ib + i, d.R - 1) * (uint32_t)d.stride_r
                                   + (uint32_t)min(s + u, d.S - 1) * (uint32_t)d.stride_s;
                const float gl = G[off];
                g[i][u] = in ? gl : 0.0f;
                lo[i][u] = hi[i][u] = 0u;
                last[i][u] = 0;
                if (MODE == LBA_STE_IMMEDIATE_OF) { lo[i][u] = P0[off]; hi[i][u] = P1[off]; }
                if (MODE == LBA_STE_RECURSIVE_OF) last[i][u] = L[off];
            }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (MODE == LBA_STE_IDENTITY) {
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[ib + i] = __builtin_fmaf(g[i][u], v[u], acc[ib + i]);
        } else if (MODE == LBA_STE_IMMEDIATE_OF) {
            masked_fmac4(acc[ib + i], lo[i], hi[i], g[i], v, d.plane_xor);
        } else {
            recursive_fmac4(acc[ib + i], k, last[i], g[i], v);
        }
    }
}

// Immediate estimator, plane words delivered through vector registers: w0..w3 hold (already complemented)
// plane words, one per lane; the word pair of fmac u sits in lanes L<u> (k0..k0+31) and L<u> + 32
// (k0+32..k0+63) of register w<u>.  v_readlane moves it to scalar registers, from there into the execution
// mask.  v_readlane ignores the execution mask, so the changed mask does not disturb the next read.
template <int L0, int L1, int L2, int L3>
__device__ __forceinline__ void masked_fmac4_lanes(float& acc, uint32_t w0, uint32_t w1, uint32_t w2, uint32_t w3,
                                                   const float (&g)[4], const float (&v)[4]) {
    // the word pair is read into a fixed aligned scalar pair so that one 64-bit move loads the execution mask.
    // The kernel runs this with every lane active (whole waves only leave early), so the mask is put back to
    // all ones instead of being saved and restored.
    asm volatile(
        "v_readlane_b32 s94, %[w0], %[a0]\n\tv_readlane_b32 s95, %[w0], %[b0]\n\t"
        "s_mov_b64 exec, s[94:95]\n\tv_fmac_f32 %[a], %[g0], %[v0]\n\t"
        "v_readlane_b32 s94, %[w1], %[a1]\n\tv_readlane_b32 s95, %[w1], %[b1]\n\t"
        "s_mov_b64 exec, s[94:95]\n\tv_fmac_f32 %[a], %[g1], %[v1]\n\t"
        "v_readlane_b32 s94, %[w2], %[a2]\n\tv_readlane_b32 s95, %[w2], %[b2]\n\t"
        "s_mov_b64 exec, s[94:95]\n\tv_fmac_f32 %[a], %[g2], %[v2]\n\t"
        "v_readlane_b32 s94, %[w3], %[a3]\n\tv_readlane_b32 s95, %[w3], %[b3]\n\t"
        "s_mov_b64 exec, s[94:95]\n\tv_fmac_f32 %[a], %[g3], %[v3]\n\t"
        "s_mov_b64 exec, -1"
        : [a] "+v"(acc)
        : [w0] "v"(w0), [w1] "v"(w1), [w2] "v"(w2), [w3] "v"(w3),
          [a0] "n"(L0), [b0] "n"(L0 + 32), [a1] "n"(L1), [b1] "n"(L1 + 32),
          [a2] "n"(L2), [b2] "n"(L2 + 32), [a3] "n"(L3), [b3] "n"(L3 + 32),
          [g0] "v"(g[0]), [g1] "v"(g[1]), [g2] "v"(g[2]), [g3] "v"(g[3]),
          [v0] "v"(v[0]), [v1] "v"(v[1]), [v2] "v"(v[2]), [v3] "v"(v[3])
        : "s94", "s95");
}

// One accumulator row I (0..15) against the four s of group UB (0..3) of a 16-s super-step.
// Word (i, u) of slab h lives in lane h*32 + a*2 + (b >> 3), register w[b & 7], with (a, b) = (i, u)
// when the plane is contiguous along s and (u, i) when it is contiguous along r.
template <bool S_CONTIG, int I, int UB>
__device__ __forceinline__ void lanes_row(float& acc, const uint32_t (&w)[8], const float (&g)[4], const float (&v)[4]) {
    constexpr int U0 = 4 * UB;
    if (S_CONTIG) {
        constexpr int L = I * 2 + (U0 >> 3);                 // the four u share a lane, registers (U0 & 7) ..
        masked_fmac4_lanes<L, L, L, L>(acc, w[(U0 & 7) + 0], w[(U0 & 7) + 1], w[(U0 & 7) + 2], w[(U0 & 7) + 3], g, v);
    } else {
        constexpr int R = I & 7, H = I >> 3;                 // one register, lanes of the four u
        masked_fmac4_lanes<(U0 + 0) * 2 + H, (U0 + 1) * 2 + H, (U0 + 2) * 2 + H, (U0 + 3) * 2 + H>(acc, w[R], w[R], w[R], w[R], g, v);
    }
}

// The 16 x 16 values g of a super-step reach the multiply-adds through LDS: the wave loads the tile with one 16-byte
// vector load per lane, a whole super-step ahead, and stores it in its own 1 KB of LDS (line p = lane / 4 holds 16
// values that are contiguous in memory: a row r0 + p when g is contiguous along s, a column s + p otherwise).  Block
// (IB, UB) then reads its 4 x 4 values with four 16-byte LDS reads in which every lane reads the same address (a
// broadcast): the value sits in a vector register of every lane, whatever the execution mask does afterwards.
// (Scalar loads delivered g before: each fed one instruction and was requested one block ahead, and their latency,
// sixteen times per super-step, was what bounded the kernel.)
template <bool S_CONTIG>
__device__ __forceinline__ float4 fetch_g_tile(const float* __restrict__ G, int r0, int s, int lane, const GradDims& d) {
    const int p = lane >> 2, c4 = (lane & 3) * 4;
    const uint32_t off = S_CONTIG ? (uint32_t)(r0 + p) * (uint32_t)d.stride_r + (uint32_t)(s + c4)
                                  : (uint32_t)(s + p) * (uint32_t)d.stride_s + (uint32_t)(r0 + c4);
    return *reinterpret_cast<const float4*>(G + off);
}

// The 16 x 64 codes of a step (16 values of s, the wave's 64 k): one 16-byte load per lane (row lane / 4, bytes
// 16 * (lane % 4) ..), stored row-major in the wave's LDS; lane k then reads byte k of every row.  (One byte load per
// lane and row, sixteen per step, took a quarter of the kernel's time.)  Needs 16-byte aligned rows of codes; a piece
// that starts at or beyond K is +0.
__device__ __forceinline__ uint4 fetch_v_tile(const uint8_t* __restrict__ V, int s, int k0, int lane, const GradDims& d) {
    const int kq = k0 + (lane & 3) * 16;
    uint4 c = make_uint4(0u, 0u, 0u, 0u);
    if (kq < d.K) c = *reinterpret_cast<const uint4*>(V + (int64_t)(s + (lane >> 2)) * d.K + kq);
    return c;
}

__device__ __forceinline__ void store_v_tile(uint8_t* vtile, uint4 c, int lane) {
    *reinterpret_cast<uint4*>(vtile + (lane >> 2) * 64 + (lane & 3) * 16) = c;
}

__device__ __forceinline__ void store_g_tile(float* tile, float4 g4, int lane) {
    *reinterpret_cast<float4*>(tile + (lane >> 2) * 16 + (lane & 3) * 4) = g4;
}

template <bool S_CONTIG, int IB, int UB>
__device__ __forceinline__ void load_g_block(float (&g)[4][4], const float* tile) {
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const float4 gv = S_CONTIG ? *reinterpret_cast<const float4*>(tile + (4 * IB + a) * 16 + 4 * UB)
                                   : *reinterpret_cast<const float4*>(tile + (4 * UB + a) * 16 + 4 * IB);
        const float ga[4] = {gv.x, gv.y, gv.z, gv.w};
#pragma unroll
        for (int b = 0; b < 4; ++b) g[S_CONTIG ? a : b][S_CONTIG ? b : a] = ga[b];
    }
}

// Block B = 4 * IB + UB of the 16 blocks of a super-step: reads its 4 x 4 values g from LDS (the other waves of the
// SIMD cover that latency: reading a block ahead cost 20 registers and a wave per SIMD, and measured slower) and runs.
// Overflows are rare where the formats fit the data: a block whose 16 word pairs hold no blocked coefficient (lanes
// beyond K carry the value +0, so their bits do not matter) takes plain multiply-adds, one instruction per 64 terms
// without the lane-mask traffic, in the same order.  dirty_lo / dirty_hi: the lanes whose words in w[0..3] / w[4..7]
// are not all ones; the block's words sit in eight fixed lanes of one of the two register groups.
template <bool S_CONTIG, int B>
__device__ __forceinline__ void lanes_block(float (&acc)[16], const float (&v)[16], const float* tile,
                                            const uint32_t (&w)[8], uint64_t dirty_lo, uint64_t dirty_hi) {
    constexpr int IB = B / 4, UB = B % 4;
    // word (i, u) of slab h: lane h*32 + a*2 + (b >> 3), register w[b & 7], (a, b) = (i, u) or (u, i) (see lanes_row)
    constexpr int AB = S_CONTIG ? IB : UB, BB = S_CONTIG ? UB : IB;            // block index along a and along b
    constexpr uint64_t lanes32 = (uint64_t)0x55u << (8 * AB + (BB >> 1));     // a = 4 AB .. 4 AB + 3, lane a*2 + (BB >> 1)
    constexpr uint64_t lanes = lanes32 | (lanes32 << 32);
    float g[4][4];
    load_g_block<S_CONTIG, IB, UB>(g, tile);
    __builtin_amdgcn_sched_barrier(0);
    if ((((BB & 1) ? dirty_hi : dirty_lo) & lanes) == 0) {     // uniform
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) acc[4 * IB + a] = __builtin_fmaf(g[a][b], v[4 * UB + b], acc[4 * IB + a]);
    } else {
        const float vv[4] = {v[4 * UB + 0], v[4 * UB + 1], v[4 * UB + 2], v[4 * UB + 3]};
        lanes_row<S_CONTIG, 4 * IB + 0, UB>(acc[4 * IB + 0], w, g[0], vv);
        lanes_row<S_CONTIG, 4 * IB + 1, UB>(acc[4 * IB + 1], w, g[1], vv);
        lanes_row<S_CONTIG, 4 * IB + 2, UB>(acc[4 * IB + 2], w, g[2], vv);
        lanes_row<S_CONTIG, 4 * IB + 3, UB>(acc[4 * IB + 3], w, g[3], vv);
    }
    __builtin_amdgcn_sched_barrier(0);
}

// 16 rows x 16 s of the immediate estimator.  The 512 plane words of the step (two slabs) are fetched with
// two 16-byte vector loads per lane (many in flight: the plane is streamed once and never reused, which
// the scalar-load path cannot sustain), turned into coefficients, and handed out lane by lane.
struct PlaneWords { uint4 x, y; };

template <bool S_CONTIG>
__device__ __forceinline__ PlaneWords fetch_plane_words(int r0, int s, int lane, const uint32_t* __restrict__ P0,
                                                        const uint32_t* __restrict__ P1, const GradDims& d) {
    const int q = lane & 31, a = q >> 1, half8 = (q & 1) * 8;
    const uint32_t* __restrict__ P = (lane & 32) ? P1 : P0;
    const uint32_t off = S_CONTIG ? (uint32_t)(r0 + a) * (uint32_t)d.stride_r + (uint32_t)(s + half8)
                                  : (uint32_t)(s + a) * (uint32_t)d.stride_s + (uint32_t)(r0 + half8);
    PlaneWords p;
    p.x = *reinterpret_cast<const uint4*>(P + off);
    p.y = *reinterpret_cast<const uint4*>(P + off + 4);
    return p;
}

template <bool S_CONTIG>
__device__ __forceinline__ void immediate_superstep(float (&acc)[16], int r0, int s, int k, int lane,
                                                    const uint8_t* __restrict__ V, const float* tile, const uint8_t* vtile,
                                                    const PlaneWords& pw, const GradDims& d) {
    const uint4 x = pw.x, y = pw.y;
    const uint32_t f = d.plane_xor;                            // OF plane: c = 1 - OF
    const uint32_t w[8] = {x.x ^ f, x.y ^ f, x.z ^ f, x.w ^ f, y.x ^ f, y.y ^ f, y.z ^ f, y.w ^ f};
    float v[16];
    if (d.v16) {                                               // uniform: the codes are in the wave's LDS tile
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = decode_e4m3(vtile[u * 64 + lane]);
    } else {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const uint32_t code = (k < d.K) ? V[(int64_t)(s + u) * d.K + k] : 0u;
            v[u] = decode_e4m3(code);
        }
    }
    const uint64_t dlo = __builtin_amdgcn_ballot_w64((w[0] & w[1] & w[2] & w[3]) != 0xFFFFFFFFu);
    const uint64_t dhi = __builtin_amdgcn_ballot_w64((w[4] & w[5] & w[6] & w[7]) != 0xFFFFFFFFu);
    lanes_block<S_CONTIG, 0>(acc, v, tile, w, dlo, dhi);   lanes_block<S_CONTIG, 1>(acc, v, tile, w, dlo, dhi);
    lanes_block<S_CONTIG, 2>(acc, v, tile, w, dlo, dhi);   lanes_block<S_CONTIG, 3>(acc, v, tile, w, dlo, dhi);
    lanes_block<S_CONTIG, 4>(acc, v, tile, w, dlo, dhi);   lanes_block<S_CONTIG, 5>(acc, v, tile, w, dlo, dhi);
    lanes_block<S_CONTIG, 6>(acc, v, tile, w, dlo, dhi);   lanes_block<S_CONTIG, 7>(acc, v, tile, w, dlo, dhi);
    lanes_block<S_CONTIG, 8>(acc, v, tile, w, dlo, dhi);   lanes_block<S_CONTIG, 9>(acc, v, tile, w, dlo, dhi);
    lanes_block<S_CONTIG, 10>(acc, v, tile, w, dlo, dhi);  lanes_block<S_CONTIG, 11>(acc, v, tile, w, dlo, dhi);
    lanes_block<S_CONTIG, 12>(acc, v, tile, w, dlo, dhi);  lanes_block<S_CONTIG, 13>(acc, v, tile, w, dlo, dhi);
    lanes_block<S_CONTIG, 14>(acc, v, tile, w, dlo, dhi);  lanes_block<S_CONTIG, 15>(acc, v, tile, w, dlo, dhi);
}

template <int MODE, bool S_CONTIG>
__global__ void __launch_bounds__(256) lba_grad_kernel(const float* __restrict__ G, const uint8_t* __restrict__ V,
                                                       const uint32_t* __restrict__ plane,
                                                       const int32_t* __restrict__ last_of,
                                                       float* __restrict__ out, const GradDims d) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int k0 = blockIdx.y * 64;
    const int k = k0 + lane;
    const int r0 = (blockIdx.x * 4 + wave) * 16;
    if (r0 >= d.R) return;                                     // whole wave (uniform)
    const int s_begin = blockIdx.z * d.s_chunk;
    const int s_end = min(d.S, s_begin + d.s_chunk);
    if (MODE == LBA_STE_IMMEDIATE_OF && d.bricks) {
        // nothing marked along this wave's part of its brick row (the usual case where the formats fit the data):
        // done before anything is fetched; the matrix-core kernel's sums are already in the output
        const uint8_t* __restrict__ br = d.bricks + ((int64_t)(k0 >> 8) * d.brick_rb + (r0 >> 7)) * d.brick_sb;
        const int b_end = (s_end + 31) >> 5;
        uint32_t any = 0u;
        int b = s_begin >> 5;
        for (; b + 8 <= b_end && !any; b += 8)
            any = (uint32_t)br[b] | br[b + 1] | br[b + 2] | br[b + 3] | br[b + 4] | br[b + 5] | br[b + 6] | br[b + 7];
        for (; b < b_end && !any; ++b) any = br[b];
        if (!any) return;                                      // uniform
    }
    const bool has_hi = k0 + 32 < d.K;                         // does the plane have a second word slab here
    const uint32_t* __restrict__ P0 = plane + (int64_t)(k0 >> 5) * d.slab;    // not dereferenced unless MODE needs it
    const uint32_t* __restrict__ P1 = has_hi ? P0 + d.slab : P0;
    const bool rows_fast = d.vec_ok && r0 + 16 <= d.R;

    float acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.0f;

    int s = s_begin;
    if (MODE == LBA_STE_IMMEDIATE_OF && rows_fast && s + 16 <= s_end) {
        __shared__ __attribute__((aligned(16))) float gtiles[4][256];      // one 16 x 16 tile of g per wave
        __shared__ __attribute__((aligned(16))) uint8_t vtiles[4][1024];    // and one 16 x 64 tile of codes
        float* tile = gtiles[wave];
        uint8_t* vtile = vtiles[wave];
        const uint8_t* __restrict__ brick_row = d.bricks ? d.bricks + ((int64_t)(k0 >> 8) * d.brick_rb + (r0 >> 7)) * d.brick_sb : nullptr;
        auto dirty = [&](int ss) { return !brick_row || brick_row[ss >> 5] != 0; };   // uniform
        // fast-forward over clean bricks, eight (256 values of s) per round of loads (s is a multiple of 32 here:
        // the slices of s start on brick boundaries)
        auto skip_clean = [&](int ss) {
            if (brick_row && (ss & 31) == 0) {
                while (ss + 256 <= s_end) {
                    const uint8_t* b8 = brick_row + (ss >> 5);
                    if ((uint32_t)b8[0] | b8[1] | b8[2] | b8[3] | b8[4] | b8[5] | b8[6] | b8[7]) break;
                    ss += 256;
                }
            }
            return ss;
        };
        int g4_for = s;                                                    // the step g4 was fetched for
        float4 g4 = fetch_g_tile<S_CONTIG>(G, r0, s, lane, d);
        auto step = [&](int ss, const PlaneWords& pw) {
            if (g4_for != ss) g4 = fetch_g_tile<S_CONTIG>(G, r0, ss, lane, d);   // the step before was skipped (clean brick)
            // LDS operations of a wave complete in order: the tiles are overwritten after the last reads of the step
            // before, and read after they are written; the wave barriers keep the compiler from moving them.
            // g was requested a whole step ahead; the codes (L2-resident, re-read by every row block) are requested
            // here, which keeps their four registers free during the step
            uint4 c4 = make_uint4(0u, 0u, 0u, 0u);
            if (d.v16) c4 = fetch_v_tile(V, ss, k0, lane, d);
            __builtin_amdgcn_wave_barrier();
            store_g_tile(tile, g4, lane);
            if (d.v16) store_v_tile(vtile, c4, lane);
            __builtin_amdgcn_wave_barrier();
            if (ss + 32 <= s_end) { g4 = fetch_g_tile<S_CONTIG>(G, r0, ss + 16, lane, d); g4_for = ss + 16; }
            immediate_superstep<S_CONTIG>(acc, r0, ss, k, lane, V, tile, vtile, pw, d);
        };
        if (S_CONTIG) {
            // two steps share the 128-byte lines of the plane's rows: both halves are requested together (a step
            // later the line has often left L2 again: the plane streams through it once)
            for (; s + 32 <= s_end; s += 32) {
                s = skip_clean(s);
                if (s + 32 > s_end) break;
                if (!dirty(s) && !dirty(s + 16)) continue;
                const PlaneWords pa = fetch_plane_words<S_CONTIG>(r0, s, lane, P0, P1, d);
                const PlaneWords pb = fetch_plane_words<S_CONTIG>(r0, s + 16, lane, P0, P1, d);
                if (dirty(s)) step(s, pa);
                if (dirty(s + 16)) step(s + 16, pb);
            }
        }
        for (; s + 16 <= s_end; s += 16) {
            s = skip_clean(s);
            if (s + 16 > s_end) break;
            if (dirty(s)) step(s, fetch_plane_words<S_CONTIG>(r0, s, lane, P0, P1, d));
        }
    }
    for (; s < s_end; s += 4) {
        if (MODE == LBA_STE_IMMEDIATE_OF && d.bricks &&
            d.bricks[((int64_t)(k0 >> 8) * d.brick_rb + (r0 >> 7)) * d.brick_sb + (s >> 5)] == 0) continue;   // uniform: a clean brick
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int su = min(s + u, d.S - 1);
            const uint32_t code = (k < d.K) ? V[(int64_t)su * d.K + k] : 0u;
            v[u] = decode_e4m3(code);
        }
        if (rows_fast && s + 4 <= s_end) {                     // uniform
#pragma unroll
            for (int ib = 0; ib < 16; ib += 4)
                grad_block<MODE, S_CONTIG, true>(acc, ib, r0, s, s_end, k, v, G, P0, P1, last_of, d);
        } else {
#pragma unroll
            for (int ib = 0; ib < 16; ib += 4)
                grad_block<MODE, S_CONTIG, false>(acc, ib, r0, s, s_end, k, v, G, P0, P1, last_of, d);
        }
    }

    if (k < d.K) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (r0 + i < d.R) {
                float* dst = out + (int64_t)(r0 + i) * d.K + k;
                // (with a brick map the output already holds the matrix-core kernel's part: zeros are not added)
                if (d.atomic) { if (!d.bricks || acc[i] != 0.0f) unsafeAtomicAdd(dst, acc[i]); }
                else          *dst = acc[i];
            }
        }
    }
}

// Brick maps of the immediate estimator from a plane, one pass: a brick is 128 rows x 32 s x 256 k of a product
// (dX: rows m, s = n; dW: rows n, s = m); its byte becomes non-zero if some coefficient in it is 0 (flip = all ones: the
// plane holds OF bits, a set bit blocks; flip = 0: it holds coefficients, a clear bit among the K valid ones blocks).
// The maps are zeroed beforehand.  One workgroup per group of rows of the [words * M][N] matrix of plane words.
struct BrickDims {
    int64_t quads;             // words * M * N / 4: 16-byte groups of plane words (N % 4 == 0: a group lies in one row)
    int32_t M, N, K, qpr;      // qpr = N / 4
    int32_t rbx, sbx, rbw, sbw;
    uint32_t flip;
};

constexpr int kBrickQuadsPerWg = 4096;                         // 64 KB of the plane per workgroup

__global__ void __launch_bounds__(256) lba_brick_map_kernel(const uint32_t* __restrict__ plane, uint8_t* __restrict__ map_dx,
                                                            uint8_t* __restrict__ map_dw, const BrickDims d) {
    const int words = (d.K + 31) >> 5;
    // the workgroup's first group: row (w, m) of the [words * M][N] matrix and position in it, computed once
    const int64_t q0 = (int64_t)blockIdx.x * kBrickQuadsPerWg;
    const int64_t row0 = q0 / d.qpr;
    const int rem0 = (int)(q0 - row0 * d.qpr);
    const int w0 = (int)(row0 / d.M);
    const int m0 = (int)(row0 - (int64_t)w0 * d.M);
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4* __restrict__ src = reinterpret_cast<const u32x4*>(plane) + q0;
    constexpr int BATCH = 8;                                   // loads in flight per lane: the pass is bound by memory
    for (int i0 = 0; i0 < kBrickQuadsPerWg / 256; i0 += BATCH) {
        u32x4 xs[BATCH];
#pragma unroll
        for (int j = 0; j < BATCH; ++j) {
            const int l = (i0 + j) * 256 + (int)threadIdx.x;
            xs[j] = (q0 + l < d.quads) ? __builtin_nontemporal_load(src + l) : u32x4{d.flip, d.flip, d.flip, d.flip};
        }
#pragma unroll
        for (int j = 0; j < BATCH; ++j) {
            const u32x4 x = xs[j];
            const uint32_t raw = (x.x ^ d.flip) | (x.y ^ d.flip) | (x.z ^ d.flip) | (x.w ^ d.flip);
            if (raw == 0u) continue;                           // the usual case: nothing blocked in these 128 steps
            const int l = (i0 + j) * 256 + (int)threadIdx.x;
            const int t = rem0 + l;
            const int dr = t / d.qpr;
            const int n = (t - dr * d.qpr) * 4;
            int w = w0, m = m0 + dr;
            while (m >= d.M) { m -= d.M; ++w; }
            const int valid = d.K - 32 * w;
            const uint32_t vmask = (w == words - 1 && valid < 32) ? ((1u << valid) - 1u) : 0xFFFFFFFFu;
            if (raw & vmask) {                                 // the four words share every brick index (n / 32, n / 128)
                uint8_t* bx = map_dx + ((int64_t)(w >> 3) * d.rbx + (m >> 7)) * d.sbx + (n >> 5);
                uint8_t* bw = map_dw + ((int64_t)(w >> 3) * d.rbw + (n >> 7)) * d.sbw + (m >> 5);
                if (!*bx) *bx = 1;                             // racing stores write the same value
                if (!*bw) *bw = 1;
            }
        }
    }
}

__global__ void lba_grad_fill_words_kernel(uint32_t* x, int64_t n, uint32_t v) {
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += step) x[i] = v;
}

// x[0..n) = 0 with a grid-stride loop (the launch caps the grid: a grid dimension holds fewer than 2^32 lanes)
__global__ void lba_grad_zero_kernel(float* x, int64_t n) {
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += step) x[i] = 0.0f;
}

static inline dim3 zero_grid(int64_t n) {
    const int64_t blocks = (n + 255) / 256;
    return dim3((unsigned)(blocks < (1 << 20) ? blocks : (1 << 20)));
}

// last_of[m, n] = highest k whose bit is set in the plane, -1 if none: one lane per output, walking
// the word slabs from the top; consecutive lanes read consecutive words.
__global__ void __launch_bounds__(256) lba_last_overflow_kernel(const uint32_t* __restrict__ plane, int32_t* __restrict__ last_of,
                                                                int64_t MN, int32_t words) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= MN) return;
    int32_t last = -1;
    for (int w = words - 1; w >= 0; --w) {
        const uint32_t x = plane[(int64_t)w * MN + i];
        if (x) { last = w * 32 + 31 - __builtin_clz(x); break; }
    }
    last_of[i] = last;
}

// Bits of a 32-bit (or, with `width` = 16, 16-bit) event field strictly above its highest set bit; all of
// them when no bit is set: the steps after the last overflow of the field.
__device__ __forceinline__ uint32_t above_last(uint32_t x, uint32_t field) {
    if (x == 0u) return field;
    const int msb = 31 - __builtin_clz(x);
    return msb == 31 ? 0u : (field & ~((2u << msb) - 1u));
}

// Coefficient plane (bit = 1: the gradient of that step passes) from the event planes; one lane per output,
// walking the word slabs from the top with the "no overflow further along the path" state.
//   immediate: c_k = 1 - OF_k.
//   recursive, sequential order: c_k = no OF at any step >= k.
//   recursive, chunked order: c_k = no OF at the steps >= k of k's chunk and no OF2 at the chunks >= k / 16.
template <int STE, int ORDER>
__global__ void __launch_bounds__(256) lba_ste_plane_kernel(const uint32_t* of1, const uint32_t* of2, uint32_t* coef,
                                                            int64_t MN, int32_t K) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= MN) return;
    const int words = (K + 31) >> 5;
    bool alive = true;                                         // sequential: no OF above; chunked: no OF2 above
    uint32_t x2 = 0u;
    for (int w = words - 1; w >= 0; --w) {
        const int valid = K - 32 * w;
        const uint32_t vmask = valid >= 32 ? 0xFFFFFFFFu : ((1u << valid) - 1u);
        const uint32_t x = of1[(int64_t)w * MN + i];
        uint32_t c;
        if (STE == LBA_STE_IMMEDIATE_OF) {
            c = ~x;
        } else if (ORDER == LBA_ORDER_SEQ) {
            c = alive ? above_last(x, 0xFFFFFFFFu) : 0u;
            alive = alive && x == 0u;
        } else {
            // chunks 2w (bits 0..15) and 2w+1 (bits 16..31); their second-level bits sit in word w / 16 of of2
            if ((w & 15) == 15 || w == words - 1) x2 = of2[(int64_t)(w >> 4) * MN + i];
            const uint32_t b = (x2 >> (2 * (w & 15))) & 3u;
            alive = alive && !(b & 2u);
            const uint32_t hi = alive ? above_last(x >> 16, 0xFFFFu) : 0u;
            alive = alive && !(b & 1u);
            const uint32_t lo = alive ? above_last(x & 0xFFFFu, 0xFFFFu) : 0u;
            c = (hi << 16) | lo;
        }
        coef[(int64_t)w * MN + i] = c & vmask;
    }
}

template <bool S_CONTIG>
static hipError_t launch_grad(int ste, const float* G, const uint8_t* V, const uint32_t* plane, const int32_t* last_of,
                              float* out, const GradDims& gp, dim3 grid, hipStream_t st) {
#define LBA_GRAD_LAUNCH(MODE) hipLaunchKernelGGL((lba_grad_kernel<MODE, S_CONTIG>), grid, dim3(256), 0, st, G, V, plane, last_of, out, gp)
    switch (ste) {
        case LBA_STE_IDENTITY:     LBA_GRAD_LAUNCH(LBA_STE_IDENTITY); break;
        case LBA_STE_IMMEDIATE_OF: LBA_GRAD_LAUNCH(LBA_STE_IMMEDIATE_OF); break;
        default:                   LBA_GRAD_LAUNCH(LBA_STE_RECURSIVE_OF); break;
    }
#undef LBA_GRAD_LAUNCH
    return hipGetLastError();
}

// One of the two products.  Splits s over grid z when the (r, k) grid alone would leave the chip idle.
// bricks: this side's brick map (immediate estimator / coefficient plane with a workspace), or NULL
// partials / partial_bytes: scratch memory in which the matrix-core path keeps the slices of a split sum, or NULL / 0
static int run_grad_side(bool dx, const float* G, const uint8_t* V, const uint32_t* plane, const int32_t* last_of,
                         float* out, int64_t M, int64_t N, int64_t K, int ste, hipStream_t st, const uint8_t* bricks = nullptr,
                         float* partials = nullptr, size_t partial_bytes = 0) {
    // coefficients that are constant inside a k tile: the matrix-core path (identity; recursive, with a sliver pass)
    if (ste == LBA_STE_IDENTITY && grad_dense_ok(G, V, nullptr, M, N, K))
        return run_grad_dense(dx, G, V, nullptr, out, M, N, K, st, nullptr, partials, partial_bytes);
    if (ste == LBA_STE_RECURSIVE_OF && grad_dense_ok(G, V, last_of, M, N, K))
        return run_grad_dense(dx, G, V, last_of, out, M, N, K, st, nullptr, partials, partial_bytes);
    if (bricks) {
        // the bricks whose coefficients are all 1 on the matrix cores (the output is overwritten, or zeroed and
        // added to); the vector kernel below then adds the other bricks
        const int rc = run_grad_dense(dx, G, V, nullptr, out, M, N, K, st, bricks, partials, partial_bytes);
        if (rc != LBA_OK) return rc;
    }
    GradDims gp;
    gp.bricks = bricks;
    gp.brick_rb = (int32_t)(((dx ? M : N) + 127) / 128);
    gp.brick_sb = (int32_t)(((dx ? N : M) + 31) / 32);
    gp.plane_xor = (ste == LBA_STE_COEF_PLANE) ? 0u : 0xFFFFFFFFu;
    if (ste == LBA_STE_COEF_PLANE) ste = LBA_STE_IMMEDIATE_OF;   // same kernel, bits taken as they are
    gp.K = (int32_t)K;
    gp.slab = M * N;
    if (dx) { gp.R = (int32_t)M; gp.S = (int32_t)N; gp.stride_r = (int32_t)N; gp.stride_s = 1; }
    else    { gp.R = (int32_t)N; gp.S = (int32_t)M; gp.stride_r = 1; gp.stride_s = (int32_t)N; }
    const int64_t gx = (gp.R + 63) / 64, gy = (K + 63) / 64;      // row blocks on x (no 65535 limit there)
    int split = 1;
    plan_grad_split(gx * gy, gp.S, &split, &gp.s_chunk);
    if (bricks) {                                              // slices of s on brick boundaries
        gp.s_chunk = (gp.s_chunk + 31) / 32 * 32;
        split = (int)((gp.S + gp.s_chunk - 1) / gp.s_chunk);
    }
    gp.atomic = (split > 1 || bricks) ? 1 : 0;
    const uintptr_t al = (uintptr_t)G | (uintptr_t)plane | (uintptr_t)last_of;
    gp.vec_ok = ((al % 16) == 0 && (N % 4) == 0) ? 1 : 0;
    gp.v16 = (((uintptr_t)V % 16) == 0 && (K % 16) == 0) ? 1 : 0;
    if (gp.atomic && !bricks) {
        const int64_t n = (int64_t)gp.R * K;
        hipLaunchKernelGGL(lba_grad_zero_kernel, zero_grid(n), dim3(256), 0, st, out, n);
        if (hipGetLastError() != hipSuccess) return LBA_ERR_LAUNCH;
    }
    const dim3 grid((unsigned)gx, (unsigned)gy, (unsigned)split);
    const hipError_t e = dx ? launch_grad<true>(ste, G, V, plane, last_of, out, gp, grid, st)
                            : launch_grad<false>(ste, G, V, plane, last_of, out, gp, grid, st);
    return e == hipSuccess ? LBA_OK : LBA_ERR_LAUNCH;
}

// bytes of the two brick maps (dX side first), each padded to a multiple of 256
void brick_bytes(int64_t M, int64_t N, int64_t K, size_t* dx_bytes, size_t* dw_bytes) {
    const size_t kb = (size_t)((K + 255) / 256);
    const size_t bx = kb * (size_t)((M + 127) / 128) * (size_t)((N + 31) / 32), bw = kb * (size_t)((N + 127) / 128) * (size_t)((M + 31) / 32);
    *dx_bytes = (bx + 255) / 256 * 256;
    *dw_bytes = (bw + 255) / 256 * 256;
}

int brick_maps_fill(void* workspace, int64_t M, int64_t N, int64_t K, bool dirty, hipStream_t st) {
    size_t bx, bw;
    brick_bytes(M, N, K, &bx, &bw);
    const int64_t words4 = (int64_t)((bx + bw) / 4);
    hipLaunchKernelGGL(lba_grad_fill_words_kernel, zero_grid(words4), dim3(256), 0, st, (uint32_t*)workspace, words4, dirty ? 0x01010101u : 0u);
    return hipGetLastError() == hipSuccess ? LBA_OK : LBA_ERR_LAUNCH;
}

int brick_maps_scan(const uint32_t* plane, void* workspace, int64_t M, int64_t N, int64_t K, uint32_t flip, hipStream_t st) {
    const int rc = brick_maps_fill(workspace, M, N, K, false, st);
    if (rc != LBA_OK) return rc;
    size_t bx, bw;
    brick_bytes(M, N, K, &bx, &bw);
    uint8_t* map_dx = (uint8_t*)workspace;
    uint8_t* map_dw = map_dx + bx;
    BrickDims bd;
    bd.quads = ((K + 31) / 32) * M * (N / 4);
    bd.M = (int32_t)M; bd.N = (int32_t)N; bd.K = (int32_t)K; bd.qpr = (int32_t)(N / 4);
    bd.rbx = (int32_t)((M + 127) / 128); bd.sbx = (int32_t)((N + 31) / 32);
    bd.rbw = (int32_t)((N + 127) / 128); bd.sbw = (int32_t)((M + 31) / 32);
    bd.flip = flip;
    const int64_t wgs = (bd.quads + kBrickQuadsPerWg - 1) / kBrickQuadsPerWg;
    if (wgs > 2147483647LL) return LBA_ERR_SHAPE;
    hipLaunchKernelGGL(lba_brick_map_kernel, dim3((unsigned)wgs), dim3(256), 0, st, plane, map_dx, map_dw, bd);
    return hipGetLastError() == hipSuccess ? LBA_OK : LBA_ERR_LAUNCH;
}

void brick_map_params(void* workspace, int64_t M, int64_t N, int64_t K, KParams* kp) {
    size_t bx, bw;
    brick_bytes(M, N, K, &bx, &bw);
    kp->map_dx = (uint8_t*)workspace;
    kp->map_dw = kp->map_dx + bx;
    kp->map_rbx = (int32_t)((M + 127) / 128); kp->map_sbx = (int32_t)((N + 31) / 32);
    kp->map_rbw = (int32_t)((N + 127) / 128); kp->map_sbw = (int32_t)((M + 31) / 32);
}

}  // namespace lba

extern "C" {

int lba_last_overflow(const uint32_t* of_mask, int32_t* last_of, int64_t M, int64_t N, int64_t K, void* hip_stream) {
    int rc = lba::validate_shapes(M, N, K);
    if (rc != LBA_OK) return rc;
    if (M * N > ((int64_t)1 << 31)) return LBA_ERR_SHAPE;      // one lane per output, fewer than 2^32 lanes per launch
    if (M == 0 || N == 0) return LBA_OK;
    if (!last_of || (K > 0 && !of_mask)) return LBA_ERR_NULL;
    const int64_t mn = M * N;
    hipLaunchKernelGGL(lba::lba_last_overflow_kernel, dim3((unsigned)((mn + 255) / 256)), dim3(256), 0,
                       (hipStream_t)hip_stream, of_mask, last_of, mn, (int32_t)((K + 31) / 32));
    return hipGetLastError() == hipSuccess ? LBA_OK : LBA_ERR_LAUNCH;
}

int lba_ste_plane(const uint32_t* of_mask, const uint32_t* of_mask2, uint32_t* coef, int64_t M, int64_t N, int64_t K,
                  int32_t ste, int32_t order, void* hip_stream) {
    int rc = lba::validate_shapes(M, N, K);
    if (rc != LBA_OK) return rc;
    if (ste != LBA_STE_IMMEDIATE_OF && ste != LBA_STE_RECURSIVE_OF) return LBA_ERR_UNSUPPORTED;
    if (order != LBA_ORDER_SEQ && order != LBA_ORDER_CHUNK16) return LBA_ERR_UNSUPPORTED;
    if (M * N > ((int64_t)1 << 31)) return LBA_ERR_SHAPE;      // one lane per output, fewer than 2^32 lanes per launch
    if (M == 0 || N == 0 || K == 0) return LBA_OK;
    if (!of_mask || !coef) return LBA_ERR_NULL;
    const bool two = ste == LBA_STE_RECURSIVE_OF && order == LBA_ORDER_CHUNK16;
    if (two && !of_mask2) return LBA_ERR_NULL;
    const int64_t mn = M * N;
    const dim3 grid((unsigned)((mn + 255) / 256)), block(256);
    hipStream_t st = (hipStream_t)hip_stream;
    if (ste == LBA_STE_IMMEDIATE_OF)
        hipLaunchKernelGGL((lba::lba_ste_plane_kernel<LBA_STE_IMMEDIATE_OF, LBA_ORDER_SEQ>), grid, block, 0, st, of_mask, of_mask2, coef, mn, (int32_t)K);
    else if (two)
        hipLaunchKernelGGL((lba::lba_ste_plane_kernel<LBA_STE_RECURSIVE_OF, LBA_ORDER_CHUNK16>), grid, block, 0, st, of_mask, of_mask2, coef, mn, (int32_t)K);
    else
        hipLaunchKernelGGL((lba::lba_ste_plane_kernel<LBA_STE_RECURSIVE_OF, LBA_ORDER_SEQ>), grid, block, 0, st, of_mask, of_mask2, coef, mn, (int32_t)K);
    return hipGetLastError() == hipSuccess ? LBA_OK : LBA_ERR_LAUNCH;
}

size_t lba_grad_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    if (M <= 0 || N <= 0 || K <= 0 || lba::validate_shapes(M, N, K) != LBA_OK || M * N > ((int64_t)1 << 30)) return 0;
    size_t a, b;
    lba::brick_bytes(M, N, K, &a, &b);
    return a + b;
}

size_t lba_grad_workspace_bytes_fast(int64_t M, int64_t N, int64_t K) {
    const size_t maps = lba_grad_workspace_bytes(M, N, K);
    if (maps == 0) return 0;
    return maps + (lba::grad_dense_partial_bytes(M, N, K) + 255) / 256 * 256;
}

static int grad_impl(const float* G, const uint8_t* A, const uint8_t* B, const uint32_t* of_mask, const int32_t* last_of,
                     float* dX, float* dW, int64_t M, int64_t N, int64_t K, int32_t ste, void* workspace, size_t workspace_bytes,
                     void* hip_stream, bool maps_ready = false);

int lba_grad(const float* G, const uint8_t* A, const uint8_t* B, const uint32_t* of_mask, const int32_t* last_of,
             float* dX, float* dW, int64_t M, int64_t N, int64_t K, int32_t ste, void* hip_stream) {
    return grad_impl(G, A, B, of_mask, last_of, dX, dW, M, N, K, ste, nullptr, 0, hip_stream);
}

int lba_grad_ws(const float* G, const uint8_t* A, const uint8_t* B, const uint32_t* of_mask, const int32_t* last_of,
                float* dX, float* dW, int64_t M, int64_t N, int64_t K, int32_t ste,
                void* workspace, size_t workspace_bytes, void* hip_stream) {
    const int rc = lba::validate_shapes(M, N, K);
    if (rc != LBA_OK) return rc;
    if (M > 0 && N > 0 && K > 0 && M * N <= ((int64_t)1 << 30)) {
        if (!workspace) return LBA_ERR_NULL;
        if (((uintptr_t)workspace % 256) != 0) return LBA_ERR_ALIGN;
        if (workspace_bytes < lba_grad_workspace_bytes(M, N, K)) return LBA_ERR_SHAPE;
    }
    return grad_impl(G, A, B, of_mask, last_of, dX, dW, M, N, K, ste, workspace, workspace_bytes, hip_stream);
}

// The brick maps of lba_grad_static: device memory that belongs to the library (every GPU the library runs on holds
// its own copy until the process ends).  In host code the array's name is only a handle: its device address is asked
// for once per device and kept.
#define LBA_GRAD_STATIC_BYTES (1 << 20)
static __device__ __align__(256) unsigned char scratch[LBA_GRAD_STATIC_BYTES];

static int static_scratch(void** out) {
    static std::mutex mu;
    static void* addr[64] = {nullptr};                         // per device
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return LBA_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LBA_ERR_LAUNCH;
        addr[dev] = p;
    }
    *out = addr[dev];
    return LBA_OK;
}

int lba_grad_premapped(const float* G, const uint8_t* A, const uint8_t* B, const uint32_t* of_mask,
                       float* dX, float* dW, int64_t M, int64_t N, int64_t K,
                       void* workspace, size_t workspace_bytes, void* hip_stream) {
    const int rc = lba::validate_shapes(M, N, K);
    if (rc != LBA_OK) return rc;
    if (M > 0 && N > 0 && K > 0 && M * N <= ((int64_t)1 << 30)) {
        if (!workspace) return LBA_ERR_NULL;
        if (((uintptr_t)workspace % 256) != 0) return LBA_ERR_ALIGN;
        if (workspace_bytes < lba_grad_workspace_bytes(M, N, K)) return LBA_ERR_SHAPE;
    }
    return grad_impl(G, A, B, of_mask, nullptr, dX, dW, M, N, K, LBA_STE_IMMEDIATE_OF, workspace, workspace_bytes, hip_stream, true);
}

int lba_grad_static(const float* G, const uint8_t* A, const uint8_t* B, const uint32_t* of_mask, const int32_t* last_of,
                    float* dX, float* dW, int64_t M, int64_t N, int64_t K, int32_t ste, void* hip_stream) {
    const int rc = lba::validate_shapes(M, N, K);
    if (rc != LBA_OK) return rc;
    if (M > 0 && N > 0 && K > 0 && M * N <= ((int64_t)1 << 30) && lba_grad_workspace_bytes(M, N, K) > (size_t)LBA_GRAD_STATIC_BYTES)
        return LBA_ERR_SHAPE;                                  // beyond the library's own scratch memory: use lba_grad_ws
    void* ws = nullptr;
    const int rs = static_scratch(&ws);
    if (rs != LBA_OK) return rs;
    return grad_impl(G, A, B, of_mask, last_of, dX, dW, M, N, K, ste, ws, (size_t)LBA_GRAD_STATIC_BYTES, hip_stream);
}

static int grad_impl(const float* G, const uint8_t* A, const uint8_t* B, const uint32_t* of_mask, const int32_t* last_of,
                     float* dX, float* dW, int64_t M, int64_t N, int64_t K, int32_t ste, void* workspace, size_t workspace_bytes,
                     void* hip_stream, bool maps_ready) {
    int rc = lba::validate_shapes(M, N, K);
    if (rc != LBA_OK) return rc;
    if (ste != LBA_STE_IDENTITY && ste != LBA_STE_IMMEDIATE_OF && ste != LBA_STE_RECURSIVE_OF &&
        ste != LBA_STE_COEF_PLANE) return LBA_ERR_UNSUPPORTED;
    if ((K + 63) / 64 > 65535) return LBA_ERR_SHAPE;           // k blocks are grid y
    if (M * N > ((int64_t)1 << 30)) return LBA_ERR_SHAPE;      // element offsets of G and of a word slab are 32-bit
    if (!dX && !dW) return LBA_ERR_NULL;
    if (K == 0) return LBA_OK;                                 // dX and dW are empty
    hipStream_t st = (hipStream_t)hip_stream;
    if (M == 0 || N == 0) {                                    // empty sums: the non-empty gradient is zero
        float* o = M == 0 ? dW : dX;
        const int64_t n = (M == 0 ? N : M) * K;
        if (o && n > 0) {
            hipLaunchKernelGGL(lba::lba_grad_zero_kernel, lba::zero_grid(n), dim3(256), 0, st, o, n);
            if (hipGetLastError() != hipSuccess) return LBA_ERR_LAUNCH;
        }
        return LBA_OK;
    }
    if (!G) return LBA_ERR_NULL;
    if ((ste == LBA_STE_IMMEDIATE_OF || ste == LBA_STE_COEF_PLANE) && !of_mask) return LBA_ERR_NULL;
    if (ste == LBA_STE_RECURSIVE_OF && !last_of) return LBA_ERR_NULL;
    if ((dX && !B) || (dW && !A)) return LBA_ERR_NULL;         // every check before the first launch
    // With a workspace, the immediate estimator (and a coefficient plane) splits the work by bricks: one pass over
    // the plane marks the bricks that hold a blocked coefficient; the others are plain dense products and run on
    // the matrix cores, the marked ones in the vector kernel that applies the plane bit by bit.  Every term is
    // added by exactly one of the two kernels.
    const uint8_t* bricks_dx = nullptr;
    const uint8_t* bricks_dw = nullptr;
    if (workspace && (ste == LBA_STE_IMMEDIATE_OF || ste == LBA_STE_COEF_PLANE) &&
        lba::grad_dense_ok(G, nullptr, nullptr, M, N, K) && ((uintptr_t)of_mask % 16) == 0) {
        size_t bx, bw;
        lba::brick_bytes(M, N, K, &bx, &bw);
        uint8_t* map_dx = (uint8_t*)workspace;
        uint8_t* map_dw = map_dx + bx;
        if (!maps_ready) {                                     // (lba_grad_premapped: the recompute call left them there)
            rc = lba::brick_maps_scan(of_mask, workspace, M, N, K, (ste == LBA_STE_COEF_PLANE) ? 0xFFFFFFFFu : 0u, st);
            if (rc != LBA_OK) return rc;
        }
        bricks_dx = map_dx;
        bricks_dw = map_dw;
    }
    // What lies behind the maps in the workspace holds the slices of a sum over s that the matrix-core kernel cuts
    // across workgroups (first of dX, then, after dX's slices have been added up, of dW).
    float* partials = nullptr;
    size_t partial_bytes = 0;
    const size_t maps_bytes = lba_grad_workspace_bytes(M, N, K);
    if (workspace && workspace_bytes > maps_bytes) {
        partials = (float*)((uint8_t*)workspace + maps_bytes);  // 256-byte aligned: the maps are padded
        partial_bytes = workspace_bytes - maps_bytes;
    }
    if (dX) {
        rc = lba::run_grad_side(true, G, B, of_mask, last_of, dX, M, N, K, ste, st, bricks_dx, partials, partial_bytes);
        if (rc != LBA_OK) return rc;
    }
    if (dW) {
        rc = lba::run_grad_side(false, G, A, of_mask, last_of, dW, M, N, K, ste, st, bricks_dw, partials, partial_bytes);
        if (rc != LBA_OK) return rc;
    }
    return LBA_OK;
}

}  // extern "C"
