// lba_grad_mfma.hip -- the gradient products whose coefficients do not depend on k inside a tile, as a
// dense contraction on the matrix cores of gfx950.
//
//   out[r, k] = sum_s g'(r, s) * value(V[s, k])          dX: r = m, s = n, V = B;  dW: r = n, s = m, V = A
//
// With the identity estimator (Sec. 4 of the paper: c = 1) g' = g and this is a plain matrix product of an
// FP32 matrix with a matrix of FP8 values.  The FP32 factor is split exactly into three bfloat16 pieces
// (g = hi + mid + lo, 8 significant bits each: truncate, subtract, truncate, subtract; every step is exact),
// an E4M3 value is a bfloat16 number as it is, so the three bfloat16 products hi*v, mid*v, lo*v are exact
// and their FP32 accumulation in v_mfma_f32_32x32x16_bf16 is the FP32 sum of products the interface
// promises (order of summation unspecified; pieces or products below the FP32 normal range, i.e. gradients
// under about 2^-100, may be flushed).  Three MFMA passes at the bfloat16 rate are about five times
// the FP32 rate of the vector units or of the FP32 MFMA.
//
// The recursive estimator under the sequential order (App. D: c = [k > last overflow index L(r, s)]) is the same
// contraction for all but a sliver of the work: inside a k tile (128 or 256 wide) starting at k0 a pair (r, s) with
// L < k0 has c = 1 for every k of the tile, a pair with L beyond the tile has c = 0, so the tile is the dense
// product with g' = [L < k0] g (the mask is applied while G is staged).  What is left are the k between L and
// the end of L's own k block, fewer than the tile width per pair: lba_grad_boundary_kernel visits every pair once
// (one workgroup per row r, its K sums in LDS, a wave per pair with lanes along k) and adds that sliver.
//
// Tiling: a workgroup of four waves owns 128 rows x 128 (or 256) k; a wave owns 64 x 64 (or 64 x 128): 2 x 2
// (2 x 4) MFMA blocks of 32 x 32, 64 (128) accumulator registers.  s advances in steps of 32: the lanes fetch 4 x 4 patches of G (FP32)
// and of V (codes), split / decode them and store bfloat16 rows [row][s] (G) and [k][s] (V, transposed) in
// LDS with a pitch of 40 elements, which makes the 16-byte fragment reads of a wave conflict-free.
// Operand fragments: lane l holds row (or column) l % 32 and the eight s values 8 * (l / 32) .. + 7 of a
// 16-deep step, the same mapping for both operands, so the contraction pairs equal s whatever order the
// hardware walks them in.  Results: register t of lane l is row 8 * (t / 4) + 4 * (l / 32) + t % 4, column l % 32.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lba.h"
#include "lba_internal.h"

namespace lba {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct DenseDims {
    int32_t R, S, K;
    int32_t s_chunk;           // s values per grid z (a multiple of 32)
    int32_t atomic;            // 1: gridDim.z > 1, combine with atomic adds into a zeroed output; 2: gridDim.z > 1, slice z
                               // is stored whole at out + z * R * K (a workspace; lba_grad_combine_kernel adds the slices)
    int32_t ld_g;              // N: G[m * N + n]
    int32_t b_chunk;           // sliver pass: s values per grid y (a multiple of 256)
    int32_t k_shift;           // log2 of the k tile of the dense pass (the sliver pass cuts k into the same blocks)
    int32_t v_vec;             // 1: every row of codes starts 4-byte aligned (V % 4 == 0, K % 4 == 0)
    int32_t brick_rb, brick_sb; // brick map of the immediate estimator: byte ((k / 256) * brick_rb + r / 128) * brick_sb + s / 32
};

// DTK (a template argument): 128 or 256 columns k per workgroup; the wider tile splits G half as often and is
// taken when it still leaves two workgroups per CU
constexpr int DTR = 128, DBS = 32, DPITCH = 40;

__device__ __forceinline__ float dense_decode_e4m3(uint32_t code) {
    float v = __builtin_amdgcn_cvt_f32_fp8((int)code, 0);
    if ((code & 0x7Fu) == 0x7Fu) v = (code & 0x80u) ? -480.0f : 480.0f;   // the two NaN codes
    return v;
}

// g = hi + mid + lo with 8 significant bits each; returns the three pieces as FP32 words whose low halves are zero
__device__ __forceinline__ void split3(float g, uint32_t& hi, uint32_t& mid, uint32_t& lo) {
    hi = __float_as_uint(g) & 0xFFFF0000u;
    const float r1 = g - __uint_as_float(hi);                  // exact: the low 16 bits of g's significand
    mid = __float_as_uint(r1) & 0xFFFF0000u;
    lo = __float_as_uint(r1 - __uint_as_float(mid));           // exact, at most 8 significant bits: low half zero
}

// two bfloat16 values (the high halves of two FP32 words) in one register, x in the low half
__device__ __forceinline__ uint32_t pack_hi(uint32_t x, uint32_t y) { return __builtin_amdgcn_perm(y, x, 0x07060302u); }

// four E4M3 codes of one word -> four FP32 values; the NaN codes are patched to +-480 on a rarely taken path
__device__ __forceinline__ void decode4(uint32_t w, float (&v)[4]) {
    typedef float v2f __attribute__((ext_vector_type(2)));
    const v2f a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
    v[0] = a[0]; v[1] = a[1]; v[2] = b[0]; v[3] = b[1];
    if ((((w & 0x7F7F7F7Fu) + 0x01010101u) & 0x80808080u) != 0u) {     // some byte has all of its low seven bits set
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t code = (w >> (8 * c)) & 0xFFu;
            if ((code & 0x7Fu) == 0x7Fu) v[c] = (code & 0x80u) ? -480.0f : 480.0f;
        }
    }
}

// S_CONTIG: G(r, s) = G[r * ld + s] (dX); else G(r, s) = G[s * ld + r] (dW).  MASKED: L (same layout as G)
// holds last-overflow indices and g' = [L < k0] g.
template <bool S_CONTIG, bool MASKED, int DTK, bool BYTES = false>
__global__ void __launch_bounds__(256, 2) lba_grad_dense_kernel(const float* __restrict__ G, const uint8_t* __restrict__ V,
                                                                const int32_t* __restrict__ L,
                                                                float* __restrict__ out, const DenseDims d,
                                                                const uint8_t* __restrict__ bricks) {
    constexpr int DNBJ = DTK / 64;                             // MFMA column blocks per wave (two waves side by side)
    static_assert(!BYTES || DTK == 128, "unaligned rows of codes: the narrow tile only");
    __shared__ __attribute__((aligned(16))) uint16_t sA[3][DTR * DPITCH];
    __shared__ __attribute__((aligned(16))) uint16_t sB[DTK * DPITCH];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wy = wave >> 1, wx = wave & 1;
    const int r0 = blockIdx.x * DTR, k0 = blockIdx.y * DTK;
    const int s_begin = blockIdx.z * d.s_chunk;
    const int s_end = min(d.S, s_begin + d.s_chunk);
    if (d.atomic == 2) out += (int64_t)blockIdx.z * d.R * d.K;     // this slice's own copy of the output (a workspace)

    // this lane's 4 x 4 patch of the G tile and of the V tile
    // Consecutive lanes take consecutive s: the eight lanes of a row write 64 contiguous bytes of LDS and the next
    // eight are 4 rows = 320 bytes = 16 banks further, so every 16 lanes of an 8-byte store cover all banks once
    // (the other order, consecutive lanes along rows, put 32 lanes on two bank pairs).  In global memory a wave
    // then reads 128 contiguous bytes of eight rows of G, or 32 bytes of eight rows of codes.
    const int a_pr = tid >> 3, a_ps = tid & 7;                 // patch row (4 rows r), patch column (4 values of s)
    const int b_ps = tid & 7, b_pk = tid >> 3;                 // 4 rows s, 4 codes k

    float4 gl[4];
    int4 ll[MASKED ? 4 : 1];                                   // last-overflow indices of the G patch: compared when the
                                                               // patch is staged, so that the loads stay in flight meanwhile
    uint32_t vl[DTK / 128][4];
    uint32_t vh[BYTES ? 4 : 1] = {};                           // unaligned rows of codes: the second aligned word of a group
    auto fetch = [&](int sb) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float4 g = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (S_CONTIG) {                                    // q: row within the patch; the float4 runs along s (S % 4 == 0 and
                                                               // s_chunk % 32 == 0: it is inside the range or outside, never across)
                const int r = r0 + 4 * a_pr + q, s = sb + 4 * a_ps;
                if (r < d.R && s < s_end) {
                    g = *reinterpret_cast<const float4*>(G + (int64_t)r * d.ld_g + s);
                    if (MASKED) ll[q] = *reinterpret_cast<const int4*>(L + (int64_t)r * d.ld_g + s);
                }
            } else {                                           // q: s within the patch; the float4 runs along r
                const int r = r0 + 4 * a_pr, s = sb + 4 * a_ps + q;
                if (r < d.R && s < s_end) {
                    g = *reinterpret_cast<const float4*>(G + (int64_t)s * d.ld_g + r);
                    if (MASKED) ll[q] = *reinterpret_cast<const int4*>(L + (int64_t)s * d.ld_g + r);
                }
            }
            gl[q] = g;
#pragma unroll
            for (int h = 0; h < DTK / 128; ++h) {
                const int sv = sb + 4 * b_ps + q, kv = k0 + 128 * h + 4 * b_pk;
                uint32_t w = 0u;                               // four codes along k; code 0 (the value +0) beyond K
                if (sv < s_end && kv < d.K) {
                    const uint8_t* __restrict__ src = V + (int64_t)sv * d.K + kv;
                    if (!BYTES) {                              // rows of codes are 4-byte aligned and K % 4 == 0
                        w = *reinterpret_cast<const uint32_t*>(src);
                    } else {                                   // the two aligned words that hold the group's valid bytes, put
                        const int nvalid = (d.K - kv) < 4 ? (d.K - kv) : 4;   // together when the patch is staged: the loads stay in flight
                        const uint32_t lo = (uint32_t)(reinterpret_cast<uintptr_t>(src) & 3u);   // (pointers derived from V stay
                        const uint8_t* __restrict__ p0 = src - lo;                              // global-memory pointers)
                        const uint8_t* __restrict__ p1 = p0 + ((lo + (uint32_t)nvalid - 1u) & ~3u);   // the same word or the next
                        w = *reinterpret_cast<const uint32_t*>(p0);
                        vh[BYTES ? q : 0] = *reinterpret_cast<const uint32_t*>(p1);
                    }
                }
                vl[h][q] = w;
            }
        }
    };

    f32x16 acc[2][DNBJ];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < DNBJ; ++j)
#pragma unroll
            for (int t = 0; t < 16; ++t) acc[i][j][t] = 0.0f;

    // Immediate estimator: a brick (128 rows x 32 s x 256 k) in which some coefficient is 0 is left to the vector
    // kernel, which applies the coefficients bit by bit; this kernel adds the bricks whose coefficients are all 1.
    const uint8_t* __restrict__ brick_row = bricks ? bricks + ((int64_t)(k0 >> 8) * d.brick_rb + (r0 >> 7)) * d.brick_sb : nullptr;
    fetch(s_begin);
    for (int sb = s_begin; sb < s_end; sb += DBS) {
        if (brick_row && brick_row[sb >> 5]) {                 // uniform over the workgroup
            if (sb + DBS < s_end) fetch(sb + DBS);
            continue;
        }
        // split / decode this step's patches into LDS
        {
            float g[4][4];                                     // [row a][s b]
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float x[4] = {gl[q].x, gl[q].y, gl[q].z, gl[q].w};
                if (MASKED) {                                  // g' = [L < k0] g (where nothing was fetched g is 0 already)
                    const int4 t = ll[MASKED ? q : 0];
                    x[0] = t.x < k0 ? x[0] : 0.0f; x[1] = t.y < k0 ? x[1] : 0.0f;
                    x[2] = t.z < k0 ? x[2] : 0.0f; x[3] = t.w < k0 ? x[3] : 0.0f;
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (S_CONTIG) g[q][e] = x[e]; else g[e][q] = x[e];
                }
            }
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                uint32_t h[4], m[4], l[4];
#pragma unroll
                for (int b = 0; b < 4; ++b) split3(g[a][b], h[b], m[b], l[b]);
                const int off = (4 * a_pr + a) * DPITCH + 4 * a_ps;
                *reinterpret_cast<uint2*>(&sA[0][off]) = make_uint2(pack_hi(h[0], h[1]), pack_hi(h[2], h[3]));
                *reinterpret_cast<uint2*>(&sA[1][off]) = make_uint2(pack_hi(m[0], m[1]), pack_hi(m[2], m[3]));
                *reinterpret_cast<uint2*>(&sA[2][off]) = make_uint2(pack_hi(l[0], l[1]), pack_hi(l[2], l[3]));
            }
            if (BYTES) {                                       // shift the groups' bytes out of their two words
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int sv = sb + 4 * b_ps + b, kv = k0 + 4 * b_pk;
                    const uint32_t sh = (uint32_t)((reinterpret_cast<uintptr_t>(V) + (uintptr_t)((int64_t)sv * d.K + kv)) & 3u) * 8u;
                    const uint32_t w = __builtin_amdgcn_alignbit(vh[BYTES ? b : 0], vl[0][b], sh);   // ({second, first} >> shift)[31:0]
                    const int left = d.K - kv;
                    vl[0][b] = (sv < s_end && left > 0) ? (left < 4 ? (w & ((1u << (8 * left)) - 1u)) : w) : 0u;
                }
            }
#pragma unroll
            for (int h = 0; h < DTK / 128; ++h) {
                float vv[4][4];                                // [row s b][code c]
#pragma unroll
                for (int b = 0; b < 4; ++b) decode4(vl[h][b], vv[b]);
#pragma unroll
                for (int c = 0; c < 4; ++c)                    // code c of each of the four rows s: an E4M3 value is a bfloat16 number
                    *reinterpret_cast<uint2*>(&sB[(128 * h + 4 * b_pk + c) * DPITCH + 4 * b_ps]) =
                        make_uint2(pack_hi(__float_as_uint(vv[0][c]), __float_as_uint(vv[1][c])),
                                   pack_hi(__float_as_uint(vv[2][c]), __float_as_uint(vv[3][c])));
            }
        }
        __syncthreads();
        if (sb + DBS < s_end) fetch(sb + DBS);                 // in flight during the MFMAs
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int so = kk * 16 + 8 * (lane >> 5);
            bf16x8 bf[DNBJ];
#pragma unroll
            for (int bj = 0; bj < DNBJ; ++bj)
                bf[bj] = *reinterpret_cast<const bf16x8*>(&sB[(wx * (DTK / 2) + bj * 32 + (lane & 31)) * DPITCH + so]);
#pragma unroll
            for (int sp = 0; sp < 3; ++sp)
#pragma unroll
                for (int bi = 0; bi < 2; ++bi) {
                    const bf16x8 af = *reinterpret_cast<const bf16x8*>(&sA[sp][(wy * 64 + bi * 32 + (lane & 31)) * DPITCH + so]);
#pragma unroll
                    for (int bj = 0; bj < DNBJ; ++bj)
                        acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bf[bj], acc[bi][bj], 0, 0, 0);
                }
        }
        __syncthreads();
    }

#pragma unroll
    for (int bi = 0; bi < 2; ++bi)
#pragma unroll
        for (int bj = 0; bj < DNBJ; ++bj) {
            const int col = k0 + wx * (DTK / 2) + bj * 32 + (lane & 31);
#pragma unroll
            for (int t = 0; t < 16; ++t) {
                const int row = r0 + wy * 64 + bi * 32 + 8 * (t >> 2) + 4 * (lane >> 5) + (t & 3);
                if (row < d.R && col < d.K) {
                    float* dst = out + (int64_t)row * d.K + col;
                    if (d.atomic == 1) unsafeAtomicAdd(dst, acc[bi][bj][t]);
                    else               *dst = acc[bi][bj][t];
                }
            }
        }
}

// The sliver of the recursive estimator that the masked dense product leaves out: for every pair (r, s) with
// L = L(r, s) >= 0 the terms g(r, s) * value(V[s, k]) for L < k < end of L's k block.  One workgroup per ROWS rows r
// keeps their K sums each in LDS; a wave takes 64 consecutive s at a time (their L and g in its lanes), then
// one pair after the other with its lanes along k.  out[r, :] += sums (the dense part is already there).
// ROWS = 2, 4, 8 or 16 (rows contiguous in memory, dW): a lane fetches its rows' values with 8- or 16-byte loads; the
// walk over s is strided by a whole row of G, so with 16 rows (64 bytes per s) every sector fetched is used in full,
// with 2 an eighth of it.  The launcher takes as many rows as have their sums in 48 KB of LDS (16 up to K = 768).
template <bool S_CONTIG, int ROWS>
__global__ void __launch_bounds__(256) lba_grad_boundary_kernel(const float* __restrict__ G, const uint8_t* __restrict__ V,
                                                                const int32_t* __restrict__ L, float* __restrict__ out,
                                                                const DenseDims d) {
    static_assert(ROWS == 1 || ((ROWS == 2 || ROWS == 4 || ROWS == 8 || ROWS == 16) && !S_CONTIG),
                  "several rows only where rows are contiguous");
    extern __shared__ float row[];                             // ROWS x K sums
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = blockIdx.x * ROWS;
    const int nrows = min(ROWS, d.R - r);                      // R % 4 == 0: 16-row groups end on a multiple of 4
    for (int k = tid; k < nrows * d.K; k += 256) row[k] = 0.0f;
    __syncthreads();
    // grid y cuts s into slices of b_chunk (a multiple of 256) when there are few rows
    const int s_lo = blockIdx.y * d.b_chunk, s_hi = min(d.S, s_lo + d.b_chunk);
    for (int s0 = s_lo + wave * 64; s0 < s_hi; s0 += 256) {
        const int s = s0 + lane;
        int32_t lv[ROWS];
        float gv[ROWS];
#pragma unroll
        for (int i = 0; i < ROWS; ++i) { lv[i] = -1; gv[i] = 0.0f; }
        if (s < s_hi) {
            const int64_t off = S_CONTIG ? (int64_t)r * d.ld_g + s : (int64_t)s * d.ld_g + r;
            if constexpr (ROWS >= 4) {                         // r % 4 == 0 and ld_g % 4 == 0: 16-byte aligned groups of 4 rows
#pragma unroll
                for (int q = 0; q < ROWS / 4; ++q) {
                    if (4 * q < nrows) {                       // uniform; a group of 4 rows exists as a whole
                        const int4 l4 = *reinterpret_cast<const int4*>(L + off + 4 * q);
                        const float4 g4 = *reinterpret_cast<const float4*>(G + off + 4 * q);
                        lv[4 * q] = l4.x; lv[4 * q + 1] = l4.y; lv[4 * q + 2] = l4.z; lv[4 * q + 3] = l4.w;
                        gv[4 * q] = g4.x; gv[4 * q + 1] = g4.y; gv[4 * q + 2] = g4.z; gv[4 * q + 3] = g4.w;
                    }
                }
            } else if constexpr (ROWS == 2) {                  // r even and ld_g % 4 == 0: 8-byte aligned; R % 4 == 0: both rows exist
                const int2 l2 = *reinterpret_cast<const int2*>(L + off);
                const float2 g2 = *reinterpret_cast<const float2*>(G + off);
                lv[0] = l2.x; lv[ROWS - 1] = l2.y; gv[0] = g2.x; gv[ROWS - 1] = g2.y;
            } else {
                lv[0] = L[off];
                gv[0] = G[off];
            }
        }
#pragma unroll
        for (int i = 0; i < ROWS; ++i) {
            uint64_t todo = __builtin_amdgcn_ballot_w64(lv[i] >= 0 && gv[i] != 0.0f);
            while (todo) {                                     // wave-uniform loop over the pairs that have a sliver
                const int j = __builtin_ctzll(todo);
                todo &= todo - 1;
                const int32_t lj = __builtin_amdgcn_readlane(lv[i], j);
                const float gj = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(gv[i]), j));
                const int k_end = min(d.K, ((lj >> d.k_shift) + 1) << d.k_shift);
                const uint8_t* __restrict__ vrow = V + (int64_t)(s0 + j) * d.K;
                for (int k = lj + 1 + lane; k < k_end; k += 64)
                    atomicAdd(&row[i * d.K + k], gj * dense_decode_e4m3(vrow[k]));
            }
        }
    }
    __syncthreads();
    for (int k = tid; k < nrows * d.K; k += 256) {
        const float x = row[k];
        if (x != 0.0f) {                                       // row[i * K + k'] belongs to out[(r + i) * K + k']: the same offset from out + r * K
            if (gridDim.y > 1) unsafeAtomicAdd(out + (int64_t)r * d.K + k, x);
            else               out[(int64_t)r * d.K + k] += x;
        }
    }
}

// out[i] = sum over the slices z of part[z * n + i], added in the order of z (the slices of a sum over s that was
// cut across workgroups, stored whole in a workspace: no atomic adds).  VEC: n % 4 == 0 and out 16-byte aligned
// (the slices are: the workspace is 256-byte aligned): four outputs per lane with 16-byte accesses.
template <bool VEC>
__global__ void __launch_bounds__(256) lba_grad_combine_kernel(const float* __restrict__ part, float* __restrict__ out, int64_t n, int slices) {
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    if (VEC) {
        const int64_t n4 = n >> 2;
        const float4* __restrict__ p4 = reinterpret_cast<const float4*>(part);
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += step) {
            float4 a = p4[i];
            for (int z0 = 1; z0 < slices; z0 += 8) {           // eight loads in flight, then the additions in the order of z
                float4 v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int z = z0 + j < slices ? z0 + j : slices - 1;   // (beyond the last slice: read it again, unused)
                    v[j] = p4[(int64_t)z * n4 + i];
                }
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (z0 + j < slices) { a.x += v[j].x; a.y += v[j].y; a.z += v[j].z; a.w += v[j].w; }
            }
            reinterpret_cast<float4*>(out)[i] = a;
        }
    } else {
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += step) {
            float acc = part[i];
            for (int z = 1; z < slices; ++z) acc += part[(int64_t)z * n + i];
            out[i] = acc;
        }
    }
}

__global__ void lba_grad_dense_zero_kernel(float* x, int64_t n) {
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += step) x[i] = 0.0f;
}

// Can the matrix-core path take this product?  16-byte rows of G (and of last_of) in both directions; with last_of
// also a row of K sums within 48 KB of LDS.  (Codes are read in 4-byte groups: one load when their rows are aligned,
// else the two aligned words around the group.)
bool grad_dense_ok(const float* G, const uint8_t* V, const int32_t* last_of, int64_t M, int64_t N, int64_t K) {
    (void)V;
    if (((uintptr_t)G % 16) != 0 || (N % 4) != 0 || (K + 127) / 128 > 65535)
        return false;
    if (last_of && (((uintptr_t)last_of % 16) != 0 || K > 12288)) return false;
    return true;
}

// Tile width, grid and slices of s of one of the two products (v_vec: rows of codes are 4-byte aligned).
struct DenseShape { int64_t gx, gy, split; bool wide; };
static DenseShape dense_shape(bool dx, int64_t M, int64_t N, int64_t K, bool v_vec, DenseDims* d) {
    DenseShape h;
    d->R = (int32_t)(dx ? M : N); d->S = (int32_t)(dx ? N : M); d->K = (int32_t)K; d->ld_g = (int32_t)N;
    h.gx = (d->R + DTR - 1) / DTR;
    // 128 x 256 tiles where they still give two workgroups per CU (K <= 128 would leave half of such a tile empty;
    // rows of codes that are not 4-byte aligned are read by the narrow kernel only)
    h.wide = K > 128 && v_vec && h.gx * ((K + 255) / 256) >= 512;
    const int dtk = h.wide ? 256 : 128;
    d->k_shift = h.wide ? 8 : 7;
    h.gy = (K + dtk - 1) / dtk;
    // enough workgroups for about two per CU: cut s into slices of a multiple of 32, doubling their number while there
    // are fewer than 384 workgroups (measured on the ResNet-50 shapes: doubling on to 512 and beyond made a second
    // round of workgroups, twice the atomic adds or slices, and a gradient sweep of 8.0 ms instead of 7.5; stopping at
    // 256 left CUs with one workgroup: 8.2 ms)
    int64_t split = 1;
    const int64_t steps = (d->S + DBS - 1) / DBS;
    while (h.gx * h.gy * split < 384 && split * 2 <= steps && split < 512) split *= 2;
    const int64_t per = (steps + split - 1) / split;
    d->s_chunk = (int32_t)(per * DBS);
    h.split = (d->S + d->s_chunk - 1) / d->s_chunk;
    return h;
}

// Bytes of workspace with which both products of a call combine their slices without atomic adds (the larger of the
// two needs, whatever the alignment of the code matrices); 0 if neither product is cut into slices.
size_t grad_dense_partial_bytes(int64_t M, int64_t N, int64_t K) {
    size_t need = 0;
    for (int dx = 0; dx < 2; ++dx)
        for (int vec = 0; vec < 2; ++vec) {
            DenseDims d;
            const DenseShape h = dense_shape(dx != 0, M, N, K, vec != 0, &d);
            if (h.split > 1) {
                const size_t b = (size_t)h.split * (size_t)d.R * (size_t)K * sizeof(float);
                if (b > need) need = b;
            }
        }
    return need;
}

// One of the two products with the identity coefficients (last_of == NULL) or the recursive ones.
// partials / partial_bytes: 256-byte aligned scratch memory for the slices of a split sum, or NULL / 0 (atomic adds).
// LBA_OK or LBA_ERR_LAUNCH.
int run_grad_dense(bool dx, const float* G, const uint8_t* V, const int32_t* last_of, float* out,
                   int64_t M, int64_t N, int64_t K, hipStream_t st, const uint8_t* bricks,
                   float* partials, size_t partial_bytes) {
    DenseDims d;
    d.brick_rb = (int32_t)(((dx ? M : N) + 127) / 128);
    d.brick_sb = (int32_t)(((dx ? N : M) + 31) / 32);
    d.v_vec = (((uintptr_t)V % 4) == 0 && (K % 4) == 0) ? 1 : 0;
    const DenseShape h = dense_shape(dx, M, N, K, d.v_vec != 0, &d);
    d.b_chunk = d.S;
    const int64_t gx = h.gx, gy = h.gy, split = h.split;
    const bool wide = h.wide;
    const int64_t n_out = (int64_t)d.R * K;
    d.atomic = split > 1 ? 1 : 0;
    float* target = out;
    if (d.atomic && partials && (size_t)split * (size_t)n_out * sizeof(float) <= partial_bytes) {
        d.atomic = 2;
        target = partials;
    }
    if (d.atomic == 1) {
        const int64_t n = n_out;
        hipLaunchKernelGGL(lba_grad_dense_zero_kernel, dim3((unsigned)((n + 255) / 256 < (1 << 20) ? (n + 255) / 256 : (1 << 20))), dim3(256), 0, st, out, n);
        if (hipGetLastError() != hipSuccess) return LBA_ERR_LAUNCH;
    }
    const dim3 grid((unsigned)gx, (unsigned)gy, (unsigned)split);
#define LBA_DENSE(SC, MK) do { if (wide)          hipLaunchKernelGGL((lba_grad_dense_kernel<SC, MK, 256>), grid, dim3(256), 0, st, G, V, last_of, target, d, bricks); \
                               else if (d.v_vec) hipLaunchKernelGGL((lba_grad_dense_kernel<SC, MK, 128>), grid, dim3(256), 0, st, G, V, last_of, target, d, bricks); \
                               else              hipLaunchKernelGGL((lba_grad_dense_kernel<SC, MK, 128, true>), grid, dim3(256), 0, st, G, V, last_of, target, d, bricks); } while (0)
    if (!last_of) { if (dx) LBA_DENSE(true, false); else LBA_DENSE(false, false); }
    else          { if (dx) LBA_DENSE(true, true);  else LBA_DENSE(false, true); }
#undef LBA_DENSE
    if (hipGetLastError() != hipSuccess) return LBA_ERR_LAUNCH;
    if (d.atomic == 2) {                                       // the slices, added in order, become the output
        const bool vec = (n_out % 4) == 0 && ((uintptr_t)out % 16) == 0;
        const int64_t blocks = ((vec ? n_out / 4 : n_out) + 255) / 256;
        const dim3 cgrid((unsigned)(blocks < (1 << 20) ? blocks : (1 << 20)));
        if (vec) hipLaunchKernelGGL(lba_grad_combine_kernel<true>, cgrid, dim3(256), 0, st, partials, out, n_out, (int)split);
        else     hipLaunchKernelGGL(lba_grad_combine_kernel<false>, cgrid, dim3(256), 0, st, partials, out, n_out, (int)split);
        if (hipGetLastError() != hipSuccess) return LBA_ERR_LAUNCH;
    }
    if (!last_of) return LBA_OK;
    // the sliver pass: one workgroup per group of rows, and with few groups also slices of s, to have about 2048
    // workgroups
    const size_t lds = (size_t)K * sizeof(float);
    int rows = 1;                                              // dW: R = N is a multiple of 4
    if (!dx) for (rows = 16; rows > 1 && (size_t)rows * lds > 49152; rows /= 2) {}
    const int64_t rgroups = (d.R + rows - 1) / rows;
    int64_t slices = rgroups >= 2048 ? 1 : (2048 + rgroups - 1) / rgroups;
    const int64_t groups = (d.S + 255) / 256;
    if (slices > groups) slices = groups;
    if (slices > 65535) slices = 65535;
    d.b_chunk = (int32_t)(((groups + slices - 1) / slices) * 256);
    slices = (d.S + d.b_chunk - 1) / d.b_chunk;
    const dim3 bgrid((unsigned)rgroups, (unsigned)slices);
    if (dx)              hipLaunchKernelGGL((lba_grad_boundary_kernel<true, 1>), bgrid, dim3(256), lds, st, G, V, last_of, out, d);
    else if (rows == 16) hipLaunchKernelGGL((lba_grad_boundary_kernel<false, 16>), bgrid, dim3(256), 16 * lds, st, G, V, last_of, out, d);
    else if (rows == 8)  hipLaunchKernelGGL((lba_grad_boundary_kernel<false, 8>), bgrid, dim3(256), 8 * lds, st, G, V, last_of, out, d);
    else if (rows == 4)  hipLaunchKernelGGL((lba_grad_boundary_kernel<false, 4>), bgrid, dim3(256), 4 * lds, st, G, V, last_of, out, d);
    else if (rows == 2)  hipLaunchKernelGGL((lba_grad_boundary_kernel<false, 2>), bgrid, dim3(256), 2 * lds, st, G, V, last_of, out, d);
    else                 hipLaunchKernelGGL((lba_grad_boundary_kernel<false, 1>), bgrid, dim3(256), lds, st, G, V, last_of, out, d);
    return hipGetLastError() == hipSuccess ? LBA_OK : LBA_ERR_LAUNCH;
}

}  // namespace lba
