// Eq.(2) on the matrix cores with an exactness guard band, shared by the append kernel (keys) and the prefill query
// sketches.  For a tile of up to 64 fp16 vectors in LDS,
//   y~[bit][vec] = sum_j (R16hi + 2^-12 R16mid)[bit][j] x[vec][j]      (v_mfma_f32_16x16x32_f16, fp32 accumulation)
// differs from the pinned fp32 multiply-add chain's value by less than guard[bit] ||x||_2 (bound derived where the
// pieces of R are made), so sign(y~) IS the chain's bit wherever |y~| exceeds that; the few bits inside the band are
// recomputed with the chain itself.  fp16 subnormals in x enter the matrix cores as they are (kernels run with fp16
// denormals enabled; a parity test feeds inputs in that range).
// fp32 vectors take the same route after stage_f32_tile has scaled each by a power of two (the sign of the projection
// and the chain's rounding are invariant under it) and split it into two fp16 pieces, x s ~ xh + 2^-12 xm: three MFMAs
// per step instead of two (the product of the two low pieces is dropped and priced into guard32), and the chain reads
// the original fp32 vector.
#pragma once

#include <hip/hip_fp16.h>

#include "internal.h"

namespace h1bkv {
namespace {

typedef _Float16 proj_f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 proj_f16x2 __attribute__((ext_vector_type(2)));
typedef float proj_f32x4 __attribute__((ext_vector_type(4)));
typedef float proj_f32x16 __attribute__((ext_vector_type(16)));

constexpr int kProjTile = 64;      // vectors per tile
constexpr int kProjThreads = 256;

// The thread index in a register the compiler cannot prove invariant across the caller's tile loop: addresses derived
// from it are recomputed per tile (a few instructions) instead of being hoisted out of the loop into registers that
// spill -- and a spill reload waits for every global load in flight.
__device__ __forceinline__ int per_tile_index(int v) {
    asm volatile("" : "+v"(v));
    return v;
}

__device__ __forceinline__ void proj_load8(const __half *p, float *out) {
    const uint4 raw = *reinterpret_cast<const uint4 *>(p);
    const __half2 *h = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float2 f = __half22float2(h[i]);
        out[2 * i] = f.x;
        out[2 * i + 1] = f.y;
    }
}

// Splits a tile of fp32 vectors for project_tile_mfma<D, true>: row(v) -> the vector's address or nullptr.  Per vector
//   s = 2^k with max |x| s in [2^12, 2^13)  (exact in fp32; fp16 pieces then neither overflow nor lose the large elements),
//   xh = fp16(x s),  xm = fp16((x s - xh) 2^12)  (the difference is exact),  band = ||x s||_2 (1 + 2^-16).
// A vector whose largest magnitude lies outside [2^-100, 2^100] (or is not finite) gets band = +inf: every one of its
// bits then counts as uncertain and comes from the chain, whose own rounding is no longer purely relative out there.
// Must be called by all 256 threads (shuffles); the caller's barrier publishes the tile.
template <int D, typename Row>
__device__ __forceinline__ void stage_f32_tile(Row row, int tile, __half *xh, __half *xm, int stride, float *band) {
    constexpr int LPR = D / 8;                                 // lanes per vector, 8 elements each
    const int tid = per_tile_index(threadIdx.x);
    for (int e0 = 0; e0 < kProjTile * D; e0 += kProjThreads * 8) {
        const int e = e0 + tid * 8, v = e / D, ch = e % D;
        const float *src = v < tile ? row(v) : nullptr;
        float x[8];
        if (src) {
            const float4 a = *reinterpret_cast<const float4 *>(src + ch), b = *reinterpret_cast<const float4 *>(src + ch + 4);
            x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = 0.0f;
        }
        uint32_t m = 0u;                                       // largest magnitude, compared as bits (non-negative floats order like integers)
#pragma unroll
        for (int i = 0; i < 8; ++i) m = max(m, __float_as_uint(x[i]) & 0x7FFFFFFFu);
#pragma unroll
        for (int o = 1; o < LPR; o <<= 1) m = max(m, (uint32_t)__shfl_xor((int)m, o));
        const int ex = (int)(m >> 23);                         // biased exponent of the largest element
        const bool in_range = ex >= 27 && ex <= 227;           // 2^-100 .. 2^100 (also excludes inf and NaN)
        const float sc = in_range ? __uint_as_float((uint32_t)(266 - ex) << 23) : (m == 0u ? 1.0f : 0.0f);
        float ss = 0.0f;
        uint32_t ph[4], pm[4];
#pragma unroll
        for (int i = 0; i < 8; i += 2) {
            const float s0 = x[i] * sc, s1 = x[i + 1] * sc;
            ss = fmaf(s0, s0, ss);
            ss = fmaf(s1, s1, ss);
            const __half h0 = __float2half_rn(s0), h1 = __float2half_rn(s1);
            const __half m0 = __float2half_rn((s0 - __half2float(h0)) * 4096.0f), m1 = __float2half_rn((s1 - __half2float(h1)) * 4096.0f);
            ph[i / 2] = (uint32_t)__half_as_ushort(h0) | ((uint32_t)__half_as_ushort(h1) << 16);
            pm[i / 2] = (uint32_t)__half_as_ushort(m0) | ((uint32_t)__half_as_ushort(m1) << 16);
        }
#pragma unroll
        for (int o = 1; o < LPR; o <<= 1) ss += __shfl_xor(ss, o);
        if (v < tile) {
            *reinterpret_cast<uint4 *>(xh + (size_t)v * stride + ch) = make_uint4(ph[0], ph[1], ph[2], ph[3]);
            *reinterpret_cast<uint4 *>(xm + (size_t)v * stride + ch) = make_uint4(pm[0], pm[1], pm[2], pm[3]);
            if (ch == 0) band[v] = (in_range || m == 0u) ? sqrtf(ss) * 1.0000153f : __uint_as_float(0x7F800000u);
        }
    }
}

// xs: the tile, row-major, `stride` halves per row (rows 16-byte aligned, stride a multiple of 8 and not of 64, so
//     that 16-byte reads down a column spread over the LDS banks);  valid(v): whether row v holds a vector.
// F32IN: the vectors are fp32 and were split by stage_f32_tile into xs (high pieces), xm (low pieces) and band (which
//     this function otherwise computes itself); source(v) is the original vector for the chain.
// w32, unsure: [kProjTile][16] 32-bit words in LDS, all zero on entry.  On return (after the caller's next barrier)
//     w32[v][0 .. b/32) holds the packed sketch of vector v.  Must be called by all 256 threads; contains barriers.
// between(): called once by every thread after the matrix-core phase, before the chain: the place to issue loads whose
//     latency the (few, long) chains can hide without their registers being held through the matrix-core phase.
template <int D, bool F32IN, typename Valid, typename Between, typename Source>
__device__ __forceinline__ void project_tile_mfma(const PoolView &pv, const __half *xs, const __half *xm, float *band_s, int stride,
                                                  int tile, Valid valid, uint32_t *w32, uint32_t *unsure, Between between,
                                                  Source source) {
    const int tid = per_tile_index(threadIdx.x), lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, kb = lane >> 4;
    const int n_tb = (tile + 15) / 16;
    const int n_bb = pv.sketch_bits / 16;                           // blocks of 16 sketch bits: wave, wave + 4, ...
    const float *guard = F32IN ? pv.guard + pv.sketch_bits : pv.guard;      // the fp32-input band follows the fp16-input one
    struct AOperands {
        uint4 hi[D / 32], mid[D / 32];
        float g[4];
    };
    auto load_a = [&](AOperands &A, int bb) {
        const size_t arow = (size_t)(16 * bb + n) * D + 8 * kb;
#pragma unroll
        for (int jb = 0; jb < D / 32; ++jb) {
            A.hi[jb] = *reinterpret_cast<const uint4 *>(pv.R16hi + arow + 32 * jb);
            A.mid[jb] = *reinterpret_cast<const uint4 *>(pv.R16mid + arow + 32 * jb);
        }
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) A.g[jj] = guard[16 * bb + 4 * kb + jj];
    };
    // the first block's pieces of R are requested before anything else: their latency runs behind the norms
    AOperands A;
    if (wave < n_bb) load_a(A, wave);
    // ---- 2-norm of every vector, once per tile: four threads per vector, 32 elements each ----
    if constexpr (!F32IN) {
        const int v = tid >> 2, part = tid & 3;
        float ss = 0.0f;
        if (v < tile && valid(v)) {
            for (int j = part * 8; j < D; j += 32) {
                float x[8];
                proj_load8(xs + (size_t)v * stride + j, x);
#pragma unroll
                for (int e = 0; e < 8; ++e) ss = fmaf(x[e], x[e], ss);
            }
        }
        ss += __shfl_xor(ss, 1);
        ss += __shfl_xor(ss, 2);
        if (part == 0) band_s[v] = sqrtf(ss) * 1.0000153f;    // fp32 rounding of the sum and the root stays below 2^-16
    }
    __syncthreads();
    for (int bb = wave; bb < n_bb; bb += 4) {
        if (bb != wave) load_a(A, bb);
#pragma unroll 1
        for (int tb = 0; tb < n_tb; ++tb) {
            proj_f32x4 yh = {0.f, 0.f, 0.f, 0.f}, ym = {0.f, 0.f, 0.f, 0.f};
            const int v = 16 * tb + n;
#pragma unroll
            for (int jb = 0; jb < D / 32; ++jb) {
                const proj_f16x8 Bx = *reinterpret_cast<const proj_f16x8 *>(xs + (size_t)v * stride + 32 * jb + 8 * kb);
                yh = __builtin_amdgcn_mfma_f32_16x16x32_f16(*reinterpret_cast<const proj_f16x8 *>(&A.hi[jb]), Bx, yh, 0, 0, 0);
                ym = __builtin_amdgcn_mfma_f32_16x16x32_f16(*reinterpret_cast<const proj_f16x8 *>(&A.mid[jb]), Bx, ym, 0, 0, 0);
                if constexpr (F32IN) {
                    const proj_f16x8 Bm = *reinterpret_cast<const proj_f16x8 *>(xm + (size_t)v * stride + 32 * jb + 8 * kb);
                    ym = __builtin_amdgcn_mfma_f32_16x16x32_f16(*reinterpret_cast<const proj_f16x8 *>(&A.hi[jb]), Bm, ym, 0, 0, 0);
                }
            }
            const float band = band_s[v];
            // element jj of this lane: bit 16 bb + 4 kb + jj of vector v
            if (v < tile && valid(v)) {
                uint32_t sbits = 0u, ubits = 0u;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const float y = fmaf(ym[jj], 0.000244140625f, yh[jj]);
                    sbits |= (y >= 0.0f ? 1u : 0u) << jj;
                    ubits |= (fabsf(y) > A.g[jj] * band ? 0u : 1u) << jj;        // also catches a NaN
                }
                const int sh = 16 * (bb & 1) + 4 * kb;
                atomicOr(&w32[v * 16 + (bb >> 1)], sbits << sh);
                if (ubits) atomicOr(&unsure[v * 16 + (bb >> 1)], ubits << sh);
            }
        }
    }
    __syncthreads();
    between();
    // ---- the chain for the bits inside the guard band: one thread per (vector, 32 bits) ----
    const int W32 = pv.sketch_bits / 32;
    for (int item = tid; item < tile * W32; item += kProjThreads) {
        const int v = item / W32, w = item - v * W32;
        if (!valid(v)) continue;
        uint32_t m = unsure[v * 16 + w];
        if (m == 0u) continue;
        uint32_t cur = w32[v * 16 + w];
        while (m) {
            const int p = __ffs(m) - 1;
            m &= m - 1u;
            const float *row = pv.R + (size_t)(32 * w + p) * D;
            float y = 0.0f;
            // 32 elements of the row at a time: all their loads are in flight before the (sequential) chain runs
#pragma unroll 1
            for (int j0 = 0; j0 < D; j0 += 32) {
                float4 rr[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) rr[q] = *reinterpret_cast<const float4 *>(row + j0 + 4 * q);
#pragma unroll
                for (int q = 0; q < 8; q += 2) {
                    float kk[8];
                    if constexpr (F32IN) {
                        const float *xv = source(v) + j0 + 4 * q;
                        const float4 a = *reinterpret_cast<const float4 *>(xv), b = *reinterpret_cast<const float4 *>(xv + 4);
                        kk[0] = a.x; kk[1] = a.y; kk[2] = a.z; kk[3] = a.w; kk[4] = b.x; kk[5] = b.y; kk[6] = b.z; kk[7] = b.w;
                    } else {
                        proj_load8(xs + (size_t)v * stride + j0 + 4 * q, kk);
                    }
                    y = __builtin_fmaf(rr[q].x, kk[0], y); y = __builtin_fmaf(rr[q].y, kk[1], y);
                    y = __builtin_fmaf(rr[q].z, kk[2], y); y = __builtin_fmaf(rr[q].w, kk[3], y);
                    y = __builtin_fmaf(rr[q + 1].x, kk[4], y); y = __builtin_fmaf(rr[q + 1].y, kk[5], y);
                    y = __builtin_fmaf(rr[q + 1].z, kk[6], y); y = __builtin_fmaf(rr[q + 1].w, kk[7], y);
                }
            }
            cur = y >= 0.0f ? (cur | (1u << p)) : (cur & ~(1u << p));
        }
        w32[v * 16 + w] = cur;
    }
}


// ------------------------------------------------------------------------------------------------------------------
// Resident form, for d <= 128: a whole kernel body.
//  * A wave keeps the pieces of R for up to 256 / d blocks of 16 bits in registers for the life of the workgroup (64
//    registers): a tile costs no loads of R, and each 16-byte read of the tile from LDS feeds all of the wave's blocks.
//    A workgroup so covers 64 * 256 / d sketch bits; wider sketches are cut into `n_parts` parts of that width, each
//    computed by workgroups of its own (which read the same vectors again: cheaper than re-reading R per tile).
//  * The next tile's fp16 vectors are requested into registers before the current tile's matrix-core phase and deposited
//    into the other of two LDS tiles afterwards (the 2-norms are taken from the registers on the way): the stream from
//    memory does not stop while the workgroup computes, and a tile costs ONE barrier.
//  * A wave assembles the 16-bit blocks it owns with two lane exchanges and stores them straight to global memory: no
//    LDS words, no atomics, no zeroing.
//  * Words with bits inside the guard band are not recomputed on the spot (one lane walking a chain of dependent loads
//    while its workgroup waits) but entered into an LDS list that all threads drain together -- looked at every 16 tiles,
//    drained when half full and after the last tile -- patching the stored words with atomics; a full list falls back to
//    recomputing on the spot.
// Rows (the caller's description of its tiles of up to 64 vectors; tile indices are the caller's):
//   int rows_in(long tile)                      number of row slots of the tile
//   size_t src(long tile, int rl)               element offset of the vector from `base`, or kProjNoRow for an empty slot
//   int page_request(long tile, int rl)         a value the destination depends on, loaded from global memory one tile
//                                               ahead of its use (the page id; 0 if there is none); valid slots only
//   uint32_t *dst(long tile, int rl, int page)  where the vector's sketch goes (32-bit words); valid slots only
// ------------------------------------------------------------------------------------------------------------------

constexpr size_t kProjNoRow = ~(size_t)0;

// Division of a 32-bit index by a divisor that is fixed for the launch, for the Rows descriptions: the quotient from the
// high half of a product with floor((2^32 - 1) / d), which falls short by at most two, corrected by comparing remainders.
// (The generic division is some thirty-five vector instructions, and one wave of the workgroup does all of them.)
struct ProjDiv {
    uint32_t d, m;
    __device__ explicit ProjDiv(uint32_t div) : d(div), m(0xFFFFFFFFu / div) {}
    __device__ void divmod(uint32_t x, uint32_t &q, uint32_t &r) const {
        q = __umulhi(x, m);
        r = x - q * d;
        if (r >= d) { r -= d; ++q; }
        if (r >= d) { r -= d; ++q; }
    }
};

// OR over the four 16-lane rows of a wave, in every lane: two row exchanges in the register file (v_permlane16_swap,
// v_permlane32_swap: after exchanging rows between two copies of x, the OR of the copies joins two different rows at every
// position), no trip through the LDS crossbar.
__device__ __forceinline__ uint32_t proj_or_rows(uint32_t x) {
    typedef unsigned pair_t __attribute__((ext_vector_type(2)));
    const pair_t a = __builtin_amdgcn_permlane16_swap(x, x, false, false);
    x = a.x | a.y;
    const pair_t b = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return b.x | b.y;
}

// Sum over aligned groups of LANES (8 or 16) neighbouring lanes, in every lane of the group, by DPP: the two exchanges
// inside a quad, then the mirror of 8 lanes (quads are uniform by then), then the mirror of 16.
template <int LANES>
__device__ __forceinline__ float proj_sum_lanes(float s) {
    static_assert(LANES == 8 || LANES == 16, "row-local DPP patterns");
    s += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, s), 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
    s += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, s), 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
    s += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, s), 0x141, 0xF, 0xF, false));  // row_half_mirror
    if (LANES == 16) s += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, s), 0x140, 0xF, 0xF, false));  // row_mirror
    return s;
}

template <int D>
struct ProjResident {
    static constexpr int NB = 256 / D;          // blocks of 16 bits per wave
    uint4 hi[NB][D / 32], mid[NB][D / 32];
    float g[NB][4];
};

// Parts a sketch of `sketch_bits` bits is cut into (64 * 256 / D bits per workgroup), 0 if there is no resident form.
template <int D>
__host__ __device__ constexpr int proj_resident_parts(int sketch_bits) {
    return D > 128 ? 0 : (sketch_bits / 64 + 256 / D - 1) / (256 / D);
}

// W: blocks per wave;  block0: the wave's first block
template <int D, bool F32IN>
__device__ __forceinline__ void load_resident(const PoolView &pv, ProjResident<D> &res, int W, int block0) {
    const int lane = threadIdx.x & 63, n = lane & 15, kb = lane >> 4;
    const float *guard = F32IN ? pv.guard + pv.sketch_bits : pv.guard;
#pragma unroll
    for (int i = 0; i < ProjResident<D>::NB; ++i) {
        const int bb = block0 + (i < W ? i : 0);                     // (unused slots repeat a valid block: no branch)
        const size_t arow = (size_t)(16 * bb + n) * D + 8 * kb;
#pragma unroll
        for (int jb = 0; jb < D / 32; ++jb) {
            res.hi[i][jb] = *reinterpret_cast<const uint4 *>(pv.R16hi + arow + 32 * jb);
            res.mid[i][jb] = *reinterpret_cast<const uint4 *>(pv.R16mid + arow + 32 * jb);
        }
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) res.g[i][jj] = guard[16 * bb + 4 * kb + jj];
    }
    // The loads are waited for here, once: each register passes through an (empty) assembly statement, after which the
    // compiler no longer counts it as the target of a load in flight.  Without this the first matrix-core instruction of
    // every tile waits for ALL outstanding loads (the counter cannot single out registers loaded before the tile loop) --
    // including the next tile's vectors that have just been requested.
#pragma unroll
    for (int i = 0; i < ProjResident<D>::NB; ++i) {
#pragma unroll
        for (int jb = 0; jb < D / 32; ++jb) {
            asm volatile("" : "+v"(res.hi[i][jb].x), "+v"(res.hi[i][jb].y), "+v"(res.hi[i][jb].z), "+v"(res.hi[i][jb].w));
            asm volatile("" : "+v"(res.mid[i][jb].x), "+v"(res.mid[i][jb].y), "+v"(res.mid[i][jb].z), "+v"(res.mid[i][jb].w));
        }
        asm volatile("" : "+v"(res.g[i][0]), "+v"(res.g[i][1]), "+v"(res.g[i][2]), "+v"(res.g[i][3]));
    }
}

// The resident pieces of R for the 32 x 32 form (d = 128, fp16 vectors, 32 sketch bits per wave): the wave's 32 rows of R
// are the MFMA's rows, the vectors its columns, so that a lane ends up with 16 bits of ONE vector.  Row i of the MFMA is
// sketch bit 16 ((i >> 2) & 1) + 4 (i >> 3) + (i & 3) of the wave's 32: accumulator element e of lane (column n, half h)
// is then bit 16 h + e -- the lane's 16 signs, shifted into a register one v_alignbit each, ARE half-word h of the
// vector's sketch word, stored as they are (no nibble assembly, no exchange between lanes).  The guard test uses the
// largest band factor of the wave's 32 bits: one threshold per vector, compared once against the smallest magnitude.
struct ProjWide {
    uint4 hi[8], mid[8];        // K steps of 16 channels
    float gmax;
};

template <bool F32IN>
__device__ __forceinline__ void load_wide(const PoolView &pv, ProjWide &res, int bit0) {
    const int lane = threadIdx.x & 63, i = lane & 31, hh = lane >> 5;
    const int bit = 16 * ((i >> 2) & 1) + 4 * (i >> 3) + (i & 3);
    const size_t arow = (size_t)(bit0 + bit) * 128 + 8 * hh;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        res.hi[s] = *reinterpret_cast<const uint4 *>(pv.R16hi + arow + 16 * s);
        res.mid[s] = *reinterpret_cast<const uint4 *>(pv.R16mid + arow + 16 * s);
    }
    float g = (F32IN ? pv.guard + pv.sketch_bits : pv.guard)[bit0 + i];
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) g = fmaxf(g, __shfl_xor(g, o));
    res.gmax = g;
    // (waited for here, once: see load_resident)
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        asm volatile("" : "+v"(res.hi[s].x), "+v"(res.hi[s].y), "+v"(res.hi[s].z), "+v"(res.hi[s].w));
        asm volatile("" : "+v"(res.mid[s].x), "+v"(res.mid[s].y), "+v"(res.mid[s].z), "+v"(res.mid[s].w));
    }
    asm volatile("" : "+v"(res.gmax));
}

// One entry per stored 32-bit sketch word that holds bits inside the guard band.
struct ProjFix {
    const void *src;       // the vector, in its boundary dtype, in global memory
    uint32_t *dst;         // the sketch word in global memory
    uint32_t mask;         // the bits to recompute
    uint32_t word;         // index of the word within the sketch: its bits are rows 32 word .. 32 word + 31 of R
};
constexpr int kProjFixCap = 256;
constexpr int kProjDrainEvery = 16;    // tiles between two looks at the list (a barrier each): about 4 entries per tile at d = b = 128
struct ProjFixList {
    int n;                 // entries requested so far (may run past the capacity: those were recomputed on the spot)
    ProjFix item[kProjFixCap];
};

// The pinned chain of Eq.(2) for row `row` of R and the vector x (boundary dtype T, global memory): y = fma(R[j], x[j], y),
// j ascending.  16 elements at a time: their loads are in flight together before the sequential chain runs (the callers
// hold the resident pieces of R next to this, so no more than that).
template <int D, typename T>
__device__ __forceinline__ float proj_chain(const float *row, const T *x) {
    float y = 0.0f;
#pragma unroll 1
    for (int j0 = 0; j0 < D; j0 += 16) {
        float4 rr[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) rr[q] = *reinterpret_cast<const float4 *>(row + j0 + 4 * q);
#pragma unroll
        for (int q = 0; q < 4; q += 2) {
            float kk[8];
            if constexpr (sizeof(T) == 2) {
                proj_load8(reinterpret_cast<const __half *>(x) + j0 + 4 * q, kk);
            } else {
                const float4 a = *reinterpret_cast<const float4 *>(x + j0 + 4 * q), b = *reinterpret_cast<const float4 *>(x + j0 + 4 * q + 4);
                kk[0] = a.x; kk[1] = a.y; kk[2] = a.z; kk[3] = a.w; kk[4] = b.x; kk[5] = b.y; kk[6] = b.z; kk[7] = b.w;
            }
            y = __builtin_fmaf(rr[q].x, kk[0], y); y = __builtin_fmaf(rr[q].y, kk[1], y);
            y = __builtin_fmaf(rr[q].z, kk[2], y); y = __builtin_fmaf(rr[q].w, kk[3], y);
            y = __builtin_fmaf(rr[q + 1].x, kk[4], y); y = __builtin_fmaf(rr[q + 1].y, kk[5], y);
            y = __builtin_fmaf(rr[q + 1].z, kk[6], y); y = __builtin_fmaf(rr[q + 1].w, kk[7], y);
        }
    }
    return y;
}

// The bits `mask` of a word whose bit p is row `row0 + p` of R, recomputed with the chain: returns the bits to set
// (the others of `mask` are to be cleared).
template <int D, typename T>
__device__ __forceinline__ uint32_t proj_chain_bits(const PoolView &pv, int row0, uint32_t mask, const T *x) {
    uint32_t set = 0u;
    while (mask) {
        const int p = __ffs(mask) - 1;
        mask &= mask - 1u;
        if (proj_chain<D, T>(pv.R + (size_t)(row0 + p) * D, x) >= 0.0f) set |= 1u << p;
    }
    return set;
}

// Drains the list: D / 16 neighbouring lanes per entry, lane c holding elements [16 c, 16 c + 16) of the vector and of the
// row of R, so that all loads of a chain are in flight at once; the chain value then travels from lane to lane (the
// order of the multiply-adds is the pinned one).  Called by all threads between two barriers.
template <int D, typename T>
__device__ __forceinline__ void proj_drain(const PoolView &pv, const ProjFixList &list) {
    constexpr int LPE = D / 16;
    const int n_fix = list.n < kProjFixCap ? list.n : kProjFixCap;
    const int tid = per_tile_index(threadIdx.x), lane = tid & 63, c = tid % LPE;
    for (int e0 = 0; e0 < n_fix; e0 += kProjThreads / LPE) {
        const int e = e0 + tid / LPE;
        const bool have = e < n_fix;
        const ProjFix f = list.item[have ? e : 0];
        uint32_t m = have ? f.mask : 0u, set = 0u;
        float xk[16];
        {
            const T *x = static_cast<const T *>(f.src) + 16 * c;
            if constexpr (sizeof(T) == 2) {
                proj_load8(reinterpret_cast<const __half *>(x), xk);
                proj_load8(reinterpret_cast<const __half *>(x) + 8, xk + 8);
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 a = *reinterpret_cast<const float4 *>(x + 4 * q);
                    xk[4 * q] = a.x; xk[4 * q + 1] = a.y; xk[4 * q + 2] = a.z; xk[4 * q + 3] = a.w;
                }
            }
        }
        while (__any(m != 0u)) {                             // (entries with several bits are rare)
            const int p = m ? __ffs(m) - 1 : 0;
            const float *row = pv.R + (size_t)(32 * (int)f.word + p) * D + 16 * c;
            float4 rr[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) rr[q] = *reinterpret_cast<const float4 *>(row + 4 * q);
            float y = 0.0f;
#pragma unroll 1
            for (int stage = 0; stage < LPE; ++stage) {
                float z = y;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    z = __builtin_fmaf(rr[q].x, xk[4 * q], z); z = __builtin_fmaf(rr[q].y, xk[4 * q + 1], z);
                    z = __builtin_fmaf(rr[q].z, xk[4 * q + 2], z); z = __builtin_fmaf(rr[q].w, xk[4 * q + 3], z);
                }
                // the value after this stage's 16 elements is the one computed by lane `stage` of the group
                y = __shfl(z, (lane & ~(LPE - 1)) + stage);
            }
            if (m) {
                if (y >= 0.0f) set |= 1u << p;
                m &= m - 1u;
            }
        }
        if (have && c == 0) {
            if (set) atomicOr(f.dst, set);
            if (f.mask & ~set) atomicAnd(f.dst, ~(f.mask & ~set));
        }
    }
}

// part, n_parts: which part of the sketch bits this workgroup computes (see above).
// WIDE: the 32 x 32 form (ProjWide); needs d = 128, fp16 vectors and 32 sketch bits per wave (128 per workgroup).
template <int D, typename T, bool WIDE, typename Rows>
__device__ __forceinline__ void resident_sketch_tiles(const PoolView &pv, const T *base, const Rows &rows, long first, long step,
                                                      long n_tiles, int part, int n_parts) {
    constexpr bool F32 = sizeof(T) == 4;
    static_assert(!WIDE || (D == 128 && !F32), "the 32 x 32 form is written for 128 fp16 channels");
    constexpr int STRIDE = D + 8, NJ = D / 32, NB = ProjResident<D>::NB;
    constexpr int NBUF = F32 ? 1 : 2;                       // (two piece tiles per fp32 tile: one buffer, one more barrier)
    constexpr int RPP = kProjThreads * 8 / D;               // rows covered by one 16-byte piece per thread
    static_assert(D == 64 || D == 128, "up to four 16-byte pieces per thread and tile");
    __shared__ __attribute__((aligned(16))) __half xs[NBUF][(F32 ? 2 : 1) * kProjTile * STRIDE];
    __shared__ float band_s[NBUF][kProjTile];
    __shared__ size_t src_s[3][kProjTile];                  // this tile's, the next one's, and the previous one's (still read by slow waves)
    __shared__ uint32_t *dst_s[2][kProjTile];
    __shared__ ProjFixList fixes;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 15, kb = lane >> 4;
    const int W = (pv.sketch_bits >> 6) / n_parts;          // blocks of 16 bits per wave
    const int block0 = (4 * part + wave) * W;               // the wave's first block
    const int pre_row = tid * 8 / D, pre_ch = tid * 8 % D;  // this thread's pieces: elements [pre_ch, pre_ch + 8) of rows pre_row + k RPP
    if (tid == 0) fixes.n = 0;
    // (named registers, not an array: an array of these stayed in scratch memory.  Empty slots read the first vector:
    // no branch around a load -- the compiler makes every load behind a branch wait for the ones before it.)
    [[maybe_unused]] uint4 pre0, pre1, pre2, pre3;
#define H1BKV_PROJ_REQUEST_ONE(K, REG, SB)                                                                  \
    if constexpr (K * RPP < kProjTile) {                                                                    \
        const size_t off = src_s[SB][pre_row + K * RPP];                                                    \
        REG = *reinterpret_cast<const uint4 *>(base + (off == kProjNoRow ? 0 : off) + pre_ch);              \
    }
#define H1BKV_PROJ_REQUEST(SB)                                                                              \
    do {                                                                                                    \
        H1BKV_PROJ_REQUEST_ONE(0, pre0, SB) H1BKV_PROJ_REQUEST_ONE(1, pre1, SB)                             \
        H1BKV_PROJ_REQUEST_ONE(2, pre2, SB) H1BKV_PROJ_REQUEST_ONE(3, pre3, SB)                             \
    } while (0)
    // deposit a piece into the LDS tile and leave its row's 2-norm (times 1 + 2^-16: above the fp32 rounding of the sum
    // and the root -- the hardware root, an ulp off at most: the correctly rounded one is an 18-instruction sequence that
    // every lane of the wave would run four times per tile) in band_s; the D / 8 lanes of a row are neighbours
#define H1BKV_PROJ_DEPOSIT_ONE(K, REG, BUF)                                                                 \
    if constexpr (K * RPP < kProjTile) {                                                                    \
        const int rl = pre_row + K * RPP;                                                                   \
        *reinterpret_cast<uint4 *>(&xs[BUF][rl * STRIDE + pre_ch]) = REG;                                   \
        const proj_f16x2 *h2 = reinterpret_cast<const proj_f16x2 *>(&REG);                                  \
        float ss = 0.0f;                                                                                    \
        _Pragma("unroll") for (int e = 0; e < 4; ++e) ss = __builtin_amdgcn_fdot2(h2[e], h2[e], ss, false); \
        ss = proj_sum_lanes<D / 8>(ss);                                                                     \
        if (pre_ch == 0) band_s[BUF][rl] = __builtin_amdgcn_sqrtf(ss) * 1.0000153f;                         \
    }
    long t = first;
    int page = 0;
    if (tid < kProjTile) src_s[0][tid] = (t < n_tiles && tid < rows.rows_in(t)) ? rows.src(t, tid) : kProjNoRow;
    __syncthreads();
    if (t < n_tiles) {
        if (tid < kProjTile && src_s[0][tid] != kProjNoRow) page = rows.page_request(t, tid);
        if constexpr (!F32) H1BKV_PROJ_REQUEST(0);
    }
    // (after the first tile's requests: the two round trips overlap, which is most of a short launch's time)
    [[maybe_unused]] ProjResident<D> res;
    [[maybe_unused]] ProjWide wres;
    if constexpr (WIDE) load_wide<F32>(pv, wres, 16 * block0);
    else load_resident<D, F32>(pv, res, W, block0);
    for (int it = 0;; t += step, ++it) {
        const bool more = t < n_tiles;
        if (!more || it % kProjDrainEvery == kProjDrainEvery - 1) {
            __syncthreads();                                 // the stores and the entries of the tiles so far are complete
            if (fixes.n > 0 && (!more || fixes.n >= kProjFixCap / 2)) {
                proj_drain<D, T>(pv, fixes);
                __syncthreads();
                if (tid == 0) fixes.n = 0;                   // (the tile's barrier below comes before the next entries)
            }
        }
        if (!more) break;
        const int buf = NBUF == 2 ? (it & 1) : 0, sb = it % 3, sb1 = (it + 1) % 3;
        const int n_here = rows.rows_in(t);
        const long t1 = t + step;
        // ---- before the barrier: this tile into LDS, its destinations, the next tile's sources ----
        if constexpr (F32) {
            __syncthreads();                                 // one tile buffer: the previous tile's readers are done
            stage_f32_tile<D>(
                [&](int rl) { return src_s[sb][rl] != kProjNoRow ? reinterpret_cast<const float *>(base + src_s[sb][rl]) : nullptr; }, n_here,
                &xs[0][0], &xs[0][kProjTile * STRIDE], STRIDE, &band_s[0][0]);
        } else {
            H1BKV_PROJ_DEPOSIT_ONE(0, pre0, buf) H1BKV_PROJ_DEPOSIT_ONE(1, pre1, buf)
            H1BKV_PROJ_DEPOSIT_ONE(2, pre2, buf) H1BKV_PROJ_DEPOSIT_ONE(3, pre3, buf)
        }
        if (tid < kProjTile) {
            dst_s[it & 1][tid] = src_s[sb][tid] != kProjNoRow ? rows.dst(t, tid, page) : nullptr;
            src_s[sb1][tid] = (t1 < n_tiles && tid < rows.rows_in(t1)) ? rows.src(t1, tid) : kProjNoRow;
        }
        __syncthreads();
        // ---- after it: the next tile's requests, then the matrix cores ----
        if (t1 < n_tiles) {
            if (tid < kProjTile && src_s[sb1][tid] != kProjNoRow) page = rows.page_request(t1, tid);
            if constexpr (!F32) H1BKV_PROJ_REQUEST(sb1);
        }
        const __half *xt = &xs[buf][0];
        [[maybe_unused]] const __half *xmt = &xs[buf][F32 ? kProjTile * STRIDE : 0];
        if constexpr (WIDE) {
#pragma unroll 1
            for (int vg = 0; vg < (n_here + 31) / 32; ++vg) {
                const int v = 32 * vg + (lane & 31), hh = lane >> 5;
                proj_f32x16 yh, ym;
#pragma unroll
                for (int e = 0; e < 16; ++e) yh[e] = ym[e] = 0.0f;
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    const proj_f16x8 Bx = *reinterpret_cast<const proj_f16x8 *>(xt + (size_t)v * STRIDE + 16 * ks + 8 * hh);
                    yh = __builtin_amdgcn_mfma_f32_32x32x16_f16(*reinterpret_cast<const proj_f16x8 *>(&wres.hi[ks]), Bx, yh, 0, 0, 0);
                    ym = __builtin_amdgcn_mfma_f32_32x32x16_f16(*reinterpret_cast<const proj_f16x8 *>(&wres.mid[ks]), Bx, ym, 0, 0, 0);
                }
                const float thr = wres.gmax * band_s[buf][v];
                const size_t my_src = src_s[sb][v];
                const bool live = my_src != kProjNoRow;
                // element e of this lane: bit 16 block0 + 16 hh + e of vector v.  The sign is read off the float's bit
                // pattern: -0.0 would come out wrong, but a zero lies inside every band and is recomputed.
                float y[16];
#pragma unroll
                for (int e = 0; e < 16; ++e) y[e] = fmaf(ym[e], 0.000244140625f, yh[e]);
                uint32_t neg = 0u;
#pragma unroll
                for (int e = 15; e >= 0; --e) neg = __builtin_amdgcn_alignbit(neg, __float_as_uint(y[e]), 31);   // (neg << 1) | sign
                float worst = fminf(fabsf(y[0]), fabsf(y[1]));
#pragma unroll
                for (int e = 2; e < 16; e += 2) worst = fminf(fminf(worst, fabsf(y[e])), fabsf(y[e + 1]));
                uint32_t bits16 = ~neg & 0xFFFFu;
                uint32_t *out = live ? dst_s[it & 1][v] : nullptr;
                const int word = block0 >> 1;                                  // the wave's 32 bits are this word of the sketch
                if (__any(live && !(worst > thr))) {                           // uniform, rare; also catches a NaN
                    uint32_t ub = 0u;
#pragma unroll
                    for (int e = 0; e < 16; ++e) ub |= (fabsf(y[e]) > thr ? 0u : 1u) << e;
                    if (live && ub) {
                        const T *x = base + my_src;
                        const uint32_t mask = ub << (16 * hh);
                        const int slot = atomicAdd(&fixes.n, 1);
                        if (slot < kProjFixCap) {
                            fixes.item[slot] = ProjFix{x, out + word, mask, (uint32_t)word};
                        } else {
                            const uint32_t set = proj_chain_bits<D, T>(pv, 32 * word, mask, x);
                            bits16 = (bits16 & ~ub) | ((set >> (16 * hh)) & ub);
                        }
                    }
                }
                // (a global address that came through LDS: see the note at the stores of the 16 x 16 form)
                if (live) *((__attribute__((address_space(1))) uint16_t *)(out + word) + hh) = (uint16_t)bits16;
            }
        } else
#pragma unroll 1
        for (int tb = 0; tb < (n_here + 15) / 16; ++tb) {
            const int v = 16 * tb + n;
            proj_f16x8 Bx[NJ];
            [[maybe_unused]] proj_f16x8 Bm[F32 ? NJ : 1];
#pragma unroll
            for (int jb = 0; jb < NJ; ++jb) {
                Bx[jb] = *reinterpret_cast<const proj_f16x8 *>(xt + (size_t)v * STRIDE + 32 * jb + 8 * kb);
                if constexpr (F32) Bm[jb] = *reinterpret_cast<const proj_f16x8 *>(xmt + (size_t)v * STRIDE + 32 * jb + 8 * kb);
            }
            const float band = band_s[buf][v];
            const size_t my_src = src_s[sb][v];
            const bool live = my_src != kProjNoRow;
            // the wave's blocks as 32-bit words: block i sits in half i & 1 of word i >> 1; this lane's nibble at 4 kb
            uint32_t sw0 = 0u, sw1 = 0u, uw0 = 0u, uw1 = 0u;
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                if (i >= W) break;                                         // uniform
                proj_f32x4 yh = {0.f, 0.f, 0.f, 0.f}, ym = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int jb = 0; jb < NJ; ++jb) {
                    yh = __builtin_amdgcn_mfma_f32_16x16x32_f16(*reinterpret_cast<const proj_f16x8 *>(&res.hi[i][jb]), Bx[jb], yh, 0, 0, 0);
                    ym = __builtin_amdgcn_mfma_f32_16x16x32_f16(*reinterpret_cast<const proj_f16x8 *>(&res.mid[i][jb]), Bx[jb], ym, 0, 0, 0);
                    if constexpr (F32)
                        ym = __builtin_amdgcn_mfma_f32_16x16x32_f16(*reinterpret_cast<const proj_f16x8 *>(&res.hi[i][jb]), Bm[jb], ym, 0, 0, 0);
                }
                // element jj of this lane: bit 16 (block0 + i) + 4 kb + jj of vector v.  The sign is read off the float's
                // bit pattern: -0.0 would come out wrong, but a zero lies inside every band and is recomputed.
                float margin[4];
                uint32_t sbits = 0u;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const float y = fmaf(ym[jj], 0.000244140625f, yh[jj]);
                    margin[jj] = fmaf(-res.g[i][jj], band, fabsf(y));      // one rounding: positive only if |y| > g band
                    sbits |= (__float_as_uint(y) >> 31) << jj;
                }
                const int sh = 16 * (i & 1) + 4 * kb;
                if (i < 2) sw0 |= (sbits ^ 0xFu) << sh;
                else sw1 |= (sbits ^ 0xFu) << sh;
                const float worst = fminf(fminf(margin[0], margin[1]), fminf(margin[2], margin[3]));
                if (__any(live && !(worst > 0.0f))) {                      // uniform, rare; also catches a NaN
                    uint32_t ubits = 0u;
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) ubits |= (margin[jj] > 0.0f ? 0u : 1u) << jj;
                    if (i < 2) uw0 |= ubits << sh;
                    else uw1 |= ubits << sh;
                }
            }
            // the four lanes of a vector (kb = 0..3) hold a nibble of every block each: OR them together
            sw0 = proj_or_rows(sw0);
            if (NB > 2 && W > 2) sw1 = proj_or_rows(sw1);
            if (__any(live && (uw0 | uw1) != 0u)) {
                uw0 = proj_or_rows(uw0);
                if (NB > 2 && W > 2) uw1 = proj_or_rows(uw1);
            }
            if (kb == 0 && live) {
                uint32_t *out = dst_s[it & 1][v];
                const T *x = base + my_src;
                const int bit0 = 16 * block0;                              // first sketch bit of this wave's blocks
#pragma unroll
                for (int j = 0; j < (NB + 1) / 2; ++j) {
                    if (2 * j >= W) break;                                 // uniform
                    uint32_t word = j == 0 ? sw0 : sw1;
                    const uint32_t mask = j == 0 ? uw0 : uw1;
                    const int row0 = bit0 + 32 * j;                        // bit p of `word` is row row0 + p of R
                    if (mask) {
                        const int slot = atomicAdd(&fixes.n, 1);
                        if (slot < kProjFixCap) {
                            fixes.item[slot] = ProjFix{x, out + (row0 >> 5), mask << (row0 & 31), (uint32_t)(row0 >> 5)};
                        } else {
                            word = (word & ~mask) | proj_chain_bits<D, T>(pv, row0, mask, x);
                        }
                    }
                    // (the pointer came through LDS: told that it is a global address, the compiler emits global stores --
                    // flat ones also count as LDS operations, and the next block's wait for its LDS reads would then wait
                    // for these stores to complete)
                    if (W == 1) *((__attribute__((address_space(1))) uint16_t *)out + block0) = (uint16_t)word;   // one block per wave: half a word
                    else *((__attribute__((address_space(1))) uint32_t *)out + (row0 >> 5)) = word;
                }
            }
        }
    }
#undef H1BKV_PROJ_REQUEST_ONE
#undef H1BKV_PROJ_REQUEST
#undef H1BKV_PROJ_DEPOSIT_ONE
}

}  // namespace
}  // namespace h1bkv
