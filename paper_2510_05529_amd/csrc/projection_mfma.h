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
typedef float proj_f32x4 __attribute__((ext_vector_type(4)));

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
// Resident form, for sketches of at most 64 * (256 / D) bits: a wave keeps the pieces of R for its blocks of 16 bits
// in registers for the life of the workgroup (64 registers), so a tile costs no loads of R at all, every 16-byte read of
// the tile from LDS feeds all of the wave's blocks, and the bits inside the guard band are not recomputed per tile (a
// handful of threads each walking a chain of dependent loads while the others wait at the barrier) but collected in an
// LDS list that all threads drain together, once per many tiles, patching the sketch words in global memory.
// ------------------------------------------------------------------------------------------------------------------

template <int D>
struct ProjResident {
    static constexpr int NB = 256 / D;          // blocks of 16 bits per wave: wave, wave + 4, ...
    uint4 hi[NB][D / 32], mid[NB][D / 32];
    float g[NB][4];
};

template <int D>
__host__ __device__ constexpr bool proj_resident_fits(int sketch_bits) {
    return sketch_bits / 64 <= 256 / D;
}

template <int D, bool F32IN>
__device__ __forceinline__ void load_resident(const PoolView &pv, ProjResident<D> &res) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n = lane & 15, kb = lane >> 4;
    const int W = pv.sketch_bits >> 6;
    const float *guard = F32IN ? pv.guard + pv.sketch_bits : pv.guard;
#pragma unroll
    for (int i = 0; i < ProjResident<D>::NB; ++i) {
        const int bb = i < W ? wave + 4 * i : wave;                  // (unused slots repeat a valid block: no branch)
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
    // including the next tile's vectors the caller has just requested.
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

// One entry per 32-bit sketch word that holds bits inside the guard band.
struct ProjFix {
    const void *src;       // the vector, in its boundary dtype, in global memory
    uint32_t *dst;         // the sketch word in global memory (written by the tile's store before the list is drained)
    uint32_t mask;         // the bits to recompute
    uint32_t word;         // index of the word within the sketch: its bits are rows 32 word .. 32 word + 31 of R
};
constexpr int kProjFixCap = 256;
struct ProjFixList {
    int n;                 // entries requested so far (may run past the capacity: those were recomputed in place)
    ProjFix item[kProjFixCap];
};

// The pinned chain of Eq.(2) for one row of R: y = fma(R[j], x[j], y), j ascending.  load8(j, out): elements j .. j+7 of
// the vector as fp32.  16 elements of the row at a time: their loads are in flight together before the sequential chain
// runs (callers hold the resident pieces of R next to this, so no more than that).
template <int D, typename Load8>
__device__ __forceinline__ float proj_chain(const float *row, Load8 load8) {
    float y = 0.0f;
#pragma unroll 1
    for (int j0 = 0; j0 < D; j0 += 16) {
        float4 rr[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) rr[q] = *reinterpret_cast<const float4 *>(row + j0 + 4 * q);
#pragma unroll
        for (int q = 0; q < 4; q += 2) {
            float kk[8];
            load8(j0 + 4 * q, kk);
            y = __builtin_fmaf(rr[q].x, kk[0], y); y = __builtin_fmaf(rr[q].y, kk[1], y);
            y = __builtin_fmaf(rr[q].z, kk[2], y); y = __builtin_fmaf(rr[q].w, kk[3], y);
            y = __builtin_fmaf(rr[q + 1].x, kk[4], y); y = __builtin_fmaf(rr[q + 1].y, kk[5], y);
            y = __builtin_fmaf(rr[q + 1].z, kk[6], y); y = __builtin_fmaf(rr[q + 1].w, kk[7], y);
        }
    }
    return y;
}

// Recomputes the listed bits with the chain and patches the words.  T: the vectors' boundary dtype.  Called by all 256
// threads between two barriers, after the stores of the tiles the entries belong to; the caller resets list.n afterwards.
template <int D, typename T>
__device__ __forceinline__ void drain_fixes(const PoolView &pv, const ProjFixList &list) {
    const int n = list.n < kProjFixCap ? list.n : kProjFixCap;
    for (int e = per_tile_index(threadIdx.x); e < n; e += kProjThreads) {
        const ProjFix f = list.item[e];
        const T *x = static_cast<const T *>(f.src);
        uint32_t m = f.mask, set = 0u, clear = 0u;
        while (m) {
            const int p = __ffs(m) - 1;
            m &= m - 1u;
            const float y = proj_chain<D>(pv.R + (size_t)(32 * f.word + p) * D, [&](int j, float *out) {
                if constexpr (sizeof(T) == 2) {
                    proj_load8(reinterpret_cast<const __half *>(x) + j, out);
                } else {
                    const float4 a = *reinterpret_cast<const float4 *>(x + j), b = *reinterpret_cast<const float4 *>(x + j + 4);
                    out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w; out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
                }
            });
            if (y >= 0.0f) set |= 1u << p;
            else clear |= 1u << p;
        }
        if (set) atomicOr(f.dst, set);
        if (clear) atomicAnd(f.dst, ~clear);
    }
}

// The tile's projections with resident pieces of R.  Arguments as project_tile_mfma, plus:
//   src(v): the vector's address in global memory (boundary dtype);  dst(v): the address of its first 32-bit sketch word
//   in global memory -- where the caller stores w32[v][..] after its next barrier.
// Words with bits inside the band are entered into `list`; when the list is full they are recomputed here, in w32.
template <int D, bool F32IN, typename Valid, typename Between, typename Src, typename Dst>
__device__ __forceinline__ void project_tile_resident(const PoolView &pv, const ProjResident<D> &res, const __half *xs, const __half *xm,
                                                      float *band_s, int stride, int tile, Valid valid, uint32_t *w32, uint32_t *unsure,
                                                      Between between, Src src, Dst dst, ProjFixList &list) {
    constexpr int NB = ProjResident<D>::NB, NJ = D / 32;
    const int tid = per_tile_index(threadIdx.x), lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, kb = lane >> 4;
    const int W = pv.sketch_bits >> 6;
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
        if (part == 0) band_s[v] = sqrtf(ss) * 1.0000153f;
    }
    __syncthreads();
#pragma unroll 1
    for (int tb = 0; tb < (tile + 15) / 16; ++tb) {
        const int v = 16 * tb + n;
        proj_f16x8 Bx[NJ];
        [[maybe_unused]] proj_f16x8 Bm[F32IN ? NJ : 1];
#pragma unroll
        for (int jb = 0; jb < NJ; ++jb) {
            Bx[jb] = *reinterpret_cast<const proj_f16x8 *>(xs + (size_t)v * stride + 32 * jb + 8 * kb);
            if constexpr (F32IN) Bm[jb] = *reinterpret_cast<const proj_f16x8 *>(xm + (size_t)v * stride + 32 * jb + 8 * kb);
        }
        const float band = band_s[v];
        const bool live = v < tile && valid(v);
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            if (i >= W) break;                                         // uniform
            proj_f32x4 yh = {0.f, 0.f, 0.f, 0.f}, ym = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int jb = 0; jb < NJ; ++jb) {
                yh = __builtin_amdgcn_mfma_f32_16x16x32_f16(*reinterpret_cast<const proj_f16x8 *>(&res.hi[i][jb]), Bx[jb], yh, 0, 0, 0);
                ym = __builtin_amdgcn_mfma_f32_16x16x32_f16(*reinterpret_cast<const proj_f16x8 *>(&res.mid[i][jb]), Bx[jb], ym, 0, 0, 0);
                if constexpr (F32IN)
                    ym = __builtin_amdgcn_mfma_f32_16x16x32_f16(*reinterpret_cast<const proj_f16x8 *>(&res.hi[i][jb]), Bm[jb], ym, 0, 0, 0);
            }
            // element jj of this lane: bit 16 bb + 4 kb + jj of vector v.  The sign is read off the float's bit pattern:
            // -0.0 would come out wrong, but a zero lies inside every band and is recomputed.
            const int bb = wave + 4 * i;
            float y[4], margin[4];
            uint32_t sbits = 0u;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                y[jj] = fmaf(ym[jj], 0.000244140625f, yh[jj]);
                margin[jj] = fmaf(-res.g[i][jj], band, fabsf(y[jj]));      // one rounding: positive only if |y| > g band
                sbits |= (__float_as_uint(y[jj]) >> 31) << jj;
            }
            sbits ^= 0xFu;
            const float worst = fminf(fminf(margin[0], margin[1]), fminf(margin[2], margin[3]));
            if (live) {
                const int sh = 16 * (bb & 1) + 4 * kb;
                atomicOr(&w32[v * 16 + (bb >> 1)], sbits << sh);
                if (!(worst > 0.0f)) {                                     // rare; also catches a NaN
                    uint32_t ubits = 0u;
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) ubits |= (margin[jj] > 0.0f ? 0u : 1u) << jj;
                    atomicOr(&unsure[v * 16 + (bb >> 1)], ubits << sh);
                }
            }
        }
    }
    __syncthreads();
    between();
    // ---- words with bits inside the guard band: into the list; recomputed here only when the list is full ----
    const int W32 = pv.sketch_bits / 32;
    for (int item = tid; item < tile * W32; item += kProjThreads) {
        const int v = item / W32, w = item - v * W32;
        if (!valid(v)) continue;
        uint32_t m = unsure[v * 16 + w];
        if (m == 0u) continue;
        const int slot = atomicAdd(&list.n, 1);
        if (slot < kProjFixCap) {
            list.item[slot] = ProjFix{src(v), dst(v) + w, m, (uint32_t)w};
            continue;
        }
        uint32_t cur = w32[v * 16 + w];
        while (m) {
            const int p = __ffs(m) - 1;
            m &= m - 1u;
            const float y = proj_chain<D>(pv.R + (size_t)(32 * w + p) * D, [&](int j, float *out) {
                if constexpr (F32IN) {
                    const float *xv = static_cast<const float *>(src(v)) + j;
                    const float4 a = *reinterpret_cast<const float4 *>(xv), b = *reinterpret_cast<const float4 *>(xv + 4);
                    out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w; out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
                } else {
                    proj_load8(xs + (size_t)v * stride + j, out);
                }
            });
            cur = y >= 0.0f ? (cur | (1u << p)) : (cur & ~(1u << p));
        }
        w32[v * 16 + w] = cur;
    }
}

}  // namespace
}  // namespace h1bkv
