// Helpers shared by the decode kernels (wave reductions, DPP moves, the AND-OR dequantisation step, sketch loads).
#pragma once

#include <hip/hip_fp16.h>

#include "internal.h"

namespace h1bkv {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxPagesPerChunk = kMaxChunk / kPage;

__device__ __forceinline__ int wave_min(int x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x = min(x, __shfl_xor(x, off));
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    return x;
}
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, false));
}
// Sum, inside each row of 16 lanes, over the lanes that hold the same channel slice (lane % LPT) of different
// tokens.  DPP row rotations: one VALU instruction per step, no LDS traffic.
template <int LPT>
__device__ __forceinline__ float row_slot_sum(float x) {
    if constexpr (LPT == 2) x += dpp_mov<0x4E>(x);    // quad_perm [2,3,0,1]: lane ^ 2
    if constexpr (LPT <= 4) x += dpp_mov<0x124>(x);   // row_ror:4
    x += dpp_mov<0x128>(x);                           // row_ror:8
    return x;
}
// x[lane] + x[lane ^ 32] (gfx950 lane-swap instruction: upper half of one operand <-> lower half of the other).
__device__ __forceinline__ float half_wave_sum(float x) {
    const unsigned u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Returns the value in a vector register whose content the compiler can no longer see as a constant.  With the
// mask and the magic number of the dequantisation step laundered this way, (x & mask) | magic is selected as ONE
// v_and_or_b32 with register operands instead of an AND and an OR with two literals -- and, unlike an inline-asm
// instruction, the result stays visible to the hazard recogniser when it feeds an MFMA.
__device__ __forceinline__ uint32_t opaque_vgpr(uint32_t v) {
    asm volatile("" : "+v"(v));
    return v;
}
// 2^x for x <= 0 as the bare hardware instruction: the library routine wraps it in a range reduction for results
// below the smallest normal number, which a softmax weight next to a weight of 1 never needs (they flush to 0 here).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ uint32_t and_or(uint32_t x, uint32_t mask, uint32_t magic) { return (x & mask) | magic; }

// Streaming loads: cache records are read once per decode step and never reused by the kernel, so the value planes
// (codes, scale/zero, fp16 values) are requested non-temporal -- they should not displace anything in the last-level
// caches on their way through.  Measured on the 32k-context benchmark (split kernel): all planes plain 281 us;
// codes only 264 us; codes and scale/zero 249 us; sketches as well 257 us -- so the sketch loads, whose result every
// lane needs first, stay plain.
typedef unsigned int nt_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream(const uint4 *p) {
    const nt_u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const nt_u32x4 *>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ uint32_t load_stream(const uint32_t *p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ uint64_t load_stream(const uint64_t *p) { return __builtin_nontemporal_load(p); }

template <int W>
struct SketchRow {
    uint64_t w[W];
};
template <int W>
__device__ __forceinline__ SketchRow<W> load_sketch(const uint64_t *p) {
    SketchRow<W> s;
    if constexpr (W == 1) {
        s.w[0] = *p;
    } else {
#pragma unroll
        for (int i = 0; i < W; i += 2) {
            const uint4 v = *reinterpret_cast<const uint4 *>(p + i);
            s.w[i] = (uint64_t)v.x | ((uint64_t)v.y << 32);
            s.w[i + 1] = (uint64_t)v.z | ((uint64_t)v.w << 32);
        }
    }
    return s;
}

}  // namespace
}  // namespace h1bkv
