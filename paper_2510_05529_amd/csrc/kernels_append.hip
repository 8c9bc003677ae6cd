// Cache append: key sketch (Sec. IV-A Eq.(2)) and 4-bit group quantisation of values (Sec. IV-B Eq.(4)),
// written into the paged planes.
//
// Work unit: a workgroup of 4 waves takes a tile of consecutive record slots of one sequence.  Slots are ordered
// head-major and, per head, start at the 8-token boundary at or below the first new position, so that a tile is
// a run of consecutive tokens of one head (contiguous output runs inside a page, whole head rows as input) and no
// 8-token block of a head is ever split between two workgroups (the token-interleaved code layout is written
// per block).  Slots before the first new token or after the last one are padding and are skipped.
//
// Sketch: lane i of a wave owns sketch bit (64*word + i): it keeps row R[bit][0..d) in registers and
// runs the fp32 chain y = fma(R[bit][j], k[j], y), j ascending from +0 -- the order that fixes every
// bit -- with k[j] broadcast from the tile in LDS.  fp16 keys stay fp16 there: the widening to fp32 is exact and
// rides on the FMA (mixed-precision FMA with an fp16 operand), which halves the LDS bytes per multiply-add -- the
// broadcast reads, not the ALUs, are what this loop saturates first.  The 64-lane ballot of (y >= 0) IS the packed
// sketch word (bit i of the word = lane i), so packing costs nothing.
//
// Quantiser: one lane per (record, 32-channel slice): min/max over the slice, combined across the
// group's lanes with wave shuffles, then zero = fp16(min), scale = fp16((max-min)/15) and
// code = clamp(rne((v - zero)/scale), 0, 15) with IEEE fp32 subtract and divide.
// Code plane layouts (PoolView::code_layout):
//   0  record-major: the 32 codes of a slice are one 16-byte store; byte m of a record = channels 2m (low), 2m+1 (high);
//   1  token-interleaved: per block of 8 tokens one 32-bit word per channel with that channel's 8 codes
//      (code_word_index / code_nibble_pos); words of partially filled blocks are read-modified-written;
//   2  the "1-bit key only" variant (Table V): no quantiser, the plane holds the values as fp16, record-major.
#include <hip/hip_fp16.h>

#include <type_traits>

#include "internal.h"
#include "projection_mfma.h"

namespace h1bkv {

namespace {

constexpr int kTile = 64;      // record slots per workgroup pass (a multiple of 8)
constexpr int kThreads = 256;
constexpr size_t kNoRow = ~(size_t)0;

__device__ __forceinline__ void load8(const __half *p, float *out) {
    const uint4 raw = *reinterpret_cast<const uint4 *>(p);
    const __half2 *h = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float2 f = __half22float2(h[i]);
        out[2 * i] = f.x;
        out[2 * i + 1] = f.y;
    }
}
__device__ __forceinline__ void load8(const float *p, float *out) {
    const float4 a = *reinterpret_cast<const float4 *>(p);
    const float4 b = *reinterpret_cast<const float4 *>(p + 4);
    out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
    out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
}

__device__ __forceinline__ void copy8(const __half *src, __half *dst) { *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(src); }
__device__ __forceinline__ void copy8(const float *src, float *dst) {
    *reinterpret_cast<float4 *>(dst) = *reinterpret_cast<const float4 *>(src);
    *reinterpret_cast<float4 *>(dst + 4) = *reinterpret_cast<const float4 *>(src + 4);
}

// Eq.(4) for one 32-channel slice x of a value vector whose quantisation group spans `lanes_per_group` neighbouring lanes
// (G / 32; all lanes of the wave must call): the group's scale and zero as fp16 bits and the slice's 32 codes, 8 per word.
__device__ __forceinline__ void quantise_slice(const float (&x)[32], int lanes_per_group, uint32_t (&packed)[4], unsigned short &sh,
                                               unsigned short &zh) {
    float mn = x[0], mx = x[0];
#pragma unroll
    for (int i = 1; i < 32; ++i) {
        mn = fminf(mn, x[i]);
        mx = fmaxf(mx, x[i]);
    }
    for (int o = 1; o < lanes_per_group; o <<= 1) {
        mn = fminf(mn, __shfl_xor(mn, o));
        mx = fmaxf(mx, __shfl_xor(mx, o));
    }
    const float delta = (mx - mn) / 15.0f;
    sh = __half_as_ushort(__float2half_rn(delta));
    zh = __half_as_ushort(__float2half_rn(mn));
    if ((zh & 0x7FFFu) == 0) zh = 0;
    const float sc = __half2float(__ushort_as_half(sh));
    const float zp = __half2float(__ushort_as_half(zh));
    packed[0] = packed[1] = packed[2] = packed[3] = 0u;
    if (sc != 0.0f) {
        // Eq.(4)'s code is clamp(rint((x - zero) / scale)) with an IEEE divide.  The quotient without the divide
        // instruction sequence: with r = RN(1 / scale) and q0 = RN(d r), q = fma(fma(-q0, scale, d), r, q0) is the
        // correctly rounded d / scale (one Newton step on a quotient that is within an ulp, exact remainder; the scale is
        // an fp16 number, so its significand is never all ones, the one case the step can miss).  Compared on the host
        // with the divide for every fp16 scale at the fp32 neighbours of every code boundary and on 2 x 10^8 random
        // quotients: no difference.  An earlier form rounded d r directly and redid words that held an element near a
        // half-integer with the divide: fp16 inputs put quotients exactly on half-integers so often that four in ten
        // (wave, word) pairs took the redo, which was two fifths of the kernel's instructions.
        // u = q + 2^23 rounds q to an integer (ties to even, as rint) in the low mantissa bits; the codes are assembled as
        // w = (w << 4) + bits(u): every bits(u) is 0x4B000000 + code, so the stray high bits sum to a constant that is
        // subtracted once per word.
        const float r = 1.0f / sc;
        const float s_fin = sc < __builtin_inff() ? sc : 0.0f;      // an overflowed scale: r = 0 and every code 0, as d / inf
#pragma unroll
        for (int wd = 0; wd < 4; ++wd) {
            uint32_t w = 0u;
#pragma unroll
            for (int i = 7; i >= 0; --i) {
                const float d = x[8 * wd + i] - zp;
                const float q0 = __fmul_rn(d, r);
                const float q = __builtin_fmaf(__builtin_fmaf(-q0, s_fin, d), r, q0);
                const float u = __fadd_rn(q, 8388608.0f);
                const float uc = __builtin_amdgcn_fmed3f(u, 8388608.0f, 8388623.0f);
                w = (w << 4) + __float_as_uint(uc);
            }
            w -= 0xFB000000u;                      // sum over i of 0x4B000000 << 4 i, modulo 2^32
            packed[wd] = w;
        }
    }
}

// bx, by, gx: the workgroup's tile index, its sequence (index into desc) and the number of workgroups that share
// the sequence's tiles -- blockIdx.x, blockIdx.y, gridDim.x when the kernel does nothing else.
// MF: the projections come from the matrix cores and only the bits inside the guard band are recomputed with the
// chain; see the projection block below (fp32 keys are scaled and split into two fp16 pieces while they are staged).
// ONE: the call appends one token per sequence (a decode step) -- a compile-time choice, because a run-time branch
// around the two ways of loading the projection row doubled the time of the prefill-sized launches.
// PART: kBoth, or only the keys' half (sketches) or the values' half (codes, scale/zero) of the work -- large appends run
// the halves as two launches: the keys' workgroups are few, long-lived and heavy in registers, the values' half is a plain
// stream that wants many light ones.
enum AppendPart { kBoth = 0, kKeys = 1, kValues = 2 };
template <int D, typename T, bool MF, bool ONE, AppendPart PART = kBoth>
__device__ __forceinline__ void append_body(const AppendArgs &a, const BatchDesc &desc, int tile, int bx, int by, int gx) {
    constexpr bool F32MF = MF && sizeof(T) == 4;              // matrix-core projection of fp32 keys: two fp16 piece tiles
    using KT = typename std::conditional<F32MF, __half, T>::type;
    constexpr int KPAD = 16 / sizeof(KT);                     // 16 bytes per row: conflict-free 16-byte reads down a column
    // the key tile in its boundary dtype; F32MF: rows [kTile, 2 kTile) hold the low pieces
    __shared__ __attribute__((aligned(16))) KT ks[F32MF ? 2 * kTile : kTile][D + KPAD];
    __shared__ float band_s[MF ? kTile : 1];          // matrix-core path: guard band norm of each key
    __shared__ uint32_t unsure[MF ? kTile : 1][16];   // matrix-core path: per token, the sketch bits that need the chain
    static_assert(kTile == kProjTile && kThreads == kProjThreads, "projection_mfma.h assumes this tile shape");
    __shared__ uint64_t words[kTile][8];              // sketch words of the tile (W <= 8)
    __shared__ size_t dst[kTile];                     // plane index of each slot: (page * H_kv + head) * 256 + slot in page
    __shared__ size_t src_off[kTile];                 // element offset of each slot's K / V row; kNoRow marks padding
    __shared__ uint32_t codes_s[kTile][D / 8 + 1];    // layout 1: codes of the tile in canonical nibble order (+1: bank spread)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    SeqDesc sd = desc.s[by];
    if (desc.pos_dev) {                               // device-resident position: the token goes where the sequence ends now
        sd.pos = desc.pos_dev[by] + desc.pos_add;
        if (sd.pos >= desc.pos_max) return;           // beyond the reserved pages: nothing is written (whole workgroup)
    }
    const PoolView &pv = a.pool;
    const int H = pv.n_kv_heads, W = pv.sketch_bits >> 6, G = pv.group_size, ng = D / G;
    const int n_new = a.n_new;
    const int off8 = sd.pos & 7;                      // slots of a head's first block that lie before the first new token
    const int L = (off8 + n_new + 7) & ~7;            // slots per head
    const int n_slots = L * H;
    const T *kbase = static_cast<const T *>(a.k) + (size_t)by * a.stride_seq;
    const T *vbase = static_cast<const T *>(a.v) + (size_t)by * a.stride_seq;

    // Row R[64 word + lane][0..d) of this lane's sketch bit lives in registers across all tiles of the workgroup.
    const int wslots = W < 4 ? W : 4, tslots = 4 / wslots;
    [[maybe_unused]] float r[MF ? 1 : D];
    [[maybe_unused]] int r_word = wave % wslots;
    [[maybe_unused]] auto load_row = [&](int word) {
        if constexpr (!MF && PART != kValues) {
            if constexpr (ONE) {
                // a decode step's append: a workgroup sketches a handful of records, so the row is read once and the
                // read should be cheap -- from R^T a wave's load of element j is one 256-byte run (from R the 64 lanes
                // read 64 different rows)
                const float *col = pv.RT + word * 64 + lane;
#pragma unroll
                for (int j = 0; j < D; ++j) r[j] = col[(size_t)j * pv.sketch_bits];
            } else {
                const float *row = pv.R + (size_t)(word * 64 + lane) * D;
#pragma unroll
                for (int j = 0; j < D; j += 4) {
                    const float4 x = *reinterpret_cast<const float4 *>(row + j);
                    r[j] = x.x; r[j + 1] = x.y; r[j + 2] = x.z; r[j + 3] = x.w;
                }
            }
        }
    };
    load_row(r_word);

    for (int slot0 = bx * tile; slot0 < n_slots; slot0 += gx * tile) {
        const int tid = per_tile_index(threadIdx.x);   // shadows the outer one: see per_tile_index
        __syncthreads();   // previous pass is done with the LDS tile
        // ---- resolve the tile once: slot -> (head, token) -> source row, destination record ----
        // (the divisions by the runtime slot count per head are done here, by one thread per slot, not in the loops)
        if constexpr (MF) {                            // the sketch words are assembled with atomic ORs: start from zero
            for (int e = tid; e < kTile * 16; e += kThreads) {
                reinterpret_cast<uint32_t *>(&words[0][0])[e] = 0u;
                (&unsure[0][0])[e] = 0u;
            }
        }
        // The source offsets need no memory access; the destination needs the block table.  That load is issued here
        // and consumed after the key tile has been requested, so the two round trips overlap.
        int my_page = 0, my_head = 0, my_pos = 0;
        if (tid < tile) {
            size_t off = kNoRow;
            if (slot0 + tid < n_slots) {
                const int head = (slot0 + tid) / L, t = (slot0 + tid) % L - off8;
                // padding slots too: a block's words start at its first slot.  Every block of a head holds at
                // least one new token, so its page has been assigned.
                const int pos = sd.pos + t;
                my_page = pv.block_table[(size_t)sd.seq_id * pv.max_pages_per_seq + pos / kPage];
                my_head = head;
                my_pos = pos;
                if (t >= 0 && t < n_new) off = (size_t)t * a.stride_tok + (size_t)head * a.stride_head;
            }
            src_off[tid] = off;
        }
        __syncthreads();
        auto valid_slot = [&](int rl) { return src_off[rl] != kNoRow; };

        // fp16 values: the slice this thread quantises first is requested now, so that its latency runs behind the key
        // staging and the projection
        constexpr bool kPrefetchV = sizeof(T) == 2;           // (fp32 values would take 32 registers next to the R row)
        [[maybe_unused]] uint4 vpre[4];
        auto prefetch_values = [&]() {
            const int rl = tid / (D / 32), slice = tid % (D / 32);
            if (rl < tile && valid_slot(rl)) {
                const uint4 *src = reinterpret_cast<const uint4 *>(vbase + src_off[rl] + slice * 32);
#pragma unroll
                for (int i = 0; i < 4; ++i) vpre[i] = src[i];
            }
        };
        // chain path: now; matrix-core path: after its MFMA phase (held through it, the 16 registers spill, and a
        // spill reload waits for every load in flight)
        if constexpr (kPrefetchV && !MF && PART != kKeys) prefetch_values();

        // ---- stage the key tile ----
        if constexpr (PART == kValues) {
        } else if constexpr (F32MF) {
            stage_f32_tile<D>([&](int rl) { return valid_slot(rl) ? kbase + src_off[rl] : nullptr; }, tile, &ks[0][0], &ks[kTile][0],
                              D + KPAD, band_s);
        } else {
            for (int e = tid * 8; e < tile * D; e += kThreads * 8) {
                const int rl = e / D, ch = e % D;
                if (valid_slot(rl)) copy8(kbase + src_off[rl] + ch, &ks[rl][ch]);
            }
        }
        if (tid < tile) dst[tid] = ((size_t)my_page * H + my_head) * kPage + (my_pos % kPage);
        __syncthreads();

        if constexpr (PART == kValues) {
        } else if constexpr (MF) {
            // ---- Eq.(2) on the matrix cores; the bits inside the guard band by the chain (projection_mfma.h) ----
            auto between = [&]() {
                if constexpr (kPrefetchV && PART != kKeys) prefetch_values();
            };
            project_tile_mfma<D, F32MF>(pv, reinterpret_cast<const __half *>(&ks[0][0]),
                                        reinterpret_cast<const __half *>(&ks[F32MF ? kTile : 0][0]), band_s, D + KPAD, tile, valid_slot,
                                        reinterpret_cast<uint32_t *>(&words[0][0]), &unsure[0][0], between,
                                        [&](int rl) { return reinterpret_cast<const float *>(kbase + src_off[rl]); });
        } else
        // ---- Eq.(2): lane = sketch bit; y = fma chain over j; ballot = packed word ----
        for (int word = wave % wslots; word < W; word += wslots) {
            if (word != r_word) {                      // only when a wave owns more than one word (b = 512)
                load_row(word);
                r_word = word;
            }
            for (int t = wave / wslots; t < tile; t += tslots) {
                if (!valid_slot(t)) continue;          // uniform over the wave
                float y = 0.0f;
#pragma unroll
                for (int j = 0; j < D; j += 8) {
                    float kk[8];
                    load8(&ks[t][j], kk);              // same address in every lane: an LDS broadcast
#pragma unroll
                    for (int i = 0; i < 8; ++i) y = __builtin_fmaf(r[j + i], kk[i], y);
                }
                const uint64_t mask = __ballot(y >= 0.0f);
                if (lane == 0) words[t][word] = mask;
            }
        }

        // ---- fp16-value variant: no quantiser, the value rounded to nearest-even fp16 ----
        if (PART != kKeys && pv.code_layout == 2) {
            __half *values = reinterpret_cast<__half *>(pv.codes);
            for (int e = tid * 8; e < tile * D; e += kThreads * 8) {
                const int rl = e / D, ch = e % D;
                if (!valid_slot(rl)) continue;
                float x[8];
                load8(vbase + src_off[rl] + ch, x);
                __half2 h[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) h[i] = __halves2half2(__float2half_rn(x[2 * i]), __float2half_rn(x[2 * i + 1]));
                *reinterpret_cast<uint4 *>(values + dst[rl] * D + ch) = *reinterpret_cast<const uint4 *>(h);
            }
        }

        // ---- Eq.(4): one lane per (slot, 32-channel slice) ----
        constexpr int LPT = D / 32;
        const int lanes_per_group = G / 32;
        for (int item = tid; PART != kKeys && pv.code_layout != 2 && item < ((tile * LPT + 63) & ~63); item += kThreads) {   // whole waves run the loop (shuffles below)
            const int rl = item / LPT, slice = item % LPT;
            const bool valid = rl < tile && valid_slot(rl);
            float x[32];
            if (kPrefetchV && valid && item == tid) {  // requested before the projection
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const __half2 *h2 = reinterpret_cast<const __half2 *>(&vpre[i]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float2 f = __half22float2(h2[e]);
                        x[8 * i + 2 * e] = f.x;
                        x[8 * i + 2 * e + 1] = f.y;
                    }
                }
            } else if (valid) {
                const T *src = vbase + src_off[rl] + slice * 32;
#pragma unroll
                for (int i = 0; i < 32; i += 8) load8(src + i, x + i);
            } else {
#pragma unroll
                for (int i = 0; i < 32; ++i) x[i] = 0.0f;
            }
            uint32_t packed[4];
            unsigned short sh, zh;
            quantise_slice(x, lanes_per_group, packed, sh, zh);
            if (valid) {
                const size_t rec = dst[rl];
                if (pv.code_layout == 0) {
                    *reinterpret_cast<uint4 *>(pv.codes + rec * (D / 2) + slice * 16) = make_uint4(packed[0], packed[1], packed[2], packed[3]);
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) codes_s[rl][slice * 4 + i] = packed[i];
                }
                if (slice % lanes_per_group == 0) pv.meta[rec * ng + slice / lanes_per_group] = (uint32_t)sh | ((uint32_t)zh << 16);
            }
        }
        __syncthreads();

        // ---- store sketch words ----
        for (int i = tid; PART != kValues && i < tile * W; i += kThreads) {
            const int rl = i / W, w = i - rl * W;
            if (valid_slot(rl)) pv.sketch[dst[rl] * W + w] = words[rl][w];
        }

        // ---- layout 1: one word per (8-token block, channel) ----
        if (PART != kKeys && pv.code_layout == 1) {
            for (int item = tid; item < (tile / 8) * D; item += kThreads) {
                const int blk = item / D, c = item % D;
                uint32_t val = 0, have = 0;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int rl = blk * 8 + j;
                    if (!valid_slot(rl)) continue;
                    const uint32_t nib = (codes_s[rl][c >> 3] >> (4 * (c & 7))) & 0xFu;
                    val |= nib << (4 * code_nibble_pos(j));
                    have |= 0xFu << (4 * code_nibble_pos(j));
                }
                if (have == 0) continue;
                // the block's 8 tokens are consecutive slots of one page: its words start at the first slot's record
                uint32_t *wp = reinterpret_cast<uint32_t *>(pv.codes + dst[blk * 8] * (D / 2)) + code_word_index(c);
                *wp = have == 0xFFFFFFFFu ? val : ((*wp & ~have) | val);
            }
        }
    }
}

template <int D, typename T, bool MF, bool ONE = false>
__global__ __launch_bounds__(kThreads, MF ? 4 : 1) void append_kernel(AppendArgs a, BatchDesc desc, int tile) {
    append_body<D, T, MF, ONE>(a, desc, tile, blockIdx.x, blockIdx.y, gridDim.x);
}

// The values' half on its own: nothing resident, few registers.
template <int D, typename T>
__global__ __launch_bounds__(kThreads, 6) void append_values_kernel(AppendArgs a, BatchDesc desc, int tile) {
    append_body<D, T, false, false, kValues>(a, desc, tile, blockIdx.x, blockIdx.y, gridDim.x);
}

// The values' half for the record-major layouts (4-bit codes per record, or fp16 values): a plain stream -- one lane per
// (record slot, 32-channel slice) in the slot order of append_body, no LDS and no barrier; the latency of the page lookup
// and of the value rows is covered by the number of waves in flight.
template <int D, typename T>
__global__ __launch_bounds__(kThreads) void append_values_stream_kernel(AppendArgs a, BatchDesc desc) {
    constexpr int LPT = D / 32;
    const PoolView &pv = a.pool;
    const SeqDesc sd = desc.s[blockIdx.y];
    const int H = pv.n_kv_heads, G = pv.group_size, ng = D / G, lanes_per_group = G / 32;
    const int off8 = sd.pos & 7, L = (off8 + a.n_new + 7) & ~7;
    const int n_items = L * H * LPT;
    const T *vbase = static_cast<const T *>(a.v) + (size_t)blockIdx.y * a.stride_seq;
    // whole waves run the loop (the quantiser exchanges minima between the lanes of a group)
    for (int item = blockIdx.x * kThreads + threadIdx.x; item < ((n_items + 63) & ~63); item += gridDim.x * kThreads) {
        const int slot = item / LPT, slice = item % LPT;
        const int head = slot / L, t = slot % L - off8;
        const bool valid = item < n_items && t >= 0 && t < a.n_new;
        float x[32];
        size_t rec = 0;
        if (valid) {
            const int pos = sd.pos + t;
            const int page = pv.block_table[(size_t)sd.seq_id * pv.max_pages_per_seq + pos / kPage];
            rec = ((size_t)page * H + head) * kPage + pos % kPage;
            const T *src = vbase + (size_t)t * a.stride_tok + (size_t)head * a.stride_head + slice * 32;
#pragma unroll
            for (int i = 0; i < 32; i += 8) load8(src + i, x + i);
        } else {
#pragma unroll
            for (int i = 0; i < 32; ++i) x[i] = 0.0f;
        }
        if (pv.code_layout == 2) {                      // fp16-value variant: the value rounded to nearest-even fp16
            if (valid) {
                __half *values = reinterpret_cast<__half *>(pv.codes) + rec * D + slice * 32;
#pragma unroll
                for (int i = 0; i < 32; i += 8) {
                    __half2 h[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) h[e] = __halves2half2(__float2half_rn(x[i + 2 * e]), __float2half_rn(x[i + 2 * e + 1]));
                    *reinterpret_cast<uint4 *>(values + i) = *reinterpret_cast<const uint4 *>(h);
                }
            }
            continue;                                   // (uniform: the layout is a property of the cache)
        }
        uint32_t packed[4];
        unsigned short sh, zh;
        quantise_slice(x, lanes_per_group, packed, sh, zh);
        if (valid) {
            *reinterpret_cast<uint4 *>(pv.codes + rec * (D / 2) + slice * 16) = make_uint4(packed[0], packed[1], packed[2], packed[3]);
            if (slice % lanes_per_group == 0) pv.meta[rec * ng + slice / lanes_per_group] = (uint32_t)sh | ((uint32_t)zh << 16);
        }
    }
}

// The keys' half on its own, with the pieces of R resident in registers (resident_sketch_tiles in projection_mfma.h):
// tiles of 64 record slots of sequence blockIdx.y, in the slot order of append_body (head-major, each head's run padded
// to 8-token blocks; the padding slots are empty).
struct KeyRows {
    const AppendArgs &a;
    SeqDesc sd;
    int L, off8, n_slots;
    ProjDiv by_L;
    __device__ int rows_in(long tile) const { return min(kTile, n_slots - (int)tile * kTile); }
    __device__ size_t src(long tile, int rl) const {
        uint32_t head, rem;
        by_L.divmod((uint32_t)((int)tile * kTile + rl), head, rem);
        const int t = (int)rem - off8;
        return t >= 0 && t < a.n_new ? (size_t)t * a.stride_tok + (size_t)head * a.stride_head : kProjNoRow;
    }
    __device__ int page_request(long tile, int rl) const {
        uint32_t head, rem;
        by_L.divmod((uint32_t)((int)tile * kTile + rl), head, rem);
        const int pos = sd.pos + (int)rem - off8;
        return a.pool.block_table[(size_t)sd.seq_id * a.pool.max_pages_per_seq + pos / kPage];
    }
    __device__ uint32_t *dst(long tile, int rl, int page) const {
        uint32_t head, rem;
        by_L.divmod((uint32_t)((int)tile * kTile + rl), head, rem);
        const int pos = sd.pos + (int)rem - off8;
        const size_t rec = ((size_t)page * a.pool.n_kv_heads + head) * kPage + pos % kPage;
        return reinterpret_cast<uint32_t *>(a.pool.sketch + rec * (a.pool.sketch_bits >> 6));
    }
};

template <int D, typename T, bool WIDE>
__global__ __launch_bounds__(kThreads, 3) void append_keys_kernel(AppendArgs a, BatchDesc desc) {
    static_assert(kTile == kProjTile && kThreads == kProjThreads, "projection_mfma.h assumes this tile shape");
    const SeqDesc sd = desc.s[blockIdx.y];
    const int off8 = sd.pos & 7, L = (off8 + a.n_new + 7) & ~7, n_slots = L * a.pool.n_kv_heads;
    const KeyRows rows{a, sd, L, off8, n_slots, ProjDiv((uint32_t)L)};
    resident_sketch_tiles<D, T, WIDE>(a.pool, static_cast<const T *>(a.k) + (size_t)blockIdx.y * a.stride_seq, rows, (long)blockIdx.x,
                                (long)gridDim.x, (long)((n_slots + kTile - 1) / kTile), (int)blockIdx.z, (int)gridDim.z);
}

// Prologue of a fused decode step: rows [0, n_seqs) of the grid append the step's new token of each sequence,
// the remaining rows sketch the step's queries (Eq.(2) applied to q, same FMA chain: thread = (query, bit), all
// loads of the thread's column of R^T issued ahead of the chain, ballot = packed word).  Neither half depends on
// the other, so one launch replaces two.
template <int D, typename T>
__global__ __launch_bounds__(kThreads) void step_prologue_kernel(AppendArgs a, BatchDesc desc, int tile, int n_seqs, QueryArgs qa) {
    if ((int)blockIdx.y < n_seqs) {
        append_body<D, T, false, true>(a, desc, tile, blockIdx.x, blockIdx.y, gridDim.x);
        return;
    }
    __shared__ float qs[4][D];
    const int b = a.pool.sketch_bits, W = b >> 6;
    const int per_block = b <= kThreads ? kThreads / b : 1;           // whole queries per workgroup pass
    const int vec0 = (((int)blockIdx.y - n_seqs) * gridDim.x + blockIdx.x) * per_block;
    const T *qbase = static_cast<const T *>(qa.q);
    for (int e = threadIdx.x; e < per_block * D; e += kThreads) {
        const int qi = e / D, vec = vec0 + qi;
        qs[qi][e % D] = vec < qa.n_vec ? (float)qbase[(size_t)vec * D + e % D] : 0.0f;
    }
    __syncthreads();
    for (int bit0 = 0; bit0 < b; bit0 += kThreads) {                  // one pass unless b = 512
        const int qi = b <= kThreads ? threadIdx.x / b : 0;
        const int bit = b <= kThreads ? threadIdx.x % b : bit0 + threadIdx.x;
        const int vec = vec0 + qi;
        float y = 0.0f;
        constexpr int CH = D < 128 ? D : 128;                         // elements of the column held at a time
#pragma unroll 1
        for (int j0 = 0; j0 < D; j0 += CH) {
            float rt[CH];
#pragma unroll
            for (int j = 0; j < CH; ++j) rt[j] = a.pool.RT[(size_t)(j0 + j) * b + bit];
#pragma unroll
            for (int j = 0; j < CH; ++j) y = __builtin_fmaf(rt[j], qs[qi][j0 + j], y);
        }
        const uint64_t mask = __ballot(y >= 0.0f);
        if ((threadIdx.x & 63) == 0 && vec < qa.n_vec) qa.q_sketch[(size_t)vec * W + (bit >> 6)] = mask;
    }
}

}  // namespace

// With qa != nullptr the launch also sketches qa->n_vec query vectors (fused decode-step prologue).
hipError_t launch_append(const AppendArgs &a, const BatchDesc &desc, int n_seqs, const QueryArgs *qa, hipStream_t st) {
    if (qa && a.n_new != 1) return hipErrorInvalidValue;   // the fused prologue is a decode step's: one token per sequence
    // Slots per head: the new tokens plus the padding down to / up to 8-token boundaries.
    int max_off = 0;
    for (int i = 0; i < n_seqs; ++i) max_off = desc.s[i].pos % 8 > max_off ? desc.s[i].pos % 8 : max_off;
    const long L = ((long)max_off + a.n_new + 7) / 8 * 8;
    const long n_slots = L * a.pool.n_kv_heads;
    // Slots per workgroup pass: a full tile for prefill-sized calls; for a decode step (one block per head) a single
    // block, so that the few records spread over many compute units.
    long tile = (n_slots * n_seqs + 255) / 256;
    tile = (tile + 7) / 8 * 8;
    tile = tile > kTile ? kTile : tile;
    const long tiles = (n_slots + tile - 1) / tile;
    // Each workgroup reads its rows of R once and keeps them in registers: with many tiles, a few resident
    // workgroups per compute unit walk all of them.
    // (the matrix-core path with streamed pieces of R keeps nothing resident: more, shorter workgroups even out the tail)
    const int D = a.pool.head_dim;
    const long wg_budget = a.proj_mfma && !qa ? 6144 : 1024;
    const long max_wgs_x = wg_budget / n_seqs > 0 ? wg_budget / n_seqs : 1;
    const unsigned gx = (unsigned)(tiles < max_wgs_x ? tiles : max_wgs_x);
    unsigned q_rows = 0;
    if (qa) {
        const int per_block = a.pool.sketch_bits <= kThreads ? kThreads / a.pool.sketch_bits : 1;
        const unsigned q_blocks = (unsigned)((qa->n_vec + per_block - 1) / per_block);
        q_rows = (q_blocks + gx - 1) / gx;
    }
    const dim3 grid(gx, (unsigned)n_seqs + q_rows);
    // Large appends whose sketch width allows resident pieces of R run as two launches: the keys' half with three
    // long-lived workgroups per compute unit (768, all in one round), the values' half as a stream of short ones.
    const long key_tiles = (n_slots + kTile - 1) / kTile;
    // (a sketch wider than one workgroup's resident pieces is cut into parts, each with workgroups of its own)
    const int parts = D == 64 ? proj_resident_parts<64>(a.pool.sketch_bits) : D == 128 ? proj_resident_parts<128>(a.pool.sketch_bits) : 0;
    const bool split = a.proj_mfma && !qa && parts > 0 && key_tiles * n_seqs * parts >= 768;
    const long max_keys_x = split && 768 / (n_seqs * parts) > 0 ? 768 / (n_seqs * parts) : 1;
    const dim3 grid_keys((unsigned)(key_tiles < max_keys_x ? key_tiles : max_keys_x), (unsigned)n_seqs, (unsigned)(parts > 0 ? parts : 1));
    const long stream_blocks = (n_slots * (D / 32) + kThreads - 1) / kThreads;
    const dim3 grid_stream((unsigned)(stream_blocks < 32768 ? stream_blocks : 32768), (unsigned)n_seqs);
    const QueryArgs qargs = qa ? *qa : QueryArgs{nullptr, nullptr, 0};
#define H1BKV_LAUNCH(DD, TT)                                                                                        \
    do {                                                                                                            \
        if (qa) hipLaunchKernelGGL((step_prologue_kernel<DD, TT>), grid, dim3(kThreads), 0, st, a, desc, (int)tile, n_seqs, qargs); \
        else if (a.n_new == 1) hipLaunchKernelGGL((append_kernel<DD, TT, false, true>), grid, dim3(kThreads), 0, st, a, desc, (int)tile); \
        else hipLaunchKernelGGL((append_kernel<DD, TT, false>), grid, dim3(kThreads), 0, st, a, desc, (int)tile);   \
    } while (0)
#define H1BKV_LAUNCH_MF(DD, TT)                                                                                        \
    do {                                                                                                               \
        if (split) {                                                                                                   \
            /* 128 fp16 channels and whole groups of 128 sketch bits: the 32 x 32 form of the tile loop */            \
            if (DD == 128 && sizeof(TT) == 2 && a.pool.sketch_bits % 128 == 0)                                         \
                hipLaunchKernelGGL((append_keys_kernel<DD, TT, DD == 128 && sizeof(TT) == 2>), grid_keys, dim3(kThreads), 0, st, a, desc); \
            else                                                                                                       \
                hipLaunchKernelGGL((append_keys_kernel<DD, TT, false>), grid_keys, dim3(kThreads), 0, st, a, desc);    \
            if (a.pool.code_layout == 1)                                                                               \
                hipLaunchKernelGGL((append_values_kernel<DD, TT>), grid, dim3(kThreads), 0, st, a, desc, (int)tile);   \
            else                                                                                                       \
                hipLaunchKernelGGL((append_values_stream_kernel<DD, TT>), grid_stream, dim3(kThreads), 0, st, a, desc); \
        } else {                                                                                                       \
            hipLaunchKernelGGL((append_kernel<DD, TT, true>), grid, dim3(kThreads), 0, st, a, desc, (int)tile);        \
        }                                                                                                              \
    } while (0)
    if (a.f16 && a.proj_mfma && !qa) {
        if (D == 64) H1BKV_LAUNCH_MF(64, __half);
        else if (D == 128) H1BKV_LAUNCH_MF(128, __half);
        else hipLaunchKernelGGL((append_kernel<256, __half, true>), grid, dim3(kThreads), 0, st, a, desc, (int)tile);
    } else if (a.proj_mfma && !qa) {                  // fp32 keys
        if (D == 64) H1BKV_LAUNCH_MF(64, float);
        else if (D == 128) H1BKV_LAUNCH_MF(128, float);
        else hipLaunchKernelGGL((append_kernel<256, float, true>), grid, dim3(kThreads), 0, st, a, desc, (int)tile);
    } else if (a.f16) {
        if (D == 64) H1BKV_LAUNCH(64, __half);
        else if (D == 128) H1BKV_LAUNCH(128, __half);
        else H1BKV_LAUNCH(256, __half);
    } else {
        if (D == 64) H1BKV_LAUNCH(64, float);
        else if (D == 128) H1BKV_LAUNCH(128, float);
        else H1BKV_LAUNCH(256, float);
    }
#undef H1BKV_LAUNCH
#undef H1BKV_LAUNCH_MF
    return hipGetLastError();
}

}  // namespace h1bkv
