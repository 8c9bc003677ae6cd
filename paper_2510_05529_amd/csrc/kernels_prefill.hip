// Prefill attention over the compressed cache: Eq.(3) and Eq.(5) for every position of a prompt chunk, causally --
// query i of a sequence attends to the cached tokens up to and including its own position, exactly the decode step
// it would have seen had the prompt been fed one token at a time.
//
// With many queries per KV head the weighted sum  sum_t p[i][t] v^[t][c]  is a dense contraction and runs on the
// matrix cores (v_mfma_f32_16x16x32_f16, fp32 accumulate); the vector ALUs score (XOR + popcount), exponentiate and
// dequantise.  One workgroup (4 waves) takes 128 consecutive query positions of one (sequence, query head) and walks
// the key tokens in tiles of 64 up to its diagonal:
//   staging   the tile's sketches go to LDS as they are; its values are dequantised ONCE per workgroup,
//             v^ = fp16(scale * code + zero), and stored channel-major so that an MFMA B operand (8 consecutive
//             tokens of one channel) is one 16-byte LDS read.  The next tile's global loads are issued before the
//             current tile is consumed, so their latency is covered.
//   scores    a wave owns 32 query rows (two MFMA row blocks).  Lane (i, kb) scores row i against tokens 8 kb .. 8 kb + 7
//             of a 32-token step: that is exactly the A-operand slot of the lane, so the weights
//             p = exp((alpha - alpha_max)/tau) are packed to fp16 in registers and never travel through LDS.
//             Running maximum per row with a lazy rescale (scores take only b+1 values, the maximum moves rarely).
//             Weights carry a factor 2^14 to keep small ones out of the fp16 subnormal range; it cancels in the
//             normalisation, which uses the row sums of the SAME fp16 weights (one more MFMA against an all-ones B).
//   causal    tiles entirely below a wave's rows take an unmasked path; tiles entirely above them are skipped.
// sketch_rows_kernel sketches the chunk's query vectors (Eq.(2), same fp32 FMA chain as the keys) with the R rows
// resident in registers, 64 vectors per LDS tile.
#include <hip/hip_fp16.h>

#include "decode_common.h"

namespace h1bkv {

namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __fp16 fp16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kTK = 64;                       // key tokens per tile
constexpr int kRB = 2;                        // 16-row blocks per wave
constexpr int kQB = kWaves * 16 * kRB;        // query positions per workgroup
constexpr int kVStride = kTK * 2 + 16;        // bytes per channel row of the value tile (16 B pad: conflict-free b128 reads)
constexpr float kPScaleLog2 = 14.0f;          // weights are stored as p * 2^14

union HalfOperand {
    uint32_t u[4];
    f16x8 v;
};

__device__ __forceinline__ int xor16_min(int x) {       // min with the lane 16 away (immediate swizzle, inside a half-wave)
    return min(x, __builtin_amdgcn_ds_swizzle(x, 0x1F | (0x10 << 10)));
}
__device__ __forceinline__ int xor32_min(int x) {       // min with the lane 32 away
    const auto r = __builtin_amdgcn_permlane32_swap((unsigned)x, (unsigned)x, false, false);
    return min((int)r[0], (int)r[1]);
}

struct StageRegs {           // one thread's share of a key tile on its way from global memory to LDS
    uint4 sk;                // 16 bytes of the tile's sketches
    uint32_t c[4];           // layout 0: 8 bytes of codes for each of two tokens;  layout 1: up to 4 code words of one block
    uint32_t m[16];          // layout 0: {scale, zero} of the two tokens;  layout 1: of the block's 8 tokens, for up to
                             //           two quantisation groups (words k and k + 1 of a thread share a group)
};

template <int W, int D, int LAYOUT>
__global__ __launch_bounds__(kThreads, 2) void prefill_kernel(PrefillArgs a, BatchDesc desc, int seq0) {
    constexpr int NCB = D / 16;
    __shared__ __attribute__((aligned(16))) unsigned char v_s[2][D * kVStride];
    __shared__ __attribute__((aligned(16))) uint64_t sk_s[2][kTK * W];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, kb = lane >> 4;
    const SeqDesc sd = desc.s[blockIdx.z];
    const int len = sd.pos, n_q = a.n_q;
    const int qb = (int)gridDim.x - 1 - (int)blockIdx.x;          // the longest-running (latest) query blocks start first
    const int row0 = qb * kQB;
    const int q0 = len - n_q;                                      // absolute position of query 0
    const int last_row = min(row0 + kQB, n_q) - 1;
    const int n_tiles = (q0 + last_row + kTK) / kTK;               // tiles that hold tokens visible to the last row

    const PoolView &pv = a.pool;
    const int H = pv.n_kv_heads, Hq = pv.n_q_heads, r = Hq / H;
    const int h = blockIdx.y, kvh = h / r;
    const int seq_g = seq0 + blockIdx.z;
    const int ng = D / pv.group_size;
    const int32_t *bt = pv.block_table + (size_t)sd.seq_id * pv.max_pages_per_seq;

    // ---- this lane's query rows ----
    int pos[kRB];                 // absolute position of row (rb, i); -1 for rows past the chunk
    uint64_t sq[kRB][W];
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) {
        const int qi = row0 + wave * 16 * kRB + rb * 16 + i;
        pos[rb] = qi < n_q ? q0 + qi : -1;
#pragma unroll
        for (int w = 0; w < W; ++w)
            sq[rb][w] = qi < n_q ? a.q_sketch[(((size_t)seq_g * n_q + qi) * Hq + h) * W + w] : 0;
    }
    const int wave_row0 = row0 + wave * 16 * kRB;
    const int wave_min_pos = q0 + wave_row0;                                       // position of the wave's first row
    const int wave_max_pos = wave_row0 < n_q ? q0 + min(wave_row0 + 16 * kRB, n_q) - 1 : -1;   // ... and of its last valid row

    f32x4 acc[kRB][NCB], accsum[kRB];
    int run_min[kRB];
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) {
        run_min[rb] = 1 << 20;
        accsum[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) acc[rb][cb] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    HalfOperand ones;
#pragma unroll
    for (int k = 0; k < 4; ++k) ones.u[k] = 0x3C003C00u;          // fp16 1.0

    // ---- staging: global -> registers (issued early) -> LDS (after the current tile has been consumed) ----
    constexpr int kItems0 = 32 * (D / 16);                        // layout 0: (token pair, 16-channel slice) items per tile
    // layout 1: a thread takes block tid / 32 of the tile's 8 blocks and words tid % 32 + 32 k of its D words
    // (word wi holds channel 16 cb + n with cb = (wi / 64) * 4 + wi % 4, n = (wi % 64) / 4: the inverse of
    // code_word_index).  Words k = 0, 1 lie in one 16-channel block, k = 2, 3 in the block 64 channels on, so the
    // thread needs the 8 tokens' {scale, zero} of at most two groups.
    constexpr int kWordsPerThread = D / 32;
    auto word_channel = [](int wi) { return 16 * ((wi >> 6) * 4 + (wi & 3)) + ((wi & 63) >> 2); };
    auto tile_rec0 = [&](int kt) {
        const int t0 = kt * kTK;
        return ((size_t)bt[t0 / kPage] * H + kvh) * kPage + (t0 % kPage);          // a tile never straddles a page
    };
    auto load_tile = [&](StageRegs &sr, int kt) {
        const size_t rec0 = tile_rec0(kt);
        if (tid < kTK * W / 2) sr.sk = reinterpret_cast<const uint4 *>(pv.sketch + rec0 * W)[tid];
        if constexpr (LAYOUT == 0) {
            if (tid < kItems0) {
                const int tp = tid / (D / 16), s16 = tid % (D / 16);
                const int g = (16 * s16) / pv.group_size;
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const size_t rec = rec0 + 2 * tp + t;
                    const uint2 c = *reinterpret_cast<const uint2 *>(pv.codes + rec * (D / 2) + s16 * 8);
                    sr.c[2 * t] = c.x;
                    sr.c[2 * t + 1] = c.y;
                    sr.m[t] = pv.meta[rec * ng + g];
                }
            }
        } else {
            const int blk = tid >> 5;
            const uint32_t *words = reinterpret_cast<const uint32_t *>(pv.codes + (rec0 + 8 * blk) * (D / 2));
#pragma unroll
            for (int k = 0; k < kWordsPerThread; ++k) sr.c[k] = words[(tid & 31) + 32 * k];
#pragma unroll
            for (int ms = 0; ms < (kWordsPerThread + 1) / 2; ++ms) {
                const int g = word_channel((tid & 31) + 64 * ms) / pv.group_size;
#pragma unroll
                for (int j = 0; j < 8; ++j) sr.m[8 * ms + j] = pv.meta[(rec0 + 8 * blk + j) * ng + g];
            }
        }
    };
    auto store_tile = [&](const StageRegs &sr, int kt, int buf) {
        const int t0 = kt * kTK;
        if (tid < kTK * W / 2) reinterpret_cast<uint4 *>(sk_s[buf])[tid] = sr.sk;
        unsigned char *vs = v_s[buf];
        if constexpr (LAYOUT == 0) {
            if (tid < kItems0) {
                const int tp = tid / (D / 16), s16 = tid % (D / 16);
                float sc[2], zp[2];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    // slots past the end of the sequence hold anything: their values must not reach the MFMA as NaN
                    const uint32_t m = t0 + 2 * tp + t < len ? sr.m[t] : 0u;
                    sc[t] = __half2float(__ushort_as_half((unsigned short)(m & 0xFFFFu)));
                    zp[t] = __half2float(__ushort_as_half((unsigned short)(m >> 16)));
                }
#pragma unroll
                for (int cc = 0; cc < 16; ++cc) {
                    const int c = (cc + s16) & 15;                 // rotate the channel order per slice: spreads the LDS banks
                    const float c0 = (float)((sr.c[c >> 3] >> (4 * (c & 7))) & 0xFu);
                    const float c1 = (float)((sr.c[2 + (c >> 3)] >> (4 * (c & 7))) & 0xFu);
                    const __half2 hv = __halves2half2(__float2half_rn(fmaf(sc[0], c0, zp[0])), __float2half_rn(fmaf(sc[1], c1, zp[1])));
                    *reinterpret_cast<__half2 *>(vs + (16 * s16 + c) * kVStride + tp * 4) = hv;
                }
            }
        } else {
            const int blk = tid >> 5;
#pragma unroll
            for (int k = 0; k < kWordsPerThread; ++k) {
                const int ch = word_channel((tid & 31) + 32 * k);
                const uint32_t x = sr.c[k];
                __half hv[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    // slots past the end of the sequence hold anything: their values must not reach the MFMA as NaN
                    const uint32_t m = t0 + 8 * blk + j < len ? sr.m[8 * (k / 2) + j] : 0u;
                    const float sc = __half2float(__ushort_as_half((unsigned short)(m & 0xFFFFu)));
                    const float zp = __half2float(__ushort_as_half((unsigned short)(m >> 16)));
                    const float code = (float)((x >> (4 * code_nibble_pos(j))) & 0xFu);
                    hv[j] = __float2half_rn(fmaf(sc, code, zp));
                }
                *reinterpret_cast<uint4 *>(vs + ch * kVStride + blk * 16) = *reinterpret_cast<const uint4 *>(hv);
            }
        }
    };

    // ---- one tile: scores, weights, MFMA ----
    auto consume_tile = [&](int kt, int buf, auto masked_tag) {
        constexpr bool kMasked = decltype(masked_tag)::value;
        const uint64_t *sks = sk_s[buf];
        const unsigned char *vs = v_s[buf];
#pragma unroll
        for (int kk = 0; kk < kTK / 32; ++kk) {
            const int tl = kk * 32 + 8 * kb;                      // first of this lane's 8 tokens, within the tile
            const int tg = kt * kTK + tl;                         // ... and its absolute position
            int ham[kRB][8], tmin[kRB];
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) tmin[rb] = 1 << 20;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const SketchRow<W> sk = load_sketch<W>(sks + (size_t)(tl + j) * W);
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) {
                    int hd = 0;
#pragma unroll
                    for (int w = 0; w < W; ++w) hd += __popcll(sq[rb][w] ^ sk.w[w]);
                    if (kMasked && tg + j > pos[rb]) hd = 1 << 20;                  // causal mask (also: rows past the chunk)
                    ham[rb][j] = hd;
                    tmin[rb] = min(tmin[rb], hd);
                }
            }
            bool changed = false;
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) {
                tmin[rb] = xor32_min(xor16_min(tmin[rb]));        // over the row's four token groups
                changed |= tmin[rb] < run_min[rb];
            }
            if (__any(changed)) {                                 // rare: the running maximum of some row moved
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) {
                    const int nm = min(run_min[rb], tmin[rb]);
                    const float f = exp2f(a.exp2_scale * (float)(nm - run_min[rb]));   // 0 while nothing was accumulated
                    run_min[rb] = nm;
                    // accumulator element j of this lane belongs to row 4 kb + j, whose factor lane 4 kb + j holds
                    float fr[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) fr[j] = __shfl(f, 4 * kb + j);
#pragma unroll
                    for (int j = 0; j < 4; ++j) accsum[rb][j] *= fr[j];
#pragma unroll
                    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc[rb][cb][j] *= fr[j];
                }
            }
            HalfOperand A[kRB];
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) {
                const float base = fmaf(a.exp2_scale, (float)run_min[rb], kPScaleLog2);
#pragma unroll
                for (int j = 0; j < 8; j += 2) {
                    float p0 = __builtin_amdgcn_exp2f(fmaf(-a.exp2_scale, (float)ham[rb][j], base));
                    float p1 = __builtin_amdgcn_exp2f(fmaf(-a.exp2_scale, (float)ham[rb][j + 1], base));
                    if (kMasked) {
                        p0 = ham[rb][j] >= (1 << 20) ? 0.0f : p0;
                        p1 = ham[rb][j + 1] >= (1 << 20) ? 0.0f : p1;
                    }
                    const fp16x2 pk = __builtin_amdgcn_cvt_pkrtz(p0, p1);
                    A[rb].u[j / 2] = *reinterpret_cast<const uint32_t *>(&pk);
                }
            }
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                const f16x8 B = *reinterpret_cast<const f16x8 *>(vs + (16 * cb + i) * kVStride + tl * 2);
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A[rb].v, B, acc[rb][cb], 0, 0, 0);
            }
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) accsum[rb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A[rb].v, ones.v, accsum[rb], 0, 0, 0);
        }
    };

    StageRegs sr;
    load_tile(sr, 0);
    store_tile(sr, 0, 0);
    __syncthreads();
    for (int kt = 0; kt < n_tiles; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < n_tiles) load_tile(sr, kt + 1);
        const int t_first = kt * kTK, t_last = t_first + kTK - 1;
        if (t_first <= wave_max_pos) {                             // else: the whole tile lies in this wave's future
            if (t_last <= wave_min_pos && wave_row0 + 16 * kRB <= n_q) consume_tile(kt, buf, std::false_type{});
            else consume_tile(kt, buf, std::true_type{});
        }
        if (kt + 1 < n_tiles) store_tile(sr, kt + 1, buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: accumulator element j of lane (n = i, kb) is row 4 kb + j, channel 16 cb + n ----
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int qi = wave_row0 + rb * 16 + 4 * kb + j;
            if (qi >= n_q) continue;
            const float inv = 1.0f / accsum[rb][j];
            float *dst = a.out + (((size_t)seq_g * n_q + qi) * Hq + h) * D + i;
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) dst[16 * cb] = acc[rb][cb][j] * inv;
        }
}

// ---- Eq.(2) for the chunk's query vectors: lane = sketch bit, R row in registers, 64 vectors per LDS tile ----
constexpr int kSketchTile = 64;

__device__ __forceinline__ void load8f(const __half *p, float *out) {
    const uint4 raw = *reinterpret_cast<const uint4 *>(p);
    const __half2 *h = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float2 f = __half22float2(h[k]);
        out[2 * k] = f.x;
        out[2 * k + 1] = f.y;
    }
}
__device__ __forceinline__ void load8f(const float *p, float *out) {
    const float4 x = *reinterpret_cast<const float4 *>(p);
    const float4 y = *reinterpret_cast<const float4 *>(p + 4);
    out[0] = x.x; out[1] = x.y; out[2] = x.z; out[3] = x.w;
    out[4] = y.x; out[5] = y.y; out[6] = y.z; out[7] = y.w;
}
__device__ __forceinline__ void copy8f(const __half *src, __half *dst) { *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(src); }
__device__ __forceinline__ void copy8f(const float *src, float *dst) {
    *reinterpret_cast<float4 *>(dst) = *reinterpret_cast<const float4 *>(src);
    *reinterpret_cast<float4 *>(dst + 4) = *reinterpret_cast<const float4 *>(src + 4);
}

template <int D, typename T>
__global__ __launch_bounds__(kThreads) void sketch_rows_kernel(PrefillArgs a, int n_seqs) {
    __shared__ __attribute__((aligned(16))) T qs[kSketchTile][D];
    __shared__ size_t src_off[kSketchTile];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const PoolView &pv = a.pool;
    const int W = pv.sketch_bits >> 6, Hq = pv.n_q_heads;
    const long n_vec = (long)n_seqs * a.n_q * Hq;
    const T *qbase = static_cast<const T *>(a.q);

    const int wslots = W < 4 ? W : 4, tslots = 4 / wslots;
    float r[D];
    int r_word = wave % wslots;
    auto load_row = [&](int word) {
        const float *row = pv.R + (size_t)(word * 64 + lane) * D;
#pragma unroll
        for (int j = 0; j < D; j += 4) {
            const float4 x = *reinterpret_cast<const float4 *>(row + j);
            r[j] = x.x; r[j + 1] = x.y; r[j + 2] = x.z; r[j + 3] = x.w;
        }
    };
    load_row(r_word);

    for (long v0 = (long)blockIdx.x * kSketchTile; v0 < n_vec; v0 += (long)gridDim.x * kSketchTile) {
        __syncthreads();
        const int n_here = (int)min((long)kSketchTile, n_vec - v0);
        if (tid < n_here) {
            const long v = v0 + tid;
            const long s = v / ((long)a.n_q * Hq), rem = v % ((long)a.n_q * Hq);
            src_off[tid] = (size_t)s * a.stride_seq + (size_t)(rem / Hq) * a.stride_tok + (size_t)(rem % Hq) * a.stride_head;
        }
        __syncthreads();
        for (int e = tid * 8; e < n_here * D; e += kThreads * 8) {
            const int rl = e / D, ch = e % D;
            copy8f(qbase + src_off[rl] + ch, &qs[rl][ch]);
        }
        __syncthreads();
        for (int word = wave % wslots; word < W; word += wslots) {
            if (word != r_word) {
                load_row(word);
                r_word = word;
            }
            for (int t = wave / wslots; t < n_here; t += tslots) {
                float y = 0.0f;
#pragma unroll
                for (int j = 0; j < D; j += 8) {
                    float kk[8];
                    load8f(&qs[t][j], kk);
#pragma unroll
                    for (int k = 0; k < 8; ++k) y = __builtin_fmaf(r[j + k], kk[k], y);
                }
                const uint64_t mask = __ballot(y >= 0.0f);
                if (lane == 0) a.q_sketch[(size_t)(v0 + t) * W + word] = mask;
            }
        }
    }
}

template <int W, int D>
hipError_t launch_prefill_layout(const PrefillArgs &a, const BatchDesc &desc, int seq0, dim3 grid, hipStream_t st) {
    if (a.pool.code_layout == 0) hipLaunchKernelGGL((prefill_kernel<W, D, 0>), grid, dim3(kThreads), 0, st, a, desc, seq0);
    else hipLaunchKernelGGL((prefill_kernel<W, D, 1>), grid, dim3(kThreads), 0, st, a, desc, seq0);
    return hipGetLastError();
}

template <int W>
hipError_t launch_prefill_d(const PrefillArgs &a, const BatchDesc &desc, int seq0, dim3 grid, hipStream_t st) {
    switch (a.pool.head_dim) {
        case 64: return launch_prefill_layout<W, 64>(a, desc, seq0, grid, st);
        case 128: return launch_prefill_layout<W, 128>(a, desc, seq0, grid, st);
        default: return hipErrorInvalidValue;      // see prefill_supported
    }
}

}  // namespace

hipError_t launch_prefill(const PrefillArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st) {
    const dim3 grid((unsigned)((a.n_q + kQB - 1) / kQB), (unsigned)a.pool.n_q_heads, (unsigned)n_seqs);
    switch (a.pool.sketch_bits) {
        case 64: return launch_prefill_d<1>(a, desc, seq0, grid, st);
        case 128: return launch_prefill_d<2>(a, desc, seq0, grid, st);
        case 256: return launch_prefill_d<4>(a, desc, seq0, grid, st);
        default: return launch_prefill_d<8>(a, desc, seq0, grid, st);
    }
}

hipError_t launch_sketch_rows(const PrefillArgs &a, int n_seqs, hipStream_t st) {
    const long n_vec = (long)n_seqs * a.n_q * a.pool.n_q_heads;
    const long tiles = (n_vec + kSketchTile - 1) / kSketchTile;
    const dim3 grid((unsigned)(tiles < 1024 ? tiles : 1024));
    const int D = a.pool.head_dim;
#define H1BKV_LAUNCH(DD, TT) hipLaunchKernelGGL((sketch_rows_kernel<DD, TT>), grid, dim3(kThreads), 0, st, a, n_seqs)
    if (D != 64 && D != 128) return hipErrorInvalidValue;      // see prefill_supported
    if (a.f16) {
        if (D == 64) H1BKV_LAUNCH(64, __half);
        else H1BKV_LAUNCH(128, __half);
    } else {
        if (D == 64) H1BKV_LAUNCH(64, float);
        else H1BKV_LAUNCH(128, float);
    }
#undef H1BKV_LAUNCH
    return hipGetLastError();
}

}  // namespace h1bkv
