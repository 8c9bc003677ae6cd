// Prefill attention over the compressed cache: Eq.(3) and Eq.(5) for every position of a prompt chunk, causally --
// query i of a sequence attends to the cached tokens up to and including its own position, exactly the decode step
// it would have seen had the prompt been fed one token at a time.
//
// With many queries per KV head both halves of the step are dense contractions and run on the matrix cores:
//   scores    alpha needs the Hamming distance of every (query, key) pair.  With the key bits unpacked to {0,1} bytes
//             and the query bits to {+4,-4} bytes,  sum_k q_k key_k = 4 (popcount(q) - ham),  so one int8 MFMA
//             (v_mfma_i32_16x16x64_i8) per 64 sketch bits yields 16 x 16 distances -- instead of 4 W XOR/popcount
//             instructions per pair on the vector ALUs.  The MFMA is issued as keys x queries, so that a lane ends
//             up holding distances of ONE query row against several tokens: the slot it has in the next MFMA.
//   weights   p = exp((alpha - alpha_ref)/tau) takes only a few hundred values (the distance from the row's reference
//             distance is an integer): one LDS table read per pair instead of an exponential, at the byte offset
//             4 (popcount(q) - ref) - score (hence the +-4).  The reference is a running minimum with slack: it is
//             renewed, and the accumulators rescaled, only when a distance falls further below it than the fp16 range
//             of the weights allows.  Weights are packed to fp16 in registers as the A operand of the second MFMA;
//             the normalisation uses the row sums of the SAME fp16 weights (one more MFMA against an all-ones B).
//   values    sum_t p[i][t] v^[t][c]  with v_mfma_f32_16x16x32_f16, fp32 accumulate.
// One workgroup (8 waves) takes 128 consecutive query positions of one (sequence, query head) -- 16 rows per wave --
// and walks the key tokens in tiles up to its diagonal.  Per tile the workgroup stages ONCE, for all its rows: the
// keys' bits as bytes, and the values dequantised, v^ = fp16(scale * code + zero), channel-major, in the token order
// the score MFMA leaves its results in (so an MFMA B operand is one 16-byte LDS read).  The next tile's global loads
// are issued before the current tile is consumed.  Tiles entirely below a wave's rows take an unmasked path; tiles
// entirely above them are skipped.
// sketch_rows_kernel sketches the chunk's query vectors (Eq.(2), same fp32 FMA chain as the keys) with the R rows
// resident in registers, 64 vectors per LDS tile.
#include <hip/hip_fp16.h>

#include <type_traits>

#include "decode_common.h"
#include "projection_mfma.h"

namespace h1bkv {

namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 h16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

// Eight waves of one 16-row block each: the same 128 query rows and the same LDS tiles per workgroup as four waves of
// two blocks, at half the registers per wave, so that four waves share a SIMD (a single wave issues a vector
// instruction only every five clocks or so; two workgroups per compute unit also cover each other's barriers).
constexpr int kPfWaves = 8;
constexpr int kPfThreads = kPfWaves * 64;
constexpr int kRB = 1;                        // 16-row blocks per wave
constexpr int kQB = kPfWaves * 16 * kRB;      // query positions per workgroup
constexpr int kCS = 8;                        // channels per staging item of the token-major layouts
constexpr float kPScaleLog2 = 4.0f;           // weights are stored as p * 2^4
constexpr float kPSlackLog2 = 11.0f;          // and may exceed 1 by up to 2^11 (p 2^4 <= 2^15 stays finite in fp16)

union HalfOperand {
    uint32_t u[4];
    f16x8 v;
};
union ByteOperand {
    uint32_t u[4];
    i32x4 v;
};

__device__ __forceinline__ int xor16_min(int x) {       // min with the lane 16 away (immediate swizzle, inside a half-wave)
    return min(x, __builtin_amdgcn_ds_swizzle(x, 0x1F | (0x10 << 10)));
}
__device__ __forceinline__ int xor32_min(int x) {       // min with the lane 32 away
    const auto r = __builtin_amdgcn_permlane32_swap((unsigned)x, (unsigned)x, false, false);
    return min((int)r[0], (int)r[1]);
}
// Bits 0..3 of x -> the low bits of bytes 0..3: the 24-bit multiply by 0x204081 puts copies of the nibble at bit
// offsets 0, 7, 14, 21, so that bit k lands on bit 8 k (full-rate multiply; three instructions with the extract).
__device__ __forceinline__ uint32_t spread4(uint32_t x) {
    return __umul24(x & 0xFu, 0x00204081u) & 0x01010101u;
}

template <int NDW>
struct StageRegs {           // one thread's share of a key tile on its way from global memory to LDS
    uint32_t skd[NDW];       // 16 sketch bits each
    uint32_t c[2];           // layout 0: kCS / 2 bytes of codes for each of two tokens;  layout 1: up to 2 code words of one block
    uint32_t m[16];          // layout 0: {scale, zero} of the two tokens;  layout 1: of the block's 8 tokens, for each
                             //           of the thread's words;  layout 2: kCS fp16 values of each of the two tokens
};

template <int W, int D, int LAYOUT>
__global__ __launch_bounds__(kPfThreads, W >= 8 ? 2 : 4) void prefill_kernel(PrefillArgs a, BatchDesc desc, int seq0) {
    constexpr int NCB = D / 16;
    constexpr int TK = W <= 2 ? 64 : 32;          // key tokens per tile (wide sketches: smaller tiles, same LDS budget)
    constexpr int NSTEP = TK / 32;                // 32-token MFMA steps per tile
    constexpr int VS = TK * 2 + 16;               // bytes per channel row of the value tile (16 B pad: conflict-free b128 reads)
    constexpr int KS = 64 * W + 16;               // bytes per token row of the key-bit tile (same padding)
    constexpr int DWT = TK * 4 * W;               // 16-bit sketch units per tile
    constexpr int NDW = DWT > kPfThreads ? DWT / kPfThreads : 1;
    __shared__ __attribute__((aligned(16))) unsigned char v_s[2][D * VS];
    __shared__ __attribute__((aligned(16))) unsigned char k_s[2][TK * KS];
    // p(e) = 2^4 exp(-2 e / (b tau)) for every distance e from a row's reference distance, e = -S .. b; one more
    // entry holds 0 for masked pairs.  One LDS read per pair replaces convert + multiply-add + exponential (a
    // quarter-rate instruction).  The reference is the smallest distance the row had seen when it was last set and
    // is only renewed (accumulators rescaled) when a distance falls more than S below it, S the largest slack whose
    // weights still fit fp16 (exp(2 S / (b tau)) <= 2^11): the best distance of a row improves by a few units many
    // times over a long context, and rescaling on each of them was a tenth of the vector work.
    __shared__ float ptab[128 * W + 2];
    // The sequence's page ids, read once: a block-table lookup per tile from global memory sits, with its full memory
    // latency, in front of every tile's loads.
    constexpr int kPagesLds = 1024;
    __shared__ int pages_s[kPagesLds];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, kb = lane >> 4;
    // grid (query head, sequence, query block x context split): workgroups are dispatched x-fastest, so the
    // longest-running (latest) query blocks of ALL heads and sequences start first and the short ones fill the tail of
    // the launch.  With n_splits > 1 (a chunk that is short against its context) a workgroup walks only its share of
    // the block's key tiles and leaves (sums, weight sum, reference distance) per row for prefill_merge_kernel.
    const SeqDesc sd = desc.s[blockIdx.y];
    const int len = sd.pos, n_q = a.n_q;
    const int n_splits = a.n_splits, split = (int)blockIdx.z % n_splits;
    const int qb = (int)gridDim.z / n_splits - 1 - (int)blockIdx.z / n_splits;
    const int row0 = qb * kQB;
    const int q0 = len - n_q;                                      // absolute position of query 0
    const int last_row = min(row0 + kQB, n_q) - 1;
    const int n_tiles = (q0 + last_row + TK) / TK;                 // tiles that hold tokens visible to the last row
    const int tile_lo = (int)((long)n_tiles * split / n_splits), tile_hi = (int)((long)n_tiles * (split + 1) / n_splits);

    const PoolView &pv = a.pool;
    const int H = pv.n_kv_heads, Hq = pv.n_q_heads, r = Hq / H;
    const int h = blockIdx.x, kvh = h / r;
    const int seq_g = seq0 + blockIdx.y;
    const int ng = D / pv.group_size;
    const int32_t *bt = pv.block_table + (size_t)sd.seq_id * pv.max_pages_per_seq;

    // ---- this lane's query rows: position, popcount, and bits 16 kb .. 16 kb + 15 of every 64-bit word as +-4 bytes ----
    // (+-4, not +-1: the score MFMA then returns 4 (popcount(q) - ham), and 4 (ham - ham_min) is the byte offset of the
    // pair's weight in the table, with no shift and no separate distance)
    int pos[kRB], pcq[kRB];       // pos: absolute position of row (rb, i), -1 for rows past the chunk;  pcq: 4 popcount(q)
    ByteOperand qpm[kRB][W];
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) {
        const int qi = row0 + wave * 16 * kRB + rb * 16 + i;
        pos[rb] = qi < n_q ? q0 + qi : -1;
        pcq[rb] = 0;
#pragma unroll
        for (int w = 0; w < W; ++w) {
            const uint64_t sq = qi < n_q ? a.q_sketch[(((size_t)seq_g * n_q + qi) * Hq + h) * W + w] : 0;
            pcq[rb] += 4 * __popcll(sq);
            const uint32_t bits = (uint32_t)(sq >> (16 * kb)) & 0xFFFFu;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t t = spread4(bits >> (4 * k));
                qpm[rb][w].u[k] = (t << 2) | ((t ^ 0x01010101u) * 0xFCu);     // bit 1 -> 0x04 (+4), bit 0 -> 0xFC (-4)
            }
        }
    }
    const int wave_row0 = row0 + wave * 16 * kRB;
    const int wave_min_pos = q0 + wave_row0;                                       // position of the wave's first row
    const int wave_max_pos = wave_row0 < n_q ? q0 + min(wave_row0 + 16 * kRB, n_q) - 1 : -1;   // ... and of its last valid row

    f32x4 acc[kRB][NCB], accsum[kRB];
    int run_min[kRB];             // 4 x the row's reference distance
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) {
        run_min[rb] = 1 << 22;
        accsum[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) acc[rb][cb] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const int S = (int)fminf(kPSlackLog2 / a.exp2_scale, (float)(64 * W));
    for (int e = threadIdx.x; e < 64 * W + S + 2; e += kPfThreads)
        ptab[e] = e <= 64 * W + S ? __builtin_amdgcn_exp2f(fmaf(-a.exp2_scale, (float)(e - S), kPScaleLog2)) : 0.0f;
    const uint32_t mask_a = opaque_vgpr(0x000F000Fu), mask_b = opaque_vgpr(0x00F000F0u);
    HalfOperand ones;
#pragma unroll
    for (int k = 0; k < 4; ++k) ones.u[k] = 0x3C003C00u;          // fp16 1.0

    // Token t of a 32-token step sits at operand position 8 ((t % 16) / 4) + 4 (t / 16) + t % 4: the score MFMA of
    // token block t / 16 leaves tokens 4 kb .. 4 kb + 3 in lane group kb, and the value MFMA wants that lane group's
    // eight tokens side by side.
    auto operand_pos = [](int t) { return (t & ~31) + 8 * ((t & 15) >> 2) + 4 * ((t >> 4) & 1) + (t & 3); };

    // ---- staging: global -> registers (issued early) -> LDS (after the current tile has been consumed) ----
    constexpr int kItems0 = (TK / 2) * (D / kCS);                 // layouts 0, 2: (token pair, channel slice) items per tile
    static_assert(kCS == 8 && kItems0 <= kPfThreads, "one staging item per thread");
    // layout 1: a thread takes one of the tile's TK / 8 blocks and words (tid % LPB) + LPB k of its D words (word wi
    // holds channel 16 cb + n with cb = (wi / 64) * 4 + wi % 4, n = (wi % 64) / 4: the inverse of code_word_index).
    // A word holds eight tokens of ONE channel: its {scale, zero} sets are those of that channel's quantisation group.
    constexpr int LPB = kPfThreads / (TK / 8);
    constexpr int kWordsPerThread = D > LPB ? D / LPB : 1;
    static_assert(kWordsPerThread <= 2, "StageRegs holds two words and their sets");
    auto word_channel = [](int wi) { return 16 * ((wi >> 6) * 4 + (wi & 3)) + ((wi & 63) >> 2); };
    {
        const int n_pages = ((n_tiles - 1) * TK) / kPage + 1;
        for (int p = tid; p < min(n_pages, kPagesLds); p += kPfThreads) pages_s[p] = bt[p];
        __syncthreads();
    }
    auto tile_rec0 = [&](int kt) {
        const int t0 = kt * TK, p = t0 / kPage;
        const int page = p < kPagesLds ? pages_s[p] : bt[p];
        return ((size_t)page * H + kvh) * kPage + (t0 % kPage);                    // a tile never straddles a page
    };
    auto load_tile = [&](StageRegs<NDW> &sr, int kt) {
        const size_t rec0 = tile_rec0(kt);
        const uint16_t *skw = reinterpret_cast<const uint16_t *>(pv.sketch + rec0 * W);
#pragma unroll
        for (int u = 0; u < NDW; ++u)
            if (tid + u * kPfThreads < DWT) sr.skd[u] = skw[tid + u * kPfThreads];
        if constexpr (LAYOUT == 0) {
            if (tid < kItems0) {
                const int tp = tid % (TK / 2), sl = tid / (TK / 2);         // token pair fastest: see the LDS writes below
                const int g = (kCS * sl) / pv.group_size;
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const size_t rec = rec0 + 2 * tp + t;
                    sr.c[t] = *reinterpret_cast<const uint32_t *>(pv.codes + rec * (D / 2) + sl * 4);
                    sr.m[t] = pv.meta[rec * ng + g];
                }
            }
        } else if constexpr (LAYOUT == 2) {              // fp16 values: 8 channels (16 bytes) of each of two tokens
            if (tid < kItems0) {
                const int tp = tid % (TK / 2), sl = tid / (TK / 2);
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const uint4 a0 = *reinterpret_cast<const uint4 *>(pv.codes + ((rec0 + 2 * tp + t) * D + kCS * sl) * 2);
                    sr.m[4 * t + 0] = a0.x; sr.m[4 * t + 1] = a0.y; sr.m[4 * t + 2] = a0.z; sr.m[4 * t + 3] = a0.w;
                }
            }
        } else {
            const int blk = tid / LPB, w0 = tid % LPB;
            const uint32_t *words = reinterpret_cast<const uint32_t *>(pv.codes + (rec0 + 8 * blk) * (D / 2));
#pragma unroll
            for (int k = 0; k < kWordsPerThread; ++k) {
                const int wi = w0 + LPB * k;
                if (wi < D) {
                    sr.c[k] = words[wi];
                    const int g = word_channel(wi) / pv.group_size;
#pragma unroll
                    for (int j = 0; j < 8; ++j) sr.m[8 * k + j] = pv.meta[(rec0 + 8 * blk + j) * ng + g];
                }
            }
        }
    };
    auto store_tile = [&](const StageRegs<NDW> &sr, int kt, int buf) {
        const int t0 = kt * TK;
        // key bits -> {0,1} bytes: 16 bits in, 16 bytes out
        unsigned char *ks = k_s[buf];
#pragma unroll
        for (int u = 0; u < NDW; ++u) {
            const int dwi = tid + u * kPfThreads;
            if (dwi < DWT) {
                const int tok = dwi / (4 * W), part = dwi % (4 * W);
                uint32_t o[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) o[k] = spread4(sr.skd[u] >> (4 * k));
                *reinterpret_cast<uint4 *>(ks + tok * KS + part * 16) = make_uint4(o[0], o[1], o[2], o[3]);
            }
        }
        unsigned char *vs = v_s[buf];
        if constexpr (LAYOUT == 0) {
            if (tid < kItems0) {
                // lanes of a half-wave hold different token pairs of one channel slice: their 4-byte writes into a
                // channel row fall into different LDS banks
                const int tp = tid % (TK / 2), sl = tid / (TK / 2);
                float sc[2], zp[2];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    // slots past the end of the sequence hold anything: their values must not reach the MFMA as NaN
                    const uint32_t m = t0 + 2 * tp + t < len ? sr.m[t] : 0u;
                    sc[t] = __half2float(__ushort_as_half((unsigned short)(m & 0xFFFFu)));
                    zp[t] = __half2float(__ushort_as_half((unsigned short)(m >> 16)));
                }
                const int p2 = operand_pos(2 * tp) * 2;            // tokens 2 tp and 2 tp + 1 stay neighbours
                // A nibble masked in place at mantissa bits 0-3 / 4-7 of a zero half-word is the fp16 subnormal
                // code 2^-24 / code 2^-20: the mixed-precision FMA reads it directly, with the scale times 2^24 / 2^20.
                const float sa[2] = {sc[0] * 16777216.0f, sc[1] * 16777216.0f}, sb[2] = {sc[0] * 1048576.0f, sc[1] * 1048576.0f};
                {
                    const uint32_t x0 = sr.c[0], x1 = sr.c[1], y0 = x0 >> 8, y1 = x1 >> 8;
                    const uint32_t t0w[4] = {x0 & mask_a, x0 & mask_b, y0 & mask_a, y0 & mask_b};
                    const uint32_t t1w[4] = {x1 & mask_a, x1 & mask_b, y1 & mask_a, y1 & mask_b};
#pragma unroll
                    for (int n = 0; n < 4; ++n) {                  // word n holds nibbles n (low half) and n + 4 (high half)
                        const __half2 h0 = *reinterpret_cast<const __half2 *>(&t0w[n]), h1 = *reinterpret_cast<const __half2 *>(&t1w[n]);
                        const float w0 = (n & 1) ? sb[0] : sa[0], w1 = (n & 1) ? sb[1] : sa[1];
                        const f32x2 lo = {fmaf(w0, __low2float(h0), zp[0]), fmaf(w1, __low2float(h1), zp[1])};
                        const f32x2 hi = {fmaf(w0, __high2float(h0), zp[0]), fmaf(w1, __high2float(h1), zp[1])};
                        const h16x2 plo = __builtin_convertvector(lo, h16x2), phi = __builtin_convertvector(hi, h16x2);
                        *reinterpret_cast<h16x2 *>(vs + (kCS * sl + n) * VS + p2) = plo;
                        *reinterpret_cast<h16x2 *>(vs + (kCS * sl + n + 4) * VS + p2) = phi;
                    }
                }
            }
        } else if constexpr (LAYOUT == 2) {
            if (tid < kItems0) {
                const int tp = tid % (TK / 2), sl = tid / (TK / 2);
                const int p2 = operand_pos(2 * tp) * 2;
                // slots past the end of the sequence hold anything: their values must not reach the MFMA as NaN
                const uint32_t keep0 = t0 + 2 * tp < len ? 0xFFFFu : 0u, keep1 = t0 + 2 * tp + 1 < len ? 0xFFFFu : 0u;
#pragma unroll
                for (int c = 0; c < kCS; ++c) {
                    const uint32_t h0 = (sr.m[c >> 1] >> (16 * (c & 1))) & keep0, h1 = (sr.m[4 + (c >> 1)] >> (16 * (c & 1))) & keep1;
                    *reinterpret_cast<uint32_t *>(vs + (kCS * sl + c) * VS + p2) = h0 | (h1 << 16);
                }
            }
        } else {
            const int blk = tid / LPB, w0 = tid % LPB;
#pragma unroll
            for (int k = 0; k < kWordsPerThread; ++k) {
                const int wi = w0 + LPB * k, ch = word_channel(wi);
                if (wi >= D) continue;
                const uint32_t x = sr.c[k], y = x >> 8;
                // nibble n of the word is token 2 n of the block, nibble n + 4 token 2 n + 1: word n below holds that
                // pair as fp16 subnormals (code 2^-24 for even n, code 2^-20 for odd n)
                const uint32_t tw[4] = {x & mask_a, x & mask_b, y & mask_a, y & mask_b};
                h16x2 hv[4];
#pragma unroll
                for (int n = 0; n < 4; ++n) {
                    float f[2];
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const int j = 2 * n + e;
                        // slots past the end of the sequence hold anything: their values must not reach the MFMA as NaN
                        const uint32_t m = t0 + 8 * blk + j < len ? sr.m[8 * k + j] : 0u;
                        const float sc = __half2float(__ushort_as_half((unsigned short)(m & 0xFFFFu)));
                        const float zp = __half2float(__ushort_as_half((unsigned short)(m >> 16)));
                        const __half2 h = *reinterpret_cast<const __half2 *>(&tw[n]);
                        f[e] = fmaf(sc * ((n & 1) ? 1048576.0f : 16777216.0f), e ? __high2float(h) : __low2float(h), zp);
                    }
                    const f32x2 pf = {f[0], f[1]};
                    hv[n] = __builtin_convertvector(pf, h16x2);
                }
                // tokens 8 blk .. 8 blk + 3 and 8 blk + 4 .. 8 blk + 7 go to two operand positions
                *reinterpret_cast<uint2 *>(vs + ch * VS + operand_pos(8 * blk) * 2) = *reinterpret_cast<const uint2 *>(&hv[0]);
                *reinterpret_cast<uint2 *>(vs + ch * VS + operand_pos(8 * blk + 4) * 2) = *reinterpret_cast<const uint2 *>(&hv[2]);
            }
        }
    };

    // ---- one tile: score MFMA, weights, value MFMA ----
    auto consume_tile = [&](int kt, int buf, auto masked_tag) {
        constexpr bool kMasked = decltype(masked_tag)::value;
        const unsigned char *ks = k_s[buf];
        const unsigned char *vs = v_s[buf];
#pragma unroll 1
        for (int st = 0; st < NSTEP; ++st) {
            // Hamming distances: lane (row i, kb) receives tokens 16 tb + 4 kb + j of the step, tb = 0, 1
            i32x4 dot[kRB][2];
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) {
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) dot[rb][tb] = i32x4{0, 0, 0, 0};
#pragma unroll
                for (int w = 0; w < W; ++w) {
                    const i32x4 K = *reinterpret_cast<const i32x4 *>(ks + (32 * st + 16 * tb + i) * KS + 64 * w + 16 * kb);
#pragma unroll
                    for (int rb = 0; rb < kRB; ++rb)
                        dot[rb][tb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(K, qpm[rb][w].v, dot[rb][tb], 0, 0, 0);
                }
            }
            const int tg = kt * TK + 32 * st + 4 * kb;            // absolute position of this lane's first token (tb = 0, j = 0)
            int dq[kRB][8], tmin[kRB];
            bool changed = false;
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) {
                int dmax = -(1 << 22);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    int d = dot[rb][j >> 2][j & 3];              // sum_k q_k key_k = 4 (popcount(q) - ham)
                    if (kMasked && tg + 16 * (j >> 2) + (j & 3) > pos[rb]) d = -(1 << 22);    // causal mask (also: rows past the chunk)
                    dq[rb][j] = d;
                    dmax = max(dmax, d);
                }
                tmin[rb] = xor32_min(xor16_min(pcq[rb] - dmax));  // 4 x the smallest distance of the step, over the row's four lane groups
                changed |= tmin[rb] < run_min[rb] - 4 * S;
            }
            if (__any(changed)) {                                 // rare: some row's best distance left the slack
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) {
                    const int nm = tmin[rb] < run_min[rb] - 4 * S ? tmin[rb] : run_min[rb];
                    const float f = exp2f(0.25f * a.exp2_scale * (float)(nm - run_min[rb]));   // 0 while nothing was accumulated
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
            // Weights from the table: p depends only on e = ham - reference, an integer in [-S, b]; masked pairs
            // are clamped to the table's zero entry.  4 (e + S) = 4 (popcount(q) - reference + S) - score is the entry's
            // byte offset.
            HalfOperand A[kRB];
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) {
#pragma unroll
                for (int j = 0; j < 8; j += 2) {
                    const int base = pcq[rb] - run_min[rb] + 4 * S;
                    int e0 = base - dq[rb][j], e1 = base - dq[rb][j + 1];
                    if (kMasked) {
                        e0 = min(e0, 4 * (64 * W + 1) + 4 * S);
                        e1 = min(e1, 4 * (64 * W + 1) + 4 * S);
                    }
                    const unsigned char *tab = reinterpret_cast<const unsigned char *>(ptab);
                    const float p0 = *reinterpret_cast<const float *>(tab + e0), p1 = *reinterpret_cast<const float *>(tab + e1);
                    // round to nearest (one packed convert on gfx950), not the truncating pack: half the weight error
                    const f32x2 pf = {p0, p1};
                    const h16x2 pk = __builtin_convertvector(pf, h16x2);
                    A[rb].u[j / 2] = *reinterpret_cast<const uint32_t *>(&pk);
                }
            }
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                const f16x8 B = *reinterpret_cast<const f16x8 *>(vs + (16 * cb + i) * VS + (32 * st + 8 * kb) * 2);
#pragma unroll
                for (int rb = 0; rb < kRB; ++rb) acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A[rb].v, B, acc[rb][cb], 0, 0, 0);
            }
#pragma unroll
            for (int rb = 0; rb < kRB; ++rb) accsum[rb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A[rb].v, ones.v, accsum[rb], 0, 0, 0);
        }
    };

    StageRegs<NDW> sr;
    if (tile_lo < tile_hi) {                                       // (a short sequence may leave a split without tiles)
        load_tile(sr, tile_lo);
        store_tile(sr, tile_lo, tile_lo & 1);
    }
    __syncthreads();
    for (int kt = tile_lo; kt < tile_hi; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < tile_hi) load_tile(sr, kt + 1);
        const int t_first = kt * TK, t_last = t_first + TK - 1;
        if (t_first <= wave_max_pos) {                             // else: the whole tile lies in this wave's future
            if (t_last <= wave_min_pos && wave_row0 + 16 * kRB <= n_q) consume_tile(kt, buf, std::false_type{});
            else consume_tile(kt, buf, std::true_type{});
        }
        if (kt + 1 < tile_hi) store_tile(sr, kt + 1, buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: accumulator element j of lane (n = i, kb) is row 4 kb + j, channel 16 cb + n ----
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int qi = wave_row0 + rb * 16 + 4 * kb + j;
            const int ref = __shfl(run_min[rb], 4 * kb + j);      // the row's reference distance sits in lane 4 kb + j
            if (qi >= n_q) continue;
            if (n_splits == 1) {
                const float inv = 1.0f / accsum[rb][j];
                float *dst = a.out + (((size_t)seq_g * n_q + qi) * Hq + h) * D + i;
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb) dst[16 * cb] = acc[rb][cb][j] * inv;
            } else {
                float *dst = a.part + ((((size_t)seq_g * n_q + qi) * Hq + h) * n_splits + split) * (D + 2);
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb) dst[16 * cb + i] = acc[rb][cb][j];
                if (i == 0) {
                    dst[D] = accsum[rb][j];
                    dst[D + 1] = __int_as_float(ref);
                }
            }
        }
}

// out = sum_s f_s o_s / sum_s f_s l_s over the context splits of one (query position, head), f_s = exp(-2 (ref_s -
// ref_min) / (b tau)): the splits' sums are relative to their own reference distances.  A split that saw no visible
// token of the row carries the initial reference (2^22) and zero sums: its factor is 0.
__global__ void prefill_merge_kernel(PrefillArgs a, int seq0) {
    const int D = a.pool.head_dim, S = a.n_splits, c = threadIdx.x;
    const size_t row = (size_t)seq0 * a.n_q * a.pool.n_q_heads + blockIdx.x;        // (sequence, position, head), flattened
    const float *p = a.part + row * S * (D + 2);
    int ref = 1 << 22;
    for (int s = 0; s < S; ++s) ref = min(ref, __float_as_int(p[(size_t)s * (D + 2) + D + 1]));
    float l = 0.0f, o = 0.0f;
    for (int s = 0; s < S; ++s) {
        const float *ps = p + (size_t)s * (D + 2);
        const float f = __builtin_amdgcn_exp2f(0.25f * a.exp2_scale * (float)(ref - __float_as_int(ps[D + 1])));
        l = fmaf(f, ps[D], l);
        o = fmaf(f, ps[c], o);
    }
    a.out[row * D + c] = o / l;
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

// The projections on the matrix cores, the bits inside the guard band by the chain (projection_mfma.h); the pieces of R
// are read per tile (any sketch width).
template <int D, typename T>
__global__ __launch_bounds__(kThreads, 4) void sketch_rows_mfma_kernel(PrefillArgs a, int n_seqs) {
    constexpr bool F32 = sizeof(T) == 4;                           // fp32 queries: scaled and split into two fp16 piece tiles
    constexpr int STRIDE = D + 8;                                  // halves per LDS row
    __shared__ __attribute__((aligned(16))) __half qs[(F32 ? 2 : 1) * kSketchTile * STRIDE];
    __shared__ size_t src_off[kSketchTile];
    __shared__ uint32_t w32[kSketchTile * 16], unsure[kSketchTile * 16];
    __shared__ float band_s[kSketchTile];
    static_assert(kSketchTile == kProjTile && kThreads == kProjThreads, "projection_mfma.h assumes this tile shape");
    const int tid = threadIdx.x;
    const PoolView &pv = a.pool;
    const int W = pv.sketch_bits >> 6, Hq = pv.n_q_heads;
    const long n_vec = (long)n_seqs * a.n_q * Hq;
    const T *qbase = static_cast<const T *>(a.q);
    for (long v0 = (long)blockIdx.x * kSketchTile; v0 < n_vec; v0 += (long)gridDim.x * kSketchTile) {
        __syncthreads();
        const int n_here = (int)min((long)kSketchTile, n_vec - v0);
        for (int e = tid; e < kSketchTile * 16; e += kThreads) {
            w32[e] = 0u;
            unsure[e] = 0u;
        }
        if (tid < n_here) {
            const long v = v0 + tid;
            const long s = v / ((long)a.n_q * Hq), rem = v % ((long)a.n_q * Hq);
            src_off[tid] = (size_t)s * a.stride_seq + (size_t)(rem / Hq) * a.stride_tok + (size_t)(rem % Hq) * a.stride_head;
        }
        __syncthreads();
        if constexpr (F32) {
            stage_f32_tile<D>([&](int rl) { return reinterpret_cast<const float *>(qbase + src_off[rl]); }, n_here, qs,
                              qs + kSketchTile * STRIDE, STRIDE, band_s);
        } else {
            for (int e = tid * 8; e < n_here * D; e += kThreads * 8) {
                const int rl = e / D, ch = e % D;
                copy8f(reinterpret_cast<const __half *>(qbase + src_off[rl] + ch), &qs[rl * STRIDE + ch]);
            }
        }
        __syncthreads();
        project_tile_mfma<D, F32>(pv, qs, qs + (F32 ? kSketchTile * STRIDE : 0), band_s, STRIDE, n_here, [](int) { return true; }, w32,
                                  unsure, []() {}, [&](int rl) { return reinterpret_cast<const float *>(qbase + src_off[rl]); });
        __syncthreads();
        // the 32-bit halves of a vector's sketch words are contiguous in w32 and in the output
        uint32_t *out = reinterpret_cast<uint32_t *>(a.q_sketch + (size_t)v0 * W);
        for (int e = tid; e < n_here * 2 * W; e += kThreads) out[e] = w32[(e / (2 * W)) * 16 + e % (2 * W)];
    }
}

// The same with the pieces of R resident in registers (d <= 128, sketches of at most 64 * 256 / d bits): three long-lived
// workgroups per compute unit walk the tiles (resident_sketch_tiles in projection_mfma.h).
struct QueryRows {
    const PrefillArgs &a;
    long n_vec;
    __device__ int rows_in(long tile) const { return (int)min((long)kSketchTile, n_vec - tile * kSketchTile); }
    __device__ size_t src(long tile, int rl) const {
        const long v = tile * kSketchTile + rl;
        const int Hq = a.pool.n_q_heads;
        long s, rem;
        if (n_vec <= 0x7FFFFFFFL) {                     // (uniform) 32-bit division: a fraction of the 64-bit one's instructions
            const uint32_t per_seq = (uint32_t)a.n_q * (uint32_t)Hq;
            s = (uint32_t)v / per_seq;
            rem = (uint32_t)v % per_seq;
        } else {
            s = v / ((long)a.n_q * Hq);
            rem = v % ((long)a.n_q * Hq);
        }
        return (size_t)s * a.stride_seq + (size_t)((uint32_t)rem / (uint32_t)Hq) * a.stride_tok +
               (size_t)((uint32_t)rem % (uint32_t)Hq) * a.stride_head;
    }
    __device__ int page_request(long, int) const { return 0; }
    __device__ uint32_t *dst(long tile, int rl, int) const {
        return reinterpret_cast<uint32_t *>(a.q_sketch + (size_t)(tile * kSketchTile + rl) * (a.pool.sketch_bits >> 6));
    }
};

template <int D, typename T>
__global__ __launch_bounds__(kThreads, 3) void sketch_rows_resident_kernel(PrefillArgs a, int n_seqs) {
    const long n_vec = (long)n_seqs * a.n_q * a.pool.n_q_heads;
    const QueryRows rows{a, n_vec};
    resident_sketch_tiles<D, T>(a.pool, static_cast<const T *>(a.q), rows, (long)blockIdx.x, (long)gridDim.x,
                                (n_vec + kSketchTile - 1) / kSketchTile, (int)blockIdx.y, (int)gridDim.y);
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
    if (a.pool.code_layout == 0) hipLaunchKernelGGL((prefill_kernel<W, D, 0>), grid, dim3(kPfThreads), 0, st, a, desc, seq0);
    else if (a.pool.code_layout == 1) hipLaunchKernelGGL((prefill_kernel<W, D, 1>), grid, dim3(kPfThreads), 0, st, a, desc, seq0);
    else hipLaunchKernelGGL((prefill_kernel<W, D, 2>), grid, dim3(kPfThreads), 0, st, a, desc, seq0);
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

hipError_t launch_prefill_merge(const PrefillArgs &a, int seq0, int n_seqs, hipStream_t st) {
    const size_t rows = (size_t)n_seqs * a.n_q * a.pool.n_q_heads;
    hipLaunchKernelGGL(prefill_merge_kernel, dim3((unsigned)rows), dim3((unsigned)a.pool.head_dim), 0, st, a, seq0);
    return hipGetLastError();
}

hipError_t launch_prefill(const PrefillArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st) {
    static_assert(kQB == kPrefillRows, "the host sizes grids and workspaces with kPrefillRows");
    const dim3 grid((unsigned)a.pool.n_q_heads, (unsigned)n_seqs, (unsigned)((a.n_q + kQB - 1) / kQB * a.n_splits));
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
    if (a.proj_mfma) {
        const dim3 fine((unsigned)(tiles < 6144 ? tiles : 6144));      // nothing stays resident: short workgroups
        // resident pieces of R: three long-lived workgroups per compute unit (768), shared by the parts of a wide sketch
        const int parts = D == 64 ? proj_resident_parts<64>(a.pool.sketch_bits) : proj_resident_parts<128>(a.pool.sketch_bits);
        const bool fits = parts > 0;
        const long res_x = parts > 0 ? 768 / parts : 1;
        const dim3 res((unsigned)(tiles < res_x ? tiles : res_x), (unsigned)(parts > 0 ? parts : 1));
#define H1BKV_LAUNCH_MF(DD, TT)                                                                                              \
    do {                                                                                                                     \
        if (fits) hipLaunchKernelGGL((sketch_rows_resident_kernel<DD, TT>), res, dim3(kThreads), 0, st, a, n_seqs);          \
        else hipLaunchKernelGGL((sketch_rows_mfma_kernel<DD, TT>), fine, dim3(kThreads), 0, st, a, n_seqs);                  \
    } while (0)
        if (a.f16) {
            if (D == 64) H1BKV_LAUNCH_MF(64, __half);
            else H1BKV_LAUNCH_MF(128, __half);
        } else {
            if (D == 64) H1BKV_LAUNCH_MF(64, float);
            else H1BKV_LAUNCH_MF(128, float);
        }
#undef H1BKV_LAUNCH_MF
    } else if (a.f16) {
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
