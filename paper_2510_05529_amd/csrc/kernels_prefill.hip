// Prefill attention over the compressed cache: Eq.(3) and Eq.(5) for every position of a prompt chunk, causally --
// query i of a sequence attends to the cached tokens up to and including its own position, exactly the decode step
// it would have seen had the prompt been fed one token at a time.
//
// With many queries per KV head both halves of the step are dense contractions and run on the matrix cores, in 32 x 32
// tiles (32 query rows per wave: every operand read from LDS feeds twice the rows of a 16-row tile, and LDS traffic,
// not matrix time, is what a 16-row formulation of this kernel was bound by):
//   scores    alpha needs the Hamming distance of every (query, key) pair.  With the key bits as fp4 numbers {0, 0.5}
//             and the negated query bits as fp4 {-4, +4},  sum_k key_k nq_k = 2 (ham - popcount(q)),  exactly, in fp32:
//             one v_mfma_scale_f32_32x32x64_f8f6f4 per 64 sketch bits (unit scales) yields 32 x 32 distances at four
//             times the fp16 rate -- instead of 4 W XOR/popcount instructions per pair on the vector ALUs.  The MFMA is
//             issued as keys x queries, so that a lane ends up holding distances of ONE query row against 16 tokens:
//             the slots it has in the next MFMA.  The block scales of the instruction are 2^-75 and 2^-74: every product
//             is then +-2 units of the smallest fp32 denormal, and with the accumulator input a per-lane constant whose
//             BIT PATTERN is (LDS address of the weight table) + 2 (popcount(q) - reference + slack), the bit pattern
//             of the result IS the LDS address of the pair's weight (the matrix cores keep denormal inputs and results
//             exact; measured).
//   weights   p = exp((alpha - alpha_ref)/tau) takes only a few hundred values (the distance from the row's reference
//             distance is an integer): one 16-bit LDS table read per pair, straight into one half of an operand
//             register -- no exponential, no conversion, no address arithmetic.  The reference is a running minimum
//             with slack: it is renewed, and the accumulators rescaled, only when a distance falls further below it
//             than the fp16 range of the weights allows (its address then lies in front of the table).
//             The normalisation uses the sums of the SAME fp16 weights (two per v_dot2).
//   values    sum_t p[i][t] v^[t][c]  with v_mfma_f32_32x32x16_f16, fp32 accumulate.
// One workgroup (8 waves; 4 for chunks of fewer than 256 positions) takes 256 (128) consecutive query positions of one
// (sequence, query head) -- 32 rows per wave -- and walks the key tokens in tiles of 64 up to its diagonal.  Per tile the workgroup stages ONCE, for all its rows: the
// keys' bits as fp4 nibbles, and the values dequantised, v^ = fp16(scale * code + zero), channel-major, in the token
// order the score MFMA leaves its results in (so an MFMA B operand is one 16-byte LDS read).  The next tile's global
// loads are issued before the current tile is consumed.  Tiles entirely below a wave's rows take an unmasked path;
// tiles entirely above them are skipped.  A head of 256 channels is served by two workgroups of 128 channels each.
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
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

constexpr int kCS = 8;                        // channels per staging item of the token-major layouts
constexpr int kTK = 64;                       // key tokens per tile
constexpr float kPScaleLog2 = 4.0f;           // weights are stored as p * 2^4
constexpr float kPSlackLog2 = 11.0f;          // and may exceed 1 by up to 2^11 (p 2^4 <= 2^15 stays finite in fp16)
constexpr int kScaleA = 0x34343434;           // E8M0 block scales of the fp4 MFMA: 2^-75 ...
constexpr int kScaleB = 0x35353535;           // ... and 2^-74: a product of fp4 0.5 and +-4 is +-2 x 2^-149

union HalfOperand {
    uint32_t u[4];
    f16x8 v;
};
union NibbleOperand {        // 32 fp4 numbers in the first four dwords (the instruction's 8-dword form is for fp8)
    uint32_t u[8];
    i32x8 v;
};

__device__ __forceinline__ float xor32_min(float x) {       // min with the lane 32 away
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fminf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

template <int NSK, int LAYOUT>
struct StageRegs {           // one thread's share of a key tile on its way from global memory to LDS
    uint32_t skd[NSK];       // 32 sketch bits each
    // layout 0: one item of (token pair, 16 channels): 8 bytes of codes per token, {scale, zero} per token
    // layout 1: 4 code words (4 neighbouring channels, one block of 8 tokens) and the block's 8 {scale, zero}
    // layout 2: 2 items of (token pair, 8 channels): 8 fp16 values per token
    uint32_t c[4];
    uint32_t m[LAYOUT == 2 ? 16 : 8];
};

// WAVES: 4 or 8 waves of 32 query rows.  Eight share every staged key tile among twice the rows (and the staging work
// among twice the threads); four keep short chunks, whose workgroups are few, spread over more compute units.
template <int W, int DTOT, int LAYOUT, int WAVES>
__global__ __launch_bounds__(WAVES * 64, 8 / WAVES) void prefill_kernel(PrefillArgs a, BatchDesc desc, int seq0) {
    constexpr int kPfThreads = WAVES * 64;
    constexpr int kQB = WAVES * 32;               // query positions per workgroup
    constexpr int D = DTOT > 128 ? 128 : DTOT;    // channels per workgroup
    constexpr int NHALF = DTOT / D;               // workgroups per head
    constexpr int NCB = D / 32;                   // 32-channel column blocks
    constexpr int TK = kTK;
    constexpr int NSTEP = TK / 32;                // 32-token MFMA steps per tile
    // bytes per channel row of the value tile.  Ten 16-byte blocks per row: 32 consecutive rows then start on 16 different
    // even bank groups (rows i and i + 16 on the same one), and the exchange below, whose key differs by one between
    // those two rows, moves one of them to the odd neighbour: the 16-byte operand reads are conflict-free.
    constexpr int VS = TK * 2 + 32;
    constexpr int KS = 32 * W + 16;               // bytes per token row of the key tile: 2 W sketch dwords, 16 B of nibbles each
    constexpr int NSKD = TK * 2 * W;              // 32-bit sketch units per tile
    constexpr int NSK = NSKD / kPfThreads > 0 ? NSKD / kPfThreads : 1;
    static_assert(NSKD % kPfThreads == 0 || NSKD < kPfThreads, "sketch dwords split evenly over the threads");
    __shared__ __attribute__((aligned(16))) unsigned char v_s[2][D * VS];
    __shared__ __attribute__((aligned(16))) unsigned char k_s[2][TK * KS];
    // p(e) = 2^4 exp(-2 e / (b tau)) as fp16 for every distance e from a row's reference distance, e = -S .. b; one
    // more entry holds 0 for masked pairs.  One LDS read per pair replaces convert + multiply-add + exponential (a
    // quarter-rate instruction).  The reference is the smallest distance the row had seen when it was last set and
    // is only renewed (accumulators rescaled) when a distance falls more than S below it, S the largest slack whose
    // weights still fit fp16 (exp(2 S / (b tau)) <= 2^11): the best distance of a row improves by a few units many
    // times over a long context, and rescaling on each of them was a tenth of the vector work.
    // In front of them sit 64 W unused entries: addresses of distances further below the reference than the slack allows
    // (never read: the reference is renewed first) then stay non-negative wherever the table lies in LDS.
    constexpr int kGuard = 64 * W;
    __shared__ _Float16 ptab[192 * W + 4];
    // The sequence's page ids, read once: a block-table lookup per tile from global memory sits, with its full memory
    // latency, in front of every tile's loads.
    constexpr int kPagesLds = 1024;
    __shared__ int pages_s[kPagesLds];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 31, g = lane >> 5;
    // Issue priorities: the two waves of a SIMD contend for its one issue slot per cycle.  The value MFMA block runs at the
    // highest priority (its instructions go the moment the matrix pipe frees, the other wave's vector work fills the
    // gaps), the staging of the next tile at the lowest, everything else in between: 4 % on the 8k prompts against equal
    // priorities, where the waves drift into doing the same phase at the same time.
    __builtin_amdgcn_s_setprio(1);
    // grid (query head [x channel half], sequence, query block x context split): workgroups are dispatched x-fastest, so
    // the longest-running (latest) query blocks of ALL heads and sequences start first and the short ones fill the tail
    // of the launch.  With n_splits > 1 (a chunk that is short against its context) a workgroup walks only its share of
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
    const int h = (int)blockIdx.x / NHALF, half = (int)blockIdx.x % NHALF, kvh = h / r;
    const int seq_g = seq0 + blockIdx.y;
    const int ng = DTOT / pv.group_size;
    const int32_t *bt = pv.block_table + (size_t)sd.seq_id * pv.max_pages_per_seq;

    // ---- this lane's query row: position, popcount, and for every 64 sketch bits the lane group's 32 bits as fp4 ----
    // Sketch dword x is spread over four operand dwords: dword j holds bits j, j + 4, ..., j + 28 of x, one per nibble --
    // (x >> j) & 0x11111111 for the keys (fp4 0.5 = 0b0001), and -4 / +4 (0b1110 / 0b0110) for a set / clear query bit.
    // The order of the K index inside an operand is free as long as both operands use the same one.
    const int wave_row0 = row0 + wave * 32;
    const int qi = wave_row0 + i;
    const int pos = qi < n_q ? q0 + qi : -1;          // absolute position of this lane's row, -1 for rows past the chunk
    int pcq = 0;                                      // popcount of the row's query sketch
    NibbleOperand qop[W];
#pragma unroll
    for (int w = 0; w < W; ++w) {
        const uint64_t sq = qi < n_q ? a.q_sketch[(((size_t)seq_g * n_q + qi) * Hq + h) * W + w] : 0;
        pcq += __popcll(sq);
        const uint32_t x = (uint32_t)(sq >> (32 * g));
#pragma unroll
        for (int j = 0; j < 4; ++j) qop[w].u[j] = 0x66666666u | (((x >> j) & 0x11111111u) << 3);
#pragma unroll
        for (int j = 4; j < 8; ++j) qop[w].u[j] = 0u;
    }
    const int wave_min_pos = q0 + wave_row0;                                       // position of the wave's first row
    const int wave_max_pos = wave_row0 < n_q ? q0 + min(wave_row0 + 32, n_q) - 1 : -1;   // ... and of its last valid row

    f32x16 acc[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[cb][v] = 0.0f;
    float lsum = 0.0f;            // this lane's share (16 of every 32 tokens) of the row's weight sum
    int ref = 64 * W;             // the row's reference distance (in distance units); the largest distance there is to begin with
    const int S = (int)fminf(kPSlackLog2 / a.exp2_scale, (float)(64 * W));
    for (int e = threadIdx.x; e < kGuard + 64 * W + S + 2; e += kPfThreads) {
        const int d = e - kGuard;                                     // distance - reference + S
        ptab[e] = d < 0 ? (_Float16)__builtin_inff()
                        : d <= 64 * W + S ? (_Float16)__builtin_amdgcn_exp2f(fmaf(-a.exp2_scale, (float)(d - S), kPScaleLog2)) : (_Float16)0.0f;
    }
    // LDS byte address of the entry for distance - reference + S = 0: what the score MFMA's results are counted from
    const uint32_t tab0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) _Float16 *)ptab + 2u * kGuard;
    const float off_zero = __uint_as_float(tab0 + 2u * (64 * W + S + 1));    // the table's zero entry
    // accumulator input of the score MFMA: bits(result) = tab0 + 2 (ham - ref + S) = LDS address of the pair's weight
    f32x16 c0;
    auto set_c0 = [&]() {
        const float v0 = __uint_as_float(tab0 + (uint32_t)(2 * (pcq - ref + S)));
#pragma unroll
        for (int v = 0; v < 16; ++v) c0[v] = v0;
    };
    set_c0();
    const uint32_t mask_a = opaque_vgpr(0x000F000Fu), mask_b = opaque_vgpr(0x00F000F0u);
    const h16x2 ones2 = {(_Float16)1.0f, (_Float16)1.0f};

    // Token t of a tile sits at operand position p(t) = t with bits 2 and 3 exchanged: the score MFMA leaves tokens
    // 8 a + 4 g + j (a = 0..3, j = 0..3) of a 32-token step in lane group g, and the value MFMA of tokens 16 m .. 16 m + 15
    // wants lane group g's eight tokens (a = 2 m, 2 m + 1) side by side at K = 8 g .. 8 g + 7.
    auto operand_pos = [](int t) { return (t & ~12) | ((t & 8) >> 1) | ((t & 4) << 1); };

    // ---- staging: global -> registers (issued early) -> LDS (after the current tile has been consumed) ----
    // Consecutive lanes take consecutive channel slices of one token pair, so that a wave's loads cover whole records
    // (a lane per token pair would touch a different cache line with every lane).  Their LDS writes then go to channel
    // rows 8 or 16 apart at one token position -- the same banks, whatever the row padding -- so the 16-byte blocks of a
    // channel row are stored exchanged: block k of row c sits at k ^ ((c >> 4) & 7).
    // What the LDS of this chip does per pass of 32 lanes (measured with address patterns of their own): 16-byte reads are
    // conflict-free iff their blocks differ mod 32 (512 bytes), 4-byte writes iff their words differ mod 64 (256 bytes).
    // With 160-byte rows and the key c >> 4 the operand reads of 32 consecutive rows meet that; the key c >> 3 does not
    // (rows i and i + 16 then share a block: every operand read took two passes).
    auto row_addr = [](int ch, int pos_halves) {       // byte offset of (channel row, operand position) in a value tile
        return ch * VS + ((((pos_halves >> 3) ^ (ch >> 4)) & 7) << 4) + ((pos_halves & 7) << 1);
    };
    static_assert(TK == 64, "a channel row is eight 16-byte blocks");
    constexpr int CS0 = 16;                                       // layout 0: channels per staging item
    constexpr int kItems0 = (TK / 2) * (D / CS0);                 // layout 0: (token pair, channel slice) items per tile
    static_assert(kItems0 <= kPfThreads, "one staging item per thread");
    // (with eight waves the items and the sketch words occupy the first four: spreading them over all eight -- 8-channel
    // items, or the sketch words on the last four -- was slower)
    constexpr int kItems2 = (TK / 2) * (D / kCS);                 // layout 2: (token pair, 8-channel slice) items per tile
    static_assert(kItems2 <= 2 * kPfThreads, "at most two staging items per thread");
    constexpr int NIT = (kItems2 + kPfThreads - 1) / kPfThreads;
    // layout 1: a thread takes one block of 8 tokens, one 16-channel column block cb and four neighbouring channels
    // 16 cb + 4 nq .. + 3 of it (one quantisation group): words (cb / 4) * 64 + (4 nq + k) * 4 + cb % 4 (code_word_index).
    constexpr int kItems1 = (TK / 8) * (D / 16) * 4;
    static_assert(kItems1 <= kPfThreads, "one staging item per thread");
    {
        const int n_pages = ((n_tiles - 1) * TK) / kPage + 1;
        for (int p = tid; p < min(n_pages, kPagesLds); p += kPfThreads) pages_s[p] = bt[p];
        __syncthreads();
    }
    // Per tile everything that depends on the tile is uniform over the workgroup (scalar registers); what depends on
    // the lane is a 32-bit offset: the loads then take a scalar base and a 32-bit lane offset, with no 64-bit vector
    // arithmetic.  Groups and group counts are powers of two: shifts, not multiplies.
    const int lg_ng = __builtin_ctz((unsigned)ng), lg_G = __builtin_ctz((unsigned)pv.group_size);
    auto tile_rec0 = [&](int kt) {
        const int t0 = kt * TK, p = t0 / kPage;
        const int page = __builtin_amdgcn_readfirstlane(p < kPagesLds ? pages_s[p] : bt[p]);
        return ((size_t)page * H + kvh) * kPage + (t0 % kPage);                    // a tile never straddles a page
    };
    using Stage = StageRegs<NSK, LAYOUT>;
    auto load_tile = [&](Stage &sr, int kt) {
        const size_t rec0 = tile_rec0(kt);
        const unsigned char *sk_base = reinterpret_cast<const unsigned char *>(pv.sketch + rec0 * W);
#pragma unroll
        for (int u = 0; u < NSK; ++u)
            if (tid + u * kPfThreads < NSKD) sr.skd[u] = *reinterpret_cast<const uint32_t *>(sk_base + (uint32_t)(tid + u * kPfThreads) * 4u);
        if constexpr (LAYOUT == 0) {
            if (tid < kItems0) {
                const unsigned char *c_base = pv.codes + rec0 * (DTOT / 2) + half * (D / 2);
                const unsigned char *m_base = reinterpret_cast<const unsigned char *>(pv.meta + (rec0 << lg_ng));
                const uint32_t tp = tid / (D / CS0), s16 = tid % (D / CS0);
                const uint32_t gq = (uint32_t)(D * half + CS0 * s16) >> lg_G;
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const uint32_t rl = 2 * tp + t;                         // record within the tile
                    const uint2 cc = *reinterpret_cast<const uint2 *>(c_base + (rl * (uint32_t)(DTOT / 2) + s16 * 8u));
                    sr.c[2 * t] = cc.x;
                    sr.c[2 * t + 1] = cc.y;
                    sr.m[t] = *reinterpret_cast<const uint32_t *>(m_base + (((rl << lg_ng) + gq) << 2));
                }
            }
        } else if constexpr (LAYOUT == 2) {              // fp16 values: 8 channels (16 bytes) of each of two tokens
            const unsigned char *v_base = pv.codes + (rec0 * DTOT + D * half) * 2;
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const int id = tid + it * kPfThreads;
                if (id >= kItems2) break;
                const uint32_t tp = id / (D / kCS), sl = id % (D / kCS);
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const uint4 a0 = *reinterpret_cast<const uint4 *>(v_base + ((2 * tp + t) * (uint32_t)DTOT + kCS * sl) * 2u);
                    uint32_t *m = sr.m + 8 * it + 4 * t;
                    m[0] = a0.x; m[1] = a0.y; m[2] = a0.z; m[3] = a0.w;
                }
            }
        } else if (tid < kItems1) {
            const uint32_t blk = tid / (D / 4), rest = tid % (D / 4);
            const uint32_t cb = rest / 4, nq = rest % 4;
            const unsigned char *w_base = pv.codes + rec0 * (DTOT / 2);
            const unsigned char *m_base = reinterpret_cast<const unsigned char *>(pv.meta + (rec0 << lg_ng));
            const uint32_t cbg = (D / 16) * half + cb;                     // column block within the whole head
#pragma unroll
            for (int k = 0; k < 4; ++k)
                sr.c[k] = *reinterpret_cast<const uint32_t *>(w_base + (8 * blk * (uint32_t)(DTOT / 2) + ((cbg >> 2) * 64 + (4 * nq + k) * 4 + (cbg & 3)) * 4u));
            const uint32_t gq = (16 * cbg + 4 * nq) >> lg_G;
#pragma unroll
            for (int j = 0; j < 8; ++j) sr.m[j] = *reinterpret_cast<const uint32_t *>(m_base + ((((8 * blk + j) << lg_ng) + gq) << 2));
        }
    };
    auto store_tile = [&](const Stage &sr, int kt, int buf) {
        const int t0 = kt * TK;
        // key bits -> fp4 nibbles: 32 bits in, 16 bytes out
        unsigned char *ks = k_s[buf];
#pragma unroll
        for (int u = 0; u < NSK; ++u) {
            const int dwi = tid + u * kPfThreads;
            if (dwi < NSKD) {
                const int tok = dwi / (2 * W), part = dwi % (2 * W);
                const uint32_t x = sr.skd[u];
                *reinterpret_cast<uint4 *>(ks + tok * KS + part * 16) =
                    make_uint4(x & 0x11111111u, (x >> 1) & 0x11111111u, (x >> 2) & 0x11111111u, (x >> 3) & 0x11111111u);
            }
        }
        unsigned char *vs = v_s[buf];
        if constexpr (LAYOUT == 0) {
            if (tid < kItems0) {
                const int tp = tid / (D / CS0), s16 = tid % (D / CS0);
                float sc[2], zp[2];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    // slots past the end of the sequence hold anything: their values must not reach the MFMA as NaN
                    const uint32_t m = t0 + 2 * tp + t < len ? sr.m[t] : 0u;
                    sc[t] = __half2float(__ushort_as_half((unsigned short)(m & 0xFFFFu)));
                    zp[t] = __half2float(__ushort_as_half((unsigned short)(m >> 16)));
                }
                const int pp = operand_pos(2 * tp);                // tokens 2 tp and 2 tp + 1 stay neighbours
                // (a lane's two rows n and n + 4 lie 32 banks apart and go out as one two-address write)
                const int wbase = row_addr(CS0 * s16, pp);
                // A nibble masked in place at mantissa bits 0-3 / 4-7 of a zero half-word is the fp16 subnormal
                // code 2^-24 / code 2^-20: the mixed-precision FMA reads it directly, with the scale times 2^24 / 2^20.
                const float sa[2] = {sc[0] * 16777216.0f, sc[1] * 16777216.0f}, sb[2] = {sc[0] * 1048576.0f, sc[1] * 1048576.0f};
#pragma unroll
                for (int k = 0; k < CS0 / 8; ++k) {                // 8 channels per code dword
                    const uint32_t x0 = sr.c[k], x1 = sr.c[2 + k], y0 = x0 >> 8, y1 = x1 >> 8;
                    const uint32_t t0w[4] = {x0 & mask_a, x0 & mask_b, y0 & mask_a, y0 & mask_b};
                    const uint32_t t1w[4] = {x1 & mask_a, x1 & mask_b, y1 & mask_a, y1 & mask_b};
#pragma unroll
                    for (int n = 0; n < 4; ++n) {                  // word n holds nibbles n (low half) and n + 4 (high half)
                        const __half2 h0 = *reinterpret_cast<const __half2 *>(&t0w[n]), h1 = *reinterpret_cast<const __half2 *>(&t1w[n]);
                        const float w0 = (n & 1) ? sb[0] : sa[0], w1 = (n & 1) ? sb[1] : sa[1];
                        const f32x2 lo = {fmaf(w0, __low2float(h0), zp[0]), fmaf(w1, __low2float(h1), zp[1])};
                        const f32x2 hi = {fmaf(w0, __high2float(h0), zp[0]), fmaf(w1, __high2float(h1), zp[1])};
                        const h16x2 plo = __builtin_convertvector(lo, h16x2), phi = __builtin_convertvector(hi, h16x2);
                        // (all channels of the item share one exchange key: the address is a lane base plus a constant)
                        static_assert(CS0 <= 16, "one key per staging item");
                        *reinterpret_cast<h16x2 *>(vs + wbase + (8 * k + n) * VS) = plo;
                        *reinterpret_cast<h16x2 *>(vs + wbase + (8 * k + n + 4) * VS) = phi;
                    }
                }
            }
        } else if constexpr (LAYOUT == 2) {
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const int id = tid + it * kPfThreads;
                if (id >= kItems2) break;
                const int tp = id / (D / kCS), sl = id % (D / kCS);
                const int pp = operand_pos(2 * tp);
                // slots past the end of the sequence hold anything: their values must not reach the MFMA as NaN
                const uint32_t keep0 = t0 + 2 * tp < len ? 0xFFFFu : 0u, keep1 = t0 + 2 * tp + 1 < len ? 0xFFFFu : 0u;
                const uint32_t *m = sr.m + 8 * it;
#pragma unroll
                for (int c = 0; c < kCS; ++c) {
                    const uint32_t h0 = (m[c >> 1] >> (16 * (c & 1))) & keep0, h1 = (m[4 + (c >> 1)] >> (16 * (c & 1))) & keep1;
                    *reinterpret_cast<uint32_t *>(vs + row_addr(kCS * sl + c, pp)) = h0 | (h1 << 16);
                }
            }
        } else if (tid < kItems1) {
            const int blk = tid / (D / 4), rest = tid % (D / 4);
            const int cb = rest / 4, nq = rest % 4;
            float sc[8], zp[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                // slots past the end of the sequence hold anything: their values must not reach the MFMA as NaN
                const uint32_t m = t0 + 8 * blk + j < len ? sr.m[j] : 0u;
                sc[j] = __half2float(__ushort_as_half((unsigned short)(m & 0xFFFFu)));
                zp[j] = __half2float(__ushort_as_half((unsigned short)(m >> 16)));
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int ch = 16 * cb + 4 * nq + k;
                const uint32_t x = sr.c[k], y = x >> 8;
                // nibble n of the word is token 2 n of the block, nibble n + 4 token 2 n + 1: word n below holds that
                // pair as fp16 subnormals (code 2^-24 for even n, code 2^-20 for odd n)
                const uint32_t tw[4] = {x & mask_a, x & mask_b, y & mask_a, y & mask_b};
                h16x2 hv[4];
#pragma unroll
                for (int n = 0; n < 4; ++n) {
                    const __half2 hh = *reinterpret_cast<const __half2 *>(&tw[n]);
                    const float mul = (n & 1) ? 1048576.0f : 16777216.0f;
                    const f32x2 pf = {fmaf(sc[2 * n] * mul, __low2float(hh), zp[2 * n]), fmaf(sc[2 * n + 1] * mul, __high2float(hh), zp[2 * n + 1])};
                    hv[n] = __builtin_convertvector(pf, h16x2);
                }
                // tokens 8 blk .. 8 blk + 3 and 8 blk + 4 .. 8 blk + 7 go to two operand positions
                *reinterpret_cast<uint2 *>(vs + row_addr(ch, operand_pos(8 * blk))) = *reinterpret_cast<const uint2 *>(&hv[0]);
                *reinterpret_cast<uint2 *>(vs + row_addr(ch, operand_pos(8 * blk + 4))) = *reinterpret_cast<const uint2 *>(&hv[2]);
            }
        }
    };

    // ---- one tile: score MFMA, weights, value MFMA ----
    auto consume_tile = [&](int kt, int buf, auto masked_tag) {
        constexpr bool kMasked = decltype(masked_tag)::value;
        const unsigned char *ks = k_s[buf];
        const unsigned char *vs = v_s[buf];
        // byte offsets of the weights of step st: lane (row i, g) receives tokens 8 a + 4 g + j of the step as element 4 a + j
        auto scores = [&](int st) {
            f32x16 off;

#pragma unroll
            for (int w = 0; w < W; ++w) {
                // the two 32-bit halves of sketch word w are the instruction's two K blocks of 32: lane group g takes half g
                NibbleOperand K;
                const uint4 kk = *reinterpret_cast<const uint4 *>(ks + (32 * st + i) * KS + (2 * w + g) * 16);
                K.u[0] = kk.x; K.u[1] = kk.y; K.u[2] = kk.z; K.u[3] = kk.w;
                K.u[4] = K.u[5] = K.u[6] = K.u[7] = 0u;
                off = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(K.v, qop[w].v, w == 0 ? c0 : off, 4, 4, 0, kScaleA, 0, kScaleB);
            }
            return off;
        };
        auto mask_step = [&](f32x16 &off, int st) {                // causal mask (also: rows past the chunk)
            const int lim = pos - (kt * TK + 32 * st + 4 * g);     // element 4 a + j is visible iff 8 a + j <= lim
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (8 * (v >> 2) + (v & 3) > lim) off[v] = off_zero;
        };
        auto row_min = [&](const f32x16 &off) {                    // smallest table address of the row in this step
            uint32_t mn = min(min(__float_as_uint(off[0]), __float_as_uint(off[1])), __float_as_uint(off[2]));
#pragma unroll
            for (int v = 3; v < 15; v += 2) mn = min(min(mn, __float_as_uint(off[v])), __float_as_uint(off[v + 1]));
            mn = min(mn, __float_as_uint(off[15]));
            const auto r2 = __builtin_amdgcn_permlane32_swap(mn, mn, false, false);    // over the row's two lane groups
            return min(r2[0], r2[1]);
        };
        // rare: some row's best distance left the slack (its table address lies in front of the table).  The step's smallest distance becomes
        // the row's reference: every address of the row grows by 2 delta, what has been accumulated shrinks by
        // exp(-2 delta / (b tau)).  Rows whose distances are all inside the slack keep their reference (delta = 0).
        auto renew = [&](f32x16 &off, uint32_t mn) {
            const int idx = ((int)mn - (int)tab0) >> 1;                               // smallest distance - reference + S
            const int delta = idx < 0 ? S - idx : 0;                                  // old reference - new one (> S)
            const float f = __builtin_amdgcn_exp2f(-a.exp2_scale * (float)delta);
            ref -= delta;
            set_c0();
            lsum *= f;
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (!kMasked || __float_as_uint(off[v]) != __float_as_uint(off_zero))
                    off[v] = __uint_as_float(__float_as_uint(off[v]) + (uint32_t)(2 * delta));
            // accumulator element 4 a + j of lane (n, g) belongs to row 8 a + 4 g + j, whose factor lane 8 a + 4 g + j holds
            float fr[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) fr[v] = __shfl(f, 8 * (v >> 2) + 4 * g + (v & 3));
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[cb][v] *= fr[v];
        };
        // Weights from the table: the result's bit pattern is the entry's LDS address.
        auto table = [&](const f32x16 &off, _Float16 *pw) {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                pw[v] = *(__attribute__((address_space(3))) const _Float16 *)(uintptr_t)__float_as_uint(off[v]);
        };
        auto pack = [&](const _Float16 *pw, HalfOperand *A) {
#pragma unroll
            for (int v = 0; v < 16; v += 2) {
                const h16x2 pk = {pw[v], pw[v + 1]};
                A[v >> 3].u[(v & 7) >> 1] = *reinterpret_cast<const uint32_t *>(&pk);
                lsum = __builtin_amdgcn_fdot2(pk, ones2, lsum, false);
            }
        };
        // Lane bases of the value operands: row i of a column block, 16-byte block (2 m' + g) ^ (the key bits that come
        // from i); the key bits that come from the column block and the step's bit are added as constants at the reads.
        const int lane_key = i >> 4;
        const int bbase[2] = {i * VS + (((0 | g) ^ lane_key) << 4), i * VS + (((2 | g) ^ lane_key) << 4)};
        auto values = [&](const HalfOperand *A, int st) {
            __builtin_amdgcn_s_setprio(3);
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
#pragma unroll
                for (int m = 0; m < 2; ++m) {
                    // row 32 cb + i, block 4 st + 2 m + g exchanged with the row's key: what depends on (cb, st, m) is a
                    // compile-time offset and a choice between two lane bases (see bbase)
                    const int mm = m ^ (cb & 1), bit2 = st ^ (cb >> 1);
                    const f16x8 B = *reinterpret_cast<const f16x8 *>(vs + bbase[mm] + (32 * cb * VS + (bit2 << 6)));
                    acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(A[m].v, B, acc[cb], 0, 0, 0);
                }
            }
            __builtin_amdgcn_s_setprio(1);
        };
        static_assert(NSTEP == 2, "the two steps of a tile are written out");

        // A wave executes in order, and a step is one long chain (scores -> minimum -> table -> value MFMAs): the second
        // step's chain up to its table reads is therefore issued among the first step's value MFMAs -- assuming that no
        // reference needs renewing; if one does, the weights are read again.
        f32x16 off0 = scores(0);
        if (kMasked) mask_step(off0, 0);
        {
            const uint32_t mn = row_min(off0);
            if (__any(mn < tab0)) renew(off0, mn);
        }
        _Float16 pw0[16], pw1[16];
        table(off0, pw0);
        f32x16 off1 = scores(1);
        HalfOperand A0[2], A1[2];
        pack(pw0, A0);
        if (kMasked) mask_step(off1, 1);
        const uint32_t mn1 = row_min(off1);
        table(off1, pw1);
        values(A0, 0);
        if (__any(mn1 < tab0)) {
            renew(off1, mn1);
            table(off1, pw1);
        }
        pack(pw1, A1);
        values(A1, 1);
    };

    // Two register sets: the loads of tile kt + 2 are issued before tile kt is consumed, so a load has two tiles of work
    // to arrive in (one tile's work is shorter than a trip to memory).
    Stage s0;
    Stage s1;
    if (tile_lo < tile_hi) {                                       // (a short sequence may leave a split without tiles)
        load_tile(s0, tile_lo);
        store_tile(s0, tile_lo, tile_lo & 1);
    }
    if (tile_lo + 1 < tile_hi) load_tile(s1, tile_lo + 1);
    __syncthreads();
    // `next` holds tile kt + 1 (requested one tile ago), `after` is free for tile kt + 2
    auto tile_step = [&](int kt, Stage &next, Stage &after) {
        const int buf = kt & 1;
        if (kt + 2 < tile_hi) load_tile(after, kt + 2);
        const int t_first = kt * TK, t_last = t_first + TK - 1;
        if (t_first <= wave_max_pos) {                             // else: the whole tile lies in this wave's future
            if (t_last <= wave_min_pos && wave_row0 + 32 <= n_q) consume_tile(kt, buf, std::false_type{});
            else consume_tile(kt, buf, std::true_type{});
        }
        __builtin_amdgcn_s_setprio(0);
        if (kt + 1 < tile_hi) store_tile(next, kt + 1, buf ^ 1);
        __builtin_amdgcn_s_setprio(1);
        __syncthreads();
    };
    for (int kt = tile_lo; kt < tile_hi; kt += 2) {
        tile_step(kt, s1, s0);
        if (kt + 1 < tile_hi) tile_step(kt + 1, s0, s1);
    }

    // ---- epilogue: accumulator element 4 a + j of lane (n = i, g) is row 8 a + 4 g + j, channel 32 cb + n ----
    const float l_row = half_wave_sum(lsum);                  // the row's two lane groups hold 16 of every 32 tokens each
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int rw = 8 * (v >> 2) + 4 * g + (v & 3);
        const int q_row = wave_row0 + rw;
        const float l = __shfl(l_row, rw);                    // the row's sums and reference sit in lane rw
        const int rref = __shfl(ref, rw);
        if (q_row >= n_q) continue;
        if (n_splits == 1) {
            const float inv = 1.0f / l;
            float *dst = a.out + (((size_t)seq_g * n_q + q_row) * Hq + h) * DTOT + D * half + i;
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) dst[32 * cb] = acc[cb][v] * inv;
        } else {
            float *dst = a.part + ((((size_t)seq_g * n_q + q_row) * Hq + h) * n_splits + split) * (DTOT + 2);
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) dst[D * half + 32 * cb + i] = acc[cb][v];
            if (i == 0 && half == 0) {
                dst[DTOT] = l;
                // the merge kernel counts references in quarter units; a split that saw no token of the row says so
                dst[DTOT + 1] = __int_as_float(l > 0.0f ? 4 * rref : 1 << 22);
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
    ProjDiv by_seq, by_heads;                           // (used when the vector index fits 32 bits)
    __device__ int rows_in(long tile) const { return (int)min((long)kSketchTile, n_vec - tile * kSketchTile); }
    __device__ size_t src(long tile, int rl) const {
        const long v = tile * kSketchTile + rl;
        const int Hq = a.pool.n_q_heads;
        if (n_vec <= 0x7FFFFFFFL) {                     // (uniform)
            uint32_t s, rem, tok, head;
            by_seq.divmod((uint32_t)v, s, rem);
            by_heads.divmod(rem, tok, head);
            return (size_t)s * a.stride_seq + (size_t)tok * a.stride_tok + (size_t)head * a.stride_head;
        }
        const long s = v / ((long)a.n_q * Hq), rem = v % ((long)a.n_q * Hq);
        return (size_t)s * a.stride_seq + (size_t)((uint32_t)rem / (uint32_t)Hq) * a.stride_tok +
               (size_t)((uint32_t)rem % (uint32_t)Hq) * a.stride_head;
    }
    __device__ int page_request(long, int) const { return 0; }
    __device__ uint32_t *dst(long tile, int rl, int) const {
        return reinterpret_cast<uint32_t *>(a.q_sketch + (size_t)(tile * kSketchTile + rl) * (a.pool.sketch_bits >> 6));
    }
};

template <int D, typename T, bool WIDE>
__global__ __launch_bounds__(kThreads, 3) void sketch_rows_resident_kernel(PrefillArgs a, int n_seqs) {
    const long n_vec = (long)n_seqs * a.n_q * a.pool.n_q_heads;
    const uint64_t per_seq = (uint64_t)a.n_q * (uint64_t)a.pool.n_q_heads;
    const QueryRows rows{a, n_vec, ProjDiv(per_seq <= 0xFFFFFFFFull ? (uint32_t)per_seq : 1u), ProjDiv((uint32_t)a.pool.n_q_heads)};
    resident_sketch_tiles<D, T, WIDE>(a.pool, static_cast<const T *>(a.q), rows, (long)blockIdx.x, (long)gridDim.x,
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

// Eq.(2) for query vectors of 256 channels: a projection row does not fit the register file next to anything else, so
// a lane holds half a row at a time and carries the chain values of 16 vectors from the first half to the second
// (the chain still runs over j = 0 .. 255 in order for every vector).
template <typename T>
__global__ __launch_bounds__(kThreads) void sketch_rows_wide_kernel(PrefillArgs a, int n_seqs) {
    constexpr int D = 256, VT = 16, HALF = 128;
    __shared__ __attribute__((aligned(16))) float qs[VT][D];
    __shared__ size_t src_off[VT];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const PoolView &pv = a.pool;
    const int W = pv.sketch_bits >> 6, Hq = pv.n_q_heads;
    const long n_vec = (long)n_seqs * a.n_q * Hq;
    const T *qbase = static_cast<const T *>(a.q);
    for (long v0 = (long)blockIdx.x * VT; v0 < n_vec; v0 += (long)gridDim.x * VT) {
        __syncthreads();
        const int n_here = (int)min((long)VT, n_vec - v0);
        if (tid < n_here) {
            const long v = v0 + tid;
            const long s = v / ((long)a.n_q * Hq), rem = v % ((long)a.n_q * Hq);
            src_off[tid] = (size_t)s * a.stride_seq + (size_t)(rem / Hq) * a.stride_tok + (size_t)(rem % Hq) * a.stride_head;
        }
        __syncthreads();
        for (int e = tid; e < n_here * D; e += kThreads) qs[e / D][e % D] = (float)qbase[src_off[e / D] + e % D];
        __syncthreads();
        for (int word = wave; word < W; word += kWaves) {
            float y[VT];
#pragma unroll
            for (int t = 0; t < VT; ++t) y[t] = 0.0f;
#pragma unroll 1
            for (int h0 = 0; h0 < D; h0 += HALF) {
                float r[HALF];
                const float *row = pv.R + (size_t)(word * 64 + lane) * D + h0;
#pragma unroll
                for (int j = 0; j < HALF; j += 4) {
                    const float4 x = *reinterpret_cast<const float4 *>(row + j);
                    r[j] = x.x; r[j + 1] = x.y; r[j + 2] = x.z; r[j + 3] = x.w;
                }
#pragma unroll 1
                for (int t = 0; t < n_here; ++t) {
                    float acc = y[0];                              // y[t], selected without dynamic register indexing
#pragma unroll
                    for (int u = 1; u < VT; ++u) acc = t == u ? y[u] : acc;
#pragma unroll
                    for (int j = 0; j < HALF; j += 4) {
                        const float4 q4 = *reinterpret_cast<const float4 *>(&qs[t][h0 + j]);
                        acc = __builtin_fmaf(r[j], q4.x, acc);
                        acc = __builtin_fmaf(r[j + 1], q4.y, acc);
                        acc = __builtin_fmaf(r[j + 2], q4.z, acc);
                        acc = __builtin_fmaf(r[j + 3], q4.w, acc);
                    }
#pragma unroll
                    for (int u = 0; u < VT; ++u) y[u] = t == u ? acc : y[u];
                }
            }
#pragma unroll
            for (int t = 0; t < VT; ++t) {
                const uint64_t mask = __ballot(y[t] >= 0.0f);
                if (lane == 0 && t < n_here) a.q_sketch[(size_t)(v0 + t) * W + word] = mask;
            }
        }
    }
}

template <int W, int D, int WAVES>
hipError_t launch_prefill_waves(const PrefillArgs &a, const BatchDesc &desc, int seq0, dim3 grid, hipStream_t st) {
    if (a.pool.code_layout == 0) hipLaunchKernelGGL((prefill_kernel<W, D, 0, WAVES>), grid, dim3(WAVES * 64), 0, st, a, desc, seq0);
    else if (a.pool.code_layout == 1) hipLaunchKernelGGL((prefill_kernel<W, D, 1, WAVES>), grid, dim3(WAVES * 64), 0, st, a, desc, seq0);
    else hipLaunchKernelGGL((prefill_kernel<W, D, 2, WAVES>), grid, dim3(WAVES * 64), 0, st, a, desc, seq0);
    return hipGetLastError();
}

template <int W, int D>
hipError_t launch_prefill_layout(const PrefillArgs &a, const BatchDesc &desc, int seq0, dim3 grid, hipStream_t st) {
    return prefill_rows(a.n_q) == 256 ? launch_prefill_waves<W, D, 8>(a, desc, seq0, grid, st)
                                      : launch_prefill_waves<W, D, 4>(a, desc, seq0, grid, st);
}

template <int W>
hipError_t launch_prefill_d(const PrefillArgs &a, const BatchDesc &desc, int seq0, dim3 grid, hipStream_t st) {
    switch (a.pool.head_dim) {
        case 64: return launch_prefill_layout<W, 64>(a, desc, seq0, grid, st);
        case 128: return launch_prefill_layout<W, 128>(a, desc, seq0, grid, st);
        default:                                   // 256 channels: two workgroups of 128 channels per head
            grid.x *= 2;
            return launch_prefill_layout<W, 256>(a, desc, seq0, grid, st);
    }
}

}  // namespace

hipError_t launch_prefill_merge(const PrefillArgs &a, int seq0, int n_seqs, hipStream_t st) {
    const size_t rows = (size_t)n_seqs * a.n_q * a.pool.n_q_heads;
    hipLaunchKernelGGL(prefill_merge_kernel, dim3((unsigned)rows), dim3((unsigned)a.pool.head_dim), 0, st, a, seq0);
    return hipGetLastError();
}

hipError_t launch_prefill(const PrefillArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st) {
    const int rows = prefill_rows(a.n_q);        // (the host sizes grids and workspaces with the same function)
    const dim3 grid((unsigned)a.pool.n_q_heads, (unsigned)n_seqs, (unsigned)((a.n_q + rows - 1) / rows * a.n_splits));
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
    if (D == 256) {                                            // (the chain; large prompts at this size are not the hot path)
        const long t16 = (n_vec + 15) / 16;
        const dim3 g16((unsigned)(t16 < 4096 ? t16 : 4096));
        if (a.f16) hipLaunchKernelGGL((sketch_rows_wide_kernel<__half>), g16, dim3(kThreads), 0, st, a, n_seqs);
        else hipLaunchKernelGGL((sketch_rows_wide_kernel<float>), g16, dim3(kThreads), 0, st, a, n_seqs);
        return hipGetLastError();
    }
    if (D != 64 && D != 128) return hipErrorInvalidValue;
    if (a.proj_mfma) {
        const dim3 fine((unsigned)(tiles < 6144 ? tiles : 6144));      // nothing stays resident: short workgroups
        // resident pieces of R: three long-lived workgroups per compute unit (768), shared by the parts of a wide sketch
        const int parts = D == 64 ? proj_resident_parts<64>(a.pool.sketch_bits) : proj_resident_parts<128>(a.pool.sketch_bits);
        const bool fits = parts > 0;
        const long res_x = parts > 0 ? 768 / parts : 1;
        const dim3 res((unsigned)(tiles < res_x ? tiles : res_x), (unsigned)(parts > 0 ? parts : 1));
#define H1BKV_LAUNCH_MF(DD, TT)                                                                                              \
    do {                                                                                                                     \
        if (fits && DD == 128 && sizeof(TT) == 2 && a.pool.sketch_bits % 128 == 0)                                            \
            hipLaunchKernelGGL((sketch_rows_resident_kernel<DD, TT, DD == 128 && sizeof(TT) == 2>), res, dim3(kThreads), 0, st, a, n_seqs); \
        else if (fits) hipLaunchKernelGGL((sketch_rows_resident_kernel<DD, TT, false>), res, dim3(kThreads), 0, st, a, n_seqs); \
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
