// Decode-step attention when several query heads share one KV head (grouped-query attention; Eq.(3), Eq.(5)).
//
// With r query heads per KV head the weighted sum  out[q][c] = sum_t p[q][t] (scale_t code_tc + zero_t)  is a skinny
// matrix product (r x T) . (T x d), and on the plain vector ALUs its r*d multiply-adds per record outrun the HBM
// stream from r = 3-4 on.  This kernel therefore runs that contraction on the matrix cores
// (v_mfma_f32_16x16x32_bf16, fp32 accumulate) and keeps the vector ALUs for what only they can do: scoring,
// softmax weights and turning nibbles into MFMA operands.  It reads the token-interleaved code layout
// (PoolView::code_layout == 1): one 32-bit word holds the 8 codes of one channel for 8 consecutive tokens.
//
//   B operand (K = 32 tokens x N = 16 channels): lane (n, kb) needs 8 consecutive tokens of channel n -- exactly
//     one code word.  A nibble masked in place at bits 0-3 or 4-7 of an otherwise zero half-word IS a bf16 number:
//     bit patterns below 2^8 (exponent field 0 or 1) are linear in their integer value, pattern m reads m 2^-133, and
//     the matrix cores take such inputs as they are (measured).  So the operand is one shift and four ANDs per code
//     word -- code 2^-133 for the tokens whose nibble sits at bits 0-3, code 2^-129 for those at bits 4-7 -- with no
//     offset to remove afterwards; the weights of a token carry the matching power of two (below).
//   A operand (M = 16 rows x K = 32 tokens): the weights w = p[q][t] * scale[t][g] of one quantisation group g,
//     split exactly into two bf16 parts (top 16 bits, and the top 16 bits of the remainder): row q carries the high
//     part and row q + RQMAX the low part, so the product keeps 16 bits of every weight at no extra MFMA cost (the M
//     dimension is far from full anyway).  Each weight is computed once (lane = (token, query-head parity)),
//     written to LDS as two half-words and read back in operand order (16 bytes per lane).
//   A lane scores and weighs the same token slot of every page, so the power of two its weights carry -- 2^64 or 2^60,
//     by where the slot's nibble sits -- is a per-lane constant folded into the exponent argument of the softmax weight;
//     the lane's sums of p and of p zero carry it too and shed it once, in the epilogue, where the accumulators are
//     multiplied by 2^69.  sum_t p zero_t  is accumulated on the vector ALU.
//
// Every wave streams on its own: it owns 64 tokens of each page of the chunk, scores them (lane = (token, query
// head parity), XOR + popcount against the query sketches in LDS), keeps a running maximum per head -- when a
// page raises it, the wave rescales its accumulators (rare: the distance to the best token so far only improves a
// few times per chunk) -- and feeds the matrix cores; no workgroup barrier and no pass over the sketches ahead of
// the values.  The four waves' (max, sum, accumulators) meet once, in the epilogue.  The partial-result format is
// that of the vector-ALU kernel, so qsketch_kernel and merge_kernel serve both.
//
// DTAU = true adds the sums the temperature derivative needs (Sec. IV-C trains tau; see kernels_decode_dtau.hip for the
// formula): a second weight p e, e = ham - running minimum, for every (token, head).  Its two bf16 parts take operand
// rows 8-11 and 12-15 next to the plain weights' rows 0-3 and 4-7 -- the MFMAs cost nothing extra, a workgroup then
// serves at most four query heads.  When a page lowers a head's running minimum by k, every e of that head grows by k:
// the distance-weighted sums take k times the plain ones before the usual rescale.
#include <type_traits>

#include "decode_common.h"

namespace h1bkv {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

union BOperand {
    uint32_t u[4];
    bf16x8 v;
};

template <int NCB4, int NG, int W>
struct PageRegs {            // what one lane holds of its wave's 64 tokens of one page
    uint64_t sk[2][W];       // sketches of tokens tk and 32 + tk
    uint4 c[2][NCB4];        // code words of (channel lane n, token block kb) for the two 32-token steps
    uint32_t m[2][NG];       // {scale, zero} of tokens tk and 32 + tk
};

template <int CTRL>
__device__ __forceinline__ int dpp_mov_i(int x) {
    return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xF, 0xF, false);
}
// Minimum over the 32 lanes that share lane / 32: DPP inside the 16-lane rows, one lane exchange across them.
__device__ __forceinline__ int half_wave_min(int x) {
    x = min(x, dpp_mov_i<0xB1>(x));      // quad_perm [1,0,3,2]
    x = min(x, dpp_mov_i<0x4E>(x));      // quad_perm [2,3,0,1]
    x = min(x, dpp_mov_i<0x124>(x));     // row_ror:4
    x = min(x, dpp_mov_i<0x128>(x));     // row_ror:8
    return min(x, __shfl_xor(x, 16));
}
__device__ __forceinline__ float half32_sum(float x) {            // over the 32 lanes that share lane / 32
#pragma unroll
    for (int off = 16; off > 0; off >>= 1) x += __shfl_xor(x, off);
    return x;
}

// RQH = 2: up to 4 query heads per workgroup (rows 0-3 high parts, 4-7 low parts); RQH = 4: up to 8 (0-7, 8-15).
// W: sketch words per token, a compile-time choice: with the width known only at run time the refill of the sketch
// registers sat behind branches, the registers they merge into were copied right after the loads, and that copy waited
// for every load in flight -- once per page.
template <int RQH, int D, int NG, int W, bool DTAU>
__global__ __launch_bounds__(kThreads, (RQH == 2 && D <= 128) ? 3 : 2) void decode_split_mfma_kernel(DecodeArgs a, BatchDesc desc, int seq0, int RQ) {
    static_assert(!DTAU || RQH == 2, "the distance-weighted rows take the second half of the 16 operand rows");
    constexpr int RQMAX = 2 * RQH;
    constexpr int NROWS = (DTAU ? 4 : 2) * RQMAX; // operand rows in use
    constexpr int NV = DTAU ? 2 : 1;              // sum sets: weight p, and weight p e
    constexpr int NCB = D / 16;                   // 16-channel column blocks
    constexpr int NCB4 = (NCB + 3) / 4;           // 16-byte loads of code words per lane and step
    constexpr int CBG = NCB / NG;                 // column blocks per quantisation group
    __shared__ float epi[kWaves][NROWS][D];       // epilogue staging of the accumulators
    __shared__ __attribute__((aligned(16))) unsigned short a_s[kWaves][2][NG][16][32];   // A operands of a page's two steps, bf16 bits
    constexpr int kMaxW = W;                      // sketch words per token, all kept in registers
    __shared__ uint64_t sq_s[RQMAX][kMaxW];
    __shared__ int pages_s[kMaxPagesPerChunk];
    __shared__ float f_s[kWaves][RQMAX];          // rescale factors on their way from the scoring lanes to the MFMA rows
    __shared__ int m_s[kWaves][RQMAX];
    __shared__ float l_s[kWaves][NV][RQMAX];
    __shared__ float zs_s[kWaves][NV][RQMAX][NG];
    __shared__ float k_s[kWaves][RQMAX];          // (DTAU) by how much a page lowered each head's running minimum

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const SeqDesc sd = desc.s[blockIdx.z];
    const int ctx = desc_pos(desc, blockIdx.z);
    const int chunk0 = blockIdx.x * a.chunk;
    if (chunk0 >= ctx) return;
    const int n_tok = min(a.chunk, ctx - chunk0);
    const int n_pages = (n_tok + kPage - 1) / kPage;

    const PoolView &pv = a.pool;
    const int H = pv.n_kv_heads, r = pv.n_q_heads / H;
    const int passes = r / RQ;
    const int kvh = blockIdx.y / passes;
    const int qh0 = kvh * r + (blockIdx.y % passes) * RQ;
    const int seq_g = seq0 + blockIdx.z;

    if (tid < n_pages) pages_s[tid] = pv.block_table[(size_t)sd.seq_id * pv.max_pages_per_seq + chunk0 / kPage + tid];
    for (int i = tid; i < RQMAX * kMaxW; i += kThreads) {
        const int q = i / kMaxW, w = i % kMaxW;
        sq_s[q][w] = (q < RQ && w < W) ? a.q_sketch[((size_t)seq_g * pv.n_q_heads + qh0 + q) * W + w] : 0;
    }
    // rows of the A operands that no query head uses stay zero for the whole kernel
    for (int i = tid; i < kWaves * 2 * NG * 16 * 32 / 2; i += kThreads) reinterpret_cast<uint32_t *>(a_s)[i] = 0u;
    __syncthreads();

    const int n = lane & 15, kb = lane >> 4;       // MFMA roles: column / row index, K block
    const int tk = lane & 31, qs = lane >> 5;      // scoring and weight roles: token, query-head parity
    f32x4 acc[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
    float zs[NV][RQH][NG], lsum[NV][RQH];
    int run_min[RQH];
#pragma unroll
    for (int qq = 0; qq < RQH; ++qq) {
        run_min[qq] = 1 << 20;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            lsum[v][qq] = 0.0f;
#pragma unroll
            for (int g = 0; g < NG; ++g) zs[v][qq][g] = 0.0f;
        }
    }
    // Tokens 2, 3, 6, 7 of a block of 8 have their nibbles at bits 4-7 of the operand halves (code 2^-129), the others at
    // bits 0-3 (code 2^-133): this lane's weights carry 2^60 or 2^64, so that every product is weight x code x 2^-69.
    const float w_exp = (tk & 2) ? 60.0f : 64.0f;
    const float w_unscale = (tk & 2) ? 0x1p-60f : 0x1p-64f;

    // One register set holds a page; each plane is requested again, for the next page, as soon as its last use in the
    // current page is behind: the sketches after scoring, the codes and scale/zero of a 32-token step after that
    // step's MFMAs.  (A second set handed over by copies cost a quarter of the loop's vector instructions and a third
    // of the registers.)
    auto page_base = [&](int pg) { return ((size_t)pages_s[pg] * H + kvh) * kPage + wave * 64; };
    auto load_sketches = [&](PageRegs<NCB4, NG, W> &pr, int pg) {
        const size_t base = page_base(pg);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const uint64_t *sp = pv.sketch + (base + 32 * t + tk) * W;
            if (W == 1) {
                pr.sk[t][0] = *sp;
            } else {
#pragma unroll
                for (int w = 0; w < kMaxW; w += 2) {
                    if (w < W) {
                        const uint4 v = *reinterpret_cast<const uint4 *>(sp + w);
                        pr.sk[t][w] = (uint64_t)v.x | ((uint64_t)v.y << 32);
                        pr.sk[t][w + 1] = (uint64_t)v.z | ((uint64_t)v.w << 32);
                    }
                }
            }
        }
    };
    auto load_step = [&](PageRegs<NCB4, NG, W> &pr, int pg, int t) {
        const size_t base = page_base(pg);
        const uint4 *cp = reinterpret_cast<const uint4 *>(pv.codes + (base + 32 * t + 8 * kb) * (D / 2)) + n;
#pragma unroll
        for (int i = 0; i < NCB4; ++i) pr.c[t][i] = load_stream(cp + i * 16);
        const uint32_t *mp = pv.meta + (base + 32 * t + tk) * NG;
#pragma unroll
        for (int g = 0; g < NG; ++g) pr.m[t][g] = load_stream(mp + g);
    };

    // more_tag: whether a page follows (std::true_type / std::false_type).  A compile-time choice, so that the refills are
    // straight-line code: the compiler then counts the loads in flight exactly and waits for the oldest only; behind a
    // run-time branch it waits for all of them.
    auto consume_page = [&](PageRegs<NCB4, NG, W> &pr, int pg, auto more_tag) {
        constexpr bool more = decltype(more_tag)::value;
        // ---- scores of this lane's two tokens against its query heads (Eq. 3) ----
        int ham[2][RQH], pmin[RQH];
        bool valid[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) valid[t] = pg * kPage + wave * 64 + 32 * t + tk < n_tok;
#pragma unroll
        for (int qq = 0; qq < RQH; ++qq) {
            uint64_t sq[kMaxW];
#pragma unroll
            for (int w = 0; w < kMaxW; ++w) sq[w] = sq_s[2 * qq + qs][w];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                int h = 0;
#pragma unroll
                for (int w = 0; w < kMaxW; ++w)
                    if (w < W) h += __popcll(sq[w] ^ pr.sk[t][w]);
                ham[t][qq] = valid[t] ? h : (1 << 20);
            }
            pmin[qq] = half_wave_min(min(ham[0][qq], ham[1][qq]));
        }
        if constexpr (more) load_sketches(pr, pg + 1);
        // ---- running maximum: rescale what has been accumulated if this page raises it ----
        bool changed = false;
#pragma unroll
        for (int qq = 0; qq < RQH; ++qq) changed |= pmin[qq] < run_min[qq];
        if (__any(changed)) {
#pragma unroll
            for (int qq = 0; qq < RQH; ++qq) {
                const int nm = min(run_min[qq], pmin[qq]);
                const float f = fast_exp2(a.exp2_scale * (float)(nm - run_min[qq]));     // <= 1; 0 when nothing was accumulated yet
                const float k = (float)(run_min[qq] - nm);                               // (all sums are still 0 the first time)
                run_min[qq] = nm;
                if constexpr (DTAU) {
                    lsum[1][qq] = (lsum[1][qq] + k * lsum[0][qq]) * f;
#pragma unroll
                    for (int g = 0; g < NG; ++g) zs[1][qq][g] = (zs[1][qq][g] + k * zs[0][qq][g]) * f;
                    if (tk == 0) k_s[wave][2 * qq + qs] = k;
                }
                lsum[0][qq] *= f;
#pragma unroll
                for (int g = 0; g < NG; ++g) zs[0][qq][g] *= f;
                if (tk == 0) f_s[wave][2 * qq + qs] = f;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            float fr[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) fr[j] = f_s[wave][(4 * kb + j) & (RQMAX - 1)];   // row -> head: high and low rows share it
            if constexpr (DTAU) {
                // rows 8-15 (lane groups kb = 2, 3) are the distance-weighted twins of rows 0-7 (kb = 0, 1), 32 lanes away
                float kr[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) kr[j] = kb >= 2 ? k_s[wave][(4 * kb + j) & (RQMAX - 1)] : 0.0f;
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[cb][j] = fmaf(kr[j], __shfl_xor(acc[cb][j], 32), acc[cb][j]);
            }
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[cb][j] *= fr[j];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        // ---- two steps of 32 tokens: weights -> A operands (both steps, then ONE hand-over through LDS) ----
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            float p[NV][RQH];
#pragma unroll
            for (int qq = 0; qq < RQH; ++qq) {
                // heads beyond RQ have an all-zero query sketch here; their rows are never read back
                p[0][qq] = valid[t] ? fast_exp2(fmaf(a.exp2_scale, (float)(run_min[qq] - ham[t][qq]), w_exp)) : 0.0f;
                lsum[0][qq] += p[0][qq];
                if constexpr (DTAU) {
                    p[1][qq] = valid[t] ? p[0][qq] * (float)(ham[t][qq] - run_min[qq]) : 0.0f;
                    lsum[1][qq] += p[1][qq];
                }
            }
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                const uint32_t m = valid[t] ? pr.m[t][g] : 0u;      // never let an unwritten slot's bits reach the arithmetic
                const float sc = __half2float(__ushort_as_half((unsigned short)(m & 0xFFFFu)));
                const float zp = __half2float(__ushort_as_half((unsigned short)(m >> 16)));
#pragma unroll
                for (int v = 0; v < NV; ++v)
#pragma unroll
                    for (int qq = 0; qq < RQH; ++qq) {
                        zs[v][qq][g] = fmaf(p[v][qq], zp, zs[v][qq][g]);
                        const float w = p[v][qq] * sc;
                        const uint32_t hi = __float_as_uint(w) & 0xFFFF0000u;
                        // the remainder is exact; its bf16 part is rounded, not cut: cutting both parts leaves every
                        // weight short by 2^-16 of itself on average, and next to the full-precision sum of p zero
                        // (which nearly cancels the code term) that bias was the kernel's largest error
                        const uint32_t lo = __float_as_uint(w - __uint_as_float(hi)) + 0x8000u;
                        a_s[wave][t][g][2 * v * RQMAX + 2 * qq + qs][tk] = (unsigned short)(hi >> 16);
                        a_s[wave][t][g][(2 * v + 1) * RQMAX + 2 * qq + qs][tk] = (unsigned short)(lo >> 16);
                    }
            }
        }
        // the operands are read by other lanes of the same wave: order the LDS writes before the reads
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // ---- code words -> B operands, MFMA ----
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                const bf16x8 A = *reinterpret_cast<const bf16x8 *>(&a_s[wave][t][g][n][8 * kb]);
#pragma unroll
                for (int j = 0; j < CBG; ++j) {
                    const int cb = g * CBG + j;
                    const uint4 c4 = pr.c[t][cb >> 2];
                    const uint32_t x = (cb & 3) == 0 ? c4.x : (cb & 3) == 1 ? c4.y : (cb & 3) == 2 ? c4.z : c4.w;
                    const uint32_t y = x >> 8;
                    BOperand b;
                    b.u[0] = x & 0x000F000Fu;                  // nibbles 0, 4 = tokens 0, 1 of the block
                    b.u[1] = x & 0x00F000F0u;                  // nibbles 1, 5 = tokens 2, 3
                    b.u[2] = y & 0x000F000Fu;                  // nibbles 2, 6 = tokens 4, 5
                    b.u[3] = y & 0x00F000F0u;                  // nibbles 3, 7 = tokens 6, 7
                    acc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, b.v, acc[cb], 0, 0, 0);
                }
            }
            if constexpr (more) load_step(pr, pg + 1, t);
        }
        // the next page overwrites the operands: its writes must not pass these reads
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };

    {
        PageRegs<NCB4, NG, W> pr;
        load_sketches(pr, 0);
        load_step(pr, 0, 0);
        load_step(pr, 0, 1);
        for (int pg = 0; pg + 1 < n_pages; ++pg) consume_page(pr, pg, std::true_type{});
        consume_page(pr, n_pages - 1, std::false_type{});
    }

    // ---------------- Epilogue: the four waves meet ----------------
#pragma unroll
    for (int v = 0; v < NV; ++v)
#pragma unroll
        for (int qq = 0; qq < RQH; ++qq) {
            lsum[v][qq] = half32_sum(lsum[v][qq] * w_unscale);
#pragma unroll
            for (int g = 0; g < NG; ++g) zs[v][qq][g] = half32_sum(zs[v][qq][g] * w_unscale);
        }
    if (4 * kb < NROWS) {
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int j = 0; j < 4; ++j) epi[wave][4 * kb + j][16 * cb + n] = acc[cb][j];
    }
    if (tk == 0) {
#pragma unroll
        for (int qq = 0; qq < RQH; ++qq) {
            m_s[wave][2 * qq + qs] = run_min[qq];
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                l_s[wave][v][2 * qq + qs] = lsum[v][qq];
#pragma unroll
                for (int g = 0; g < NG; ++g) zs_s[wave][v][2 * qq + qs][g] = zs[v][qq][g];
            }
        }
    }
    __syncthreads();
    const size_t part = ((size_t)seq_g * pv.n_q_heads + qh0) * a.n_splits + blockIdx.x;
    for (int e = tid; e < RQ * D; e += kThreads) {
        const int q = e / D, c = e % D, g = c / (D / NG);
        int hm = 1 << 20;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) hm = min(hm, m_s[w][q]);
        float o = 0.0f, l = 0.0f, oh = 0.0f, lh = 0.0f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            if (DTAU && m_s[w][q] >= (1 << 20)) continue;                           // a wave that saw no valid token
            const float f = fast_exp2(a.exp2_scale * (float)(hm - m_s[w][q]));      // 0 for a wave that saw no valid token
            float val[NV];
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const int hi_row = 2 * v * RQMAX + q, lo_row = hi_row + RQMAX;
                val[v] = fmaf(0x1p69f, epi[w][hi_row][c] + epi[w][lo_row][c], zs_s[w][v][q][g]);   // products were weight x code x 2^-69
            }
            o = fmaf(f, val[0], o);
            l = fmaf(f, l_s[w][0][q], l);
            if constexpr (DTAU) {
                const float k = (float)(m_s[w][q] - hm);                            // the wave counted e from its own minimum
                oh = fmaf(f, fmaf(k, val[0], val[NV - 1]), oh);
                lh = fmaf(f, fmaf(k, l_s[w][0][q], l_s[w][NV - 1][q]), lh);
            }
        }
        a.part_o[(part + (size_t)q * a.n_splits) * D + c] = o;
        if constexpr (DTAU) a.part_oh[(part + (size_t)q * a.n_splits) * D + c] = oh;
        if (c == 0) {
            float *ml = a.part_ml + (part + (size_t)q * a.n_splits) * (DTAU ? 4 : 2);
            ml[0] = __int_as_float(hm);
            ml[1] = l;
            if constexpr (DTAU) ml[2] = lh;
        }
    }
}

template <int RQH, int D, int NG, bool DTAU>
hipError_t launch_w(const DecodeArgs &a, const BatchDesc &desc, int seq0, dim3 grid, int rq, hipStream_t st) {
    switch (a.pool.sketch_bits) {
        case 64: H1BKV_LAUNCH_TIMED((decode_split_mfma_kernel<RQH, D, NG, 1, DTAU>), grid, dim3(kThreads), st, a, desc, seq0, rq); break;
        case 128: H1BKV_LAUNCH_TIMED((decode_split_mfma_kernel<RQH, D, NG, 2, DTAU>), grid, dim3(kThreads), st, a, desc, seq0, rq); break;
        case 256: H1BKV_LAUNCH_TIMED((decode_split_mfma_kernel<RQH, D, NG, 4, DTAU>), grid, dim3(kThreads), st, a, desc, seq0, rq); break;
        case 512: H1BKV_LAUNCH_TIMED((decode_split_mfma_kernel<RQH, D, NG, 8, DTAU>), grid, dim3(kThreads), st, a, desc, seq0, rq); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int RQH, int D, bool DTAU>
hipError_t launch_ng(const DecodeArgs &a, const BatchDesc &desc, int seq0, dim3 grid, int rq, hipStream_t st) {
    const int ng = D / a.pool.group_size;
    if (ng == 1) return launch_w<RQH, D, 1, DTAU>(a, desc, seq0, grid, rq, st);
    if (ng == 2) return launch_w<RQH, D, 2, DTAU>(a, desc, seq0, grid, rq, st);
    if (ng == 4) return launch_w<RQH, D, 4, DTAU>(a, desc, seq0, grid, rq, st);
    if constexpr (D == 256) {
        if (ng == 8) return launch_w<RQH, D, 8, DTAU>(a, desc, seq0, grid, rq, st);
    }
    return hipErrorInvalidValue;
}

template <int RQH, bool DTAU>
hipError_t launch_d(const DecodeArgs &a, const BatchDesc &desc, int seq0, dim3 grid, int rq, hipStream_t st) {
    switch (a.pool.head_dim) {
        case 64: return launch_ng<RQH, 64, DTAU>(a, desc, seq0, grid, rq, st);
        case 128: return launch_ng<RQH, 128, DTAU>(a, desc, seq0, grid, rq, st);
        case 256:                                  // four query heads per workgroup at most: the epilogue's LDS staging
            if constexpr (RQH == 2) return launch_ng<RQH, 256, DTAU>(a, desc, seq0, grid, rq, st);
            return hipErrorInvalidValue;
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_decode_split_mfma(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st) {
    const int r = a.pool.n_q_heads / a.pool.n_kv_heads;
    const int rq = mfma_heads_per_wg(r, a.pool.head_dim);
    const dim3 grid((unsigned)a.n_splits, (unsigned)(a.pool.n_kv_heads * (r / rq)), (unsigned)n_seqs);
    return rq <= 4 ? launch_d<2, false>(a, desc, seq0, grid, rq, st) : launch_d<4, false>(a, desc, seq0, grid, rq, st);
}

// The same with the distance-weighted sums of the temperature derivative: at most four query heads per workgroup.
hipError_t launch_decode_dtau_split_mfma(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st) {
    const int r = a.pool.n_q_heads / a.pool.n_kv_heads;
    const int rq = r % 4 == 0 ? 4 : (r % 3 == 0 ? 3 : (r % 2 == 0 ? 2 : 1));
    const dim3 grid((unsigned)a.n_splits, (unsigned)(a.pool.n_kv_heads * (r / rq)), (unsigned)n_seqs);
    return launch_d<2, true>(a, desc, seq0, grid, rq, st);
}

}  // namespace h1bkv
