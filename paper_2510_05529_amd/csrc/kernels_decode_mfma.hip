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
//     one code word.  Three shifts and four AND-ORs put the nibbles into the mantissas of bf16 128.0 constants:
//     the register pair reads as 128 + code, exact in bf16.
//   A operand (M = 16 rows x K = 32 tokens): the weights w = p[q][t] * scale[t][g] of one quantisation group g,
//     split exactly into two bf16 parts (top 16 bits, and the top 16 bits of the remainder): row q carries the high
//     part and row q + RQMAX the low part, so the product keeps 16 bits of every weight at no extra MFMA cost (the M
//     dimension is far from full anyway).  Each weight is computed once (lane = (token, query-head parity)),
//     written to LDS as two half-words and read back in operand order (16 bytes per lane).
//   The constant 128 of the B operand is removed with the row sums of A, which one more MFMA against an all-ones B
//     delivers in the same rounding as the main products;  sum_t p zero_t  is accumulated on the vector ALU.
//
// Phase A (scores, chunk maximum, softmax weights into LDS) and the partial-result format are those of the
// vector-ALU kernel, so qsketch_kernel and merge_kernel serve both.
#include "decode_common.h"

namespace h1bkv {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

union BOperand {
    uint32_t u[4];
    bf16x8 v;
};

template <int NCB4, int NG>
struct StepRegs {            // what one lane holds of one 32-token step
    uint4 c[NCB4];           // code words of its (channel lane n, token block kb): 4 column blocks per 16 bytes
    uint32_t m[NG];          // {scale, zero} of its (token, groups) for the weight computation
};

// RQH = 2: up to 4 query heads per workgroup (rows 0-3 high parts, 4-7 low parts); RQH = 4: up to 8 (0-7, 8-15).
template <int RQH, int D, int NG>
__global__ __launch_bounds__(kThreads) void decode_split_mfma_kernel(DecodeArgs a, BatchDesc desc, int seq0, int RQ) {
    constexpr int RQMAX = 2 * RQH;
    constexpr int NCB = D / 16;                   // 16-channel column blocks
    constexpr int NCB4 = (NCB + 3) / 4;           // 16-byte loads of code words per lane and step
    constexpr int CBG = NCB / NG;                 // column blocks per quantisation group
    constexpr int CHUNK_MAX = RQMAX > 4 ? kMaxChunk / 2 : kMaxChunk;
    constexpr int P_FLOATS = RQMAX * CHUNK_MAX, EPI_FLOATS = kWaves * 16 * D;
    __shared__ float smem[P_FLOATS > EPI_FLOATS ? P_FLOATS : EPI_FLOATS];   // p_t (ham_t before that); epilogue staging
    __shared__ __attribute__((aligned(16))) unsigned short a_s[kWaves][NG][16][32];   // A operands, bf16 bits
    __shared__ uint64_t sq_s[RQMAX][8];
    __shared__ int pages_s[kMaxPagesPerChunk];
    __shared__ int red_i[RQMAX][kWaves];
    __shared__ float red_f[RQMAX][kWaves];
    __shared__ float sum_s[kWaves][NG][16];
    __shared__ float zs_s[kWaves][RQMAX][NG];
    float(*p_s)[CHUNK_MAX] = reinterpret_cast<float(*)[CHUNK_MAX]>(smem);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const SeqDesc sd = desc.s[blockIdx.z];
    const int ctx = sd.pos;
    const int chunk0 = blockIdx.x * a.chunk;
    if (chunk0 >= ctx) return;
    const int n_tok = min(a.chunk, ctx - chunk0);
    const int n_pages = (n_tok + kPage - 1) / kPage;

    const PoolView &pv = a.pool;
    const int H = pv.n_kv_heads, r = pv.n_q_heads / H, W = pv.sketch_bits >> 6;
    const int passes = r / RQ;
    const int kvh = blockIdx.y / passes;
    const int qh0 = kvh * r + (blockIdx.y % passes) * RQ;
    const int seq_g = seq0 + blockIdx.z;

    if (tid < n_pages) pages_s[tid] = pv.block_table[(size_t)sd.seq_id * pv.max_pages_per_seq + chunk0 / kPage + tid];
    for (int i = tid; i < RQ * W; i += kThreads) sq_s[i / W][i % W] = a.q_sketch[((size_t)seq_g * pv.n_q_heads + qh0 + i / W) * W + i % W];
    // rows of the A operands that no query head uses stay zero for the whole kernel
    for (int i = tid; i < kWaves * NG * 16 * 32 / 2; i += kThreads) reinterpret_cast<uint32_t *>(a_s)[i] = 0u;
    __syncthreads();

    // ---------------- Phase A: scores (thread = token) ----------------
    int hmin[RQMAX];
#pragma unroll
    for (int q = 0; q < RQMAX; ++q) hmin[q] = 1 << 20;
    // pages are taken four at a time: all their sketch loads are in flight before the first popcount
    for (int k0 = 0; k0 < n_pages; k0 += 4) {
        uint64_t s[4][8];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (k0 + kk < n_pages) {
                const uint64_t *sp = pv.sketch + (((size_t)pages_s[k0 + kk] * H + kvh) * kPage + tid) * W;
                if (W == 1) {
                    s[kk][0] = sp[0];
                } else {
#pragma unroll
                    for (int w = 0; w < 8; w += 2) {
                        if (w < W) {
                            const uint4 v = *reinterpret_cast<const uint4 *>(sp + w);
                            s[kk][w] = (uint64_t)v.x | ((uint64_t)v.y << 32);
                            s[kk][w + 1] = (uint64_t)v.z | ((uint64_t)v.w << 32);
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (k0 + kk < n_pages) {
                const int k = k0 + kk;
                const bool valid = k * kPage + tid < n_tok;
#pragma unroll
                for (int q = 0; q < RQMAX; ++q) {
                    if (q < RQ) {
                        int h = 0;
#pragma unroll
                        for (int w = 0; w < 8; ++w)
                            if (w < W) h += __popcll(sq_s[q][w] ^ s[kk][w]);
                        p_s[q][k * kPage + tid] = __int_as_float(h);
                        if (valid) hmin[q] = min(hmin[q], h);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int q = 0; q < RQMAX; ++q) {
        const int m = wave_min(hmin[q]);
        if (lane == 0) red_i[q][wave] = m;
    }
    __syncthreads();
    float lsum[RQMAX];
#pragma unroll
    for (int q = 0; q < RQMAX; ++q) {
        hmin[q] = min(min(red_i[q][0], red_i[q][1]), min(red_i[q][2], red_i[q][3]));
        lsum[q] = 0.0f;
    }
    for (int k = 0; k < n_pages; ++k) {
        const bool valid = k * kPage + tid < n_tok;
#pragma unroll
        for (int q = 0; q < RQMAX; ++q) {
            // heads beyond RQ get weight 0, so their operand rows contribute nothing
            const float p = (q < RQ && valid) ? exp2f(a.exp2_scale * (float)(hmin[q] - __float_as_int(p_s[q][k * kPage + tid]))) : 0.0f;
            p_s[q][k * kPage + tid] = p;
            lsum[q] += p;
        }
    }
#pragma unroll
    for (int q = 0; q < RQMAX; ++q) {
        const float l = wave_sum(lsum[q]);
        if (lane == 0) red_f[q][wave] = l;
    }
    __syncthreads();

    // ---------------- Phase B: weighted sum on the matrix cores ----------------
    const int n = lane & 15, kb = lane >> 4;       // MFMA roles: column / row index, K block
    const int tk = lane & 31, qs = lane >> 5;      // weight roles: token of the step, query-head parity
    f32x4 acc[NCB], accsum[NG];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int g = 0; g < NG; ++g) accsum[g] = f32x4{0.f, 0.f, 0.f, 0.f};
    float zs[RQH][NG];
#pragma unroll
    for (int qq = 0; qq < RQH; ++qq)
#pragma unroll
        for (int g = 0; g < NG; ++g) zs[qq][g] = 0.0f;
    const uint32_t mask = opaque_vgpr(0x000F000Fu), magic = opaque_vgpr(0x43004300u);    // bf16 128.0 in both halves
    BOperand ones;
#pragma unroll
    for (int i = 0; i < 4; ++i) ones.u[i] = 0x3F803F80u;       // bf16 1.0

    // step s of this wave: page s / 2, tokens [wave * 64 + (s & 1) * 32, + 32) of that page
    const int n_steps = 2 * n_pages;
    auto load_step = [&](StepRegs<NCB4, NG> &sr, int s) {
        const size_t base = ((size_t)pages_s[s >> 1] * H + kvh) * kPage + wave * 64 + (s & 1) * 32;
        const uint4 *cp = reinterpret_cast<const uint4 *>(pv.codes + (base + 8 * kb) * (D / 2)) + n;
#pragma unroll
        for (int i = 0; i < NCB4; ++i) sr.c[i] = cp[i * 16];
        const uint32_t *mp = pv.meta + (base + tk) * NG;
#pragma unroll
        for (int g = 0; g < NG; ++g) sr.m[g] = mp[g];
    };
    auto consume_step = [&](const StepRegs<NCB4, NG> &sr, int s) {
        const int idx = (s >> 1) * kPage + wave * 64 + (s & 1) * 32 + tk;
        const bool valid = idx < n_tok;
        float p[RQH];
#pragma unroll
        for (int qq = 0; qq < RQH; ++qq) p[qq] = p_s[2 * qq + qs][idx];
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const uint32_t m = valid ? sr.m[g] : 0u;           // never let an unwritten slot's bits reach the arithmetic
            const float sc = __half2float(__ushort_as_half((unsigned short)(m & 0xFFFFu)));
            const float zp = __half2float(__ushort_as_half((unsigned short)(m >> 16)));
#pragma unroll
            for (int qq = 0; qq < RQH; ++qq) {
                zs[qq][g] = fmaf(p[qq], zp, zs[qq][g]);
                const float w = p[qq] * sc;
                const uint32_t hi = __float_as_uint(w) & 0xFFFF0000u;
                const uint32_t lo = __float_as_uint(w - __uint_as_float(hi));   // exact
                a_s[wave][g][2 * qq + qs][tk] = (unsigned short)(hi >> 16);
                a_s[wave][g][RQMAX + 2 * qq + qs][tk] = (unsigned short)(lo >> 16);
            }
        }
        // the operands are read by other lanes of the same wave: order the LDS writes before the reads
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const bf16x8 A = *reinterpret_cast<const bf16x8 *>(&a_s[wave][g][n][8 * kb]);
#pragma unroll
            for (int j = 0; j < CBG; ++j) {
                const int cb = g * CBG + j;
                const uint4 c4 = sr.c[cb >> 2];
                const uint32_t x = (cb & 3) == 0 ? c4.x : (cb & 3) == 1 ? c4.y : (cb & 3) == 2 ? c4.z : c4.w;
                BOperand b;
                b.u[0] = and_or(x, mask, magic);           // nibbles 0, 4 = tokens 0, 1 of the block
                b.u[1] = and_or(x >> 4, mask, magic);      // nibbles 1, 5 = tokens 2, 3
                b.u[2] = and_or(x >> 8, mask, magic);      // nibbles 2, 6 = tokens 4, 5
                b.u[3] = and_or(x >> 12, mask, magic);     // nibbles 3, 7 = tokens 6, 7
                acc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, b.v, acc[cb], 0, 0, 0);
            }
            accsum[g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, ones.v, accsum[g], 0, 0, 0);
        }
        // the next step overwrites the operands: its writes must not pass these reads
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    {
        StepRegs<NCB4, NG> A, B;
        load_step(A, 0);
        int s = 0;
        while (true) {
            if (s + 1 < n_steps) load_step(B, s + 1);
            consume_step(A, s);
            if (++s >= n_steps) break;
            if (s + 1 < n_steps) load_step(A, s + 1);
            consume_step(B, s);
            if (++s >= n_steps) break;
        }
    }

    // ---------------- Epilogue ----------------
#pragma unroll
    for (int qq = 0; qq < RQH; ++qq)
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int off = 16; off > 0; off >>= 1) zs[qq][g] += __shfl_xor(zs[qq][g], off);   // over the 32 tokens of a half-wave
    __syncthreads();                                   // every wave is done reading p_s
    float *epi = smem;                                 // [wave][row 16][channel D]
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int j = 0; j < 4; ++j) epi[((size_t)wave * 16 + 4 * kb + j) * D + 16 * cb + n] = acc[cb][j];
    if (n == 0) {
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int j = 0; j < 4; ++j) sum_s[wave][g][4 * kb + j] = accsum[g][j];
    }
    if (tk == 0) {
#pragma unroll
        for (int qq = 0; qq < RQH; ++qq)
#pragma unroll
            for (int g = 0; g < NG; ++g) zs_s[wave][2 * qq + qs][g] = zs[qq][g];
    }
    __syncthreads();
    const size_t part = ((size_t)seq_g * pv.n_q_heads + qh0) * a.n_splits + blockIdx.x;
    for (int e = tid; e < RQ * D; e += kThreads) {
        const int q = e / D, c = e % D, g = c / (D / NG);
        float o = 0.0f, ws = 0.0f, z = 0.0f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            o += epi[((size_t)w * 16 + q) * D + c] + epi[((size_t)w * 16 + RQMAX + q) * D + c];
            ws += sum_s[w][g][q] + sum_s[w][g][RQMAX + q];
            z += zs_s[w][q][g];
        }
        a.part_o[(part + (size_t)q * a.n_splits) * D + c] = fmaf(-128.0f, ws, o) + z;   // B held 128 + code
    }
    if (tid < RQ) {
        float *ml = a.part_ml + (part + (size_t)tid * a.n_splits) * 2;
        ml[0] = __int_as_float(hmin[tid]);
        ml[1] = red_f[tid][0] + red_f[tid][1] + red_f[tid][2] + red_f[tid][3];
    }
}

template <int RQH, int D>
hipError_t launch_ng(const DecodeArgs &a, const BatchDesc &desc, int seq0, dim3 grid, int rq, hipStream_t st) {
    const int ng = D / a.pool.group_size;
    if (ng == 1) hipLaunchKernelGGL((decode_split_mfma_kernel<RQH, D, 1>), grid, dim3(kThreads), 0, st, a, desc, seq0, rq);
    else if (ng == 2) hipLaunchKernelGGL((decode_split_mfma_kernel<RQH, D, 2>), grid, dim3(kThreads), 0, st, a, desc, seq0, rq);
    else if (ng == 4) hipLaunchKernelGGL((decode_split_mfma_kernel<RQH, D, 4>), grid, dim3(kThreads), 0, st, a, desc, seq0, rq);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

template <int RQH>
hipError_t launch_d(const DecodeArgs &a, const BatchDesc &desc, int seq0, dim3 grid, int rq, hipStream_t st) {
    switch (a.pool.head_dim) {
        case 64: return launch_ng<RQH, 64>(a, desc, seq0, grid, rq, st);
        case 128: return launch_ng<RQH, 128>(a, desc, seq0, grid, rq, st);
        default: return launch_ng<RQH, 256>(a, desc, seq0, grid, rq, st);
    }
}

}  // namespace

hipError_t launch_decode_split_mfma(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st) {
    const int r = a.pool.n_q_heads / a.pool.n_kv_heads;
    const int rq = mfma_heads_per_wg(r);
    const dim3 grid((unsigned)a.n_splits, (unsigned)(a.pool.n_kv_heads * (r / rq)), (unsigned)n_seqs);
    return rq <= 4 ? launch_d<2>(a, desc, seq0, grid, rq, st) : launch_d<4>(a, desc, seq0, grid, rq, st);
}

}  // namespace h1bkv
