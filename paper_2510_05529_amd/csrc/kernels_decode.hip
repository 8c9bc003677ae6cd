// Decode-step attention over the compressed cache (Sec. IV-A Eq.(3), Sec. IV-C Eq.(5)).
//
// decode_split_kernel: one workgroup (4 waves) per (context chunk, KV head [x query-head pass], sequence).
//   Phase A  thread = token: stream the chunk's packed sketches (16 B/lane at b = 128), Hamming distance
//            by XOR + popcount against the RQ query sketches that share this KV head, block-wide minimum
//            distance (= maximum score alpha), then p_t = exp((alpha_t - alpha_max)/tau) into LDS and sum p.
//            Scores only take b+1 values and alpha_max is known before any value byte is touched, so the
//            accumulators are never rescaled.
//   Phase B  lane = (token, 32-channel slice): each lane reads one aligned 16-byte run of nibbles (exactly
//            32 codes) and the 4-byte {scale, zero} pair of its group, so a wave instruction covers 1 KiB of
//            contiguous codes.  Dequantisation is folded into the weights:
//              sum_t p_t (scale_t code_tc + zero_t) = sum_t (p_t scale_t) code_tc + sum_t p_t zero_t,
//            and the int4 -> float step rides on the FMA itself (nibbles OR-ed into the mantissa of an fp16
//            constant, read by a mixed-precision FMA): 15 VALU instructions per 8 elements.
//            Loads for the next page are in flight while the current page is consumed.
//   Epilogue sums over the token slots of a 16-lane row with DPP rotations, over rows and waves through LDS,
//            and writes the chunk's partial (min distance, sum p, unnormalised output) to the workspace.
// merge_kernel: log-sum-exp merge of the chunk partials of one (sequence, query head).
// qsketch_kernel: s_q = sign(R q) with the same fp32 FMA chain as the keys (lane = bit, ballot = word).
#include "decode_common.h"

namespace h1bkv {

namespace {

template <int LPT>
struct PageRegs {            // what one lane holds of one page: LPT x (16 B of codes + 4 B of scale/zero)
    uint4 c[LPT];
    uint32_t m[LPT];
};

template <int RQ, int W, int LPT>
__global__ __launch_bounds__(kThreads, RQ >= 4 ? 2 : 1) void decode_split_kernel(DecodeArgs a, BatchDesc desc, int seq0) {
    constexpr int D = 32 * LPT;
    constexpr int TPW = 64 / LPT;                 // tokens covered by one wave-wide load
    constexpr int ROWS = LPT == 8 ? 2 : 4;        // 16-lane rows of a wave that reach the LDS stage of the epilogue
    constexpr int NPART = kWaves * ROWS;
    constexpr int EPI_STRIDE = D + 2 * LPT;       // per (partial, q): D sums, LPT zero-sums, LPT weight-sums
    constexpr int P_FLOATS = RQ * kMaxChunk, EPI_FLOATS = NPART * RQ * EPI_STRIDE;
    // p_t of the chunk during phases A/B; reused for the partial sums of the epilogue.
    __shared__ float smem[P_FLOATS > EPI_FLOATS ? P_FLOATS : EPI_FLOATS];
    __shared__ int pages_s[kMaxPagesPerChunk];
    __shared__ int red_i[RQ][kWaves];
    __shared__ float red_f[RQ][kWaves];
    float(*p_s)[kMaxChunk] = reinterpret_cast<float(*)[kMaxChunk]>(smem);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const SeqDesc sd = desc.s[blockIdx.z];
    const int ctx = sd.pos;
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
    const int ng = D / pv.group_size;

    if (tid < n_pages) pages_s[tid] = pv.block_table[(size_t)sd.seq_id * pv.max_pages_per_seq + chunk0 / kPage + tid];

    uint64_t sq[RQ][W];
#pragma unroll
    for (int q = 0; q < RQ; ++q)
#pragma unroll
        for (int w = 0; w < W; ++w) sq[q][w] = a.q_sketch[((size_t)seq_g * pv.n_q_heads + qh0 + q) * W + w];
    __syncthreads();

    const int slice = lane % LPT;
    const int tok_w = wave * 64 + lane / LPT;              // token (within a page) of this lane's first load
    const int meta_col = (slice * 32) / pv.group_size;
    const uint32_t mask = opaque_vgpr(0x00F000F0u), magic = opaque_vgpr(0x64006400u);

    auto load_page = [&](PageRegs<LPT> &pr, int pg) {
        const size_t base = ((size_t)pages_s[pg] * H + kvh) * kPage;
        const uint4 *cp = reinterpret_cast<const uint4 *>(pv.codes) + (base * LPT + wave * 64 * LPT + lane);
#pragma unroll
        for (int it = 0; it < LPT; ++it) {
            pr.c[it] = cp[it * 64];
            pr.m[it] = pv.meta[(base + tok_w + it * TPW) * ng + meta_col];
        }
    };
    // With 4 query heads per lane the 128 accumulators leave no room for a second page buffer: those variants run
    // single-buffered at 2 waves per SIMD and rely on the other resident waves to cover the load latency.
    constexpr bool kDoubleBuffer = RQ < 4;
    PageRegs<LPT> A;
    [[maybe_unused]] PageRegs<LPT> B;

    // ---------------- Phase A: scores ----------------
    int ham[RQ][kMaxPagesPerChunk];
    int hmin[RQ];
#pragma unroll
    for (int q = 0; q < RQ; ++q) hmin[q] = 1 << 20;
    {
        SketchRow<W> s[kMaxPagesPerChunk];
#pragma unroll
        for (int k = 0; k < kMaxPagesPerChunk; ++k)
            if (k < n_pages) s[k] = load_sketch<W>(pv.sketch + (((size_t)pages_s[k] * H + kvh) * kPage + tid) * W);
        // The first page of values is requested right behind the sketches, before any score is computed, so
        // that its latency is covered by phase A instead of being paid after it.
        load_page(A, 0);
#pragma unroll
        for (int k = 0; k < kMaxPagesPerChunk; ++k) {
            if (k < n_pages) {
                const bool valid = k * kPage + tid < n_tok;
#pragma unroll
                for (int q = 0; q < RQ; ++q) {
                    int h = 0;
#pragma unroll
                    for (int w = 0; w < W; ++w) h += __popcll(sq[q][w] ^ s[k].w[w]);
                    ham[q][k] = h;
                    if (valid) hmin[q] = min(hmin[q], h);
                }
            }
        }
    }
#pragma unroll
    for (int q = 0; q < RQ; ++q) {
        const int m = wave_min(hmin[q]);
        if (lane == 0) red_i[q][wave] = m;
    }
    __syncthreads();
    float lsum[RQ];
#pragma unroll
    for (int q = 0; q < RQ; ++q) {
        hmin[q] = min(min(red_i[q][0], red_i[q][1]), min(red_i[q][2], red_i[q][3]));
        lsum[q] = 0.0f;
    }
#pragma unroll
    for (int k = 0; k < kMaxPagesPerChunk; ++k) {
        if (k < n_pages) {
            const bool valid = k * kPage + tid < n_tok;
#pragma unroll
            for (int q = 0; q < RQ; ++q) {
                const float p = valid ? exp2f(a.exp2_scale * (float)(hmin[q] - ham[q][k])) : 0.0f;
                p_s[q][k * kPage + tid] = p;
                lsum[q] += p;
            }
        }
    }
#pragma unroll
    for (int q = 0; q < RQ; ++q) {
        const float l = wave_sum(lsum[q]);
        if (lane == 0) red_f[q][wave] = l;
    }
    __syncthreads();

    // ---------------- Phase B: weighted sum of dequantised values ----------------
    // A nibble is turned into an fp16 number without a convert instruction: shifted to mantissa bits 4-7 of
    // 1024.0 (0x6400) and OR-ed in, it reads as 1024 + 16 code, two nibbles (n and n+4 of a dword) per 32-bit
    // operation; the fp32 FMA takes the fp16 halves directly (mixed-precision FMA) with weight p scale / 16.
    // The constant part, 64 times the running sum of weights, is taken off at the end.  (Leaving even nibbles
    // at bits 0-3 would save two shifts per dword but puts a 1024-fold offset under the fp32 accumulation.)
    float acc[RQ][32];
    float zs[RQ], wsum[RQ];
#pragma unroll
    for (int q = 0; q < RQ; ++q) {
        zs[q] = 0.0f;
        wsum[q] = 0.0f;
#pragma unroll
        for (int i = 0; i < 32; ++i) acc[q][i] = 0.0f;
    }
    auto consume_page = [&](const PageRegs<LPT> &pr, int pg) {
#pragma unroll
        for (int it = 0; it < LPT; ++it) {
            const int idx = pg * kPage + tok_w + it * TPW;
            const uint32_t m = idx < n_tok ? pr.m[it] : 0u;    // never let an unwritten slot's bits reach the FMAs
            const float sc = __half2float(__ushort_as_half((unsigned short)(m & 0xFFFFu)));
            const float zp = __half2float(__ushort_as_half((unsigned short)(m >> 16)));
            float w16[RQ];
#pragma unroll
            for (int q = 0; q < RQ; ++q) {
                const float p = p_s[q][idx];
                const float w = p * sc;
                w16[q] = w * 0.0625f;
                zs[q] = fmaf(p, zp, zs[q]);
                wsum[q] += w;
            }
            const uint32_t x[4] = {pr.c[it].x, pr.c[it].y, pr.c[it].z, pr.c[it].w};
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) {
                const uint32_t t[4] = {and_or(x[dw] << 4, mask, magic), and_or(x[dw], mask, magic),
                                       and_or(x[dw] >> 4, mask, magic), and_or(x[dw] >> 8, mask, magic)};
#pragma unroll
                for (int n = 0; n < 4; ++n) {               // t[n] holds nibbles n (low half) and n + 4 (high half)
                    const __half2 h = *reinterpret_cast<const __half2 *>(&t[n]);
                    const float lo = __low2float(h), hi = __high2float(h);
#pragma unroll
                    for (int q = 0; q < RQ; ++q) {
                        acc[q][8 * dw + n] = fmaf(w16[q], lo, acc[q][8 * dw + n]);
                        acc[q][8 * dw + n + 4] = fmaf(w16[q], hi, acc[q][8 * dw + n + 4]);
                    }
                }
            }
        }
    };

    if constexpr (kDoubleBuffer) {
        int pg = 0;
        while (true) {
            if (pg + 1 < n_pages) load_page(B, pg + 1);
            consume_page(A, pg);
            if (++pg >= n_pages) break;
            if (pg + 1 < n_pages) load_page(A, pg + 1);
            consume_page(B, pg);
            if (++pg >= n_pages) break;
        }
    } else {
        for (int pg = 0; pg < n_pages; ++pg) {
            if (pg > 0) load_page(A, pg);
            consume_page(A, pg);
        }
    }

    // ---------------- Epilogue ----------------
    // Token slots of a 16-lane row are summed with DPP rotations; rows and waves meet in LDS.
#pragma unroll
    for (int q = 0; q < RQ; ++q) {
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            acc[q][i] = row_slot_sum<LPT>(acc[q][i]);
            if constexpr (ROWS == 2) acc[q][i] = half_wave_sum(acc[q][i]);
        }
        zs[q] = row_slot_sum<LPT>(zs[q]);
        wsum[q] = row_slot_sum<LPT>(wsum[q]);
        if constexpr (ROWS == 2) {
            zs[q] = half_wave_sum(zs[q]);
            wsum[q] = half_wave_sum(wsum[q]);
        }
    }
    __syncthreads();                                   // every wave is done reading p_s
    float *epi = smem;
    const int row = lane >> 4;
    if ((lane & 15) < LPT && row < ROWS) {
#pragma unroll
        for (int q = 0; q < RQ; ++q) {
            float *dst = epi + ((size_t)(wave * ROWS + row) * RQ + q) * EPI_STRIDE;
#pragma unroll
            for (int i = 0; i < 32; i += 4)
                *reinterpret_cast<float4 *>(dst + slice * 32 + i) = make_float4(acc[q][i], acc[q][i + 1], acc[q][i + 2], acc[q][i + 3]);
            dst[D + slice] = zs[q];
            dst[D + LPT + slice] = wsum[q];
        }
    }
    __syncthreads();
    const size_t part = ((size_t)seq_g * pv.n_q_heads + qh0) * a.n_splits + blockIdx.x;
    for (int e = tid; e < RQ * D; e += kThreads) {
        const int q = e / D, c = e % D;
        float o = 0.0f, z = 0.0f, ws = 0.0f;
#pragma unroll
        for (int pt = 0; pt < NPART; ++pt) {
            const float *src = epi + ((size_t)pt * RQ + q) * EPI_STRIDE;
            o += src[c];
            z += src[D + c / 32];
            ws += src[D + LPT + c / 32];
        }
        a.part_o[(part + (size_t)q * a.n_splits) * D + c] = fmaf(-64.0f, ws, o) + z;   // (1024 + 16 code) / 16 = 64 + code
    }
    if (tid < RQ) {
        float *ml = a.part_ml + (part + (size_t)tid * a.n_splits) * 2;
        ml[0] = __int_as_float(hmin[tid]);
        ml[1] = red_f[tid][0] + red_f[tid][1] + red_f[tid][2] + red_f[tid][3];
    }
}

// out = sum_s e^{(alpha_s - alpha_max)/tau} o_s / sum_s e^{(alpha_s - alpha_max)/tau} l_s over the chunks of one head.
// One block per (sequence, query head); thread = (channel, chunk lane): the chunks are strided over
// kMergeThreads / d lanes and met in LDS, so a 128k context (64 chunks) costs 16 dependent steps, not 64.
constexpr int kMergeThreads = 512;
__global__ __launch_bounds__(kMergeThreads) void merge_kernel(DecodeArgs a, BatchDesc desc, int seq0) {
    __shared__ int hmin_s[kMergeThreads / 64];
    __shared__ float lo_s[kMergeThreads][2];
    const int D = a.pool.head_dim;
    const int qh = blockIdx.x, seq_g = seq0 + blockIdx.y;
    const int ctx = desc.s[blockIdx.y].pos;
    const int n = (ctx + a.chunk - 1) / a.chunk;
    const size_t part = ((size_t)seq_g * a.pool.n_q_heads + qh) * a.n_splits;
    const int tid = threadIdx.x, c = tid % D, sl = tid / D, n_sl = kMergeThreads / D;
    float *out = a.out + ((size_t)seq_g * a.pool.n_q_heads + qh) * D;
    if (n == 0) {
        if (sl == 0) out[c] = 0.0f;
        return;
    }
    int hmin = 1 << 20;
    for (int s = tid; s < n; s += kMergeThreads) hmin = min(hmin, __float_as_int(a.part_ml[(part + s) * 2]));
    hmin = wave_min(hmin);
    if ((tid & 63) == 0) hmin_s[tid >> 6] = hmin;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kMergeThreads / 64; ++w) hmin = min(hmin, hmin_s[w]);
    float l = 0.0f, o = 0.0f;
#pragma unroll 4
    for (int s = sl; s < n; s += n_sl) {
        const float w = exp2f(a.exp2_scale * (float)(hmin - __float_as_int(a.part_ml[(part + s) * 2])));
        l = fmaf(w, a.part_ml[(part + s) * 2 + 1], l);
        o = fmaf(w, a.part_o[(part + s) * D + c], o);
    }
    lo_s[tid][0] = l;
    lo_s[tid][1] = o;
    __syncthreads();
    if (sl == 0) {
        for (int k = 1; k < n_sl; ++k) {
            l += lo_s[k * D + c][0];
            o += lo_s[k * D + c][1];
        }
        out[c] = o / l;
    }
}

// One wave per (query vector, sketch word): lane = bit.
template <typename T>
__global__ void qsketch_kernel(DecodeArgs a, int seq0) {
    __shared__ float qs[256];
    const int D = a.pool.head_dim, b = a.pool.sketch_bits, W = b >> 6;
    const size_t vec = (size_t)seq0 * a.pool.n_q_heads + blockIdx.x;
    const T *q = static_cast<const T *>(a.q) + vec * D;
    for (int j = threadIdx.x; j < D; j += blockDim.x) qs[j] = (float)q[j];
    __syncthreads();
    const int bit = threadIdx.x;
    float y = 0.0f;
#pragma unroll 16
    for (int j = 0; j < D; ++j) y = __builtin_fmaf(a.pool.RT[(size_t)j * b + bit], qs[j], y);
    const uint64_t mask = __ballot(y >= 0.0f);
    if ((threadIdx.x & 63) == 0) a.q_sketch[vec * W + (threadIdx.x >> 6)] = mask;
}

template <int RQ, int W>
hipError_t launch_split_lpt(const DecodeArgs &a, const BatchDesc &desc, int seq0, dim3 grid, hipStream_t st) {
    switch (a.pool.head_dim) {
        case 64: hipLaunchKernelGGL((decode_split_kernel<RQ, W, 2>), grid, dim3(kThreads), 0, st, a, desc, seq0); break;
        case 128: hipLaunchKernelGGL((decode_split_kernel<RQ, W, 4>), grid, dim3(kThreads), 0, st, a, desc, seq0); break;
        default: hipLaunchKernelGGL((decode_split_kernel<RQ, W, 8>), grid, dim3(kThreads), 0, st, a, desc, seq0); break;
    }
    return hipGetLastError();
}

template <int RQ>
hipError_t launch_split_w(const DecodeArgs &a, const BatchDesc &desc, int seq0, dim3 grid, hipStream_t st) {
    switch (a.pool.sketch_bits) {
        case 64: return launch_split_lpt<RQ, 1>(a, desc, seq0, grid, st);
        case 128: return launch_split_lpt<RQ, 2>(a, desc, seq0, grid, st);
        case 256: return launch_split_lpt<RQ, 4>(a, desc, seq0, grid, st);
        default: return launch_split_lpt<RQ, 8>(a, desc, seq0, grid, st);
    }
}

}  // namespace

// Query heads handled per workgroup: the largest of 4, 2, 1 that divides r.
static int q_per_wg(int r) { return r % 4 == 0 ? 4 : (r % 2 == 0 ? 2 : 1); }

hipError_t launch_decode_split(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st) {
    const int r = a.pool.n_q_heads / a.pool.n_kv_heads;
    const int rq = q_per_wg(r);
    const dim3 grid((unsigned)a.n_splits, (unsigned)(a.pool.n_kv_heads * (r / rq)), (unsigned)n_seqs);
    switch (rq) {
        case 4: return launch_split_w<4>(a, desc, seq0, grid, st);
        case 2: return launch_split_w<2>(a, desc, seq0, grid, st);
        default: return launch_split_w<1>(a, desc, seq0, grid, st);
    }
}

hipError_t launch_merge(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st) {
    hipLaunchKernelGGL(merge_kernel, dim3((unsigned)a.pool.n_q_heads, (unsigned)n_seqs), dim3(kMergeThreads), 0, st, a, desc, seq0);
    return hipGetLastError();
}

hipError_t launch_qsketch(const DecodeArgs &a, int seq0, int n_seqs, hipStream_t st) {
    const dim3 grid((unsigned)(n_seqs * a.pool.n_q_heads)), block((unsigned)a.pool.sketch_bits);
    if (a.f16) hipLaunchKernelGGL((qsketch_kernel<__half>), grid, block, 0, st, a, seq0);
    else hipLaunchKernelGGL((qsketch_kernel<float>), grid, block, 0, st, a, seq0);
    return hipGetLastError();
}

}  // namespace h1bkv
