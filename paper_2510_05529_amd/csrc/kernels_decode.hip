// Decode-step attention over the compressed cache (Sec. IV-A Eq.(3), Sec. IV-C Eq.(5)).
//
// decode_split_kernel: one workgroup (4 waves) per (context chunk, KV head [x query-head pass], sequence); every
//   wave streams on its own over its 64 tokens of each page of the chunk, with no workgroup barrier until the end.
//   Scoring role  lane = token: packed sketch (16 B/lane at b = 128), Hamming distance by XOR + popcount against the
//            RQ query sketches that share this KV head, wave-wide minimum (= maximum score alpha) by DPP.  The wave
//            keeps a running maximum per head; when a page raises it the accumulators are rescaled (scores only
//            take b+1 values, so this happens a handful of times per chunk).  p_t = exp((alpha_t - alpha_max)/tau).
//   Value role    lane = (token, 32-channel slice): each lane reads one aligned 16-byte run of nibbles (exactly
//            32 codes) and the 4-byte {scale, zero} pair of its group, so a wave instruction covers 1 KiB of
//            contiguous codes; p_t comes from the scoring lane by a lane permute.  Dequantisation is folded into
//            the weights:  sum_t p_t (scale_t code_tc + zero_t) = sum_t (p_t scale_t) code_tc + sum_t p_t zero_t,
//            and the int4 -> float step rides on the FMA itself (a masked nibble is read as an fp16 subnormal by a
//            mixed-precision FMA): 13 VALU instructions per 8 elements.
//            Loads for the next page (sketches, codes, scale/zero) are in flight while the current page is consumed.
//   Epilogue sums over the token slots of a 16-lane row with DPP rotations, over rows and waves through LDS (each
//            wave's part scaled to the common maximum), and writes the chunk's partial (min distance, sum p,
//            unnormalised output) to the workspace.
// merge_kernel: log-sum-exp merge of the chunk partials of one (sequence, query head).
// qsketch_kernel: s_q = sign(R q) with the same fp32 FMA chain as the keys (lane = bit, ballot = word).
#include "decode_common.h"

namespace h1bkv {

namespace {

template <int W, int LPT>
struct PageRegs {            // what one lane holds of its wave's 64 tokens of one page
    SketchRow<W> sk;         // sketch of token `lane` (scoring role)
    uint4 c[LPT];            // LPT x 16 B of codes and
    uint32_t m[LPT];         //       4 B of scale/zero of token it * TPW + lane / LPT, slice lane % LPT (value role)
};

// Minimum over the wave, result in every lane: DPP inside the 16-lane rows, two lane exchanges across them.
__device__ __forceinline__ int wave_min_dpp(int x) {
    x = min(x, __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xF, 0xF, false));    // quad_perm [1,0,3,2]
    x = min(x, __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xF, 0xF, false));    // quad_perm [2,3,0,1]
    x = min(x, __builtin_amdgcn_update_dpp(0, x, 0x124, 0xF, 0xF, false));   // row_ror:4
    x = min(x, __builtin_amdgcn_update_dpp(0, x, 0x128, 0xF, 0xF, false));   // row_ror:8
    x = min(x, __shfl_xor(x, 16));
    return min(x, __shfl_xor(x, 32));
}

// DTAU = true adds the distance-weighted sums of the temperature derivative (Sec. IV-C; formula in
// kernels_decode_dtau.hip): every query head carries a second accumulator set with weight p e, e = ham - running
// minimum >= 0; when a page lowers the minimum by k, the second set takes k times the first before the usual rescale.
template <int RQH, int W, int LPT, bool DTAU>
__global__ __launch_bounds__(kThreads, RQH * (DTAU ? 2 : 1) >= 4 ? 2 : 1) void decode_split_kernel(DecodeArgs a, BatchDesc desc, int seq0) {
    constexpr int NV = DTAU ? 2 : 1;              // sum sets per query head: weight p, and weight p e
    constexpr int RQ = RQH * NV;                  // accumulator sets: set NV q + v of query head q
    constexpr int D = 32 * LPT;
    constexpr int TPW = 64 / LPT;                 // tokens covered by one wave-wide load of codes
    constexpr int ROWS = LPT == 8 ? 2 : 4;        // 16-lane rows of a wave that reach the LDS stage of the epilogue
    constexpr int NPART = kWaves * ROWS;
    constexpr int EPI_STRIDE = D + LPT;           // per (partial, q): D sums, LPT zero-sums
    __shared__ float epi[NPART * RQ * EPI_STRIDE];
    __shared__ int pages_s[kMaxPagesPerChunk];
    __shared__ int m_s[kWaves][RQH];
    __shared__ float l_s[kWaves][RQ];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const SeqDesc sd = desc.s[blockIdx.z];
    const PoolView &pv = a.pool;
    const int chunk0 = blockIdx.x * a.chunk;
    // The chunk's page ids and the query sketches do not depend on the context length: they are requested first, so that
    // a length that lives in device memory (desc_pos) is one more load in flight, not a round trip in front of them.
    // (Table entries past the sequence's pages are read too and never used.)
    int my_page = 0;
    if (tid < a.chunk / kPage && chunk0 / kPage + tid < pv.max_pages_per_seq)
        my_page = pv.block_table[(size_t)sd.seq_id * pv.max_pages_per_seq + chunk0 / kPage + tid];
    const int H = pv.n_kv_heads, r = pv.n_q_heads / H;
    const int passes = r / RQH;
    const int kvh = blockIdx.y / passes;
    const int qh0 = kvh * r + (blockIdx.y % passes) * RQH;
    const int seq_g = seq0 + blockIdx.z;
    const int ng = D / pv.group_size;
    uint64_t sq[RQH][W];
#pragma unroll
    for (int q = 0; q < RQH; ++q)
#pragma unroll
        for (int w = 0; w < W; ++w) sq[q][w] = a.q_sketch[((size_t)seq_g * pv.n_q_heads + qh0 + q) * W + w];

    const int ctx = desc_pos(desc, blockIdx.z);
    if (chunk0 >= ctx) return;
    const int n_tok = min(a.chunk, ctx - chunk0);
    const int n_pages = (n_tok + kPage - 1) / kPage;
    if (tid < n_pages) pages_s[tid] = my_page;
    __syncthreads();

    // Every wave streams on its own: it owns tokens [64 wave, 64 wave + 64) of each page of the chunk.
    const int slice = lane % LPT;
    const int tok_v = lane / LPT;                          // value role: token (within a 64-token share) of the first load
    const int meta_col = (slice * 32) / pv.group_size;
    const uint32_t mask_a = opaque_vgpr(0x000F000Fu), mask_b = opaque_vgpr(0x00F000F0u);

    float acc[RQ][32];
    float zs[RQ], lsum[RQ];
    int run_min[RQH];
#pragma unroll
    for (int q = 0; q < RQH; ++q) run_min[q] = 1 << 20;
#pragma unroll
    for (int q = 0; q < RQ; ++q) {
        zs[q] = 0.0f;
        lsum[q] = 0.0f;
#pragma unroll
        for (int i = 0; i < 32; ++i) acc[q][i] = 0.0f;
    }

    auto load_page = [&](PageRegs<W, LPT> &pr, int pg) {
        const size_t base = ((size_t)pages_s[pg] * H + kvh) * kPage + wave * 64;
        pr.sk = load_sketch<W>(pv.sketch + (base + lane) * W);
        const uint4 *cp = reinterpret_cast<const uint4 *>(pv.codes) + (base * LPT + lane);
#pragma unroll
        for (int it = 0; it < LPT; ++it) {
            pr.c[it] = load_stream(cp + it * 64);
            pr.m[it] = load_stream(pv.meta + (base + tok_v + it * TPW) * ng + meta_col);
        }
    };

    // A nibble is turned into an fp16 number without a convert instruction and without an offset: masked in place
    // at mantissa bits 0-3 or 4-7 of an otherwise zero half-word it IS the fp16 subnormal code 2^-24 or code 2^-20
    // (two nibbles, n and n + 4 of a dword, per AND; one shift by 8 bits reaches the other four).  The fp32 FMA takes
    // the fp16 halves directly (mixed-precision FMA, fp16 denormals are enabled) with the weight p scale scaled by
    // 2^24 or 2^20 -- exact powers of two, so the products are the exact p scale code.
    auto consume_page = [&](const PageRegs<W, LPT> &pr, int pg) {
        // ---- scoring role: lane = token (Eq. 3), running maximum per query head ----
        const bool valid = pg * kPage + wave * 64 + lane < n_tok;
        float p[RQ];
#pragma unroll
        for (int q = 0; q < RQH; ++q) {
            int h = 0;
#pragma unroll
            for (int w = 0; w < W; ++w) h += __popcll(sq[q][w] ^ pr.sk.w[w]);
            const int pmin = wave_min_dpp(valid ? h : (1 << 20));
            if (pmin < run_min[q]) {                       // uniform over the wave; rare after the first pages
                const float f = fast_exp2(a.exp2_scale * (float)(pmin - run_min[q]));   // 0 while nothing has been accumulated
                if constexpr (DTAU) {
                    const float k = (float)(run_min[q] - pmin);      // every e grows by k (all sums are still 0 the first time)
                    lsum[NV * q + 1] = (lsum[NV * q + 1] + k * lsum[NV * q]) * f;
                    zs[NV * q + 1] = (zs[NV * q + 1] + k * zs[NV * q]) * f;
#pragma unroll
                    for (int i = 0; i < 32; ++i) acc[NV * q + 1][i] = (acc[NV * q + 1][i] + k * acc[NV * q][i]) * f;
                }
                run_min[q] = pmin;
                lsum[NV * q] *= f;
                zs[NV * q] *= f;
#pragma unroll
                for (int i = 0; i < 32; ++i) acc[NV * q][i] *= f;
            }
            p[NV * q] = valid ? fast_exp2(a.exp2_scale * (float)(run_min[q] - h)) : 0.0f;
            lsum[NV * q] += p[NV * q];
            if constexpr (DTAU) {
                p[NV * q + 1] = valid ? p[NV * q] * (float)(h - run_min[q]) : 0.0f;
                lsum[NV * q + 1] += p[NV * q + 1];
            }
        }
        // ---- value role: lane = (token, 32-channel slice) ----
#pragma unroll
        for (int it = 0; it < LPT; ++it) {
            const int src_lane = it * TPW + tok_v;         // the lane that scored this lane's token
            const bool vvalid = pg * kPage + wave * 64 + src_lane < n_tok;
            const uint32_t m = vvalid ? pr.m[it] : 0u;     // never let an unwritten slot's bits reach the FMAs
            const float sc = __half2float(__ushort_as_half((unsigned short)(m & 0xFFFFu)));
            const float zp = __half2float(__ushort_as_half((unsigned short)(m >> 16)));
            float wa[RQ], wb[RQ];
#pragma unroll
            for (int q = 0; q < RQ; ++q) {
                const float pt = __shfl(p[q], src_lane);
                const float w = pt * sc;
                wa[q] = w * 16777216.0f;                   // a nibble at mantissa bits 0-3 reads as code 2^-24
                wb[q] = w * 1048576.0f;                    //          at mantissa bits 4-7 as code 2^-20
                zs[q] = fmaf(pt, zp, zs[q]);
            }
            const uint32_t x[4] = {pr.c[it].x, pr.c[it].y, pr.c[it].z, pr.c[it].w};
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) {
                const uint32_t y = x[dw] >> 8;
                // t[n] holds nibbles n (low half) and n + 4 (high half) as fp16 subnormals
                const uint32_t t[4] = {x[dw] & mask_a, x[dw] & mask_b, y & mask_a, y & mask_b};
#pragma unroll
                for (int n = 0; n < 4; ++n) {
                    const __half2 h = *reinterpret_cast<const __half2 *>(&t[n]);
                    const float lo = __low2float(h), hi = __high2float(h);
#pragma unroll
                    for (int q = 0; q < RQ; ++q) {
                        const float wq = (n & 1) ? wb[q] : wa[q];
                        acc[q][8 * dw + n] = fmaf(wq, lo, acc[q][8 * dw + n]);
                        acc[q][8 * dw + n + 4] = fmaf(wq, hi, acc[q][8 * dw + n + 4]);
                    }
                }
            }
        }
    };

    // With 4 query heads per lane the 128 accumulators leave no room for a second page buffer: those variants run
    // single-buffered at 2 waves per SIMD and rely on the other resident waves to cover the load latency.
    constexpr bool kDoubleBuffer = RQ < 4;
    PageRegs<W, LPT> A;
    [[maybe_unused]] PageRegs<W, LPT> B;
    load_page(A, 0);
    if constexpr (kDoubleBuffer) {
        // The last page is consumed in a copy of the code without a prefetch in front of it: with the prefetch behind a
        // run-time branch, the compiler must assume at the join that it did not happen, waits for the current page's
        // registers as if they were the youngest loads, and so waits for most of the prefetch it has just issued.
        int pg = 0;
        while (true) {
            if (pg + 1 >= n_pages) {
                consume_page(A, pg);
                break;
            }
            load_page(B, pg + 1);
            consume_page(A, pg);
            ++pg;
            if (pg + 1 >= n_pages) {
                consume_page(B, pg);
                break;
            }
            load_page(A, pg + 1);
            consume_page(B, pg);
            ++pg;
        }
    } else {
        for (int pg = 0; pg < n_pages; ++pg) {
            if (pg > 0) load_page(A, pg);
            consume_page(A, pg);
        }
    }

    // ---------------- Epilogue: the four waves meet ----------------
    // Token slots of a 16-lane row are summed with DPP rotations; rows and waves meet in LDS.
#pragma unroll
    for (int q = 0; q < RQ; ++q) {
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            acc[q][i] = row_slot_sum<LPT>(acc[q][i]);
            if constexpr (ROWS == 2) acc[q][i] = half_wave_sum(acc[q][i]);
        }
        zs[q] = row_slot_sum<LPT>(zs[q]);
        if constexpr (ROWS == 2) {
            zs[q] = half_wave_sum(zs[q]);
        }
        lsum[q] = wave_sum(lsum[q]);
    }
    const int row = lane >> 4;
    if ((lane & 15) < LPT && row < ROWS) {
#pragma unroll
        for (int q = 0; q < RQ; ++q) {
            float *dst = epi + ((size_t)(wave * ROWS + row) * RQ + q) * EPI_STRIDE;
#pragma unroll
            for (int i = 0; i < 32; i += 4)
                *reinterpret_cast<float4 *>(dst + slice * 32 + i) = make_float4(acc[q][i], acc[q][i + 1], acc[q][i + 2], acc[q][i + 3]);
            dst[D + slice] = zs[q];
        }
    }
    if (lane == 0) {
#pragma unroll
        for (int q = 0; q < RQH; ++q) m_s[wave][q] = run_min[q];
#pragma unroll
        for (int q = 0; q < RQ; ++q) l_s[wave][q] = lsum[q];
    }
    __syncthreads();
    const size_t part = ((size_t)seq_g * pv.n_q_heads + qh0) * a.n_splits + blockIdx.x;
    for (int e = tid; e < RQH * D; e += kThreads) {
        const int q = e / D, c = e % D;
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
                float ow = 0.0f, z = 0.0f;
#pragma unroll
                for (int rw = 0; rw < ROWS; ++rw) {
                    const float *src = epi + ((size_t)(w * ROWS + rw) * RQ + NV * q + v) * EPI_STRIDE;
                    ow += src[c];
                    z += src[D + c / 32];
                }
                val[v] = ow + z;
            }
            o = fmaf(f, val[0], o);
            l = fmaf(f, l_s[w][NV * q], l);
            if constexpr (DTAU) {
                const float k = (float)(m_s[w][q] - hm);                            // the wave counted e from its own minimum
                oh = fmaf(f, fmaf(k, val[0], val[NV - 1]), oh);
                lh = fmaf(f, fmaf(k, l_s[w][NV * q], l_s[w][NV * q + 1]), lh);
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

// out = sum_s e^{(alpha_s - alpha_max)/tau} o_s / sum_s e^{(alpha_s - alpha_max)/tau} l_s over the chunks of one head.
// One block per (sequence, query head); thread = (channel, chunk lane): the chunks are strided over
// kMergeThreads / d lanes and met in LDS, so a 128k context (64 chunks) costs 16 dependent steps, not 64.
constexpr int kMergeThreads = 512;
__global__ __launch_bounds__(kMergeThreads) void merge_kernel(DecodeArgs a, BatchDesc desc, int seq0) {
    __shared__ int hmin_s[kMergeThreads / 64];
    __shared__ float lo_s[kMergeThreads][2];
    const int D = a.pool.head_dim;
    const int qh = blockIdx.x, seq_g = seq0 + blockIdx.y;
    const int ctx = desc_pos(desc, blockIdx.y);
    if (desc.advance) {                       // (uniform) device-resident positions: this is the step's last kernel
        __syncthreads();
        if (threadIdx.x == 0) advance_positions_when_all_read(desc, a.pool.ticket, gridDim.x * gridDim.y, (int)gridDim.y);
    }
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
        const float w = fast_exp2(a.exp2_scale * (float)(hmin - __float_as_int(a.part_ml[(part + s) * 2])));
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

// The same merge for large batches of short contexts (at most kMergeFewChunks chunks, thousands of heads): a thread owns
// (head, channel) and walks the head's chunks itself, 512 / d heads per block -- one block per head is thousands of
// blocks of 512 threads with a handful of loads each (11.9 -> 6.4 us at 128 sequences x 32 heads).
constexpr int kMergeFewChunks = 8;
__global__ __launch_bounds__(kMergeThreads) void merge_few_kernel(DecodeArgs a, BatchDesc desc, int seq0, int n_seqs) {
    const int D = a.pool.head_dim, Hq = a.pool.n_q_heads;
    const int c = threadIdx.x % D;
    const int head = blockIdx.x * (kMergeThreads / D) + threadIdx.x / D;       // (sequence, query head) of this launch, flattened
    const bool mine = head < n_seqs * Hq;
    const int ctx = mine ? desc_pos(desc, head / Hq) : 0;
    if (desc.advance) {                       // (uniform) device-resident positions: this is the step's last kernel
        __syncthreads();
        if (threadIdx.x == 0) advance_positions_when_all_read(desc, a.pool.ticket, gridDim.x, n_seqs);
    }
    if (!mine) return;
    const int s_local = head / Hq, qh = head % Hq, seq_g = seq0 + s_local;
    const int n = (ctx + a.chunk - 1) / a.chunk;
    const size_t part = ((size_t)seq_g * Hq + qh) * a.n_splits;
    float *out = a.out + ((size_t)seq_g * Hq + qh) * D;
    if (n == 0) {
        out[c] = 0.0f;
        return;
    }
    int hm[kMergeFewChunks];
    float ls[kMergeFewChunks], os[kMergeFewChunks];
    int hmin = 1 << 20;
#pragma unroll
    for (int s = 0; s < kMergeFewChunks; ++s) {
        if (s < n) {
            hm[s] = __float_as_int(a.part_ml[(part + s) * 2]);
            ls[s] = a.part_ml[(part + s) * 2 + 1];
            os[s] = a.part_o[(part + s) * D + c];
            hmin = min(hmin, hm[s]);
        }
    }
    float l = 0.0f, o = 0.0f;
#pragma unroll
    for (int s = 0; s < kMergeFewChunks; ++s) {
        if (s < n) {
            const float w = fast_exp2(a.exp2_scale * (float)(hmin - hm[s]));
            l = fmaf(w, ls[s], l);
            o = fmaf(w, os[s], o);
        }
    }
    out[c] = o / l;
}

// One wave per (query vector, sketch word): lane = bit.  All d loads of the lane's column of R^T are issued before
// the FMA chain starts (the chain itself must stay sequential: its order fixes the bits), so the kernel costs
// one memory round trip, not d of them.
template <typename T, int D>
__global__ void qsketch_kernel(DecodeArgs a, int seq0) {
    __shared__ float qs[D];
    const int b = a.pool.sketch_bits, W = b >> 6;
    const size_t vec = (size_t)seq0 * a.pool.n_q_heads + blockIdx.x;
    const T *q = static_cast<const T *>(a.q) + vec * D;
    const int bit = threadIdx.x;
    for (int j = threadIdx.x; j < D; j += blockDim.x) qs[j] = (float)q[j];
    __syncthreads();
    // at most 128 elements of the column at a time (256 would not fit the register file next to anything else)
    constexpr int CH = D < 128 ? D : 128;
    float y = 0.0f;
#pragma unroll 1
    for (int j0 = 0; j0 < D; j0 += CH) {
        float rt[CH];
#pragma unroll
        for (int j = 0; j < CH; ++j) rt[j] = a.pool.RT[(size_t)(j0 + j) * b + bit];
#pragma unroll
        for (int j = 0; j < CH; ++j) y = __builtin_fmaf(rt[j], qs[j0 + j], y);
    }
    const uint64_t mask = __ballot(y >= 0.0f);
    if ((threadIdx.x & 63) == 0) a.q_sketch[vec * W + (threadIdx.x >> 6)] = mask;
}

template <int RQ, int W, bool DTAU>
hipError_t launch_split_lpt(const DecodeArgs &a, const BatchDesc &desc, int seq0, dim3 grid, hipStream_t st) {
    switch (a.pool.head_dim) {
        case 64: H1BKV_LAUNCH_TIMED((decode_split_kernel<RQ, W, 2, DTAU>), grid, dim3(kThreads), st, a, desc, seq0); break;
        case 128: H1BKV_LAUNCH_TIMED((decode_split_kernel<RQ, W, 4, DTAU>), grid, dim3(kThreads), st, a, desc, seq0); break;
        default: H1BKV_LAUNCH_TIMED((decode_split_kernel<RQ, W, 8, DTAU>), grid, dim3(kThreads), st, a, desc, seq0); break;
    }
    return hipGetLastError();
}

template <int RQ, bool DTAU = false>
hipError_t launch_split_w(const DecodeArgs &a, const BatchDesc &desc, int seq0, dim3 grid, hipStream_t st) {
    switch (a.pool.sketch_bits) {
        case 64: return launch_split_lpt<RQ, 1, DTAU>(a, desc, seq0, grid, st);
        case 128: return launch_split_lpt<RQ, 2, DTAU>(a, desc, seq0, grid, st);
        case 256: return launch_split_lpt<RQ, 4, DTAU>(a, desc, seq0, grid, st);
        default: return launch_split_lpt<RQ, 8, DTAU>(a, desc, seq0, grid, st);
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

// The same with the distance-weighted sums of the temperature derivative: one query head (two accumulator sets) per
// workgroup pass.
hipError_t launch_decode_dtau_split(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st) {
    const dim3 grid((unsigned)a.n_splits, (unsigned)a.pool.n_q_heads, (unsigned)n_seqs);
    return launch_split_w<1, true>(a, desc, seq0, grid, st);
}

hipError_t launch_merge(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st) {
    const int heads = n_seqs * a.pool.n_q_heads;
    if (a.n_splits <= kMergeFewChunks && heads >= 2048 && kMergeThreads % a.pool.head_dim == 0) {
        const int per_block = kMergeThreads / a.pool.head_dim;
        hipLaunchKernelGGL(merge_few_kernel, dim3((unsigned)((heads + per_block - 1) / per_block)), dim3(kMergeThreads), 0, st, a, desc, seq0, n_seqs);
    } else {
        hipLaunchKernelGGL(merge_kernel, dim3((unsigned)a.pool.n_q_heads, (unsigned)n_seqs), dim3(kMergeThreads), 0, st, a, desc, seq0);
    }
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_qsketch_t(const DecodeArgs &a, int seq0, int n_seqs, hipStream_t st) {
    const dim3 grid((unsigned)(n_seqs * a.pool.n_q_heads)), block((unsigned)a.pool.sketch_bits);
    switch (a.pool.head_dim) {
        case 64: hipLaunchKernelGGL((qsketch_kernel<T, 64>), grid, block, 0, st, a, seq0); break;
        case 128: hipLaunchKernelGGL((qsketch_kernel<T, 128>), grid, block, 0, st, a, seq0); break;
        default: hipLaunchKernelGGL((qsketch_kernel<T, 256>), grid, block, 0, st, a, seq0); break;
    }
    return hipGetLastError();
}

hipError_t launch_qsketch(const DecodeArgs &a, int seq0, int n_seqs, hipStream_t st) {
    return a.f16 ? launch_qsketch_t<__half>(a, seq0, n_seqs, st) : launch_qsketch_t<float>(a, seq0, n_seqs, st);
}

}  // namespace h1bkv
