// Decode-step attention for the "1-bit key only" variant (Table V ablation, Sec. VI-E): keys are packed sketches
// scored by XOR + popcount (Sec. IV-A Eq.(3)), values are kept as fp16, so Eq.(5) is softmax(alpha/tau) fp16(V).
//
// Same streaming structure as the 4-bit kernel: one workgroup (4 waves) per (context chunk, KV head [x query-head
// pass], sequence); every wave streams on its own over its 64 tokens of each page with a running maximum per query
// head; the waves meet once, in the epilogue.
//   Scoring role  lane = token (16-byte sketch load at b = 128), wave minimum of the Hamming distance by DPP.
//   Value role    lane = (token, 8-channel slice): one 16-byte load = 8 fp16 channels, so a wave instruction reads
//            1 KiB of contiguous values (64 / (d/8) tokens); p_t comes from the scoring lane by a lane swizzle and
//            the fp16 -> fp32 widening rides on the mixed-precision FMA.  2d + 8W bytes per token against d FMAs per
//            query head: HBM-bound for every r the kernel serves (up to 8 query heads per pass).
//   Slots past the end of the context can hold anything (also NaN bit patterns): the last, partial share of a wave
//   takes a masked path that zeroes them; full shares take the plain path.
// DTAU = true adds the distance-weighted sums of the temperature derivative (Sec. IV-C; formula in
// kernels_decode_dtau.hip): every query head carries a second accumulator set with weight p e, e = ham - running
// minimum; when a page lowers the minimum by k the second set takes k times the first before the usual rescale.
#include <type_traits>
#include <utility>

#include "decode_common.h"

namespace h1bkv {

namespace {

__device__ __forceinline__ int wave_min_dpp16(int x) {
    x = min(x, __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xF, 0xF, false));    // quad_perm [1,0,3,2]
    x = min(x, __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xF, 0xF, false));    // quad_perm [2,3,0,1]
    x = min(x, __builtin_amdgcn_update_dpp(0, x, 0x124, 0xF, 0xF, false));   // row_ror:4
    x = min(x, __builtin_amdgcn_update_dpp(0, x, 0x128, 0xF, 0xF, false));   // row_ror:8
    x = min(x, __shfl_xor(x, 16));
    return min(x, __shfl_xor(x, 32));
}

// Compile-time loop: body(std::integral_constant<int, I>{}) for I = 0 .. N-1 (the lane-swizzle pattern below must
// be an immediate).
template <int N, typename F, int... I>
__device__ __forceinline__ void static_for_impl(F &&body, std::integer_sequence<int, I...>) {
    (body(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F &&body) {
    static_for_impl<N>(body, std::make_integer_sequence<int, N>{});
}

// Broadcast, inside every aligned group of GROUP lanes (8, 16 or 32), the value of the group's lane IDX: a lane
// swizzle with an immediate pattern (lane' = (lane & and_mask) | or_mask within each half-wave) -- no index register,
// unlike a general lane permute.
template <int GROUP, int IDX>
__device__ __forceinline__ float group_pick(float x) {
    constexpr int and_mask = 0x1F & ~(GROUP - 1);
    return __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(x), and_mask | (IDX << 5)));
}

// Register budget: one batch of value loads (up to 16 x 16 B per lane) plus 8 accumulators per query head; the
// latency of the single-buffered loads is covered by the other resident waves (4 per SIMD at one query head).
template <int RQ, int W, int D, bool DTAU>
__global__ __launch_bounds__(kThreads, RQ * (DTAU ? 2 : 1) >= 8 ? 2 : (RQ * (DTAU ? 2 : 1) >= 4 ? 3 : 4)) void decode_split_f16v_kernel(DecodeArgs a, BatchDesc desc, int seq0) {
    constexpr int LPT = D / 8;                    // lanes per token
    constexpr int TPW = 64 / LPT;                 // tokens covered by one wave-wide load of values
    constexpr int NV = DTAU ? 2 : 1;              // sum sets per query head: weight p, and weight p e
    constexpr int RQV = RQ * NV;                  // accumulator sets: set NV q + v
    __shared__ float epi[kWaves][RQV][D];
    __shared__ int pages_s[kMaxPagesPerChunk];
    __shared__ int m_s[kWaves][RQ];
    __shared__ float l_s[kWaves][RQV];

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

    uint64_t sq[RQ][W];
#pragma unroll
    for (int q = 0; q < RQ; ++q)
#pragma unroll
        for (int w = 0; w < W; ++w) {
            // the same for every lane: keep it in scalar registers
            const uint64_t x = a.q_sketch[((size_t)seq_g * pv.n_q_heads + qh0 + q) * W + w];
            const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x), hi = __builtin_amdgcn_readfirstlane((uint32_t)(x >> 32));
            sq[q][w] = (uint64_t)lo | ((uint64_t)hi << 32);
        }
    __syncthreads();

    const int slice = lane % LPT;
    const int tok_v = lane / LPT;

    float acc[RQV][8];
    float lsum[RQV];
    int run_min[RQ];
#pragma unroll
    for (int q = 0; q < RQ; ++q) run_min[q] = 1 << 20;
#pragma unroll
    for (int q = 0; q < RQV; ++q) {
        lsum[q] = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[q][i] = 0.0f;
    }

    // Value loads per batch: a share's loads are taken in batches that fit the register budget next to the
    // accumulators (16 x 16 B per lane at one or two query heads and d <= 128, 8 otherwise).
    constexpr int LPB = (RQV >= 4 || LPT > 16) ? (LPT < 8 ? LPT : 8) : LPT;
    constexpr int NB = LPT / LPB;

    // Token order inside a wave's 64-token share: the value loads cover TPW consecutive tokens per instruction
    // (lane = (token tok_v, slice)), so load `it` of lane group tok_v holds token it * TPW + tok_v.  The scoring lanes
    // are laid out to match: lane (tok_v, it) scores exactly that token, so a value lane finds its weight in lane
    // `it` of its own LPT-lane group.
    const int tok_s = slice * TPW + tok_v;                 // scoring role: this lane's token within the share

    auto consume_share = [&](int pg, auto masked_tag) {
        constexpr bool kMasked = decltype(masked_tag)::value;
        const int tok0 = pg * kPage + wave * 64;
        const size_t base = ((size_t)pages_s[pg] * H + kvh) * kPage + wave * 64;
        const SketchRow<W> sk = load_sketch<W>(pv.sketch + (base + tok_s) * W);
        const uint4 *vp = reinterpret_cast<const uint4 *>(pv.codes) + (base * LPT + lane);
        uint4 v[LPB];
#pragma unroll
        for (int it = 0; it < LPB; ++it) v[it] = load_stream(vp + it * 64);
        // ---- scoring role (Eq. 3), running maximum per query head ----
        const bool valid = !kMasked || tok0 + tok_s < n_tok;
        float p[RQV];
#pragma unroll
        for (int q = 0; q < RQ; ++q) {
            int h = 0;
#pragma unroll
            for (int w = 0; w < W; ++w) h += __popcll(sq[q][w] ^ sk.w[w]);
            const int pmin = wave_min_dpp16(valid ? h : (1 << 20));
            if (pmin < run_min[q]) {                       // uniform over the wave; rare after the first pages
                const float f = fast_exp2(a.exp2_scale * (float)(pmin - run_min[q]));
                if constexpr (DTAU) {
                    const float k = (float)(run_min[q] - pmin);      // every e grows by k (all sums are still 0 the first time)
                    lsum[NV * q + 1] = (lsum[NV * q + 1] + k * lsum[NV * q]) * f;
#pragma unroll
                    for (int i = 0; i < 8; ++i) acc[NV * q + 1][i] = (acc[NV * q + 1][i] + k * acc[NV * q][i]) * f;
                }
                run_min[q] = pmin;
                lsum[NV * q] *= f;
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[NV * q][i] *= f;
            }
            p[NV * q] = valid ? fast_exp2(a.exp2_scale * (float)(run_min[q] - h)) : 0.0f;
            lsum[NV * q] += p[NV * q];
            if constexpr (DTAU) {
                p[NV * q + 1] = valid ? p[NV * q] * (float)(h - run_min[q]) : 0.0f;
                lsum[NV * q + 1] += p[NV * q + 1];
            }
        }
        // ---- value role: lane = (token, 8-channel slice) ----
        static_for<NB>([&](auto nbc) {
            constexpr int nb = decltype(nbc)::value;
            if constexpr (nb > 0) {
                __builtin_amdgcn_sched_barrier(0);         // keep the next batch's loads behind this point
#pragma unroll
                for (int it = 0; it < LPB; ++it) v[it] = load_stream(vp + (nb * LPB + it) * 64);
            }
            static_for<LPB>([&](auto itc) {
                constexpr int it = decltype(itc)::value;
                constexpr int load = nb * LPB + it;
                // with many query heads the scheduler would otherwise pull every load's swizzles up front and spill
                if constexpr (RQV >= 4 && it > 0) __builtin_amdgcn_sched_barrier(0);
                uint4 x = v[it];
                if (kMasked && tok0 + load * TPW + tok_v >= n_tok) x = make_uint4(0u, 0u, 0u, 0u);
                const __half2 *h2 = reinterpret_cast<const __half2 *>(&x);
                float pt[RQV];
#pragma unroll
                for (int q = 0; q < RQV; ++q) pt[q] = group_pick<LPT, load>(p[q]);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float lo = __low2float(h2[i]), hi = __high2float(h2[i]);
#pragma unroll
                    for (int q = 0; q < RQV; ++q) {
                        acc[q][2 * i] = fmaf(pt[q], lo, acc[q][2 * i]);
                        acc[q][2 * i + 1] = fmaf(pt[q], hi, acc[q][2 * i + 1]);
                    }
                }
            });
        });
    };

    for (int pg = 0; pg < n_pages; ++pg) {
        if (pg * kPage + wave * 64 + 64 <= n_tok) consume_share(pg, std::false_type{});
        else consume_share(pg, std::true_type{});
    }

    // ---------------- Epilogue: token slots of a wave, then the four waves ----------------
#pragma unroll
    for (int q = 0; q < RQV; ++q) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int off = LPT; off < 64; off <<= 1) acc[q][i] += __shfl_xor(acc[q][i], off);
        lsum[q] = wave_sum(lsum[q]);
    }
    if (tok_v == 0) {
#pragma unroll
        for (int q = 0; q < RQV; ++q) {
            *reinterpret_cast<float4 *>(&epi[wave][q][slice * 8]) = make_float4(acc[q][0], acc[q][1], acc[q][2], acc[q][3]);
            *reinterpret_cast<float4 *>(&epi[wave][q][slice * 8 + 4]) = make_float4(acc[q][4], acc[q][5], acc[q][6], acc[q][7]);
        }
    }
    if (lane == 0) {
#pragma unroll
        for (int q = 0; q < RQ; ++q) m_s[wave][q] = run_min[q];
#pragma unroll
        for (int q = 0; q < RQV; ++q) l_s[wave][q] = lsum[q];
    }
    __syncthreads();
    const size_t part = ((size_t)seq_g * pv.n_q_heads + qh0) * a.n_splits + blockIdx.x;
    for (int e = tid; e < RQ * D; e += kThreads) {
        const int q = e / D, c = e % D;
        int hm = 1 << 20;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) hm = min(hm, m_s[w][q]);
        float o = 0.0f, l = 0.0f, oh = 0.0f, lh = 0.0f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            if (DTAU && m_s[w][q] >= (1 << 20)) continue;                           // a wave that saw no valid token
            const float f = fast_exp2(a.exp2_scale * (float)(hm - m_s[w][q]));      // 0 for a wave that saw no valid token
            o = fmaf(f, epi[w][NV * q][c], o);
            l = fmaf(f, l_s[w][NV * q], l);
            if constexpr (DTAU) {
                const float k = (float)(m_s[w][q] - hm);                            // the wave counted e from its own minimum
                oh = fmaf(f, fmaf(k, epi[w][NV * q][c], epi[w][NV * q + 1][c]), oh);
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

template <int RQ, int W, bool DTAU>
hipError_t launch_d(const DecodeArgs &a, const BatchDesc &desc, int seq0, dim3 grid, hipStream_t st) {
    if (a.pool.head_dim == 64) {
        H1BKV_LAUNCH_TIMED((decode_split_f16v_kernel<RQ, W, 64, DTAU>), grid, dim3(kThreads), st, a, desc, seq0);
    } else if constexpr (RQ * (DTAU ? 2 : 1) <= 4) {                 // 8 accumulator sets only fit next to a d = 64 batch
        if (a.pool.head_dim == 128) H1BKV_LAUNCH_TIMED((decode_split_f16v_kernel<RQ, W, 128, DTAU>), grid, dim3(kThreads), st, a, desc, seq0);
        else H1BKV_LAUNCH_TIMED((decode_split_f16v_kernel<RQ, W, 256, DTAU>), grid, dim3(kThreads), st, a, desc, seq0);
    } else {
        return hipErrorInvalidConfiguration;
    }
    return hipGetLastError();
}

template <int RQ, bool DTAU>
hipError_t launch_w(const DecodeArgs &a, const BatchDesc &desc, int seq0, dim3 grid, hipStream_t st) {
    switch (a.pool.sketch_bits) {
        case 64: return launch_d<RQ, 1, DTAU>(a, desc, seq0, grid, st);
        case 128: return launch_d<RQ, 2, DTAU>(a, desc, seq0, grid, st);
        case 256: return launch_d<RQ, 4, DTAU>(a, desc, seq0, grid, st);
        default: return launch_d<RQ, 8, DTAU>(a, desc, seq0, grid, st);
    }
}

}  // namespace

hipError_t launch_decode_split_f16v(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st) {
    const int r = a.pool.n_q_heads / a.pool.n_kv_heads;
    // query heads per workgroup pass: the largest of 8 (d = 64 only), 4, 2, 1 that divides r
    const int rq = (r % 8 == 0 && a.pool.head_dim == 64) ? 8 : (r % 4 == 0 ? 4 : (r % 2 == 0 ? 2 : 1));
    const dim3 grid((unsigned)a.n_splits, (unsigned)(a.pool.n_kv_heads * (r / rq)), (unsigned)n_seqs);
    switch (rq) {
        case 8: return launch_w<8, false>(a, desc, seq0, grid, st);
        case 4: return launch_w<4, false>(a, desc, seq0, grid, st);
        case 2: return launch_w<2, false>(a, desc, seq0, grid, st);
        default: return launch_w<1, false>(a, desc, seq0, grid, st);
    }
}

// The same with the distance-weighted sums of the temperature derivative: two accumulator sets per query head, so
// at most two query heads per pass.
hipError_t launch_decode_dtau_split_f16v(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st) {
    const int r = a.pool.n_q_heads / a.pool.n_kv_heads;
    const int rq = r % 2 == 0 ? 2 : 1;
    const dim3 grid((unsigned)a.n_splits, (unsigned)(a.pool.n_kv_heads * (r / rq)), (unsigned)n_seqs);
    return rq == 2 ? launch_w<2, true>(a, desc, seq0, grid, st) : launch_w<1, true>(a, desc, seq0, grid, st);
}

}  // namespace h1bkv
