// Decode-step attention together with its derivative with respect to the softmax temperature tau -- the one scalar
// that the finetuning stage trains next to V_proj (Sec. IV-C, Eq.(5)):
//   out = sum_t p_t v^_t / l,   p_t = exp(alpha_t / tau),  l = sum_t p_t,
//   d out / d tau = -(1/tau^2) ( sum_t p_t alpha_t v^_t / l - (sum_t p_t alpha_t / l) out ).
// With alpha = 1 - 2 ham / b (Eq.(3)) this is  (2 / (b tau^2)) ( oh / l - (lh / l) out )  for the distance-weighted
// sums  lh = sum p e,  oh = sum p e v^,  where e = ham - ham_min >= 0 (a constant shift of e leaves the bracket
// unchanged).  Counting e from the running minimum keeps lh and oh small next to l and o -- the tokens that carry
// weight have small e -- which is what the covariance in the bracket needs in fp32.
//
// decode_dtau_split_kernel is the vector-ALU decode kernel (record-major codes, one query head per workgroup pass,
// every wave streaming on its own with a running minimum) with a second set of sums whose weight is p e instead of p.
// When a page lowers the running minimum by k, every e grows by k:  lh += k l,  oh += k o,  then the usual rescale.
// merge_dtau_kernel merges the chunk partials the same way and applies the formula above.
#include "decode_common.h"

namespace h1bkv {

namespace {

template <int W, int LPT>
struct PageRegsT {           // what one lane holds of its wave's 64 tokens of one page
    SketchRow<W> sk;         // sketch of token `lane` (scoring role)
    uint4 c[LPT];            // LPT x 16 B of codes and
    uint32_t m[LPT];         //       4 B of scale/zero of token it * TPW + lane / LPT, slice lane % LPT (value role)
};

__device__ __forceinline__ int wave_min_dpp_t(int x) {
    x = min(x, __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xF, 0xF, false));    // quad_perm [1,0,3,2]
    x = min(x, __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xF, 0xF, false));    // quad_perm [2,3,0,1]
    x = min(x, __builtin_amdgcn_update_dpp(0, x, 0x124, 0xF, 0xF, false));   // row_ror:4
    x = min(x, __builtin_amdgcn_update_dpp(0, x, 0x128, 0xF, 0xF, false));   // row_ror:8
    x = min(x, __shfl_xor(x, 16));
    return min(x, __shfl_xor(x, 32));
}

// Index 0 of every pair of sums carries weight p, index 1 weight p e.
template <int W, int LPT>
__global__ __launch_bounds__(kThreads, 1) void decode_dtau_split_kernel(DecodeArgs a, BatchDesc desc, int seq0) {
    constexpr int D = 32 * LPT;
    constexpr int TPW = 64 / LPT;                 // tokens covered by one wave-wide load of codes
    constexpr int ROWS = LPT == 8 ? 2 : 4;        // 16-lane rows of a wave that reach the LDS stage of the epilogue
    constexpr int NPART = kWaves * ROWS;
    constexpr int EPI_STRIDE = D + 2 * LPT;       // per (partial, sum set): D sums, LPT zero-sums, LPT weight-sums
    __shared__ float epi[NPART * 2 * EPI_STRIDE];
    __shared__ int pages_s[kMaxPagesPerChunk];
    __shared__ int m_s[kWaves];
    __shared__ float l_s[kWaves][2];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const SeqDesc sd = desc.s[blockIdx.z];
    const int ctx = sd.pos;
    const int chunk0 = blockIdx.x * a.chunk;
    if (chunk0 >= ctx) return;
    const int n_tok = min(a.chunk, ctx - chunk0);
    const int n_pages = (n_tok + kPage - 1) / kPage;

    const PoolView &pv = a.pool;
    const int H = pv.n_kv_heads, r = pv.n_q_heads / H;
    const int qh = blockIdx.y, kvh = qh / r;
    const int seq_g = seq0 + blockIdx.z;
    const int ng = D / pv.group_size;

    if (tid < n_pages) pages_s[tid] = pv.block_table[(size_t)sd.seq_id * pv.max_pages_per_seq + chunk0 / kPage + tid];
    uint64_t sq[W];
#pragma unroll
    for (int w = 0; w < W; ++w) sq[w] = a.q_sketch[((size_t)seq_g * pv.n_q_heads + qh) * W + w];
    __syncthreads();

    const int slice = lane % LPT;
    const int tok_v = lane / LPT;
    const int meta_col = (slice * 32) / pv.group_size;
    const uint32_t mask = opaque_vgpr(0x00F000F0u), magic = opaque_vgpr(0x64006400u);

    float acc[2][32], zs[2], wsum[2], lsum[2];
    int run_min = 1 << 20;
#pragma unroll
    for (int v = 0; v < 2; ++v) {
        zs[v] = wsum[v] = lsum[v] = 0.0f;
#pragma unroll
        for (int i = 0; i < 32; ++i) acc[v][i] = 0.0f;
    }

    auto load_page = [&](PageRegsT<W, LPT> &pr, int pg) {
        const size_t base = ((size_t)pages_s[pg] * H + kvh) * kPage + wave * 64;
        pr.sk = load_sketch<W>(pv.sketch + (base + lane) * W);
        const uint4 *cp = reinterpret_cast<const uint4 *>(pv.codes) + (base * LPT + lane);
#pragma unroll
        for (int it = 0; it < LPT; ++it) {
            pr.c[it] = load_stream(cp + it * 64);
            pr.m[it] = load_stream(pv.meta + (base + tok_v + it * TPW) * ng + meta_col);
        }
    };

    auto consume_page = [&](const PageRegsT<W, LPT> &pr, int pg) {
        // ---- scoring role: lane = token (Eq. 3), running minimum of the distance ----
        const bool valid = pg * kPage + wave * 64 + lane < n_tok;
        int h = 0;
#pragma unroll
        for (int w = 0; w < W; ++w) h += __popcll(sq[w] ^ pr.sk.w[w]);
        const int pmin = wave_min_dpp_t(valid ? h : (1 << 20));
        if (pmin < run_min) {                          // uniform over the wave; rare after the first pages
            const float k = (float)(run_min - pmin);   // every e grows by k (all sums are still 0 the first time)
            const float f = fast_exp2(a.exp2_scale * (float)(pmin - run_min));
            run_min = pmin;
            lsum[1] = (lsum[1] + k * lsum[0]) * f;
            zs[1] = (zs[1] + k * zs[0]) * f;
            wsum[1] = (wsum[1] + k * wsum[0]) * f;
            lsum[0] *= f;
            zs[0] *= f;
            wsum[0] *= f;
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                acc[1][i] = (acc[1][i] + k * acc[0][i]) * f;
                acc[0][i] *= f;
            }
        }
        const float p = valid ? fast_exp2(a.exp2_scale * (float)(run_min - h)) : 0.0f;
        const float pe = valid ? p * (float)(h - run_min) : 0.0f;
        lsum[0] += p;
        lsum[1] += pe;
        // ---- value role: lane = (token, 32-channel slice); see the decode kernel for the dequantisation ----
#pragma unroll
        for (int it = 0; it < LPT; ++it) {
            const int src_lane = it * TPW + tok_v;
            const bool vvalid = pg * kPage + wave * 64 + src_lane < n_tok;
            const uint32_t m = vvalid ? pr.m[it] : 0u;
            const float sc = __half2float(__ushort_as_half((unsigned short)(m & 0xFFFFu)));
            const float zp = __half2float(__ushort_as_half((unsigned short)(m >> 16)));
            const float pt[2] = {__shfl(p, src_lane), __shfl(pe, src_lane)};
            float w16[2];
#pragma unroll
            for (int v = 0; v < 2; ++v) {
                const float w = pt[v] * sc;
                w16[v] = w * 0.0625f;
                zs[v] = fmaf(pt[v], zp, zs[v]);
                wsum[v] += w;
            }
            const uint32_t x[4] = {pr.c[it].x, pr.c[it].y, pr.c[it].z, pr.c[it].w};
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) {
                const uint32_t t[4] = {and_or(x[dw] << 4, mask, magic), and_or(x[dw], mask, magic),
                                       and_or(x[dw] >> 4, mask, magic), and_or(x[dw] >> 8, mask, magic)};
#pragma unroll
                for (int n = 0; n < 4; ++n) {
                    const __half2 hh = *reinterpret_cast<const __half2 *>(&t[n]);
                    const float lo = __low2float(hh), hi = __high2float(hh);
#pragma unroll
                    for (int v = 0; v < 2; ++v) {
                        acc[v][8 * dw + n] = fmaf(w16[v], lo, acc[v][8 * dw + n]);
                        acc[v][8 * dw + n + 4] = fmaf(w16[v], hi, acc[v][8 * dw + n + 4]);
                    }
                }
            }
        }
    };

    PageRegsT<W, LPT> A, B;
    load_page(A, 0);
    {
        int pg = 0;
        while (true) {
            if (pg + 1 < n_pages) load_page(B, pg + 1);
            consume_page(A, pg);
            if (++pg >= n_pages) break;
            if (pg + 1 < n_pages) load_page(A, pg + 1);
            consume_page(B, pg);
            if (++pg >= n_pages) break;
        }
    }

    // ---------------- Epilogue: the four waves meet ----------------
#pragma unroll
    for (int v = 0; v < 2; ++v) {
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            acc[v][i] = row_slot_sum<LPT>(acc[v][i]);
            if constexpr (ROWS == 2) acc[v][i] = half_wave_sum(acc[v][i]);
        }
        zs[v] = row_slot_sum<LPT>(zs[v]);
        wsum[v] = row_slot_sum<LPT>(wsum[v]);
        if constexpr (ROWS == 2) {
            zs[v] = half_wave_sum(zs[v]);
            wsum[v] = half_wave_sum(wsum[v]);
        }
        lsum[v] = wave_sum(lsum[v]);
    }
    const int row = lane >> 4;
    if ((lane & 15) < LPT && row < ROWS) {
#pragma unroll
        for (int v = 0; v < 2; ++v) {
            float *dst = epi + ((size_t)(wave * ROWS + row) * 2 + v) * EPI_STRIDE;
#pragma unroll
            for (int i = 0; i < 32; i += 4)
                *reinterpret_cast<float4 *>(dst + slice * 32 + i) = make_float4(acc[v][i], acc[v][i + 1], acc[v][i + 2], acc[v][i + 3]);
            dst[D + slice] = zs[v];
            dst[D + LPT + slice] = wsum[v];
        }
    }
    if (lane == 0) {
        m_s[wave] = run_min;
        l_s[wave][0] = lsum[0];
        l_s[wave][1] = lsum[1];
    }
    __syncthreads();
    const size_t part = ((size_t)seq_g * pv.n_q_heads + qh) * a.n_splits + blockIdx.x;
    for (int c = tid; c < D; c += kThreads) {
        int hm = 1 << 20;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) hm = min(hm, m_s[w]);
        float o = 0.0f, oh = 0.0f, l = 0.0f, lh = 0.0f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            if (m_s[w] >= (1 << 20)) continue;                                   // a wave that saw no valid token
            const float f = fast_exp2(a.exp2_scale * (float)(hm - m_s[w]));
            const float k = (float)(m_s[w] - hm);                                // the wave counted e from its own minimum
            float val[2];
#pragma unroll
            for (int v = 0; v < 2; ++v) {
                float ow = 0.0f, z = 0.0f, ws = 0.0f;
#pragma unroll
                for (int rw = 0; rw < ROWS; ++rw) {
                    const float *src = epi + ((size_t)(w * ROWS + rw) * 2 + v) * EPI_STRIDE;
                    ow += src[c];
                    z += src[D + c / 32];
                    ws += src[D + LPT + c / 32];
                }
                val[v] = fmaf(-64.0f, ws, ow) + z;                               // (1024 + 16 code) / 16 = 64 + code
            }
            o = fmaf(f, val[0], o);
            oh = fmaf(f, fmaf(k, val[0], val[1]), oh);
            l = fmaf(f, l_s[w][0], l);
            lh = fmaf(f, fmaf(k, l_s[w][0], l_s[w][1]), lh);
        }
        a.part_o[part * D + c] = o;
        a.part_oh[part * D + c] = oh;
        if (c == 0) {
            float *ml = a.part_ml + part * 4;
            ml[0] = __int_as_float(hm);
            ml[1] = l;
            ml[2] = lh;
        }
    }
}

// One block per (sequence, query head), thread = channel; chunks are walked in order (the derivative is a
// finetuning-side quantity, its merge is not latency-critical).
__global__ void merge_dtau_kernel(DecodeArgs a, BatchDesc desc, int seq0, float dtau_scale) {
    const int D = a.pool.head_dim;
    const int qh = blockIdx.x, seq_g = seq0 + blockIdx.y;
    const int ctx = desc.s[blockIdx.y].pos;
    const int n = (ctx + a.chunk - 1) / a.chunk;
    const size_t part = ((size_t)seq_g * a.pool.n_q_heads + qh) * a.n_splits;
    const int c = threadIdx.x;
    const size_t oi = ((size_t)seq_g * a.pool.n_q_heads + qh) * D + c;
    if (n == 0) {
        a.out[oi] = 0.0f;
        a.dout[oi] = 0.0f;
        return;
    }
    int hmin = 1 << 20;
    for (int s = 0; s < n; ++s) hmin = min(hmin, __float_as_int(a.part_ml[(part + s) * 4]));
    float l = 0.0f, lh = 0.0f, o = 0.0f, oh = 0.0f;
    for (int s = 0; s < n; ++s) {
        const float *ml = a.part_ml + (part + s) * 4;
        const int hm = __float_as_int(ml[0]);
        const float f = fast_exp2(a.exp2_scale * (float)(hmin - hm));
        const float k = (float)(hm - hmin);
        const float os = a.part_o[(part + s) * D + c];
        l = fmaf(f, ml[1], l);
        lh = fmaf(f, fmaf(k, ml[1], ml[2]), lh);
        o = fmaf(f, os, o);
        oh = fmaf(f, fmaf(k, os, a.part_oh[(part + s) * D + c]), oh);
    }
    const float out = o / l;
    a.out[oi] = out;
    a.dout[oi] = dtau_scale * (oh / l - (lh / l) * out);       // dtau_scale = 2 / (b tau^2)
}

template <int W>
hipError_t launch_dtau_lpt(const DecodeArgs &a, const BatchDesc &desc, int seq0, dim3 grid, hipStream_t st) {
    switch (a.pool.head_dim) {
        case 64: hipLaunchKernelGGL((decode_dtau_split_kernel<W, 2>), grid, dim3(kThreads), 0, st, a, desc, seq0); break;
        case 128: hipLaunchKernelGGL((decode_dtau_split_kernel<W, 4>), grid, dim3(kThreads), 0, st, a, desc, seq0); break;
        default: hipLaunchKernelGGL((decode_dtau_split_kernel<W, 8>), grid, dim3(kThreads), 0, st, a, desc, seq0); break;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_decode_dtau_split(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st) {
    const dim3 grid((unsigned)a.n_splits, (unsigned)a.pool.n_q_heads, (unsigned)n_seqs);
    switch (a.pool.sketch_bits) {
        case 64: return launch_dtau_lpt<1>(a, desc, seq0, grid, st);
        case 128: return launch_dtau_lpt<2>(a, desc, seq0, grid, st);
        case 256: return launch_dtau_lpt<4>(a, desc, seq0, grid, st);
        default: return launch_dtau_lpt<8>(a, desc, seq0, grid, st);
    }
}

hipError_t launch_merge_dtau(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, float dtau_scale, hipStream_t st) {
    hipLaunchKernelGGL(merge_dtau_kernel, dim3((unsigned)a.pool.n_q_heads, (unsigned)n_seqs), dim3((unsigned)a.pool.head_dim), 0, st, a,
                       desc, seq0, dtau_scale);
    return hipGetLastError();
}

}  // namespace h1bkv
