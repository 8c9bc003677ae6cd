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
//            i.e. one int->float convert and one fp32 FMA per element, plus one FMA per 32 elements.
//            Loads for the next page are in flight while the current page is consumed.
//   Epilogue sums over the token slots of a wave by lane exchange, over waves through LDS, and writes the
//            chunk's partial (min distance, sum p, unnormalised output) to the workspace.
// merge_kernel: log-sum-exp merge of the chunk partials of one (sequence, query head).
// qsketch_kernel: s_q = sign(R q) with the same fp32 FMA chain as the keys (lane = bit, ballot = word).
#include <hip/hip_fp16.h>

#include "internal.h"

namespace h1bkv {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxPagesPerChunk = kMaxChunk / kPage;

__device__ __forceinline__ int wave_min(int x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x = min(x, __shfl_xor(x, off));
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    return x;
}
// Sum over the lanes that hold the same channel slice (lane % LPT) of different tokens.
template <int LPT>
__device__ __forceinline__ float slot_sum(float x) {
#pragma unroll
    for (int off = 32; off >= LPT; off >>= 1) x += __shfl_xor(x, off);
    return x;
}

template <int W>
struct SketchRow {
    uint64_t w[W];
};
template <int W>
__device__ __forceinline__ SketchRow<W> load_sketch(const uint64_t *p) {
    SketchRow<W> s;
    if constexpr (W == 1) {
        s.w[0] = *p;
    } else {
#pragma unroll
        for (int i = 0; i < W; i += 2) {
            const uint4 v = *reinterpret_cast<const uint4 *>(p + i);
            s.w[i] = (uint64_t)v.x | ((uint64_t)v.y << 32);
            s.w[i + 1] = (uint64_t)v.z | ((uint64_t)v.w << 32);
        }
    }
    return s;
}

template <int LPT>
struct PageRegs {            // what one lane holds of one page: LPT x (16 B of codes + 4 B of scale/zero)
    uint4 c[LPT];
    uint32_t m[LPT];
};

template <int RQ, int W, int LPT>
__global__ __launch_bounds__(kThreads) void decode_split_kernel(DecodeArgs a, BatchDesc desc, int seq0) {
    constexpr int D = 32 * LPT;
    constexpr int TPW = 64 / LPT;     // tokens covered by one wave-wide load
    __shared__ float p_s[RQ][kMaxChunk];
    __shared__ int pages_s[kMaxPagesPerChunk];
    __shared__ int red_i[RQ][kWaves];
    __shared__ float red_f[RQ][kWaves];
    __shared__ float wave_o[kWaves][RQ][D];
    __shared__ float wave_z[kWaves][RQ][LPT];

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
    float acc[RQ][32];
    float zs[RQ];
#pragma unroll
    for (int q = 0; q < RQ; ++q) {
        zs[q] = 0.0f;
#pragma unroll
        for (int i = 0; i < 32; ++i) acc[q][i] = 0.0f;
    }
    const int slice = lane % LPT;
    const int tok_w = wave * 64 + lane / LPT;              // token (within a page) of this lane's first load
    const int meta_col = (slice * 32) / pv.group_size;

    auto load_page = [&](PageRegs<LPT> &pr, int pg) {
        const size_t base = ((size_t)pages_s[pg] * H + kvh) * kPage;
        const uint4 *cp = reinterpret_cast<const uint4 *>(pv.codes) + (base * LPT + wave * 64 * LPT + lane);
#pragma unroll
        for (int it = 0; it < LPT; ++it) {
            pr.c[it] = cp[it * 64];
            pr.m[it] = pv.meta[(base + tok_w + it * TPW) * ng + meta_col];
        }
    };
    auto consume_page = [&](const PageRegs<LPT> &pr, int pg) {
#pragma unroll
        for (int it = 0; it < LPT; ++it) {
            const int idx = pg * kPage + tok_w + it * TPW;
            const uint32_t m = idx < n_tok ? pr.m[it] : 0u;    // never let an unwritten slot's bits reach the FMAs
            const float sc = __half2float(__ushort_as_half((unsigned short)(m & 0xFFFFu)));
            const float zp = __half2float(__ushort_as_half((unsigned short)(m >> 16)));
            float wlo[RQ], whi[RQ];
#pragma unroll
            for (int q = 0; q < RQ; ++q) {
                const float p = p_s[q][idx];
                wlo[q] = p * sc;
                whi[q] = wlo[q] * 0.0625f;                    // high nibbles are converted as 16*code
                zs[q] = fmaf(p, zp, zs[q]);
            }
            const uint32_t x[4] = {pr.c[it].x, pr.c[it].y, pr.c[it].z, pr.c[it].w};
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) {
                const uint32_t lo = x[dw] & 0x0F0F0F0Fu, hi = x[dw] & 0xF0F0F0F0u;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float flo = (float)((lo >> (8 * k)) & 0xFFu);
                    const float fhi = (float)((hi >> (8 * k)) & 0xFFu);
#pragma unroll
                    for (int q = 0; q < RQ; ++q) {
                        acc[q][8 * dw + 2 * k] = fmaf(wlo[q], flo, acc[q][8 * dw + 2 * k]);
                        acc[q][8 * dw + 2 * k + 1] = fmaf(whi[q], fhi, acc[q][8 * dw + 2 * k + 1]);
                    }
                }
            }
        }
    };

    {
        PageRegs<LPT> A, B;
        load_page(A, 0);
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

    // ---------------- Epilogue ----------------
#pragma unroll
    for (int q = 0; q < RQ; ++q) {
#pragma unroll
        for (int i = 0; i < 32; ++i) acc[q][i] = slot_sum<LPT>(acc[q][i]);
        zs[q] = slot_sum<LPT>(zs[q]);
    }
    if (lane < LPT) {
#pragma unroll
        for (int q = 0; q < RQ; ++q) {
#pragma unroll
            for (int i = 0; i < 32; ++i) wave_o[wave][q][lane * 32 + i] = acc[q][i];
            wave_z[wave][q][lane] = zs[q];
        }
    }
    __syncthreads();
    const size_t part = ((size_t)seq_g * pv.n_q_heads + qh0) * a.n_splits + blockIdx.x;
    for (int e = tid; e < RQ * D; e += kThreads) {
        const int q = e / D, c = e % D;
        float o = 0.0f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) o += wave_o[w][q][c] + wave_z[w][q][c / 32];
        a.part_o[(part + (size_t)q * a.n_splits) * D + c] = o;
    }
    if (tid < RQ) {
        float *ml = a.part_ml + (part + (size_t)tid * a.n_splits) * 2;
        ml[0] = __int_as_float(hmin[tid]);
        ml[1] = red_f[tid][0] + red_f[tid][1] + red_f[tid][2] + red_f[tid][3];
    }
}

// out = sum_s e^{(alpha_s - alpha_max)/tau} o_s / sum_s e^{(alpha_s - alpha_max)/tau} l_s over the chunks of one head.
__global__ void merge_kernel(DecodeArgs a, BatchDesc desc, int seq0) {
    const int D = a.pool.head_dim;
    const int qh = blockIdx.x, seq_g = seq0 + blockIdx.y;
    const int ctx = desc.s[blockIdx.y].pos;
    const int n = (ctx + a.chunk - 1) / a.chunk;
    const size_t part = ((size_t)seq_g * a.pool.n_q_heads + qh) * a.n_splits;
    const int c = threadIdx.x;
    float *out = a.out + ((size_t)seq_g * a.pool.n_q_heads + qh) * D;
    if (n == 0) {
        out[c] = 0.0f;
        return;
    }
    int hmin = 1 << 20;
    for (int s = 0; s < n; ++s) hmin = min(hmin, __float_as_int(a.part_ml[(part + s) * 2]));
    float l = 0.0f, o = 0.0f;
    for (int s = 0; s < n; ++s) {
        const float w = exp2f(a.exp2_scale * (float)(hmin - __float_as_int(a.part_ml[(part + s) * 2])));
        l = fmaf(w, a.part_ml[(part + s) * 2 + 1], l);
        o = fmaf(w, a.part_o[(part + s) * D + c], o);
    }
    out[c] = o / l;
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
    hipLaunchKernelGGL(merge_kernel, dim3((unsigned)a.pool.n_q_heads, (unsigned)n_seqs), dim3((unsigned)a.pool.head_dim), 0, st, a, desc, seq0);
    return hipGetLastError();
}

hipError_t launch_qsketch(const DecodeArgs &a, int seq0, int n_seqs, hipStream_t st) {
    const dim3 grid((unsigned)(n_seqs * a.pool.n_q_heads)), block((unsigned)a.pool.sketch_bits);
    if (a.f16) hipLaunchKernelGGL((qsketch_kernel<__half>), grid, block, 0, st, a, seq0);
    else hipLaunchKernelGGL((qsketch_kernel<float>), grid, block, 0, st, a, seq0);
    return hipGetLastError();
}

}  // namespace h1bkv
