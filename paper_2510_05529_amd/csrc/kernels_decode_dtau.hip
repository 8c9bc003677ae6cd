// Decode-step attention together with its derivative with respect to the softmax temperature tau -- the one scalar
// that the finetuning stage trains next to V_proj (Sec. IV-C, Eq.(5)):
//   out = sum_t p_t v^_t / l,   p_t = exp(alpha_t / tau),  l = sum_t p_t,
//   d out / d tau = -(1/tau^2) ( sum_t p_t alpha_t v^_t / l - (sum_t p_t alpha_t / l) out ).
// With alpha = 1 - 2 ham / b (Eq.(3)) this is  (2 / (b tau^2)) ( oh / l - (lh / l) out )  for the distance-weighted
// sums  lh = sum p e,  oh = sum p e v^,  where e = ham - ham_min >= 0 (a constant shift of e leaves the bracket
// unchanged).  Counting e from the running minimum keeps lh and oh small next to l and o -- the tokens that carry
// weight have small e -- which is what the covariance in the bracket needs in fp32.
//
// The three split kernels (vector-ALU, matrix-core, fp16-value) carry, with their DTAU flag, a second set of sums whose
// weight is p e instead of p.  When a page lowers the running minimum by k, every e grows by k:  lh += k l,  oh += k o,
// then the usual rescale.  merge_dtau_kernel, here, merges the chunk partials the same way and applies the formula above.
#include "decode_common.h"

namespace h1bkv {

namespace {

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
#pragma unroll 8
    for (int s = 0; s < n; ++s) hmin = min(hmin, __float_as_int(a.part_ml[(part + s) * 4]));
    float l = 0.0f, lh = 0.0f, o = 0.0f, oh = 0.0f;
    // (unrolled: the loads of several chunks are in flight together -- a long context has dozens of chunks, and one
    // round trip per chunk was three times the plain merge's time)
#pragma unroll 8
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

}  // namespace

hipError_t launch_merge_dtau(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, float dtau_scale, hipStream_t st) {
    hipLaunchKernelGGL(merge_dtau_kernel, dim3((unsigned)a.pool.n_q_heads, (unsigned)n_seqs), dim3((unsigned)a.pool.head_dim), 0, st, a,
                       desc, seq0, dtau_scale);
    return hipGetLastError();
}

}  // namespace h1bkv
