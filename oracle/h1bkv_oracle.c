/*
 * H1B-KV CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct implementation of what the H1B-KV hot path computes, written
 * from the paper (arxiv 2510.05529).  It exists so that the HIP library can be checked element by
 * element against something that shares no code with it.  Only the tests, the smoke check and the
 * benchmark's cpu-baseline leg may load it; the product never does.
 *
 * What it follows:
 *   Eq.(2)  Sec. IV-A   key sketch      s_k = sign(R k), stored as b bits
 *   Eq.(3)  Sec. IV-A   binary score    alpha_t = (1/b) s_t^T s_q
 *   Eq.(4)  Sec. IV-B   4-bit affine value quantisation with a scale and a zero point
 *   Eq.(5)  Sec. IV-C   out = softmax(alpha / tau) V_dequant
 *
 * Readings of what the paper leaves open (each one is also what the HIP path implements):
 *   - sign(0) = +1: bit i is 1 iff y_i >= 0 (so -0.0 gives 1 and NaN gives 0).
 *   - Floating point decides integers here (sketch bits, int4 codes), so those decisions are taken
 *     in fp32 with a fixed operation order: y_i = fma(R[i][j], k[j], y_i) for j = 0..d-1 from +0.0f;
 *     the quantiser is the fp32 sequence sub, IEEE divide, round-half-even written out below.
 *     Everything that stays floating point (scores, softmax, weighted sum) is done in fp64.
 *   - One R for all heads; bit i goes to word i/64, bit position i%64 (LSB first).
 *   - Quantisation is per group of G consecutive channels of one value vector, min-anchored:
 *     zero = fp16(min), scale = fp16((max-min)/15), code = clamp(rne((v-zero)/scale), 0, 15),
 *     dequant = scale*code + zero.  This is Eq.(4) with the real-valued zero point -min/scale
 *     moved inside the rounding, which is what keeps the round-trip error within scale/2.
 *   - Channel 2m is the low nibble and channel 2m+1 the high nibble of byte m.
 *   - A group whose fp16 scale is 0 stores codes 0 (dequantises to zero).
 *   - Attention is over every cached token, no mask; query head h reads KV head h / (H_q/H_kv).
 *
 * Parity pins (tests/test_oracle_*.py): brute-force +-1 dot products, the identity
 * <s_q,s_k> = b - 2 popcount(s_q xor s_k), Prop. 1's expectation 1 - 2 theta/pi, round-trip error
 * <= scale/2, closed forms of Eq.(5) (T=1, equal sketches, tau -> inf, two-level), exact rational
 * arithmetic on tiny cases, and numpy's float16 for the half conversions.  The fp16-value variant at the end
 * of the file is pinned by tests/test_oracle_f16v.py (numpy float16 storage, closed forms, agreement with the
 * 4-bit functions on values both formats hold exactly, the explicit +-1 rendering); prefill attention by
 * tests/test_oracle_prefill.py (per-prefix decode steps, causality, the explicit causal +-1 rendering); the
 * temperature derivative by tests/test_oracle_dtau.py (central differences of the float64 rendering, a two-level
 * closed form, the large-tau covariance limit, cases where it must vanish).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------- IEEE binary16 <-> binary32, written out (no hardware or compiler half type) ---------- */

float h1bkv_oracle_half_to_float(uint16_t h) {
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t exp = (h >> 10) & 0x1Fu;
    uint32_t man = h & 0x3FFu;
    uint32_t bits;
    if (exp == 0) {
        if (man == 0) {
            bits = sign;                                   /* +-0 */
        } else {                                           /* subnormal: value = man * 2^-24 */
            float v = (float)man * 5.9604644775390625e-08f; /* exact: man < 2^10, 2^-24 a power of two */
            memcpy(&bits, &v, 4);
            bits |= sign;
        }
    } else if (exp == 31) {
        bits = sign | 0x7F800000u | (man << 13);           /* inf / nan */
    } else {
        bits = sign | ((exp + 112u) << 23) | (man << 13);  /* rebias 15 -> 127 */
    }
    float f;
    memcpy(&f, &bits, 4);
    return f;
}

uint16_t h1bkv_oracle_float_to_half(float f) {              /* round to nearest, ties to even */
    uint32_t x;
    memcpy(&x, &f, 4);
    uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
    uint32_t ax = x & 0x7FFFFFFFu;
    if (ax >= 0x7F800000u)                                 /* inf or nan */
        return (uint16_t)(sign | 0x7C00u | ((ax > 0x7F800000u) ? 0x200u : 0u));
    if (ax >= 0x477FF000u)                                 /* >= 65520 rounds to inf */
        return (uint16_t)(sign | 0x7C00u);
    if (ax <= 0x33000000u)                                 /* <= 2^-25 rounds to 0 (2^-25 itself ties to even) */
        return sign;
    int e = (int)(ax >> 23) - 127;                         /* unbiased exponent, -25 .. 15 */
    uint32_t m = (ax & 0x7FFFFFu) | 0x800000u;             /* 24-bit significand */
    int shift = (e < -14) ? (13 + (-14 - e)) : 13;         /* bits to drop (subnormal results drop more) */
    uint32_t kept = m >> shift;
    uint32_t rem = m & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (kept & 1u))) kept++;
    uint32_t out;
    if (e < -14) out = kept;                               /* subnormal (a carry to 0x400 is the smallest normal) */
    else out = ((uint32_t)(e + 15) << 10) + (kept - 0x400u); /* carry out of the mantissa bumps the exponent */
    return (uint16_t)(sign | out);
}

/* ---------- Eq.(2): sketch n vectors x[n][d] with R[b][d]; out[n][b/64] ---------- */

static void sketch_one(const float *R, int b, int d, const float *k, uint64_t *s) {
    for (int w = 0; w < b / 64; ++w) s[w] = 0;
    for (int i = 0; i < b; ++i) {
        float y = 0.0f;
        for (int j = 0; j < d; ++j) y = fmaf(R[(int64_t)i * d + j], k[j], y);
        if (y >= 0.0f) s[i / 64] |= (uint64_t)1 << (i % 64);
    }
}

void h1bkv_oracle_sketch(const float *R, int b, int d, const float *x, int64_t n, uint64_t *out) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n; ++r) sketch_one(R, b, d, x + r * d, out + r * (b / 64));
}

/* ---------- Eq.(4): quantise n vectors v[n][d] in groups of G channels ---------- */

static void quantize_one(const float *x, int d, int G, uint8_t *c, uint16_t *scale, uint16_t *zero) {
    int ng = d / G;
    for (int m = 0; m < d / 2; ++m) c[m] = 0;
    for (int g = 0; g < ng; ++g) {
        float mn = x[g * G], mx = x[g * G];
        for (int j = 1; j < G; ++j) {
            float e = x[g * G + j];
            if (e < mn) mn = e;
            if (e > mx) mx = e;
        }
        float delta = (mx - mn) / 15.0f;
        uint16_t sh = h1bkv_oracle_float_to_half(delta);
        uint16_t zh = h1bkv_oracle_float_to_half(mn);
        if ((zh & 0x7FFFu) == 0) zh = 0;                   /* a zero minimum is stored as +0 */
        scale[g] = sh;
        zero[g] = zh;
        float sc = h1bkv_oracle_half_to_float(sh);
        float zp = h1bkv_oracle_half_to_float(zh);
        for (int j = 0; j < G; ++j) {
            int ch = g * G + j;
            int q = 0;
            if (sc != 0.0f) {
                float t = rintf((x[ch] - zp) / sc);         /* default rounding mode: half to even */
                if (t < 0.0f) t = 0.0f;
                if (t > 15.0f) t = 15.0f;
                q = (int)t;
            }
            c[ch / 2] |= (uint8_t)(q << (4 * (ch & 1)));
        }
    }
}

void h1bkv_oracle_quantize(const float *v, int64_t n, int d, int G,
                           uint8_t *codes /*[n][d/2]*/, uint16_t *scale /*[n][d/G]*/, uint16_t *zero /*[n][d/G]*/) {
    int ng = d / G;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n; ++r)
        quantize_one(v + r * d, d, G, codes + r * (d / 2), scale + r * ng, zero + r * ng);
}

/* dequantised values scale*code + zero as fp64 (exact: fp16 scale times a 4-bit code plus an fp16 zero) */
void h1bkv_oracle_dequantize(const uint8_t *codes, const uint16_t *scale, const uint16_t *zero,
                             int64_t n, int d, int G, double *out /*[n][d]*/) {
    int ng = d / G;
    for (int64_t r = 0; r < n; ++r)
        for (int ch = 0; ch < d; ++ch) {
            int q = (codes[r * (d / 2) + ch / 2] >> (4 * (ch & 1))) & 0xF;
            double sc = (double)h1bkv_oracle_half_to_float(scale[r * ng + ch / G]);
            double zp = (double)h1bkv_oracle_half_to_float(zero[r * ng + ch / G]);
            out[r * d + ch] = sc * (double)q + zp;
        }
}

/* ---------- Eq.(3): Hamming distances of one query sketch against T cached sketches ---------- */

void h1bkv_oracle_hamming(const uint64_t *sq, const uint64_t *sk /*[T][W]*/, int64_t T, int W, int32_t *ham) {
    for (int64_t t = 0; t < T; ++t) {
        int h = 0;
        for (int w = 0; w < W; ++w) h += __builtin_popcountll(sq[w] ^ sk[t * W + w]);
        ham[t] = h;
    }
}

/* ---------- Eq.(3)+(5) for one (sequence, query head): out[d] ---------- */

void h1bkv_oracle_decode_one(const uint64_t *sq /*[W]*/, const uint64_t *sk /*[T][W]*/,
                             const uint8_t *codes /*[T][d/2]*/, const uint16_t *scale /*[T][d/G]*/,
                             const uint16_t *zero /*[T][d/G]*/, int64_t T, int b, int d, int G, double tau,
                             float *out /*[d]*/) {
    int W = b / 64, ng = d / G;
    double acc[1024];
    for (int c = 0; c < d; ++c) acc[c] = 0.0;
    if (T <= 0) {
        for (int c = 0; c < d; ++c) out[c] = 0.0f;
        return;
    }
    /* alpha_t = (b - 2 ham_t) / b ; m = max_t alpha_t */
    double m = -2.0;
    for (int64_t t = 0; t < T; ++t) {
        int h = 0;
        for (int w = 0; w < W; ++w) h += __builtin_popcountll(sq[w] ^ sk[t * W + w]);
        double alpha = (double)(b - 2 * h) / (double)b;
        if (alpha > m) m = alpha;
    }
    double l = 0.0;
    for (int64_t t = 0; t < T; ++t) {
        int h = 0;
        for (int w = 0; w < W; ++w) h += __builtin_popcountll(sq[w] ^ sk[t * W + w]);
        double alpha = (double)(b - 2 * h) / (double)b;
        double p = exp((alpha - m) / tau);
        l += p;
        for (int c = 0; c < d; ++c) {
            int q = (codes[t * (d / 2) + c / 2] >> (4 * (c & 1))) & 0xF;
            double sc = (double)h1bkv_oracle_half_to_float(scale[t * ng + c / G]);
            double zp = (double)h1bkv_oracle_half_to_float(zero[t * ng + c / G]);
            acc[c] += p * (sc * (double)q + zp);
        }
    }
    for (int c = 0; c < d; ++c) out[c] = (float)(acc[c] / l);
}

/*
 * Eq.(5) and its derivative with respect to the temperature, the one scalar the finetuning stage trains next to
 * V_proj (Sec. IV-C):  with p_t = exp(alpha_t / tau), l = sum p_t, out = sum p_t v_t / l,
 *   d out / d tau = -(1 / tau^2) ( sum p_t alpha_t v_t / l  -  (sum p_t alpha_t / l) out ),
 * i.e. minus the softmax-weighted covariance of the scores with the values, over tau^2.  Same inputs as
 * h1bkv_oracle_decode_one; dout [d] is zero for T <= 1.
 */
void h1bkv_oracle_decode_one_dtau(const uint64_t *sq, const uint64_t *sk, const uint8_t *codes, const uint16_t *scale,
                                  const uint16_t *zero, int64_t T, int b, int d, int G, double tau, float *out,
                                  float *dout) {
    int W = b / 64, ng = d / G;
    double acc[1024], acca[1024];
    for (int c = 0; c < d; ++c) acc[c] = acca[c] = 0.0;
    if (T <= 0) {
        for (int c = 0; c < d; ++c) out[c] = dout[c] = 0.0f;
        return;
    }
    double m = -2.0;
    for (int64_t t = 0; t < T; ++t) {
        int h = 0;
        for (int w = 0; w < W; ++w) h += __builtin_popcountll(sq[w] ^ sk[t * W + w]);
        double alpha = (double)(b - 2 * h) / (double)b;
        if (alpha > m) m = alpha;
    }
    double l = 0.0, la = 0.0;
    for (int64_t t = 0; t < T; ++t) {
        int h = 0;
        for (int w = 0; w < W; ++w) h += __builtin_popcountll(sq[w] ^ sk[t * W + w]);
        double alpha = (double)(b - 2 * h) / (double)b;
        double p = exp((alpha - m) / tau);
        l += p;
        la += p * alpha;
        for (int c = 0; c < d; ++c) {
            int q = (codes[t * (d / 2) + c / 2] >> (4 * (c & 1))) & 0xF;
            double sc = (double)h1bkv_oracle_half_to_float(scale[t * ng + c / G]);
            double zp = (double)h1bkv_oracle_half_to_float(zero[t * ng + c / G]);
            double v = sc * (double)q + zp;
            acc[c] += p * v;
            acca[c] += p * alpha * v;
        }
    }
    for (int c = 0; c < d; ++c) {
        double o = acc[c] / l;
        out[c] = (float)o;
        dout[c] = (float)(-(acca[c] / l - (la / l) * o) / (tau * tau));
    }
}

void h1bkv_oracle_decode_batch_dtau(const float *R, int b, int d, int G, int B, int Hq, int Hkv, int64_t Tcap,
                                    const int32_t *ctx_len, const float *q, const uint64_t *sketches,
                                    const uint8_t *codes, const uint16_t *scale, const uint16_t *zero, double tau,
                                    float *out, float *dout) {
    int W = b / 64, ng = d / G, r = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
    for (int s = 0; s < B; ++s)
        for (int h = 0; h < Hq; ++h) {
            uint64_t sq[16];
            sketch_one(R, b, d, q + ((int64_t)s * Hq + h) * d, sq);
            int64_t base = ((int64_t)s * Hkv + h / r) * Tcap;
            int64_t o = ((int64_t)s * Hq + h) * d;
            h1bkv_oracle_decode_one_dtau(sq, sketches + base * W, codes + base * (d / 2), scale + base * ng,
                                         zero + base * ng, ctx_len[s], b, d, G, tau, out + o, dout + o);
        }
}

/*
 * One decode step over a whole batch held in canonical layout:
 *   sketches [B][H_kv][Tcap][W], codes [B][H_kv][Tcap][d/2], scale/zero [B][H_kv][Tcap][d/G],
 *   q [B][H_q][d] (fp32 values), ctx_len[B] <= Tcap, out [B][H_q][d].
 * The query is sketched with the same recipe as the keys; query head h reads KV head h / (H_q/H_kv).
 */
void h1bkv_oracle_decode_batch(const float *R, int b, int d, int G, int B, int Hq, int Hkv, int64_t Tcap,
                               const int32_t *ctx_len, const float *q, const uint64_t *sketches,
                               const uint8_t *codes, const uint16_t *scale, const uint16_t *zero, double tau,
                               float *out) {
    int W = b / 64, ng = d / G, r = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
    for (int s = 0; s < B; ++s)
        for (int h = 0; h < Hq; ++h) {
            uint64_t sq[16];
            sketch_one(R, b, d, q + ((int64_t)s * Hq + h) * d, sq);
            int64_t base = ((int64_t)s * Hkv + h / r) * Tcap;
            h1bkv_oracle_decode_one(sq, sketches + base * W, codes + base * (d / 2), scale + base * ng,
                                    zero + base * ng, ctx_len[s], b, d, G, tau, out + ((int64_t)s * Hq + h) * d);
        }
}

/*
 * Prefill attention (Eq.(3) + Eq.(5) applied to every position of a prompt chunk): the last n_q cached positions
 * of each sequence are the queries; query i of sequence s (absolute position ctx_len[s] - n_q + i) attends to the
 * cached tokens up to and including its own position, i.e. to the first ctx_len[s] - n_q + i + 1 tokens -- the
 * decode step it would have seen had the prompt been fed one token at a time.
 *   q [B][n_q][H_q][d] (fp32 values), out [B][n_q][H_q][d]; planes as in h1bkv_oracle_decode_batch.
 */
void h1bkv_oracle_prefill_batch(const float *R, int b, int d, int G, int B, int Hq, int Hkv, int64_t Tcap,
                                const int32_t *ctx_len, int64_t n_q, const float *q, const uint64_t *sketches,
                                const uint8_t *codes, const uint16_t *scale, const uint16_t *zero, double tau,
                                float *out) {
    int W = b / 64, ng = d / G, r = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 4) collapse(3)
    for (int s = 0; s < B; ++s)
        for (int64_t i = 0; i < n_q; ++i)
            for (int h = 0; h < Hq; ++h) {
                uint64_t sq[16];
                int64_t vec = ((int64_t)s * n_q + i) * Hq + h;
                sketch_one(R, b, d, q + vec * d, sq);
                int64_t base = ((int64_t)s * Hkv + h / r) * Tcap;
                int64_t visible = (int64_t)ctx_len[s] - n_q + i + 1;
                h1bkv_oracle_decode_one(sq, sketches + base * W, codes + base * (d / 2), scale + base * ng,
                                        zero + base * ng, visible, b, d, G, tau, out + vec * d);
            }
}

/*
 * Cache append for a batch in boundary layout k, v [B][n_new][H_kv][d] (fp32 values) into canonical
 * planes at token positions [t0, t0+n_new): sketches [B][H_kv][Tcap][W] etc.
 */
void h1bkv_oracle_append_batch(const float *R, int b, int d, int G, int B, int Hkv, int64_t Tcap, int64_t t0,
                               int64_t n_new, const float *k, const float *v, uint64_t *sketches,
                               uint8_t *codes, uint16_t *scale, uint16_t *zero) {
    int W = b / 64, ng = d / G;
#pragma omp parallel for schedule(dynamic, 16) collapse(3)
    for (int s = 0; s < B; ++s)
        for (int h = 0; h < Hkv; ++h)
            for (int64_t t = 0; t < n_new; ++t) {
                int64_t src = (((int64_t)s * n_new + t) * Hkv + h) * d;
                int64_t dst = ((int64_t)s * Hkv + h) * Tcap + t0 + t;
                sketch_one(R, b, d, k + src, sketches + dst * W);
                quantize_one(v + src, d, G, codes + dst * (d / 2), scale + dst * ng, zero + dst * ng);
            }
}

/*
 * ---------- "1-bit key only" variant (Table V ablation, Sec. VI-E): sketched keys, fp16 values ----------
 * Keys and scores are exactly as above (Eq.(2), Eq.(3)); values skip Eq.(4) and are kept as IEEE binary16
 * numbers (the paper's FP16 value storage), so Eq.(5) reads  out = softmax(alpha / tau) fp16(V).
 * A stored value is the input rounded to nearest-even binary16 (unchanged if the input already is fp16).
 */
void h1bkv_oracle_decode_one_f16v(const uint64_t *sq /*[W]*/, const uint64_t *sk /*[T][W]*/,
                                  const uint16_t *v16 /*[T][d] fp16 bit patterns*/, int64_t T, int b, int d,
                                  double tau, float *out /*[d]*/) {
    int W = b / 64;
    double acc[1024];
    for (int c = 0; c < d; ++c) acc[c] = 0.0;
    if (T <= 0) {
        for (int c = 0; c < d; ++c) out[c] = 0.0f;
        return;
    }
    double m = -2.0;
    for (int64_t t = 0; t < T; ++t) {
        int h = 0;
        for (int w = 0; w < W; ++w) h += __builtin_popcountll(sq[w] ^ sk[t * W + w]);
        double alpha = (double)(b - 2 * h) / (double)b;
        if (alpha > m) m = alpha;
    }
    double l = 0.0;
    for (int64_t t = 0; t < T; ++t) {
        int h = 0;
        for (int w = 0; w < W; ++w) h += __builtin_popcountll(sq[w] ^ sk[t * W + w]);
        double alpha = (double)(b - 2 * h) / (double)b;
        double p = exp((alpha - m) / tau);
        l += p;
        for (int c = 0; c < d; ++c) acc[c] += p * (double)h1bkv_oracle_half_to_float(v16[t * d + c]);
    }
    for (int c = 0; c < d; ++c) out[c] = (float)(acc[c] / l);
}

/*
 * The same with the temperature derivative (Sec. IV-C, Eq.(5); see h1bkv_oracle_decode_one_dtau):
 *   d out / d tau = -(1 / tau^2) ( sum p_t alpha_t v_t / l  -  (sum p_t alpha_t / l) out ),  v_t the stored fp16 value.
 */
void h1bkv_oracle_decode_one_dtau_f16v(const uint64_t *sq, const uint64_t *sk, const uint16_t *v16, int64_t T, int b,
                                       int d, double tau, float *out, float *dout) {
    int W = b / 64;
    double acc[1024], acca[1024];
    for (int c = 0; c < d; ++c) acc[c] = acca[c] = 0.0;
    if (T <= 0) {
        for (int c = 0; c < d; ++c) out[c] = dout[c] = 0.0f;
        return;
    }
    double m = -2.0;
    for (int64_t t = 0; t < T; ++t) {
        int h = 0;
        for (int w = 0; w < W; ++w) h += __builtin_popcountll(sq[w] ^ sk[t * W + w]);
        double alpha = (double)(b - 2 * h) / (double)b;
        if (alpha > m) m = alpha;
    }
    double l = 0.0, la = 0.0;
    for (int64_t t = 0; t < T; ++t) {
        int h = 0;
        for (int w = 0; w < W; ++w) h += __builtin_popcountll(sq[w] ^ sk[t * W + w]);
        double alpha = (double)(b - 2 * h) / (double)b;
        double p = exp((alpha - m) / tau);
        l += p;
        la += p * alpha;
        for (int c = 0; c < d; ++c) {
            double v = (double)h1bkv_oracle_half_to_float(v16[t * d + c]);
            acc[c] += p * v;
            acca[c] += p * alpha * v;
        }
    }
    for (int c = 0; c < d; ++c) {
        double o = acc[c] / l;
        out[c] = (float)o;
        dout[c] = (float)(-(acca[c] / l - (la / l) * o) / (tau * tau));
    }
}

void h1bkv_oracle_decode_batch_dtau_f16v(const float *R, int b, int d, int B, int Hq, int Hkv, int64_t Tcap,
                                         const int32_t *ctx_len, const float *q, const uint64_t *sketches,
                                         const uint16_t *v16, double tau, float *out, float *dout) {
    int W = b / 64, r = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
    for (int s = 0; s < B; ++s)
        for (int h = 0; h < Hq; ++h) {
            uint64_t sq[16];
            sketch_one(R, b, d, q + ((int64_t)s * Hq + h) * d, sq);
            int64_t base = ((int64_t)s * Hkv + h / r) * Tcap;
            int64_t o = ((int64_t)s * Hq + h) * d;
            h1bkv_oracle_decode_one_dtau_f16v(sq, sketches + base * W, v16 + base * d, ctx_len[s], b, d, tau, out + o,
                                              dout + o);
        }
}

/* Batch forms in canonical layout: sketches [B][H_kv][Tcap][W], values [B][H_kv][Tcap][d] fp16 bit patterns. */
void h1bkv_oracle_decode_batch_f16v(const float *R, int b, int d, int B, int Hq, int Hkv, int64_t Tcap,
                                    const int32_t *ctx_len, const float *q, const uint64_t *sketches,
                                    const uint16_t *v16, double tau, float *out) {
    int W = b / 64, r = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
    for (int s = 0; s < B; ++s)
        for (int h = 0; h < Hq; ++h) {
            uint64_t sq[16];
            sketch_one(R, b, d, q + ((int64_t)s * Hq + h) * d, sq);
            int64_t base = ((int64_t)s * Hkv + h / r) * Tcap;
            h1bkv_oracle_decode_one_f16v(sq, sketches + base * W, v16 + base * d, ctx_len[s], b, d, tau,
                                         out + ((int64_t)s * Hq + h) * d);
        }
}

void h1bkv_oracle_append_batch_f16v(const float *R, int b, int d, int B, int Hkv, int64_t Tcap, int64_t t0,
                                    int64_t n_new, const float *k, const float *v, uint64_t *sketches,
                                    uint16_t *v16) {
    int W = b / 64;
#pragma omp parallel for schedule(dynamic, 16) collapse(3)
    for (int s = 0; s < B; ++s)
        for (int h = 0; h < Hkv; ++h)
            for (int64_t t = 0; t < n_new; ++t) {
                int64_t src = (((int64_t)s * n_new + t) * Hkv + h) * d;
                int64_t dst = ((int64_t)s * Hkv + h) * Tcap + t0 + t;
                sketch_one(R, b, d, k + src, sketches + dst * W);
                for (int c = 0; c < d; ++c) v16[dst * d + c] = h1bkv_oracle_float_to_half(v[src + c]);
            }
}

int h1bkv_oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
