/*
 * h1bkv.h -- C ABI of the MI355X (gfx950) H1B-KV library: decode-step attention over a hybrid
 * compressed KV cache (keys = packed 1-bit random-projection sketches, values = 4-bit
 * group-quantised codes), and the cache-append step that produces it (arxiv 2510.05529, Sec. IV).
 *
 * Conventions that hold for every entry point
 *   - Return value: H1BKV_OK (0) or a negative H1BKV_E* code; nothing throws, aborts or prints.
 *   - "dev" pointers are device (HIP global memory) addresses on the handle's device; "host" pointers
 *     are ordinary host memory.  The caller owns every buffer it passes (pool, Q/K/V, out, workspace)
 *     and the stream; the library owns only the host-side handle and its page bookkeeping.
 *   - All arguments are validated on the host before any device work; a call that returns an error
 *     has changed neither the cache contents nor the bookkeeping.
 *   - h1bkv_append_kv and h1bkv_decode_attn only enqueue kernels on `hip_stream` (a hipStream_t, NULL
 *     for the default stream) and return without synchronising.  All calls on one handle must be
 *     ordered by the caller (one stream, or explicit dependencies) and made from one thread at a time.
 *   - The calling thread's current HIP device must be the handle's device.
 *   - Layouts are row-major with the last index fastest.  Notation: b = sketch_bits, W = b/64,
 *     d = head_dim, G = group_size, n_g = d/G, r = n_q_heads / n_kv_heads.
 */
#ifndef H1BKV_H
#define H1BKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct h1bkv_cache h1bkv_cache; /* opaque host-side handle */

enum { H1BKV_F32 = 0, H1BKV_F16 = 1 };  /* dtype of Q, K, V at the boundary */

enum {
    H1BKV_OK = 0,
    H1BKV_EINVAL = -1,     /* an argument value is not allowed (bad dtype, tau <= 0, duplicate seq id ...) */
    H1BKV_ENULL = -2,      /* a required pointer is NULL */
    H1BKV_ESHAPE = -3,     /* a shape/config constraint is violated (see h1bkv_config) */
    H1BKV_ENOSPACE = -4,   /* page pool exhausted, or a sequence would exceed max_pages_per_seq */
    H1BKV_ERANGE = -5,     /* sequence id / head / token range out of bounds */
    H1BKV_EWORKSPACE = -6, /* workspace or pool smaller than required */
    H1BKV_EHIP = -7,       /* a HIP runtime call failed (launch, copy, wrong current device) */
    H1BKV_ENODEVICE = -8   /* the handle is bookkeeping-only (device == H1BKV_DEVICE_NONE) and the call needs a GPU */
};

#define H1BKV_DEVICE_NONE (-1)
#define H1BKV_PAGE_TOKENS 256

/*
 * Cache geometry.  Constraints (violations give H1BKV_ESHAPE):
 *   n_kv_heads >= 1, n_q_heads a multiple of n_kv_heads (query head h reads KV head h / r);
 *   head_dim in {64, 128, 256};  sketch_bits in {64, 128, 256, 512} (the paper's ablation puts the
 *   useful lower bound at b = 64, Sec. VI-E/F);  group_size in {32, 64, 128} and dividing head_dim;
 *   in_dtype H1BKV_F32 or H1BKV_F16;  page_tokens 0 (= default) or H1BKV_PAGE_TOKENS;
 *   max_seqs, max_pages, max_pages_per_seq >= 1;
 *   value_bits 0 or 4 (= the method: 4-bit group-quantised values, Eq.(4)) or 16 (the "1-bit key only" ablation of
 *   Table V / Sec. VI-E: keys are sketches, values are kept as fp16; group_size is then unused but still checked).
 * device: HIP device ordinal, or H1BKV_DEVICE_NONE for a bookkeeping-only handle that runs all
 * validation and page accounting but never touches a GPU (capacity planning, host-side tests).
 */
typedef struct {
    int32_t n_q_heads, n_kv_heads, head_dim;
    int32_t sketch_bits;
    int32_t group_size;
    int32_t in_dtype;
    int32_t page_tokens;
    int32_t max_seqs, max_pages, max_pages_per_seq;
    int32_t device;
    int32_t value_bits;
    uint64_t seed;          /* used only when h1bkv_create is given no projection: seed of the library's own draw */
} h1bkv_config;

/* Library version, major*10000 + minor*100 + patch. */
int h1bkv_version(void);

/* Static description of an error code (never NULL). */
const char *h1bkv_strerror(int code);

/*
 * Device bytes the caller must provide as the pool for this geometry (0 if cfg is NULL or invalid).
 * The pool holds R, its transpose and its fp16 pieces, the block table, and three planes per page:
 * sketches [page][H_kv][256][W] u64 (Eq.(2)), codes [page][H_kv][256][d/2] u8 and
 * {fp16 scale, fp16 zero} pairs [page][H_kv][256][n_g] (Eq.(4)).  With value_bits = 16 the last two planes are
 * replaced by one plane of fp16 values [page][H_kv][256][d].
 */
size_t h1bkv_pool_bytes(const h1bkv_config *cfg);

/*
 * Create a handle over `pool_dev` (pool_bytes >= h1bkv_pool_bytes(cfg), 256-byte aligned; ignored and
 * may be NULL for a bookkeeping-only handle).  R_host [b][d] fp32 is the fixed Gaussian projection of
 * Eq.(2) (Sec. III: R_ij ~ N(0,1), drawn once, shared by keys and queries of every head); it is
 * copied to the device here, synchronously.  All sequences start empty, all pages free.
 * R_host == NULL: the library draws R itself from cfg->seed -- a splitmix64 stream (state += 0x9E3779B97F4A7C15, then
 * the two xor-shift-multiply rounds with 0xBF58476D1CE4E5B9 and 0x94D049BB133111EB and a final xor-shift by 31), a
 * uniform u = ((x >> 11) + 0.5) 2^-53 per draw, and per pair of consecutive elements (2p, 2p+1) of the row-major
 * array two draws u1, u2 giving sqrt(-2 ln u1) cos(2 pi u2) and sqrt(-2 ln u1) sin(2 pi u2), computed in double and
 * rounded to fp32.  The values depend on the host's libm in the last place; read what was drawn with
 * h1bkv_get_projection.
 */
int h1bkv_create(const h1bkv_config *cfg, void *pool_dev, size_t pool_bytes, const float *R_host,
                 h1bkv_cache **out);

/* Free the host handle.  The pool stays the caller's.  NULL is accepted. */
int h1bkv_destroy(h1bkv_cache *c);

/* Copy R [b][d] back to host memory (from the handle's host copy). */
int h1bkv_get_projection(const h1bkv_cache *c, float *R_host_out);

/* Bookkeeping (host only, no device work). */
int h1bkv_seq_len(const h1bkv_cache *c, int32_t seq_id, int32_t *len_out);
int h1bkv_free_pages(const h1bkv_cache *c, int32_t *n_out);
int h1bkv_reset_seq(h1bkv_cache *c, int32_t seq_id);                      /* length 0, pages returned */
int h1bkv_truncate_seq(h1bkv_cache *c, int32_t seq_id, int32_t new_len);  /* 0 <= new_len <= length   */

/*
 * Cache append (Sec. IV-A Eq.(2) and Sec. IV-B Eq.(4)): for each of the n_seqs sequences named in
 * seq_ids_host (distinct ids), append n_new >= 1 tokens at positions [len, len + n_new).
 * For every (sequence, token, KV head):
 *   sketch bit i = ( sum_j R[i][j] k[j] >= 0 ), the sum taken in fp32 as a chain of fused multiply-adds
 *   over j = 0..d-1 from +0; bit i is stored in word i/64 at bit position i%64;
 *   per group of G channels of v: zero = fp16(min), scale = fp16((max - min)/15),
 *   code = clamp(round_half_even((v - zero)/scale), 0, 15) in fp32 (code 0 when scale is 0);
 *   with value_bits = 16 instead: the value rounded to nearest-even fp16 (an fp16 input is stored unchanged).
 * k_dev, v_dev: [n_seqs][n_new][n_kv_heads][d] in in_dtype, addressed with the given strides (in
 * elements; the channel stride is 1).  Inputs must be finite.  Pages are taken from the free list as
 * needed (H1BKV_ENOSPACE if they do not suffice; then nothing is appended).
 */
int h1bkv_append_kv(h1bkv_cache *c, const int32_t *seq_ids_host, int32_t n_seqs, int32_t n_new,
                    const void *k_dev, const void *v_dev, int64_t stride_seq, int64_t stride_tok,
                    int64_t stride_head, void *hip_stream);

/*
 * Workspace bytes h1bkv_decode_attn needs for up to n_seqs sequences of up to max_ctx tokens
 * (query sketches plus per-chunk partial results); monotone in both arguments.
 */
size_t h1bkv_decode_workspace_bytes(const h1bkv_cache *c, int32_t n_seqs, int32_t max_ctx);

/*
 * Decode-step attention (Sec. IV-A Eq.(3), Sec. IV-C Eq.(5)): for every sequence s in seq_ids_host
 * and every query head h, with T = current length of s:
 *   s_q = sign(R q) (same recipe as the keys);  alpha_t = (b - 2 popcount(s_q xor s_t)) / b;
 *   out = sum_t softmax_t(alpha_t / tau) * (scale_t * code_t + zero_t)   over all T cached tokens
 * (no mask; T == 0 gives zeros; with value_bits = 16 the bracket is the stored fp16 value).  q_dev [n_seqs][n_q_heads][d] in in_dtype, dense;
 * out_dev [n_seqs][n_q_heads][d] fp32; tau > 0 and finite.  The context is processed in chunks whose
 * partial (max, sum, weighted sum) results are merged by a log-sum-exp step; accumulation is fp32.
 * workspace_dev: >= h1bkv_decode_workspace_bytes(c, n_seqs, longest T), 256-byte aligned.
 */
int h1bkv_decode_attn(h1bkv_cache *c, const int32_t *seq_ids_host, int32_t n_seqs, const void *q_dev,
                      float tau, float *out_dev, void *workspace_dev, size_t workspace_bytes,
                      void *hip_stream);

/*
 * h1bkv_decode_attn for callers that cannot allocate device memory or hand over a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, same kernels and same results, but
 * the query sketches and per-chunk partial results live in a static device array of H1BKV_STATIC_SCRATCH_BYTES inside
 * the library (one copy per GPU, held until the process ends; its address is looked up when a handle is created on
 * the device).  The call allocates nothing on the device.  A call whose sketches and partials do not fit (they
 * grow with n_seqs x n_q_heads x chunks of the longest context) returns H1BKV_EWORKSPACE and launches nothing.  Every
 * call on a GPU, from any handle, uses that GPU's one array and nothing in it needs clearing between calls (each call
 * overwrites what it reads): calls that overlap in time on one GPU -- two streams, two handles -- race; order them.
 */
#define H1BKV_STATIC_SCRATCH_BYTES (16u << 20)
int h1bkv_decode_attn_static(h1bkv_cache *c, const int32_t *seq_ids_host, int32_t n_seqs, const void *q_dev,
                             float tau, float *out_dev, void *hip_stream);

/*
 * One decode step in one call: h1bkv_append_kv with n_new = 1 (k_dev, v_dev: [n_seqs][n_kv_heads][d], sequence
 * and head strides in elements) followed by h1bkv_decode_attn over the grown context, with the same results as
 * the two calls (Sec. IV: a generated token's key and value are cached, then its query attends to the cache).
 * The new token's append and the query sketches do not depend on each other and share one kernel launch, so the
 * step costs three launches instead of four.  workspace as for h1bkv_decode_attn with the lengths after the append.
 * Validation covers both halves before anything is changed or enqueued; if a launch of the decode half fails, the
 * appended token is taken back (lengths and page assignments as before the call).
 * Under HIP graph capture: token positions, context lengths and page assignments travel in the kernel arguments, so a
 * captured step is frozen at the position it was captured at -- replaying it rewrites the same slot and attends over
 * the same length, and the host bookkeeping advanced once, at capture.  A graph is therefore valid for one position
 * (re-capture per token, launch eagerly, or use h1bkv_decode_step_dev below).
 */
int h1bkv_decode_step(h1bkv_cache *c, const int32_t *seq_ids_host, int32_t n_seqs, const void *k_dev,
                      const void *v_dev, int64_t stride_seq, int64_t stride_head, const void *q_dev, float tau,
                      float *out_dev, void *workspace_dev, size_t workspace_bytes, void *hip_stream);

/*
 * The decode step with device-resident positions, for callers that replay one captured step token after token
 * (Sec. IV: the same append-then-attend step; only where the lengths live differs).
 *   h1bkv_reserve_seq     assigns pages for the next n_tokens positions of a sequence now (block table updated in stream
 *                         order); its length does not change.  H1BKV_ENOSPACE if the pool or the per-sequence page limit
 *                         cannot hold them; nothing changes then.  h1bkv_truncate_seq / h1bkv_reset_seq give reserved
 *                         pages beyond the new length back.  h1bkv_reserved_tokens: positions that have a page.
 *   h1bkv_decode_step_dev as h1bkv_decode_step, but the number of tokens sequence seq_ids_host[i] holds is read by the
 *                         kernels from pos_dev[i] (int32, device memory, 4-byte aligned) when they run: the new token is
 *                         written at position pos_dev[i], the query attends over pos_dev[i] + 1 tokens, and with
 *                         advance = 1 the step's last kernel adds one to pos_dev[i].  advance = 0 leaves the positions
 *                         alone: the layers of a model, each with a cache of its own, share ONE position array, all but
 *                         the last layer's step pass 0 and the last one moves the token on for all of them (anything
 *                         but 0 or 1: H1BKV_EINVAL).  No kernel touches a position >= max_pos: every sequence
 *                         must have pages for max_pos tokens (H1BKV_ERANGE otherwise), launches and workspace
 *                         (>= h1bkv_decode_workspace_bytes(c, n_seqs, max_pos)) are sized for max_pos, and a sequence
 *                         that has reached max_pos is left as it is (no append, attention over its max_pos tokens, no
 *                         advance).  The host's lengths are NOT changed: captured in a HIP graph, the step can be replayed
 *                         max_pos - pos times, each replay one token further.  The caller writes the initial lengths
 *                         into pos_dev (h1bkv_seq_len) before the first step and must not run other calls on these
 *                         sequences in between.
 *   h1bkv_set_seq_len     tells the host bookkeeping the length the device has reached (>= the current length, within
 *                         the reserved pages; H1BKV_ERANGE otherwise), after which every other call sees the grown
 *                         sequence.
 */
int h1bkv_reserve_seq(h1bkv_cache *c, int32_t seq_id, int32_t n_tokens, void *hip_stream);
int h1bkv_reserved_tokens(const h1bkv_cache *c, int32_t seq_id, int32_t *n_out);
int h1bkv_decode_step_dev(h1bkv_cache *c, const int32_t *seq_ids_host, int32_t n_seqs, const void *k_dev,
                          const void *v_dev, int64_t stride_seq, int64_t stride_head, const void *q_dev, float tau,
                          float *out_dev, int32_t *pos_dev, int32_t max_pos, int32_t advance, void *workspace_dev,
                          size_t workspace_bytes, void *hip_stream);
int h1bkv_set_seq_len(h1bkv_cache *c, int32_t seq_id, int32_t new_len);

/*
 * Decode-step attention together with its derivative with respect to the temperature (Sec. IV-C: tau is the scalar the
 * finetuning stage trains; Eq.(5)):  out as h1bkv_decode_attn, and
 *   dout_dtau = -(1/tau^2) ( sum_t p_t alpha_t v_t / l - (sum_t p_t alpha_t / l) out ),  p_t = exp(alpha_t / tau), l = sum_t p_t
 * -- the softmax-weighted covariance of scores and dequantised values over -tau^2; zero for T <= 1.
 * out_dev, dout_dtau_dev: [n_seqs][n_q_heads][d] fp32.  Every cache geometry h1bkv_decode_attn serves is supported
 * (4-bit and fp16 values, any number of query heads per KV head).  workspace_dev: >=
 * h1bkv_decode_dtau_workspace_bytes(c, n_seqs, longest T), 256-byte aligned.  Other arguments as h1bkv_decode_attn.
 */
size_t h1bkv_decode_dtau_workspace_bytes(const h1bkv_cache *c, int32_t n_seqs, int32_t max_ctx);
int h1bkv_decode_attn_dtau(h1bkv_cache *c, const int32_t *seq_ids_host, int32_t n_seqs, const void *q_dev, float tau,
                           float *out_dev, float *dout_dtau_dev, void *workspace_dev, size_t workspace_bytes,
                           void *hip_stream);

/*
 * Prefill attention (Sec. IV-A Eq.(3), Sec. IV-C Eq.(5) applied to every position of a prompt chunk): the n_q most
 * recent cached positions of every sequence are the queries.  Query i of sequence s (absolute position
 * len_s - n_q + i) attends to the cached tokens up to and including its own position, with the same scores, softmax
 * and dequantised values as h1bkv_decode_attn -- the result of feeding the chunk one token at a time
 * (append the chunk's keys and values with h1bkv_append_kv first).  Every sequence must hold at least n_q tokens
 * (H1BKV_ERANGE otherwise).  q_dev [n_seqs][n_q][n_q_heads][d] in in_dtype with strides in elements (channel
 * stride 1, rows 16-byte aligned); out_dev [n_seqs][n_q][n_q_heads][d] fp32, dense.  The weighted sum runs on the
 * matrix cores with fp16 operands (weights and dequantised values rounded to fp16, fp32 accumulation).
 * Every cache geometry is supported (a head of 256 channels is served as two halves of 128); with value_bits = 16 the
 * stored fp16 values are used as they are.
 * workspace_dev: >= h1bkv_prefill_workspace_bytes(c, n_seqs, n_q), 256-byte aligned: the chunk's query sketches and, for
 * chunks too short to fill the chip with one workgroup per 128 (from 256 positions on: 256) query positions, the per-row partial results of up to
 * 16 context splits (a chunk of a few hundred positions over a long context is split over the context as well, and
 * the splits are merged by a second kernel -- the same exact re-association as in h1bkv_decode_attn).
 */
size_t h1bkv_prefill_workspace_bytes(const h1bkv_cache *c, int32_t n_seqs, int32_t n_q);
int h1bkv_prefill_attn(h1bkv_cache *c, const int32_t *seq_ids_host, int32_t n_seqs, int32_t n_q, const void *q_dev,
                       int64_t stride_seq, int64_t stride_tok, int64_t stride_head, float tau, float *out_dev,
                       void *workspace_dev, size_t workspace_bytes, void *hip_stream);

/*
 * Tuning override for the context chunk of h1bkv_decode_attn: tokens per chunk, a multiple of
 * H1BKV_PAGE_TOKENS up to 8192, or 0 for the built-in choice.  Results do not depend on it beyond
 * fp32 summation order.
 */
int h1bkv_set_decode_chunk(h1bkv_cache *c, int32_t chunk_tokens);

/*
 * Tuning switch for the key projection of Eq.(2) in prefill-sized h1bkv_append_kv calls (n_new >= 16), in
 * h1bkv_prefill_attn's query sketches and in h1bkv_decode_attn's when a call brings thousands of
 * queries: 1 (default) computes the projections on the matrix cores from a two-piece fp16 split of R (and, for fp32
 * inputs, of the vectors, each scaled by a power of two first) and recomputes, with the fp32 multiply-add chain stated
 * at h1bkv_append_kv, every bit whose projection lies inside a guard band around zero that bounds the difference
 * between the two evaluations -- the stored bits are those of the chain either way; 0 always runs the chain.
 */
int h1bkv_set_projection_path(h1bkv_cache *c, int32_t use_matrix_cores);

/*
 * Test hook for the error paths: the nth kernel launch (nth >= 1) attempted on this handle from now on is not made and
 * is reported as a failed launch (the call returns H1BKV_EHIP after restoring the bookkeeping); 0 disarms.  A
 * bookkeeping-only handle counts the launches it would have made.  Nothing faults: the launch is skipped on the host.
 */
int h1bkv_debug_fail_launch(h1bkv_cache *c, int32_t nth);

/*
 * Canonical, layout-independent view of cached records (synchronous: waits for the device first).
 * Tokens [t0, t0+n) of (seq_id, kv_head) to host arrays: sketch_out [n][W] u64, codes_out [n][d/2] u8
 * (channel 2m low nibble, 2m+1 high nibble of byte m), scale_out / zero_out [n][n_g] fp16 bit patterns.
 * With value_bits = 16, codes_out / codes_in is the value plane instead, [n][d] fp16 bit patterns (2d bytes per
 * token), and scale/zero must be NULL (H1BKV_EINVAL otherwise).
 * Any output pointer may be NULL to skip that plane.  h1bkv_import_tokens is the mirror image and
 * overwrites existing positions; h1bkv_extend_seq reserves n_new uninitialised positions (pages and
 * block-table update on `hip_stream`) so that a saved cache can be restored with import.
 */
int h1bkv_export_tokens(const h1bkv_cache *c, int32_t seq_id, int32_t kv_head, int32_t t0, int32_t n,
                        uint64_t *sketch_out, uint8_t *codes_out, uint16_t *scale_out, uint16_t *zero_out);
int h1bkv_import_tokens(h1bkv_cache *c, int32_t seq_id, int32_t kv_head, int32_t t0, int32_t n,
                        const uint64_t *sketch_in, const uint8_t *codes_in, const uint16_t *scale_in,
                        const uint16_t *zero_in);
int h1bkv_extend_seq(h1bkv_cache *c, int32_t seq_id, int32_t n_new, void *hip_stream);

/*
 * Per-kernel timing for benchmarks.  After h1bkv_profile_enable(c, capacity > 0, kernel_mask), every launch of
 * the library's kernels whose kind is in kernel_mask (bit 1 << H1BKV_K_*) on this handle is bracketed by a pair
 * of HIP events on the launch stream (up to `capacity` launches per kind; later ones are not recorded).
 * h1bkv_profile_read waits for the recorded events and writes the elapsed milliseconds of each recorded launch
 * of `kernel` to ms_out (at most cap values) and their number to n_out, then clears that kind's records.
 * capacity == 0 disables recording and releases the events.  Launches enqueued while the stream is being captured into
 * a HIP graph are not timed.
 * A kind whose work takes two kernels (H1BKV_K_APPEND of a large append: the keys' half and the values' half;
 * H1BKV_K_PREFILL with a context split: the attention kernel and its merge) is bracketed once around both.
 * H1BKV_K_DECODE_SPLIT is the exception to the bracket: its two events are attached to the kernel's own dispatch and
 * hold the kernel's start and end, the duration a kernel trace reports (events recorded around a launch also count
 * the 2-3 microseconds between command packets, which is 4 % of a 70-microsecond kernel).
 */
enum { H1BKV_K_APPEND = 0, H1BKV_K_QSKETCH = 1, H1BKV_K_DECODE_SPLIT = 2, H1BKV_K_MERGE = 3, H1BKV_K_PREFILL = 4,
       H1BKV_K_COUNT = 5 };
int h1bkv_profile_enable(h1bkv_cache *c, int32_t capacity, uint32_t kernel_mask);
/* Bracket only every `stride`-th launch of each selected kind (stride >= 1; 1 = every launch, the default): an
 * event pair costs a few microseconds on the stream, which a benchmark of sub-millisecond steps can thin out. */
int h1bkv_profile_stride(h1bkv_cache *c, int32_t stride);
int h1bkv_profile_read(h1bkv_cache *c, int32_t kernel, float *ms_out, int32_t cap, int32_t *n_out);

/*
 * Plain device-to-device streaming copy of n_bytes (a multiple of 16; both pointers 16-byte aligned)
 * with the library's own 16-byte-per-lane grid-stride kernel, enqueued on hip_stream.  It exists as
 * the known-size reference against which hardware traffic counters and the achievable HBM rate are
 * calibrated; it is not part of the attention path.
 */
int h1bkv_stream_copy(void *dst_dev, const void *src_dev, size_t n_bytes, void *hip_stream);

/*
 * Read-only counterpart: streams n_bytes (a multiple of 16, 16-byte aligned) from src_dev with 16-byte loads,
 * XOR-folds them and writes 16 bytes per workgroup to sink_dev (>= 128 KiB).  Its rate is the HBM read
 * ceiling a streaming kernel can reach on this device, against which the decode kernel is also reported.
 */
int h1bkv_stream_read(const void *src_dev, size_t n_bytes, void *sink_dev, void *hip_stream);
/*
 * The same launch, timed: waits for the kernel (the one synchronous call among these helpers) and writes its duration
 * in milliseconds to ms_out (host), taken from events attached to the kernel's dispatch as for H1BKV_K_DECODE_SPLIT above,
 * so that the ceiling and the decode kernel are measured the same way.  n_bytes > 0.
 */
int h1bkv_stream_read_ms(const void *src_dev, size_t n_bytes, void *sink_dev, void *hip_stream, float *ms_out);

#ifdef __cplusplus
}
#endif
#endif /* H1BKV_H */
