// Shared declarations between the host side (cache.cpp) and the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "h1bkv.h"

namespace h1bkv {

constexpr int kPage = H1BKV_PAGE_TOKENS;   // tokens per page
constexpr int kMaxSeqsPerLaunch = 128;     // sequences described by one kernel-argument block
constexpr int kMaxChunk = 8192;            // largest context chunk one decode workgroup handles
constexpr int kPublishPairs = 240;         // block-table updates carried by one publish launch

// Per-launch sequence descriptors travel as a kernel argument (no host->device copy, nothing to keep
// alive after the launch returns).  `pos` is the first new position for append and the context length
// for decode.
struct SeqDesc {
    int32_t seq_id;
    int32_t pos;
};
struct BatchDesc {
    SeqDesc s[kMaxSeqsPerLaunch];
    // Device-resident positions (h1bkv_decode_step_dev; nullptr otherwise): pos_dev[i] is the number of tokens sequence
    // s[i] holds, read by the kernels when they run -- a captured launch then follows the sequence as it grows.  The
    // position a kernel works on is pos_dev[i] + pos_add, never beyond pos_max (the tokens the caller reserved pages for).
    const int32_t *pos_dev = nullptr;
    int32_t pos_add = 0;
    int32_t pos_max = 0;
    int32_t advance = 0;     // the step's last kernel (the merge) adds one to every position once all its workgroups have read theirs
};

// The position of sequence i of a launch: the descriptor's, or the device-resident one.
__device__ __forceinline__ int desc_pos(const BatchDesc &d, int i) {
    if (d.pos_dev) {
        const int p = d.pos_dev[i] + d.pos_add;
        return p < d.pos_max ? p : d.pos_max;
    }
    return d.s[i].pos;
}

// Device-resident positions, end of a step: called by every workgroup of the step's last kernel right after all its
// threads have read their positions (the caller's barrier), by one thread.  The workgroup that arrives last -- every
// other one holds its position in registers by then -- moves the n sequences of the launch one token on and leaves the
// counter at zero for the next launch.  (No kernel of the step reads a position after this point; the next step's
// kernels start after this one has ended.)
__device__ __forceinline__ void advance_positions_when_all_read(const BatchDesc &d, uint32_t *ticket, unsigned n_workgroups, int n) {
    if (atomicAdd(ticket, 1u) != n_workgroups - 1) return;
    atomicExch(ticket, 0u);
    int32_t *pos = const_cast<int32_t *>(d.pos_dev);
    for (int i = 0; i < n; ++i)
        if (pos[i] < d.pos_max) pos[i] += 1;
}

struct TablePairs {
    int32_t n;
    int32_t index[kPublishPairs];   // flat index into block_table [max_seqs][max_pages_per_seq]
    int32_t page[kPublishPairs];
};

// Device view of the pool.
struct PoolView {
    const float *R;          // [b][d]
    const float *RT;         // [d][b]
    // Matrix-core projection (prefill-sized appends, prefill query sketches): R split into two fp16 pieces,
    // R ~ R16hi + 2^-12 R16mid, and per row the guard band factor: a projection whose magnitude exceeds
    // guard[i] * ||k||_2 has the sign of the pinned fp32 chain for certain (see make_projection_pieces in cache.cpp).
    const uint16_t *R16hi;   // [b][d] fp16 bits
    const uint16_t *R16mid;  // [b][d] fp16 bits
    const float *guard;      // [2][b]: the band factors for fp16 inputs, then those for fp32 inputs (split into two pieces too)
    int32_t *block_table;    // [max_seqs][max_pages_per_seq]
    uint32_t *ticket;        // one counter (zero between launches): workgroups of a merge that have read their positions
    uint64_t *sketch;        // [page][H_kv][256][W]
    uint8_t *codes;          // [page][H_kv][256][d/2]
    uint32_t *meta;          // [page][H_kv][256][n_g]  low half = fp16 scale, high half = fp16 zero
    int32_t max_pages_per_seq;
    int32_t n_kv_heads, n_q_heads, head_dim, sketch_bits, group_size;
    int32_t code_layout;     // 0: record-major nibbles; 1: token-interleaved words (see below);
                             // 2: no codes -- `codes` holds fp16 values [page][H_kv][256][d], `meta` is unused
};

// Code plane layout 1 (used when several query heads share a KV head and the weighted sum runs on the matrix
// cores): per (page, head) the 256 tokens form 32 blocks of 8 tokens; a block is d 32-bit words, one per
// channel, each holding the channel's 8 codes.  Token j of the block sits at nibble j/2 (j even) or 4 + j/2
// (j odd), so that nibbles n and n+4 -- which one AND-OR turns into the two fp16/bf16 halves of a register --
// are consecutive tokens, i.e. consecutive K indices of an MFMA operand.  Channel c = 16*cb + n is word
// (cb/4)*64 + n*4 + cb%4: the 16 lanes n of an MFMA column block read 16 bytes each (4 column blocks), contiguously.
__host__ __device__ inline int code_nibble_pos(int j) { return (j & 1) ? 4 + (j >> 1) : (j >> 1); }
__host__ __device__ inline int code_word_index(int c) {
    const int cb = c >> 4, n = c & 15;
    return (cb >> 2) * 64 + n * 4 + (cb & 3);
}

struct AppendArgs {
    PoolView pool;
    const void *k, *v;
    int64_t stride_seq, stride_tok, stride_head;
    int32_t n_new;
    int32_t f16;
    int32_t proj_mfma;       // sketch bits from the matrix-core projection plus exact recomputation inside the guard band
};

struct QueryArgs {            // query vectors sketched by the fused decode-step prologue
    const void *q;            // [n_vec][d] in the cache's input dtype
    uint64_t *q_sketch;       // [n_vec][W]
    int32_t n_vec;
};

struct DecodeArgs {
    PoolView pool;
    const void *q;            // [n_seqs][H_q][d]
    uint64_t *q_sketch;       // workspace: [n_seqs][H_q][W]
    float *part_ml;           // workspace: [n_seqs][H_q][S][2]  (min Hamming distance as int bits, sum of p)
    float *part_o;            // workspace: [n_seqs][H_q][S][d]
    float *out;               // [n_seqs][H_q][d]
    float *part_oh;           // temperature-derivative path only: workspace [n_seqs][H_q][S][d], distance-weighted sums
    float *dout;              // temperature-derivative path only: [n_seqs][H_q][d]
    int32_t n_splits;         // S: chunks of the longest context in the call
    int32_t chunk;            // tokens per chunk (multiple of the page size)
    int32_t f16;
    float exp2_scale;         // 2 log2(e) / (b tau): p = exp2(exp2_scale * (ham_min - ham))
};

struct PrefillArgs {
    PoolView pool;
    const void *q;            // [n_seqs][n_q][H_q][d] in the cache's input dtype, addressed with the strides below
    int64_t stride_seq, stride_tok, stride_head;
    uint64_t *q_sketch;       // workspace: [n_seqs][n_q][H_q][W]
    float *out;               // [n_seqs][n_q][H_q][d]
    float *part;              // workspace: [n_seqs][n_q][H_q][n_splits][d + 2] partial results (n_splits > 1 only):
                              //   d unnormalised sums, the weight sum, the reference distance (x 4, as int bits)
    int32_t n_q;              // query positions per sequence: the last n_q cached positions
    int32_t n_splits;         // context splits per query block: each workgroup walks 1 / n_splits of the block's key tiles
    int32_t f16;
    int32_t proj_mfma;        // query sketches from the matrix-core projection (fp16 queries)
    float exp2_scale;         // 2 log2(e) / (b tau)
};

// Query positions per prefill workgroup: 256 (eight waves) from 256 positions per chunk on, 128 (four waves) below.
inline int prefill_rows(int n_q) { return n_q >= 256 ? 256 : 128; }
constexpr int kPrefillMaxSplits = 16;
// Most context splits a prefill call of n_seqs x n_q query positions can use: enough workgroups to fill the chip when
// the chunk is short (a long prompt alone already brings thousands of workgroups: one split).
inline int prefill_max_splits(int n_q_heads, int n_seqs, int n_q) {
    const int rows = prefill_rows(n_q);
    const int64_t wgs = (int64_t)n_q_heads * n_seqs * ((n_q + rows - 1) / rows);
    // One workgroup per place the chip has for them (256 compute units x 1 of eight waves or 2 of four) and no more: a split
    // costs partial results and a merge, and halves what a workgroup gets out of its prologue (8k prompts in chunks of
    // 512 positions: 1.80 ms of attention per prompt batch with one split, 2.36 with two; chunks of 128: 3.51 ms with
    // four splits, 4.49 with eight, 5.97 with two).
    const int64_t fill = rows == 256 ? 256 : 512;
    const int64_t s = (fill + wgs - 1) / wgs;
    return (int)(s < 1 ? 1 : s > kPrefillMaxSplits ? kPrefillMaxSplits : s);
}

// Query heads one matrix-core decode workgroup serves: the largest divisor of r that is at most 8 (4 at 256 channels).
inline int mfma_heads_per_wg(int r, int head_dim) {
    for (int q = head_dim > 128 ? 4 : 8; q > 1; --q)
        if (r % q == 0) return q;
    return 1;
}
// The matrix-core decode path (and with it code layout 1) is used from 3 query heads per KV head on, for every
// geometry (256 channels: four query heads per workgroup at most, two waves per SIMD).
inline bool mfma_decode_supported(int r, int head_dim, int group_size, int sketch_bits) {
    (void)head_dim; (void)group_size; (void)sketch_bits;
    return r >= 3;
}
// Largest context chunk of one decode workgroup.
inline int max_decode_chunk(int, int) { return kMaxChunk; }

// Launchers (kernels_*.hip).  Each returns hipGetLastError() of its launch.
hipError_t launch_publish(const TablePairs &pairs, int32_t *block_table, hipStream_t st);
// Profiling of the split-decode kernels (and of the timed read-only stream): the events of the current profiling slot are attached to the kernel's own
// dispatch (they then hold the start and the end of the kernel itself, what a kernel trace reports) instead of being
// recorded around the launch, where they also count the few microseconds between command packets.  The bracket in
// cache.cpp hands them over, the launch takes them; without profiling both are null and the launch is an ordinary one.
struct DispatchEvents {
    hipEvent_t start = nullptr, stop = nullptr;
};
void set_dispatch_events(hipEvent_t start, hipEvent_t stop);
DispatchEvents take_dispatch_events();
#define H1BKV_LAUNCH_TIMED(kernel, grid, block, st, ...)                                                  \
    do {                                                                                                   \
        const DispatchEvents ev_ = take_dispatch_events();                                                 \
        if (ev_.start) hipExtLaunchKernelGGL(kernel, grid, block, 0, st, ev_.start, ev_.stop, 0, __VA_ARGS__); \
        else hipLaunchKernelGGL(kernel, grid, block, 0, st, __VA_ARGS__);   /* (the shorter path on the host) */ \
    } while (0)

hipError_t launch_append(const AppendArgs &a, const BatchDesc &desc, int n_seqs, const QueryArgs *qa, hipStream_t st);
hipError_t launch_qsketch(const DecodeArgs &a, int seq0, int n_seqs, hipStream_t st);
hipError_t launch_decode_split(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st);
hipError_t launch_decode_split_mfma(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st);
hipError_t launch_decode_split_f16v(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st);
hipError_t launch_decode_dtau_split(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st);
hipError_t launch_decode_dtau_split_mfma(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st);
hipError_t launch_decode_dtau_split_f16v(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st);
hipError_t launch_merge_dtau(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, float dtau_scale, hipStream_t st);
hipError_t launch_merge(const DecodeArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st);
hipError_t launch_sketch_rows(const PrefillArgs &a, int n_seqs, hipStream_t st);
hipError_t launch_prefill_merge(const PrefillArgs &a, int seq0, int n_seqs, hipStream_t st);
hipError_t launch_prefill(const PrefillArgs &a, const BatchDesc &desc, int seq0, int n_seqs, hipStream_t st);
hipError_t launch_stream_copy(void *dst, const void *src, size_t n_bytes, hipStream_t st);
hipError_t launch_stream_read(const void *src, size_t n_bytes, void *sink, hipStream_t st);

}  // namespace h1bkv
