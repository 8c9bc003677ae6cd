// Host side of the H1B-KV library: handle, argument validation, page bookkeeping, launch sequencing,
// canonical export/import and the per-kernel event timer.  No arithmetic of the method lives here.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "internal.h"

using namespace h1bkv;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Layout {
    size_t off_R, off_RT, off_R16hi, off_R16mid, off_guard, off_bt, off_sketch, off_codes, off_meta, total;
};

bool config_ok(const h1bkv_config *c) {
    if (!c) return false;
    if (c->n_kv_heads < 1 || c->n_q_heads < 1 || c->n_q_heads % c->n_kv_heads != 0) return false;
    if (c->head_dim != 64 && c->head_dim != 128 && c->head_dim != 256) return false;
    if (c->sketch_bits != 64 && c->sketch_bits != 128 && c->sketch_bits != 256 && c->sketch_bits != 512) return false;
    if (c->group_size != 32 && c->group_size != 64 && c->group_size != 128) return false;
    if (c->head_dim % c->group_size != 0) return false;
    if (c->in_dtype != H1BKV_F32 && c->in_dtype != H1BKV_F16) return false;
    if (c->page_tokens != 0 && c->page_tokens != kPage) return false;
    if (c->max_seqs < 1 || c->max_pages < 1 || c->max_pages_per_seq < 1) return false;
    if (c->device < H1BKV_DEVICE_NONE) return false;
    if (c->value_bits != 0 && c->value_bits != 4 && c->value_bits != 16) return false;
    return true;
}

Layout make_layout(const h1bkv_config &c) {
    Layout L{};
    const size_t b = c.sketch_bits, d = c.head_dim, W = b / 64, ng = d / c.group_size;
    const size_t rec = (size_t)c.max_pages * c.n_kv_heads * kPage;
    size_t o = 0;
    L.off_R = o;       o = align_up(o + b * d * sizeof(float));
    L.off_RT = o;      o = align_up(o + b * d * sizeof(float));
    L.off_R16hi = o;   o = align_up(o + b * d * sizeof(uint16_t));
    L.off_R16mid = o;  o = align_up(o + b * d * sizeof(uint16_t));
    L.off_guard = o;   o = align_up(o + 2 * b * sizeof(float));
    // (64 more words behind the block table: the first is the merge kernels' arrival counter)
    L.off_bt = o;      o = align_up(o + ((size_t)c.max_seqs * c.max_pages_per_seq + 64) * sizeof(int32_t));
    L.off_sketch = o;  o = align_up(o + rec * W * 8);
    const bool f16v = c.value_bits == 16;
    L.off_codes = o;   o = align_up(o + rec * (f16v ? 2 * d : d / 2));
    L.off_meta = o;    o = align_up(o + (f16v ? 0 : rec * ng * 4));
    L.total = o;
    return L;
}

// fp16 pieces of R are made with the host compiler's own binary16 type: a cast to _Float16 rounds to nearest even,
// a cast back is exact; the bit pattern is what the device reads.
inline uint16_t half_bits(_Float16 h) {
    uint16_t u;
    std::memcpy(&u, &h, sizeof u);
    return u;
}

// Pieces of R for the matrix-core projection and the guard band that keeps the sketch bits exactly those of the
// pinned fp32 chain (Eq.(2): bit = (y >= 0) with y = fma-chain over j).
//   hi = fp16(R), mid = fp16((R - hi) 2^12):  R = hi + 2^-12 mid + delta, |delta| tiny.
// The kernel computes y~ = sum_j (hi_j + 2^-12 mid_j) k_j with fp32 accumulation (products of two fp16 numbers are
// exact in fp32).  Against the chain value y:
//   |y~ - y| <= sum_j |delta_j| |k_j|                       (pieces)             <= ||delta||_2 ||k||_2
//            + (rounding of the chain: d steps of 2^-24 relative to sum |R_j k_j|)  <= d 2^-24 ||R||_2 ||k||_2
//            + (rounding of the matrix-core accumulation, any order, two piece sums and their combination;
//               allowed three times the chain's)                                     <= 3 d 2^-24 ||R||_2 ||k||_2
//            + (a piece that is an fp16 subnormal may be read as zero)              <= ||flush||_2 ||k||_2.
// guard[i] is twice the sum of these row factors; a bit with |y~| <= guard[i] ||k||_2 is recomputed with the chain.
// fp32 inputs are scaled by a power of two and split the same way, k s = kh + 2^-12 km + eps (stage_f32_tile), and the
// kernel leaves out the product of the two low pieces; guard[b + i] prices that in:
//            + (input pieces: |eps_j| <= 2^-22 |k_j s| + 2^-37)                       <= 2^-21 ||R||_2 ||k s||_2
//            + (dropped 2^-24 sum mid_j km_j, |mid_j| <= 2 |R_j|, |km_j| <= 2 |k_j s|) <= 2^-22 ||R||_2 ||k s||_2
//            + (a third piece sum in the matrix-core accumulation: four times the chain's instead of three).
void make_projection_pieces(const float *R, int b, int d, std::vector<uint16_t> &hi, std::vector<uint16_t> &mid,
                            std::vector<float> &guard) {
    hi.resize((size_t)b * d);
    mid.resize((size_t)b * d);
    guard.resize(2 * (size_t)b);
    for (int i = 0; i < b; ++i) {
        double n2 = 0.0, delta2 = 0.0, flush2 = 0.0;
        for (int j = 0; j < d; ++j) {
            const size_t e = (size_t)i * d + j;
            const double r = (double)R[e];
            const _Float16 h16 = (_Float16)R[e];
            const double h = (double)h16;
            const _Float16 m16 = (_Float16)(float)((r - h) * 4096.0);   // r - h is exact in double, and in float after scaling
            const double m = (double)m16;
            hi[e] = half_bits(h16);
            mid[e] = half_bits(m16);
            const double delta = r - (h + m / 4096.0);
            n2 += r * r;
            delta2 += delta * delta;
            double fl = 0.0;
            if ((hi[e] & 0x7C00u) == 0) fl += std::fabs(h);
            if ((mid[e] & 0x7C00u) == 0) fl += std::fabs(m) / 4096.0;
            flush2 += fl * fl;
        }
        const double g = 2.0 * (std::sqrt(delta2) + 4.0 * d * std::ldexp(1.0, -24) * std::sqrt(n2) + std::sqrt(flush2));
        guard[i] = std::nextafter((float)g, INFINITY);
        const double g32 = 2.0 * (std::sqrt(delta2) + (5.0 * d * std::ldexp(1.0, -24) + std::ldexp(1.0, -21) + std::ldexp(1.0, -22)) * std::sqrt(n2) +
                                  std::sqrt(flush2));
        guard[(size_t)b + i] = std::nextafter((float)g32, INFINITY);
    }
}

// Projection drawn by the library when the caller passes none (Sec. III: R_ij ~ N(0,1), fixed once): a splitmix64
// stream from the seed, two draws per pair of consecutive elements, Box-Muller in double, rounded to fp32.
struct SplitMix64 {
    uint64_t s;
    uint64_t next() {
        s += 0x9E3779B97F4A7C15ull;
        uint64_t z = s;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    double uniform() { return ((double)(next() >> 11) + 0.5) * 0x1p-53; }   // in (0, 1)
};

void draw_projection(uint64_t seed, std::vector<float> &R) {
    SplitMix64 g{seed};
    for (size_t e = 0; e + 1 < R.size(); e += 2) {
        const double u1 = g.uniform(), u2 = g.uniform();
        const double rad = std::sqrt(-2.0 * std::log(u1)), ang = 6.283185307179586476925 * u2;
        R[e] = (float)(rad * std::cos(ang));
        R[e + 1] = (float)(rad * std::sin(ang));
    }
}

// Scratch of h1bkv_decode_attn_static: one array per GPU the library runs on, resident until the process ends.  In host
// code the array's name is only a stand-in for the symbol; its device address is looked up once per device
// (scratch_for_device) and that pointer is what kernels and everything else receive.
static __device__ __align__(256) unsigned char scratch[H1BKV_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
unsigned char *scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device `dev` (looked up on first use), or nullptr.
unsigned char *scratch_for_device(int dev) {
    if (dev < 0 || dev >= kMaxDevices) return nullptr;
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
        scratch_ptr[dev] = static_cast<unsigned char *>(p);
    }
    return scratch_ptr[dev];
}

// Device-resident sequence positions of h1bkv_decode_step_dev: pos[i] tokens are cached for the call's i-th sequence,
// and no kernel works beyond max_pos.
struct DevicePositions {
    const int32_t *pos;
    int32_t max_pos;
    int32_t advance;       // the step's last kernel moves the positions one token on
};

struct EventPair {
    hipEvent_t a, b;
};

}  // namespace

namespace h1bkv {
namespace {
thread_local DispatchEvents g_dispatch_events;     // (a handle is driven by one thread at a time)
}
void set_dispatch_events(hipEvent_t start, hipEvent_t stop) { g_dispatch_events = DispatchEvents{start, stop}; }
DispatchEvents take_dispatch_events() {
    const DispatchEvents e = g_dispatch_events;
    g_dispatch_events = DispatchEvents{};
    return e;
}
}  // namespace h1bkv

struct h1bkv_cache {
    h1bkv_config cfg;
    Layout lay;
    int W, ng, r;
    int code_layout;   // 0 record-major, 1 token-interleaved (matrix-core decode); see internal.h
    bool dry;
    char *pool;
    std::vector<float> R;
    std::vector<int32_t> seq_len;
    std::vector<std::vector<int32_t>> seq_pages;
    std::vector<int32_t> free_list;     // stack of free page ids
    mutable std::vector<char> seen;     // scratch of the duplicate-id check
    int32_t chunk_override;
    int32_t proj_mfma;     // 1: matrix-core projection where it applies (default); 0: always the plain fp32 chain
    int32_t fail_countdown;   // test hook: > 0 counts launch attempts down, the one that reaches 0 is skipped and reported failed
    // profiling
    int32_t prof_cap;
    uint32_t prof_mask;
    int32_t prof_stride;
    int32_t prof_seen[H1BKV_K_COUNT];
    std::vector<EventPair> prof_events[H1BKV_K_COUNT];
    int32_t prof_used[H1BKV_K_COUNT];

    PoolView view() const {
        PoolView v{};
        if (pool) {              // (a bookkeeping-only handle has no pool: its view carries the geometry only)
            v.R = reinterpret_cast<const float *>(pool + lay.off_R);
            v.RT = reinterpret_cast<const float *>(pool + lay.off_RT);
            v.R16hi = reinterpret_cast<const uint16_t *>(pool + lay.off_R16hi);
            v.R16mid = reinterpret_cast<const uint16_t *>(pool + lay.off_R16mid);
            v.guard = reinterpret_cast<const float *>(pool + lay.off_guard);
            v.block_table = reinterpret_cast<int32_t *>(pool + lay.off_bt);
            v.ticket = reinterpret_cast<uint32_t *>(v.block_table + (size_t)cfg.max_seqs * cfg.max_pages_per_seq);
            v.sketch = reinterpret_cast<uint64_t *>(pool + lay.off_sketch);
            v.codes = reinterpret_cast<uint8_t *>(pool + lay.off_codes);
            v.meta = reinterpret_cast<uint32_t *>(pool + lay.off_meta);
        }
        v.max_pages_per_seq = cfg.max_pages_per_seq;
        v.n_kv_heads = cfg.n_kv_heads;
        v.n_q_heads = cfg.n_q_heads;
        v.head_dim = cfg.head_dim;
        v.sketch_bits = cfg.sketch_bits;
        v.group_size = cfg.group_size;
        v.code_layout = code_layout;
        return v;
    }
};

namespace {

int check_device(const h1bkv_cache *c) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != c->cfg.device) return H1BKV_EHIP;
    return H1BKV_OK;
}

// (events recorded into a graph under capture hold no times: such launches are not timed)
inline bool capturing(hipStream_t st) {
    hipStreamCaptureStatus s = hipStreamCaptureStatusNone;
    return hipStreamIsCapturing(st, &s) == hipSuccess && s != hipStreamCaptureStatusNone;
}

// Event bracket around one kernel launch; inert unless profiling is enabled.  The split-decode kernel's events ride on its
// dispatch instead (see H1BKV_LAUNCH_TIMED): recorded around the launch they only serve a launch that did not take them.
struct Timed {
    h1bkv_cache *c;
    int kind;
    hipStream_t st;
    int slot;
    Timed(h1bkv_cache *c_, int kind_, hipStream_t st_) : c(c_), kind(kind_), st(st_), slot(-1) {
        if (c->prof_cap > 0 && ((c->prof_mask >> kind) & 1u) && c->prof_used[kind] < c->prof_cap && !capturing(st) &&
            c->prof_seen[kind]++ % c->prof_stride == 0) {
            slot = c->prof_used[kind]++;
            if (kind == H1BKV_K_DECODE_SPLIT) set_dispatch_events(c->prof_events[kind][slot].a, c->prof_events[kind][slot].b);
            else (void)hipEventRecord(c->prof_events[kind][slot].a, st);
        }
    }
    ~Timed() {
        if (slot < 0) return;
        if (kind == H1BKV_K_DECODE_SPLIT) {
            const DispatchEvents left = take_dispatch_events();
            if (left.start) {                        // nothing was launched (an error path): leave valid, empty timings
                (void)hipEventRecord(c->prof_events[kind][slot].a, st);
                (void)hipEventRecord(c->prof_events[kind][slot].b, st);
            }
        } else {
            (void)hipEventRecord(c->prof_events[kind][slot].b, st);
        }
    }
};

void release_events(h1bkv_cache *c) {
    for (int k = 0; k < H1BKV_K_COUNT; ++k) {
        for (auto &e : c->prof_events[k]) {
            (void)hipEventDestroy(e.a);
            (void)hipEventDestroy(e.b);
        }
        c->prof_events[k].clear();
        c->prof_used[k] = 0;
    }
    c->prof_cap = 0;
}

// Gate in front of every kernel launch (also the launches a bookkeeping-only handle skips): false when the failure
// armed with h1bkv_debug_fail_launch falls on this attempt -- the launch is then not made and reported as failed.
bool launch_allowed(h1bkv_cache *c) { return !(c->fail_countdown > 0 && --c->fail_countdown == 0); }

int pages_for(int32_t len) { return (len + kPage - 1) / kPage; }

// Pages that must be newly taken so that seq can hold new_len tokens, or a negative error.
int pages_needed(const h1bkv_cache *c, int32_t seq, int64_t new_len) {
    if (new_len > (int64_t)c->cfg.max_pages_per_seq * kPage) return H1BKV_ENOSPACE;
    return std::max(0, pages_for((int32_t)new_len) - (int)c->seq_pages[seq].size());   // (reserved pages may already cover it)
}

// Take pages for seq up to new_len and queue the block-table updates.
void take_pages(h1bkv_cache *c, int32_t seq, int32_t new_len, std::vector<int32_t> &upd_index,
                std::vector<int32_t> &upd_page) {
    auto &pg = c->seq_pages[seq];
    while ((int)pg.size() < pages_for(new_len)) {
        int32_t p = c->free_list.back();
        c->free_list.pop_back();
        upd_index.push_back(seq * c->cfg.max_pages_per_seq + (int32_t)pg.size());
        upd_page.push_back(p);
        pg.push_back(p);
    }
}

int publish(h1bkv_cache *c, const std::vector<int32_t> &idx, const std::vector<int32_t> &page, hipStream_t st) {
    size_t done = 0;
    while (done < idx.size()) {
        TablePairs tp;
        tp.n = (int32_t)std::min<size_t>(kPublishPairs, idx.size() - done);
        for (int i = 0; i < tp.n; ++i) {
            tp.index[i] = idx[done + i];
            tp.page[i] = page[done + i];
        }
        if (!launch_allowed(c)) return H1BKV_EHIP;
        if (!c->dry && launch_publish(tp, c->view().block_table, st) != hipSuccess) return H1BKV_EHIP;
        done += tp.n;
    }
    return H1BKV_OK;
}

int check_seq_ids(const h1bkv_cache *c, const int32_t *ids, int32_t n) {
    if (!ids) return H1BKV_ENULL;
    if (n < 1) return H1BKV_EINVAL;
    std::vector<char> &seen = c->seen;        // sized max_seqs at creation: no allocation per call
    std::fill(seen.begin(), seen.end(), 0);
    for (int i = 0; i < n; ++i) {
        if (ids[i] < 0 || ids[i] >= c->cfg.max_seqs) return H1BKV_ERANGE;
        if (seen[ids[i]]) return H1BKV_EINVAL;
        seen[ids[i]] = 1;
    }
    return H1BKV_OK;
}

// Chunk (tokens) the decode uses for a call of n_seqs sequences whose longest context is max_ctx:
// the largest page multiple (<= kMaxChunk) that still leaves enough workgroups to fill the chip.
// dtau: the call also computes the temperature derivative (its vector kernel takes one QUERY head per workgroup).
int choose_chunk(const h1bkv_cache *c, int n_seqs, int max_ctx, bool dtau = false) {
    if (c->chunk_override > 0) return c->chunk_override;
    const bool per_query_head = dtau && c->code_layout != 1;
    const int64_t heads = (int64_t)n_seqs * (per_query_head ? c->cfg.n_q_heads : c->cfg.n_kv_heads);
    // the matrix-core kernel gains from long streams per workgroup: two workgroups per compute unit (512 on the chip) are
    // enough, and more of them only add prologues, epilogues and partial results (measured over eight grouped-query
    // geometries from 50 MB to 470 MB, contexts of 4k to 128k tokens: the chunk that gives 512 workgroups was the fastest
    // in every one -- 63.7 us against 74.6 with 1024 workgroups at 16 x 8 KV heads x 32768 tokens, 40.3 against 47.8 at
    // 64 x 8 x 4096, 14.5 against 16.6 at 2 x 8 x 32768, 65.0 against 66.3 at 4 x 8 x 131072)
    // The vector kernel with two query heads per workgroup (r = 2) behaves the same way (8 x 16 KV heads x 32768 tokens:
    // 69.0 us with 512 workgroups, 93.4 with 4096; 16 x 4 x 65536: 89.4 against 138.2); with one head per workgroup the
    // chunk hardly matters from 1024 tokens on, and 4096 workgroups keep the tail of the launch short.  The derivative's
    // vector kernel carries two sets of sums per head, like two heads: 265.7 us with 8192-token chunks at 16 x 32 heads x
    // 32768 tokens, 276.9 with 4096, 296.6 with 2048.
    // (the fp16-value kernel with several heads per workgroup likewise, if less so: 8 x 8 KV heads x 16384 tokens, r = 4:
    // 63.5 us with 512 workgroups, 68.2 with 4096)
    const bool two_sets = (c->code_layout == 0 && (c->r >= 2 || dtau)) || (c->code_layout == 2 && c->r >= 2);
    const int64_t target_wgs = (c->code_layout == 1 || two_sets) ? 512 : 4096;
    int chunk = max_decode_chunk(c->r, c->code_layout);
    // Small problems: a workgroup's fixed cost (prologue, four-wave epilogue, partial results) is that of two or three
    // pages of streaming, so below 1024-token chunks only a quarter of the target (at least 1024) is insisted on (measured at 8 x 32
    // heads x 4096 tokens: 25.8 us with one page per workgroup, 21.2 us with four).
    // Tiny problems (up to 1280 (head, page) units in all: one sequence of a 7B-shaped model at 8k-10k tokens) cannot give
    // every compute unit four workgroups of several pages; there one workgroup per compute unit with up to four pages
    // is best (measured at 1 x 32 heads x 8192 tokens, records from HBM: 12.4 us with one page per workgroup, 11.7 with
    // two, 11.2 with four, 13.9 with eight).
    const bool tiny = heads * ((max_ctx + kPage - 1) / kPage) <= 1280;
    while (chunk > kPage) {
        const int64_t wgs = heads * ((max_ctx + chunk - 1) / chunk);
        if (wgs >= target_wgs || (chunk <= 1024 && wgs >= std::max<int64_t>(target_wgs / 4, 1024))) break;
        if (tiny && chunk <= 1024 && wgs >= 256) break;
        chunk /= 2;
    }
    return chunk;
}

}  // namespace

extern "C" {

int h1bkv_version(void) { return 100; }

const char *h1bkv_strerror(int code) {
    switch (code) {
        case H1BKV_OK: return "ok";
        case H1BKV_EINVAL: return "invalid argument value";
        case H1BKV_ENULL: return "required pointer is NULL";
        case H1BKV_ESHAPE: return "shape or configuration constraint violated";
        case H1BKV_ENOSPACE: return "page pool exhausted or sequence page limit reached";
        case H1BKV_ERANGE: return "sequence id, head or token range out of bounds";
        case H1BKV_EWORKSPACE: return "workspace or pool too small";
        case H1BKV_EHIP: return "HIP runtime call failed or wrong current device";
        case H1BKV_ENODEVICE: return "bookkeeping-only handle: call needs a GPU";
        default: return "unknown error code";
    }
}

size_t h1bkv_pool_bytes(const h1bkv_config *cfg) {
    if (!config_ok(cfg)) return 0;
    return make_layout(*cfg).total;
}

int h1bkv_create(const h1bkv_config *cfg, void *pool_dev, size_t pool_bytes, const float *R_host, h1bkv_cache **out) {
    if (!cfg || !out) return H1BKV_ENULL;
    if (!config_ok(cfg)) return H1BKV_ESHAPE;
    const bool dry = cfg->device == H1BKV_DEVICE_NONE;
    Layout lay = make_layout(*cfg);
    if (!dry) {
        if (!pool_dev) return H1BKV_ENULL;
        if (reinterpret_cast<uintptr_t>(pool_dev) % kAlign != 0) return H1BKV_EINVAL;
        if (pool_bytes < lay.total) return H1BKV_EWORKSPACE;
    }
    h1bkv_cache *c = new (std::nothrow) h1bkv_cache();
    if (!c) return H1BKV_EINVAL;
    c->cfg = *cfg;
    c->cfg.page_tokens = kPage;
    c->lay = lay;
    c->W = cfg->sketch_bits / 64;
    c->ng = cfg->head_dim / cfg->group_size;
    c->r = cfg->n_q_heads / cfg->n_kv_heads;
    c->cfg.value_bits = cfg->value_bits == 16 ? 16 : 4;
    c->code_layout = c->cfg.value_bits == 16 ? 2 : mfma_decode_supported(cfg->n_q_heads / cfg->n_kv_heads, cfg->head_dim, cfg->group_size, cfg->sketch_bits) ? 1 : 0;
    c->dry = dry;
    c->pool = static_cast<char *>(pool_dev);
    const size_t nR = (size_t)cfg->sketch_bits * cfg->head_dim;
    if (R_host) {
        c->R.assign(R_host, R_host + nR);
    } else {
        c->R.resize(nR);           // nR is even: b is a multiple of 64
        draw_projection(cfg->seed, c->R);
    }
    R_host = c->R.data();
    c->seq_len.assign(cfg->max_seqs, 0);
    c->seq_pages.assign(cfg->max_seqs, {});
    c->seen.assign(cfg->max_seqs, 0);
    c->free_list.resize(cfg->max_pages);
    for (int i = 0; i < cfg->max_pages; ++i) c->free_list[i] = cfg->max_pages - 1 - i;  // page 0 is taken first
    c->chunk_override = 0;
    c->proj_mfma = 1;
    c->fail_countdown = 0;
    c->prof_cap = 0;
    c->prof_mask = 0;
    c->prof_stride = 1;
    for (int k = 0; k < H1BKV_K_COUNT; ++k) c->prof_seen[k] = 0;
    for (int k = 0; k < H1BKV_K_COUNT; ++k) c->prof_used[k] = 0;
    if (!dry) {
        if (check_device(c) != H1BKV_OK) {
            delete c;
            return H1BKV_EHIP;
        }
        std::vector<float> RT(nR);
        for (int i = 0; i < cfg->sketch_bits; ++i)
            for (int j = 0; j < cfg->head_dim; ++j) RT[(size_t)j * cfg->sketch_bits + i] = R_host[(size_t)i * cfg->head_dim + j];
        bool ok = hipDeviceSynchronize() == hipSuccess;
        ok = ok && scratch_for_device(cfg->device) != nullptr;
        ok = ok && hipMemcpy(c->pool + lay.off_R, R_host, nR * sizeof(float), hipMemcpyHostToDevice) == hipSuccess;
        ok = ok && hipMemcpy(c->pool + lay.off_RT, RT.data(), nR * sizeof(float), hipMemcpyHostToDevice) == hipSuccess;
        std::vector<uint16_t> hi, mid;
        std::vector<float> guard;
        make_projection_pieces(R_host, cfg->sketch_bits, cfg->head_dim, hi, mid, guard);
        ok = ok && hipMemcpy(c->pool + lay.off_R16hi, hi.data(), nR * sizeof(uint16_t), hipMemcpyHostToDevice) == hipSuccess;
        ok = ok && hipMemcpy(c->pool + lay.off_R16mid, mid.data(), nR * sizeof(uint16_t), hipMemcpyHostToDevice) == hipSuccess;
        ok = ok && hipMemcpy(c->pool + lay.off_guard, guard.data(), guard.size() * sizeof(float), hipMemcpyHostToDevice) == hipSuccess;
        ok = ok && hipMemset(c->pool + lay.off_bt, 0, ((size_t)cfg->max_seqs * cfg->max_pages_per_seq + 64) * sizeof(int32_t)) == hipSuccess;
        ok = ok && hipDeviceSynchronize() == hipSuccess;
        if (!ok) {
            delete c;
            return H1BKV_EHIP;
        }
    }
    *out = c;
    return H1BKV_OK;
}

int h1bkv_destroy(h1bkv_cache *c) {
    if (!c) return H1BKV_OK;
    release_events(c);
    delete c;
    return H1BKV_OK;
}

int h1bkv_get_projection(const h1bkv_cache *c, float *R_host_out) {
    if (!c || !R_host_out) return H1BKV_ENULL;
    std::memcpy(R_host_out, c->R.data(), c->R.size() * sizeof(float));
    return H1BKV_OK;
}

int h1bkv_seq_len(const h1bkv_cache *c, int32_t seq_id, int32_t *len_out) {
    if (!c || !len_out) return H1BKV_ENULL;
    if (seq_id < 0 || seq_id >= c->cfg.max_seqs) return H1BKV_ERANGE;
    *len_out = c->seq_len[seq_id];
    return H1BKV_OK;
}

int h1bkv_free_pages(const h1bkv_cache *c, int32_t *n_out) {
    if (!c || !n_out) return H1BKV_ENULL;
    *n_out = (int32_t)c->free_list.size();
    return H1BKV_OK;
}

int h1bkv_truncate_seq(h1bkv_cache *c, int32_t seq_id, int32_t new_len) {
    if (!c) return H1BKV_ENULL;
    if (seq_id < 0 || seq_id >= c->cfg.max_seqs) return H1BKV_ERANGE;
    if (new_len < 0 || new_len > c->seq_len[seq_id]) return H1BKV_ERANGE;
    auto &pg = c->seq_pages[seq_id];
    while ((int)pg.size() > pages_for(new_len)) {
        c->free_list.push_back(pg.back());
        pg.pop_back();
    }
    c->seq_len[seq_id] = new_len;
    return H1BKV_OK;
}

int h1bkv_reset_seq(h1bkv_cache *c, int32_t seq_id) { return h1bkv_truncate_seq(c, seq_id, 0); }

int h1bkv_set_decode_chunk(h1bkv_cache *c, int32_t chunk_tokens) {
    if (!c) return H1BKV_ENULL;
    if (chunk_tokens != 0 && (chunk_tokens < kPage || chunk_tokens > max_decode_chunk(c->r, c->code_layout) || chunk_tokens % kPage != 0)) return H1BKV_EINVAL;
    c->chunk_override = chunk_tokens;
    return H1BKV_OK;
}

int h1bkv_debug_fail_launch(h1bkv_cache *c, int32_t nth) {
    if (!c) return H1BKV_ENULL;
    if (nth < 0) return H1BKV_EINVAL;
    c->fail_countdown = nth;
    return H1BKV_OK;
}

int h1bkv_set_projection_path(h1bkv_cache *c, int32_t use_matrix_cores) {
    if (!c) return H1BKV_ENULL;
    if (use_matrix_cores != 0 && use_matrix_cores != 1) return H1BKV_EINVAL;
    c->proj_mfma = use_matrix_cores;
    return H1BKV_OK;
}

int h1bkv_extend_seq(h1bkv_cache *c, int32_t seq_id, int32_t n_new, void *hip_stream) {
    if (!c) return H1BKV_ENULL;
    if (seq_id < 0 || seq_id >= c->cfg.max_seqs) return H1BKV_ERANGE;
    if (n_new < 1) return H1BKV_EINVAL;
    const int64_t new_len = (int64_t)c->seq_len[seq_id] + n_new;
    const int need = pages_needed(c, seq_id, new_len);
    if (need < 0) return need;
    if (need > (int)c->free_list.size()) return H1BKV_ENOSPACE;
    if (!c->dry) {
        int rc = check_device(c);
        if (rc != H1BKV_OK) return rc;
    }
    std::vector<int32_t> ui, up;
    const int32_t old_len = c->seq_len[seq_id];
    take_pages(c, seq_id, (int32_t)new_len, ui, up);
    c->seq_len[seq_id] = (int32_t)new_len;
    const int rc = publish(c, ui, up, static_cast<hipStream_t>(hip_stream));
    if (rc != H1BKV_OK) h1bkv_truncate_seq(c, seq_id, old_len);   // pages back, length as before
    return rc;
}

// Everything h1bkv_append_kv checks before it touches the bookkeeping.
static int validate_append(const h1bkv_cache *c, const int32_t *seq_ids_host, int32_t n_seqs, int32_t n_new, const void *k_dev,
                           const void *v_dev, int64_t stride_seq, int64_t stride_tok, int64_t stride_head) {
    int rc = check_seq_ids(c, seq_ids_host, n_seqs);
    if (rc != H1BKV_OK) return rc;
    if (n_new < 1) return H1BKV_EINVAL;
    if (!c->dry && (!k_dev || !v_dev)) return H1BKV_ENULL;
    if (stride_seq < 0 || stride_tok < 0 || stride_head < c->cfg.head_dim) return H1BKV_EINVAL;
    const int elt = c->cfg.in_dtype == H1BKV_F16 ? 2 : 4;
    if (!c->dry) {
        // rows are read with 16-byte loads
        if (reinterpret_cast<uintptr_t>(k_dev) % 16 || reinterpret_cast<uintptr_t>(v_dev) % 16) return H1BKV_EINVAL;
        if ((stride_seq * elt) % 16 || (stride_tok * elt) % 16 || (stride_head * elt) % 16) return H1BKV_EINVAL;
    }
    int64_t need_total = 0;
    for (int i = 0; i < n_seqs; ++i) {
        const int need = pages_needed(c, seq_ids_host[i], (int64_t)c->seq_len[seq_ids_host[i]] + n_new);
        if (need < 0) return need;
        need_total += need;
    }
    if (need_total > (int64_t)c->free_list.size()) return H1BKV_ENOSPACE;
    return c->dry ? H1BKV_OK : check_device(c);
}

// Takes pages, publishes them and launches the append kernel(s).  With q_dev != nullptr each launch also sketches
// the queries of its sequences into q_sketch_dev (fused decode-step prologue).  Arguments are already validated.
// With dev != nullptr the positions are device-resident (h1bkv_decode_step_dev): the pages were reserved beforehand, the
// kernels read where each sequence ends, and the host's lengths do not change.
static int enqueue_append(h1bkv_cache *c, const int32_t *seq_ids_host, int32_t n_seqs, int32_t n_new, const void *k_dev,
                          const void *v_dev, int64_t stride_seq, int64_t stride_tok, int64_t stride_head, const void *q_dev,
                          uint64_t *q_sketch_dev, hipStream_t st, const DevicePositions *dev = nullptr) {
    const int elt = c->cfg.in_dtype == H1BKV_F16 ? 2 : 4;
    std::vector<int32_t> ui, up;
    if (!dev)
        for (int i = 0; i < n_seqs; ++i) take_pages(c, seq_ids_host[i], c->seq_len[seq_ids_host[i]] + n_new, ui, up);
    int rc = publish(c, ui, up, st);
    if (rc == H1BKV_OK) {
        AppendArgs a{};
        a.pool = c->view();
        a.stride_seq = stride_seq;
        a.stride_tok = stride_tok;
        a.stride_head = stride_head;
        a.n_new = n_new;
        a.f16 = c->cfg.in_dtype == H1BKV_F16;
        // prefill-sized appends take the matrix-core projection; short ones (a decode step's single token) stay on the
        // plain chain, which is launch-bound there anyway
        a.proj_mfma = n_new >= 16 && c->proj_mfma;
        for (int s0 = 0; s0 < n_seqs && rc == H1BKV_OK; s0 += kMaxSeqsPerLaunch) {
            const int n = std::min(kMaxSeqsPerLaunch, n_seqs - s0);
            BatchDesc desc;
            for (int i = 0; i < n; ++i) desc.s[i] = SeqDesc{seq_ids_host[s0 + i], dev ? 0 : c->seq_len[seq_ids_host[s0 + i]]};
            if (dev) {
                desc.pos_dev = dev->pos + s0;
                desc.pos_add = 0;
                desc.pos_max = dev->max_pos;
            }
            if (!c->dry) {
                a.k = static_cast<const char *>(k_dev) + (size_t)s0 * stride_seq * elt;
                a.v = static_cast<const char *>(v_dev) + (size_t)s0 * stride_seq * elt;
            }
            QueryArgs qa{};
            if (q_dev) {
                const size_t vec0 = (size_t)s0 * c->cfg.n_q_heads;
                qa.q = static_cast<const char *>(q_dev) + vec0 * c->cfg.head_dim * elt;
                qa.q_sketch = q_sketch_dev + vec0 * c->W;
                qa.n_vec = n * c->cfg.n_q_heads;
            }
            if (!launch_allowed(c)) {
                rc = H1BKV_EHIP;
            } else if (!c->dry) {
                Timed t(c, H1BKV_K_APPEND, st);
                if (launch_append(a, desc, n, q_dev ? &qa : nullptr, st) != hipSuccess) rc = H1BKV_EHIP;
            }
        }
    }
    if (rc != H1BKV_OK) {
        // A launch failed: give the pages taken above back, so the bookkeeping is as it was before the call (with
        // device-resident positions none were taken, and the reserved ones stay).
        if (!dev)
            for (int i = 0; i < n_seqs; ++i) h1bkv_truncate_seq(c, seq_ids_host[i], c->seq_len[seq_ids_host[i]]);
        return rc;
    }
    if (!dev)
        for (int i = 0; i < n_seqs; ++i) c->seq_len[seq_ids_host[i]] += n_new;
    return H1BKV_OK;
}

int h1bkv_append_kv(h1bkv_cache *c, const int32_t *seq_ids_host, int32_t n_seqs, int32_t n_new, const void *k_dev,
                    const void *v_dev, int64_t stride_seq, int64_t stride_tok, int64_t stride_head, void *hip_stream) {
    if (!c) return H1BKV_ENULL;
    const int rc = validate_append(c, seq_ids_host, n_seqs, n_new, k_dev, v_dev, stride_seq, stride_tok, stride_head);
    if (rc != H1BKV_OK) return rc;
    return enqueue_append(c, seq_ids_host, n_seqs, n_new, k_dev, v_dev, stride_seq, stride_tok, stride_head, nullptr, nullptr,
                          static_cast<hipStream_t>(hip_stream));
}

size_t h1bkv_decode_workspace_bytes(const h1bkv_cache *c, int32_t n_seqs, int32_t max_ctx) {
    if (!c || n_seqs < 1 || max_ctx < 0) return 0;
    const size_t heads = (size_t)n_seqs * c->cfg.n_q_heads;
    const size_t max_splits = std::max(1, pages_for(max_ctx));   // worst case: one page per chunk
    size_t o = align_up(heads * c->W * 8);
    o = align_up(o + heads * max_splits * 2 * sizeof(float));
    o = align_up(o + heads * max_splits * c->cfg.head_dim * sizeof(float));
    return o;
}

// Workspace bytes one decode call really uses: query sketches and the partial results of the chunks it will launch
// (h1bkv_decode_workspace_bytes is the bound for any chunk choice).
static size_t decode_workspace_used(const h1bkv_cache *c, int32_t n_seqs, int max_ctx) {
    const int chunk = choose_chunk(c, n_seqs, max_ctx);
    const size_t S = std::max(1, (max_ctx + chunk - 1) / chunk);
    const size_t heads = (size_t)n_seqs * c->cfg.n_q_heads;
    size_t o = align_up(heads * c->W * 8);
    o = align_up(o + heads * S * 2 * sizeof(float));
    o = align_up(o + heads * S * c->cfg.head_dim * sizeof(float));
    return o;
}

// Everything h1bkv_decode_attn checks; `grow` tokens are about to be appended to every sequence first.  With
// static_ws the workspace is the library's own scratch array: the call must fit into it.
static int validate_decode(const h1bkv_cache *c, const int32_t *seq_ids_host, int32_t n_seqs, const void *q_dev, float tau,
                           const float *out_dev, const void *workspace_dev, size_t workspace_bytes, int grow,
                           bool static_ws = false) {
    int rc = check_seq_ids(c, seq_ids_host, n_seqs);
    if (rc != H1BKV_OK) return rc;
    if (!(tau > 0.0f) || !std::isfinite(tau)) return H1BKV_EINVAL;
    int max_ctx = 0;
    for (int i = 0; i < n_seqs; ++i) max_ctx = std::max(max_ctx, c->seq_len[seq_ids_host[i]] + grow);
    if (static_ws && decode_workspace_used(c, n_seqs, max_ctx) > (size_t)H1BKV_STATIC_SCRATCH_BYTES) return H1BKV_EWORKSPACE;
    if (c->dry) return H1BKV_ENODEVICE;
    if (!q_dev || !out_dev || (!static_ws && !workspace_dev)) return H1BKV_ENULL;
    if (reinterpret_cast<uintptr_t>(workspace_dev) % kAlign || reinterpret_cast<uintptr_t>(q_dev) % 16 ||
        reinterpret_cast<uintptr_t>(out_dev) % 16)
        return H1BKV_EINVAL;
    if (!static_ws && workspace_bytes < h1bkv_decode_workspace_bytes(c, n_seqs, max_ctx)) return H1BKV_EWORKSPACE;
    return check_device(c);
}

// Launches (query sketch,) split decode and merge for validated arguments.
// With dev != nullptr the context lengths are device-resident: every sequence attends over pos[i] + 1 tokens (the token the
// step's prologue has just appended included), and the launch is sized for max_pos tokens.
static int enqueue_decode(h1bkv_cache *c, const int32_t *seq_ids_host, int32_t n_seqs, const void *q_dev, float tau,
                          float *out_dev, void *workspace_dev, bool sketches_done, hipStream_t st,
                          const DevicePositions *dev = nullptr) {
    int max_ctx = dev ? dev->max_pos : 0;
    if (!dev)
        for (int i = 0; i < n_seqs; ++i) max_ctx = std::max(max_ctx, c->seq_len[seq_ids_host[i]]);
    const int chunk = choose_chunk(c, n_seqs, max_ctx);
    const int S = std::max(1, (max_ctx + chunk - 1) / chunk);
    const size_t heads = (size_t)n_seqs * c->cfg.n_q_heads;
    char *ws = static_cast<char *>(workspace_dev);
    DecodeArgs a{};
    a.pool = c->view();
    a.q = q_dev;
    a.q_sketch = reinterpret_cast<uint64_t *>(ws);
    size_t o = align_up(heads * c->W * 8);
    a.part_ml = reinterpret_cast<float *>(ws + o);
    o = align_up(o + heads * S * 2 * sizeof(float));
    a.part_o = reinterpret_cast<float *>(ws + o);
    a.out = out_dev;
    a.n_splits = S;
    a.chunk = chunk;
    a.f16 = c->cfg.in_dtype == H1BKV_F16;
    a.exp2_scale = (float)(2.0 * 1.4426950408889634 / ((double)c->cfg.sketch_bits * (double)tau));

    for (int s0 = 0; s0 < n_seqs; s0 += kMaxSeqsPerLaunch) {
        const int n = std::min(kMaxSeqsPerLaunch, n_seqs - s0);
        BatchDesc desc;
        for (int i = 0; i < n; ++i) desc.s[i] = SeqDesc{seq_ids_host[s0 + i], dev ? 0 : c->seq_len[seq_ids_host[s0 + i]]};
        if (dev) {
            desc.pos_dev = dev->pos + s0;
            desc.pos_add = 1;
            desc.pos_max = dev->max_pos;
            desc.advance = dev->advance;      // (read by the merge kernels only)
        }
        if (!sketches_done) {
            Timed t(c, H1BKV_K_QSKETCH, st);
            // Thousands of fp16 queries (large batches): the prefill path's matrix-core projection with its guard band
            // (same bits as the chain); the queries are then one position per sequence.
            const bool mfma_q = c->proj_mfma && c->cfg.head_dim <= 128 && (int64_t)n * c->cfg.n_q_heads >= 2048;
            if (mfma_q) {
                PrefillArgs pa{};
                pa.pool = a.pool;
                pa.q = static_cast<const char *>(q_dev) + (size_t)s0 * c->cfg.n_q_heads * c->cfg.head_dim * (a.f16 ? 2 : 4);
                pa.stride_seq = (int64_t)c->cfg.n_q_heads * c->cfg.head_dim;
                pa.stride_tok = 0;
                pa.stride_head = c->cfg.head_dim;
                pa.q_sketch = a.q_sketch + (size_t)s0 * c->cfg.n_q_heads * c->W;
                pa.n_q = 1;
                pa.f16 = a.f16;
                pa.proj_mfma = 1;
                if (!launch_allowed(c) || launch_sketch_rows(pa, n, st) != hipSuccess) return H1BKV_EHIP;
            } else if (!launch_allowed(c) || launch_qsketch(a, s0, n, st) != hipSuccess) {
                return H1BKV_EHIP;
            }
        }
        if (!launch_allowed(c)) return H1BKV_EHIP;
        {
            Timed t(c, H1BKV_K_DECODE_SPLIT, st);
            const hipError_t e = c->code_layout == 2   ? launch_decode_split_f16v(a, desc, s0, n, st)
                                 : c->code_layout == 1 ? launch_decode_split_mfma(a, desc, s0, n, st)
                                                       : launch_decode_split(a, desc, s0, n, st);
            if (e != hipSuccess) return H1BKV_EHIP;
        }
        if (!launch_allowed(c)) return H1BKV_EHIP;
        {
            Timed t(c, H1BKV_K_MERGE, st);
            if (launch_merge(a, desc, s0, n, st) != hipSuccess) return H1BKV_EHIP;
        }
    }
    return H1BKV_OK;
}

int h1bkv_decode_attn(h1bkv_cache *c, const int32_t *seq_ids_host, int32_t n_seqs, const void *q_dev, float tau,
                      float *out_dev, void *workspace_dev, size_t workspace_bytes, void *hip_stream) {
    if (!c) return H1BKV_ENULL;
    const int rc = validate_decode(c, seq_ids_host, n_seqs, q_dev, tau, out_dev, workspace_dev, workspace_bytes, 0);
    if (rc != H1BKV_OK) return rc;
    return enqueue_decode(c, seq_ids_host, n_seqs, q_dev, tau, out_dev, workspace_dev, false, static_cast<hipStream_t>(hip_stream));
}

int h1bkv_decode_attn_static(h1bkv_cache *c, const int32_t *seq_ids_host, int32_t n_seqs, const void *q_dev, float tau,
                             float *out_dev, void *hip_stream) {
    if (!c) return H1BKV_ENULL;
    const int rc = validate_decode(c, seq_ids_host, n_seqs, q_dev, tau, out_dev, nullptr, 0, 0, true);
    if (rc != H1BKV_OK) return rc;
    // the address of this device's copy of the array was looked up when the handle was created; nothing is allocated here
    unsigned char *ws = scratch_for_device(c->cfg.device);
    if (!ws) return H1BKV_EHIP;
    return enqueue_decode(c, seq_ids_host, n_seqs, q_dev, tau, out_dev, ws, false, static_cast<hipStream_t>(hip_stream));
}

int h1bkv_decode_step(h1bkv_cache *c, const int32_t *seq_ids_host, int32_t n_seqs, const void *k_dev, const void *v_dev,
                      int64_t stride_seq, int64_t stride_head, const void *q_dev, float tau, float *out_dev,
                      void *workspace_dev, size_t workspace_bytes, void *hip_stream) {
    if (!c) return H1BKV_ENULL;
    // both halves are validated before anything changes
    int rc = validate_decode(c, seq_ids_host, n_seqs, q_dev, tau, out_dev, workspace_dev, workspace_bytes, 1);
    if (rc != H1BKV_OK) return rc;
    rc = validate_append(c, seq_ids_host, n_seqs, 1, k_dev, v_dev, stride_seq, 0, stride_head);
    if (rc != H1BKV_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    // the query sketches sit at the start of the workspace (see enqueue_decode)
    rc = enqueue_append(c, seq_ids_host, n_seqs, 1, k_dev, v_dev, stride_seq, 0, stride_head, q_dev,
                        static_cast<uint64_t *>(workspace_dev), st);
    if (rc != H1BKV_OK) return rc;
    rc = enqueue_decode(c, seq_ids_host, n_seqs, q_dev, tau, out_dev, workspace_dev, true, st);
    if (rc != H1BKV_OK) {
        // the decode half failed to launch: take the appended token back, so that the call has changed no length and no
        // page assignment (the record written past the old length is invisible and will be overwritten)
        for (int i = 0; i < n_seqs; ++i) h1bkv_truncate_seq(c, seq_ids_host[i], c->seq_len[seq_ids_host[i]] - 1);
    }
    return rc;
}

int h1bkv_reserve_seq(h1bkv_cache *c, int32_t seq_id, int32_t n_tokens, void *hip_stream) {
    if (!c) return H1BKV_ENULL;
    if (seq_id < 0 || seq_id >= c->cfg.max_seqs) return H1BKV_ERANGE;
    if (n_tokens < 0) return H1BKV_EINVAL;
    const int64_t upto = (int64_t)c->seq_len[seq_id] + n_tokens;
    const int need = pages_needed(c, seq_id, upto);
    if (need < 0) return need;
    if (need > (int)c->free_list.size()) return H1BKV_ENOSPACE;
    if (!c->dry) {
        const int rc = check_device(c);
        if (rc != H1BKV_OK) return rc;
    }
    std::vector<int32_t> ui, up;
    take_pages(c, seq_id, (int32_t)upto, ui, up);
    const int rc = publish(c, ui, up, static_cast<hipStream_t>(hip_stream));
    if (rc != H1BKV_OK) h1bkv_truncate_seq(c, seq_id, c->seq_len[seq_id]);   // the pages taken go back
    return rc;
}

int h1bkv_reserved_tokens(const h1bkv_cache *c, int32_t seq_id, int32_t *n_out) {
    if (!c || !n_out) return H1BKV_ENULL;
    if (seq_id < 0 || seq_id >= c->cfg.max_seqs) return H1BKV_ERANGE;
    *n_out = (int32_t)c->seq_pages[seq_id].size() * kPage;
    return H1BKV_OK;
}

int h1bkv_set_seq_len(h1bkv_cache *c, int32_t seq_id, int32_t new_len) {
    if (!c) return H1BKV_ENULL;
    if (seq_id < 0 || seq_id >= c->cfg.max_seqs) return H1BKV_ERANGE;
    if (new_len < c->seq_len[seq_id] || pages_for(new_len) > (int)c->seq_pages[seq_id].size()) return H1BKV_ERANGE;
    c->seq_len[seq_id] = new_len;
    return H1BKV_OK;
}

int h1bkv_decode_step_dev(h1bkv_cache *c, const int32_t *seq_ids_host, int32_t n_seqs, const void *k_dev, const void *v_dev,
                          int64_t stride_seq, int64_t stride_head, const void *q_dev, float tau, float *out_dev,
                          int32_t *pos_dev, int32_t max_pos, int32_t advance, void *workspace_dev, size_t workspace_bytes,
                          void *hip_stream) {
    if (!c) return H1BKV_ENULL;
    int rc = check_seq_ids(c, seq_ids_host, n_seqs);
    if (rc != H1BKV_OK) return rc;
    if (!(tau > 0.0f) || !std::isfinite(tau) || max_pos < 1 || (advance != 0 && advance != 1)) return H1BKV_EINVAL;
    // every position the kernels may touch has a page already: nothing is assigned while the step runs (or replays)
    for (int i = 0; i < n_seqs; ++i)
        if (pages_for(max_pos) > (int)c->seq_pages[seq_ids_host[i]].size()) return H1BKV_ERANGE;
    if (stride_seq < 0 || stride_head < c->cfg.head_dim) return H1BKV_EINVAL;
    if (c->dry) return H1BKV_ENODEVICE;
    if (!k_dev || !v_dev || !q_dev || !out_dev || !pos_dev || !workspace_dev) return H1BKV_ENULL;
    const int elt = c->cfg.in_dtype == H1BKV_F16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(k_dev) % 16 || reinterpret_cast<uintptr_t>(v_dev) % 16 ||
        reinterpret_cast<uintptr_t>(q_dev) % 16 || reinterpret_cast<uintptr_t>(out_dev) % 16 ||
        reinterpret_cast<uintptr_t>(pos_dev) % 4 || reinterpret_cast<uintptr_t>(workspace_dev) % kAlign ||
        (stride_seq * elt) % 16 || (stride_head * elt) % 16)
        return H1BKV_EINVAL;
    if (workspace_bytes < h1bkv_decode_workspace_bytes(c, n_seqs, max_pos)) return H1BKV_EWORKSPACE;
    rc = check_device(c);
    if (rc != H1BKV_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const DevicePositions dev{pos_dev, max_pos, advance};
    rc = enqueue_append(c, seq_ids_host, n_seqs, 1, k_dev, v_dev, stride_seq, 0, stride_head, q_dev,
                        static_cast<uint64_t *>(workspace_dev), st, &dev);
    if (rc != H1BKV_OK) return rc;
    // (the merge, the step's last kernel, advances the positions if asked to; if a launch fails before it they stay as
    // they are and the appended records lie past every sequence's end)
    return enqueue_decode(c, seq_ids_host, n_seqs, q_dev, tau, out_dev, workspace_dev, true, st, &dev);
}

size_t h1bkv_decode_dtau_workspace_bytes(const h1bkv_cache *c, int32_t n_seqs, int32_t max_ctx) {
    if (!c || n_seqs < 1 || max_ctx < 0) return 0;
    const size_t heads = (size_t)n_seqs * c->cfg.n_q_heads;
    const size_t max_splits = std::max(1, pages_for(max_ctx));   // worst case: one page per chunk
    size_t o = align_up(heads * c->W * 8);
    o = align_up(o + heads * max_splits * 4 * sizeof(float));
    o = align_up(o + heads * max_splits * c->cfg.head_dim * sizeof(float));
    o = align_up(o + heads * max_splits * c->cfg.head_dim * sizeof(float));
    return o;
}

int h1bkv_decode_attn_dtau(h1bkv_cache *c, const int32_t *seq_ids_host, int32_t n_seqs, const void *q_dev, float tau,
                           float *out_dev, float *dout_dtau_dev, void *workspace_dev, size_t workspace_bytes,
                           void *hip_stream) {
    if (!c) return H1BKV_ENULL;
    int rc = check_seq_ids(c, seq_ids_host, n_seqs);
    if (rc != H1BKV_OK) return rc;
    if (!(tau > 0.0f) || !std::isfinite(tau)) return H1BKV_EINVAL;
    if (c->dry) return H1BKV_ENODEVICE;
    if (!q_dev || !out_dev || !dout_dtau_dev || !workspace_dev) return H1BKV_ENULL;
    if (reinterpret_cast<uintptr_t>(workspace_dev) % kAlign || reinterpret_cast<uintptr_t>(q_dev) % 16 ||
        reinterpret_cast<uintptr_t>(out_dev) % 16 || reinterpret_cast<uintptr_t>(dout_dtau_dev) % 16)
        return H1BKV_EINVAL;
    int max_ctx = 0;
    for (int i = 0; i < n_seqs; ++i) max_ctx = std::max(max_ctx, c->seq_len[seq_ids_host[i]]);
    if (workspace_bytes < h1bkv_decode_dtau_workspace_bytes(c, n_seqs, max_ctx)) return H1BKV_EWORKSPACE;
    rc = check_device(c);
    if (rc != H1BKV_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);

    const int chunk = choose_chunk(c, n_seqs, max_ctx, true);
    const int S = std::max(1, (max_ctx + chunk - 1) / chunk);
    const size_t heads = (size_t)n_seqs * c->cfg.n_q_heads;
    char *ws = static_cast<char *>(workspace_dev);
    DecodeArgs a{};
    a.pool = c->view();
    a.q = q_dev;
    a.q_sketch = reinterpret_cast<uint64_t *>(ws);
    size_t o = align_up(heads * c->W * 8);
    a.part_ml = reinterpret_cast<float *>(ws + o);
    o = align_up(o + heads * S * 4 * sizeof(float));
    a.part_o = reinterpret_cast<float *>(ws + o);
    o = align_up(o + heads * S * c->cfg.head_dim * sizeof(float));
    a.part_oh = reinterpret_cast<float *>(ws + o);
    a.out = out_dev;
    a.dout = dout_dtau_dev;
    a.n_splits = S;
    a.chunk = chunk;
    a.f16 = c->cfg.in_dtype == H1BKV_F16;
    a.exp2_scale = (float)(2.0 * 1.4426950408889634 / ((double)c->cfg.sketch_bits * (double)tau));
    const float dtau_scale = (float)(2.0 / ((double)c->cfg.sketch_bits * (double)tau * (double)tau));
    for (int s0 = 0; s0 < n_seqs; s0 += kMaxSeqsPerLaunch) {
        const int n = std::min(kMaxSeqsPerLaunch, n_seqs - s0);
        BatchDesc desc;
        for (int i = 0; i < n; ++i) desc.s[i] = SeqDesc{seq_ids_host[s0 + i], c->seq_len[seq_ids_host[s0 + i]]};
        {
            Timed t(c, H1BKV_K_QSKETCH, st);
            if (!launch_allowed(c) || launch_qsketch(a, s0, n, st) != hipSuccess) return H1BKV_EHIP;
        }
        {
            Timed t(c, H1BKV_K_DECODE_SPLIT, st);
            if (!launch_allowed(c)) return H1BKV_EHIP;
            const hipError_t e = c->code_layout == 2   ? launch_decode_dtau_split_f16v(a, desc, s0, n, st)
                                 : c->code_layout == 1 ? launch_decode_dtau_split_mfma(a, desc, s0, n, st)
                                                       : launch_decode_dtau_split(a, desc, s0, n, st);
            if (e != hipSuccess) return H1BKV_EHIP;
        }
        {
            Timed t(c, H1BKV_K_MERGE, st);
            if (!launch_allowed(c) || launch_merge_dtau(a, desc, s0, n, dtau_scale, st) != hipSuccess) return H1BKV_EHIP;
        }
    }
    return H1BKV_OK;
}

size_t h1bkv_prefill_workspace_bytes(const h1bkv_cache *c, int32_t n_seqs, int32_t n_q) {
    if (!c || n_seqs < 1 || n_q < 1) return 0;
    const size_t rows = (size_t)n_seqs * n_q * c->cfg.n_q_heads;
    const int splits = prefill_max_splits(c->cfg.n_q_heads, n_seqs, n_q);
    size_t o = align_up(rows * c->W * 8);                                        // the chunk's query sketches
    if (splits > 1) o = align_up(o + rows * splits * (c->cfg.head_dim + 2) * sizeof(float));   // partial results per context split
    return o;
}

int h1bkv_prefill_attn(h1bkv_cache *c, const int32_t *seq_ids_host, int32_t n_seqs, int32_t n_q, const void *q_dev,
                       int64_t stride_seq, int64_t stride_tok, int64_t stride_head, float tau, float *out_dev,
                       void *workspace_dev, size_t workspace_bytes, void *hip_stream) {
    if (!c) return H1BKV_ENULL;
    int rc = check_seq_ids(c, seq_ids_host, n_seqs);
    if (rc != H1BKV_OK) return rc;
    if (n_q < 1 || !(tau > 0.0f) || !std::isfinite(tau)) return H1BKV_EINVAL;
    for (int i = 0; i < n_seqs; ++i)
        if (c->seq_len[seq_ids_host[i]] < n_q) return H1BKV_ERANGE;
    if (stride_seq < 0 || stride_tok < 0 || stride_head < c->cfg.head_dim) return H1BKV_EINVAL;
    if (c->dry) return H1BKV_ENODEVICE;
    if (!q_dev || !out_dev || !workspace_dev) return H1BKV_ENULL;
    const int elt = c->cfg.in_dtype == H1BKV_F16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(workspace_dev) % kAlign || reinterpret_cast<uintptr_t>(q_dev) % 16 ||
        reinterpret_cast<uintptr_t>(out_dev) % 16 || (stride_seq * elt) % 16 || (stride_tok * elt) % 16 || (stride_head * elt) % 16)
        return H1BKV_EINVAL;
    if (workspace_bytes < h1bkv_prefill_workspace_bytes(c, n_seqs, n_q)) return H1BKV_EWORKSPACE;
    rc = check_device(c);
    if (rc != H1BKV_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);

    PrefillArgs a{};
    a.pool = c->view();
    a.q = q_dev;
    a.stride_seq = stride_seq;
    a.stride_tok = stride_tok;
    a.stride_head = stride_head;
    a.q_sketch = static_cast<uint64_t *>(workspace_dev);
    a.part = reinterpret_cast<float *>(static_cast<char *>(workspace_dev) + align_up((size_t)n_seqs * n_q * c->cfg.n_q_heads * c->W * 8));
    a.out = out_dev;
    a.n_q = n_q;
    // a chunk that is short against its context is split over the context as well: every split at least a page long
    int max_len = 0;
    for (int i = 0; i < n_seqs; ++i) max_len = std::max(max_len, c->seq_len[seq_ids_host[i]]);
    a.n_splits = std::max(1, std::min(prefill_max_splits(c->cfg.n_q_heads, n_seqs, n_q), max_len / kPage));
    a.f16 = c->cfg.in_dtype == H1BKV_F16;
    a.proj_mfma = c->proj_mfma && (int64_t)n_seqs * n_q * c->cfg.n_q_heads >= 64;
    a.exp2_scale = (float)(2.0 * 1.4426950408889634 / ((double)c->cfg.sketch_bits * (double)tau));
    {
        Timed t(c, H1BKV_K_QSKETCH, st);
        if (!launch_allowed(c) || launch_sketch_rows(a, n_seqs, st) != hipSuccess) return H1BKV_EHIP;
    }
    for (int s0 = 0; s0 < n_seqs; s0 += kMaxSeqsPerLaunch) {
        const int n = std::min(kMaxSeqsPerLaunch, n_seqs - s0);
        BatchDesc desc;
        for (int i = 0; i < n; ++i) desc.s[i] = SeqDesc{seq_ids_host[s0 + i], c->seq_len[seq_ids_host[s0 + i]]};
        Timed t(c, H1BKV_K_PREFILL, st);
        if (!launch_allowed(c) || launch_prefill(a, desc, s0, n, st) != hipSuccess) return H1BKV_EHIP;
        if (a.n_splits > 1 && (!launch_allowed(c) || launch_prefill_merge(a, s0, n, st) != hipSuccess)) return H1BKV_EHIP;
    }
    return H1BKV_OK;
}

static int xfer_tokens(const h1bkv_cache *c, int32_t seq_id, int32_t kv_head, int32_t t0, int32_t n, bool to_host,
                       uint64_t *sk, uint8_t *codes, uint16_t *scale, uint16_t *zero) {
    if (!c) return H1BKV_ENULL;
    if (seq_id < 0 || seq_id >= c->cfg.max_seqs || kv_head < 0 || kv_head >= c->cfg.n_kv_heads) return H1BKV_ERANGE;
    if (t0 < 0 || n < 0 || (int64_t)t0 + n > c->seq_len[seq_id]) return H1BKV_ERANGE;
    if (c->dry) return H1BKV_ENODEVICE;
    if ((scale == nullptr) != (zero == nullptr)) return H1BKV_ENULL;
    if (c->code_layout == 2 && scale) return H1BKV_EINVAL;          // fp16 values carry no scale/zero
    int rc = check_device(c);
    if (rc != H1BKV_OK) return rc;
    if (hipDeviceSynchronize() != hipSuccess) return H1BKV_EHIP;
    const PoolView pv = c->view();
    const size_t W = c->W, hb = c->code_layout == 2 ? 2 * (size_t)c->cfg.head_dim : c->cfg.head_dim / 2, ng = c->ng;
    std::vector<uint32_t> meta;
    const hipMemcpyKind kind = to_host ? hipMemcpyDeviceToHost : hipMemcpyHostToDevice;
    int32_t t = t0;
    while (t < t0 + n) {
        const int32_t page = c->seq_pages[seq_id][t / kPage];
        const int32_t slot = t % kPage;
        const int32_t run = std::min(kPage - slot, t0 + n - t);
        const size_t rec = ((size_t)page * c->cfg.n_kv_heads + kv_head) * kPage + slot;
        const size_t i = (size_t)(t - t0);
        bool ok = true;
        if (sk) {
            void *dev = pv.sketch + rec * W;
            ok = ok && hipMemcpy(to_host ? (void *)(sk + i * W) : dev, to_host ? dev : (void *)(sk + i * W), run * W * 8, kind) == hipSuccess;
        }
        if (codes && c->code_layout != 1) {
            void *dev = pv.codes + rec * hb;
            ok = ok && hipMemcpy(to_host ? (void *)(codes + i * hb) : dev, to_host ? dev : (void *)(codes + i * hb), run * hb, kind) == hipSuccess;
        }
        if (codes && c->code_layout == 1) {
            // token-interleaved words: move whole 8-token blocks and pick / patch the nibbles of the requested tokens
            const int d = c->cfg.head_dim;
            const int32_t b0 = slot / 8 * 8, b1 = (slot + run + 7) / 8 * 8;
            std::vector<uint32_t> blk((size_t)(b1 - b0) / 8 * d);
            void *dev = pv.codes + (rec - slot + b0) * hb;
            ok = ok && hipMemcpy(blk.data(), dev, blk.size() * 4, hipMemcpyDeviceToHost) == hipSuccess;
            for (int32_t s = slot; s < slot + run; ++s) {
                uint32_t *w = blk.data() + (size_t)(s - b0) / 8 * d;
                const int sh = 4 * code_nibble_pos(s & 7);
                uint8_t *canon = codes + (i + (s - slot)) * hb;
                for (int ch = 0; ch < d; ++ch) {
                    uint32_t &word = w[code_word_index(ch)];
                    if (to_host) {
                        const uint8_t nib = (word >> sh) & 0xF;
                        canon[ch / 2] = (ch & 1) ? (uint8_t)((canon[ch / 2] & 0x0F) | (nib << 4)) : (uint8_t)((canon[ch / 2] & 0xF0) | nib);
                    } else {
                        const uint32_t nib = (canon[ch / 2] >> (4 * (ch & 1))) & 0xF;
                        word = (word & ~(0xFu << sh)) | (nib << sh);
                    }
                }
            }
            if (!to_host) ok = ok && hipMemcpy(dev, blk.data(), blk.size() * 4, hipMemcpyHostToDevice) == hipSuccess;
        }
        if (scale) {
            void *dev = pv.meta + rec * ng;
            meta.resize(run * ng);
            if (to_host) {
                ok = ok && hipMemcpy(meta.data(), dev, run * ng * 4, kind) == hipSuccess;
                for (size_t e = 0; e < run * ng; ++e) {
                    scale[i * ng + e] = (uint16_t)(meta[e] & 0xFFFFu);
                    zero[i * ng + e] = (uint16_t)(meta[e] >> 16);
                }
            } else {
                for (size_t e = 0; e < run * ng; ++e) meta[e] = (uint32_t)scale[i * ng + e] | ((uint32_t)zero[i * ng + e] << 16);
                ok = ok && hipMemcpy(dev, meta.data(), run * ng * 4, kind) == hipSuccess;
            }
        }
        if (!ok) return H1BKV_EHIP;
        t += run;
    }
    return H1BKV_OK;
}

int h1bkv_export_tokens(const h1bkv_cache *c, int32_t seq_id, int32_t kv_head, int32_t t0, int32_t n,
                        uint64_t *sketch_out, uint8_t *codes_out, uint16_t *scale_out, uint16_t *zero_out) {
    return xfer_tokens(c, seq_id, kv_head, t0, n, true, sketch_out, codes_out, scale_out, zero_out);
}

int h1bkv_import_tokens(h1bkv_cache *c, int32_t seq_id, int32_t kv_head, int32_t t0, int32_t n,
                        const uint64_t *sketch_in, const uint8_t *codes_in, const uint16_t *scale_in,
                        const uint16_t *zero_in) {
    return xfer_tokens(c, seq_id, kv_head, t0, n, false, const_cast<uint64_t *>(sketch_in), const_cast<uint8_t *>(codes_in),
                       const_cast<uint16_t *>(scale_in), const_cast<uint16_t *>(zero_in));
}

int h1bkv_profile_enable(h1bkv_cache *c, int32_t capacity, uint32_t kernel_mask) {
    if (!c) return H1BKV_ENULL;
    if (capacity < 0) return H1BKV_EINVAL;
    if (c->dry) return capacity == 0 ? H1BKV_OK : H1BKV_ENODEVICE;
    release_events(c);
    if (capacity == 0) return H1BKV_OK;
    int rc = check_device(c);
    if (rc != H1BKV_OK) return rc;
    c->prof_mask = kernel_mask;
    for (int k = 0; k < H1BKV_K_COUNT; ++k) {
        if (!((kernel_mask >> k) & 1u)) continue;
        c->prof_events[k].resize(capacity);
        for (auto &e : c->prof_events[k]) {
            if (hipEventCreate(&e.a) != hipSuccess || hipEventCreate(&e.b) != hipSuccess) return H1BKV_EHIP;
        }
    }
    c->prof_cap = capacity;
    return H1BKV_OK;
}

int h1bkv_profile_stride(h1bkv_cache *c, int32_t stride) {
    if (!c) return H1BKV_ENULL;
    if (stride < 1) return H1BKV_EINVAL;
    c->prof_stride = stride;
    for (int k = 0; k < H1BKV_K_COUNT; ++k) c->prof_seen[k] = 0;
    return H1BKV_OK;
}

int h1bkv_profile_read(h1bkv_cache *c, int32_t kernel, float *ms_out, int32_t cap, int32_t *n_out) {
    if (!c || !n_out || (!ms_out && cap > 0)) return H1BKV_ENULL;
    if (kernel < 0 || kernel >= H1BKV_K_COUNT || cap < 0) return H1BKV_EINVAL;
    int n = 0;
    for (int i = 0; i < c->prof_used[kernel]; ++i) {
        auto &e = c->prof_events[kernel][i];
        if (hipEventSynchronize(e.b) != hipSuccess) return H1BKV_EHIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, e.a, e.b) != hipSuccess) return H1BKV_EHIP;
        if (n < cap) ms_out[n++] = ms;
    }
    c->prof_used[kernel] = 0;
    *n_out = n;
    return H1BKV_OK;
}

int h1bkv_stream_copy(void *dst_dev, const void *src_dev, size_t n_bytes, void *hip_stream) {
    if (!dst_dev || !src_dev) return H1BKV_ENULL;
    if (n_bytes % 16 || reinterpret_cast<uintptr_t>(dst_dev) % 16 || reinterpret_cast<uintptr_t>(src_dev) % 16) return H1BKV_EINVAL;
    if (n_bytes == 0) return H1BKV_OK;
    return launch_stream_copy(dst_dev, src_dev, n_bytes, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? H1BKV_OK : H1BKV_EHIP;
}

int h1bkv_stream_read(const void *src_dev, size_t n_bytes, void *sink_dev, void *hip_stream) {
    if (!src_dev || !sink_dev) return H1BKV_ENULL;
    if (n_bytes % 16 || reinterpret_cast<uintptr_t>(src_dev) % 16 || reinterpret_cast<uintptr_t>(sink_dev) % 16) return H1BKV_EINVAL;
    if (n_bytes == 0) return H1BKV_OK;
    return launch_stream_read(src_dev, n_bytes, sink_dev, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? H1BKV_OK : H1BKV_EHIP;
}

int h1bkv_stream_read_ms(const void *src_dev, size_t n_bytes, void *sink_dev, void *hip_stream, float *ms_out) {
    if (!ms_out) return H1BKV_ENULL;
    *ms_out = 0.0f;
    if (!src_dev || !sink_dev) return H1BKV_ENULL;
    if (n_bytes == 0 || n_bytes % 16 || reinterpret_cast<uintptr_t>(src_dev) % 16 || reinterpret_cast<uintptr_t>(sink_dev) % 16) return H1BKV_EINVAL;
    hipEvent_t a = nullptr, b = nullptr;
    if (hipEventCreate(&a) != hipSuccess) return H1BKV_EHIP;
    if (hipEventCreate(&b) != hipSuccess) {
        (void)hipEventDestroy(a);
        return H1BKV_EHIP;
    }
    set_dispatch_events(a, b);
    bool ok = launch_stream_read(src_dev, n_bytes, sink_dev, static_cast<hipStream_t>(hip_stream)) == hipSuccess;
    (void)take_dispatch_events();                    // (a launch that failed early has not taken them)
    ok = ok && hipEventSynchronize(b) == hipSuccess && hipEventElapsedTime(ms_out, a, b) == hipSuccess;
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    return ok ? H1BKV_OK : H1BKV_EHIP;
}

}  // extern "C"
