// C ABI of the Kascade hot path: argument checks, launch planning, workspace carving.
// No device allocation and no synchronisation.  The attention calls keep nothing between calls; the only
// process-wide state is what the two aids at the end of the header own: the tuning overrides
// (kascade_tuning_set, four integers) and the per-kernel timing records (kascade_profile_*).
#include "../../include/kascade.h"

#include <hip/hip_ext.h>
#include <limits.h>
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <vector>

#include "kernels.h"

using namespace kascade;

namespace {

enum { kPerHeadSets = 0, kSharedSets = 1, kPreSoftmax = 2 };   // anchor variants behind one implementation

constexpr size_t kAlign = 256;
constexpr int kTargetBlocks = 1024;   // about four workgroups per compute unit (256 CUs)

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
int64_t round_up_i(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// Tuning overrides (kascade_tuning_set): 0 = the library's own plan.  Test and measurement aids.
std::atomic<int> g_tuning[KASCADE_TUNE_COUNT];
int tuning(int knob) { return g_tuning[knob].load(std::memory_order_relaxed); }

int check_desc(const kascade_desc* d, bool prefill) {
    if (!d) return KASCADE_INVALID_ARG;
    if (d->batch <= 0 || d->n_q_heads <= 0 || d->n_kv_heads <= 0) return KASCADE_INVALID_ARG;
    if (d->n_q_heads % d->n_kv_heads) return KASCADE_INVALID_ARG;
    if (prefill && d->batch != 1) return KASCADE_INVALID_ARG;
    // sequences and key heads are grid dimensions y / z of the decode kernels
    if (d->batch > 65535 || d->n_kv_heads > 65535) return KASCADE_UNSUPPORTED;
    if (d->head_dim != 64 && d->head_dim != 128) return KASCADE_UNSUPPORTED;
    if (d->dtype != KASCADE_F32 && d->dtype != KASCADE_BF16 && d->dtype != KASCADE_F16) return KASCADE_UNSUPPORTED;
    // heads per key head: the vector-ALU kernels are built for 1, 2, 4 and 8; the matrix-unit decode kernels
    // (bf16) take any group up to 16; prefill workgroups hold 128 / G whole tokens
    const int G = d->n_q_heads / d->n_kv_heads;
    const bool pow2 = G == 1 || G == 2 || G == 4 || G == 8;
    const bool any_group = !prefill && d->dtype != KASCADE_F32 && G <= 16;
    if (!pow2 && !any_group) return KASCADE_UNSUPPORTED;
    if (!(d->softmax_scale >= 0.f) || isinf(d->softmax_scale)) return KASCADE_INVALID_ARG;
    const int64_t es = d->dtype == KASCADE_F32 ? 4 : 2;
    const int64_t strides[] = {d->q_stride[0], d->q_stride[2], d->kv_stride[0], d->kv_stride[1], d->kv_stride[2],
                               prefill ? d->q_stride[1] : 0};
    for (int64_t s : strides) {
        if (s < 0) return KASCADE_INVALID_ARG;
        if ((s * es) % 16) return KASCADE_MISALIGNED;
    }
    if (d->kv_stride[2] < d->head_dim || d->q_stride[2] < d->head_dim || d->o_stride[2] < d->head_dim)
        return KASCADE_INVALID_ARG;
    return KASCADE_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

Shape make_shape(const kascade_desc* d) {
    Shape s;
    s.B = d->batch; s.Hq = d->n_q_heads; s.Hkv = d->n_kv_heads; s.D = d->head_dim;
    s.G = s.Hq / s.Hkv;
    s.dtype = d->dtype;
    const double scale = d->softmax_scale > 0.f ? (double)d->softmax_scale : 1.0 / sqrt((double)d->head_dim);
    s.scale_log2 = (float)(scale * 1.4426950408889634074);
    for (int i = 0; i < 3; ++i) { s.q_stride[i] = d->q_stride[i]; s.kv_stride[i] = d->kv_stride[i]; s.o_stride[i] = d->o_stride[i]; }
    return s;
}

// rows per workgroup for `n_rows` rows in each of `pairs` (sequence, key head) problems
DecodePlan plan_rows(int64_t n_rows, int pairs, int target_blocks, int min_chunk, int max_chunks, int forced_chunk) {
    DecodePlan p;
    if (max_chunks > kMaxChunks) max_chunks = kMaxChunks;
    int64_t want = (target_blocks + pairs - 1) / pairs;
    if (want < 1) want = 1;
    int64_t chunk = round_up_i((n_rows + want - 1) / want, 256);
    if (chunk < min_chunk) chunk = min_chunk;
    const int64_t floor_chunk = round_up_i((n_rows + max_chunks - 1) / max_chunks, 256);
    if (chunk < floor_chunk) chunk = floor_chunk;
    if (forced_chunk > 0) chunk = round_up_i(forced_chunk, 64);
    if (chunk < floor_chunk) chunk = floor_chunk;
    p.chunk = (int)chunk;
    p.n_chunks = (int)((n_rows + chunk - 1) / chunk);
    if (p.n_chunks < 1) p.n_chunks = 1;
    return p;
}
// gather, bf16 with 256-byte rows: at most 512 workgroups, so that the
// grid is resident at two workgroups per compute unit and runs the form of the kernel that keeps a wave's
// whole 64-row group in flight; each (sequence, key head) gets 512 / pairs chunks of whole 256-row passes.
// Measured against every other split from batch 1 x 131072 to batch 64 x 131072 (10 % budgets): equal or
// up to 13 % faster than about four smaller workgroups per compute unit; the matrix-unit kernel that
// serves groups of eight heads is fastest with the same split.  Other shapes keep that older rule.
DecodePlan plan_gather(const Shape& s, int64_t k_max) {
    const int pairs = s.B * s.Hkv;
    const int forced = tuning(KASCADE_TUNE_GATHER_CHUNK);
    if (k_max < 1) k_max = 1;   // a size query may ask about an empty budget
    if (s.dtype != 0 && s.D == 128 && forced == 0) {
        int64_t n = 512 / pairs;
        n = n < 1 ? 1 : (n > 64 ? 64 : n);
        DecodePlan p;
        p.chunk = (int)round_up_i((k_max + n - 1) / n, 256);
        p.n_chunks = (int)((k_max + p.chunk - 1) / p.chunk);
        if (p.n_chunks < 1) p.n_chunks = 1;
        return p;
    }
    DecodePlan p = plan_rows(k_max, pairs, kTargetBlocks, 256, 64, forced);
    // 256 rows are a single pass of a workgroup; if that still leaves three or more workgroups per compute
    // unit, two passes per workgroup amortise its start-up and merge better (measured, cold caches)
    if (p.chunk == 256 && forced == 0 && (int64_t)p.n_chunks * pairs >= 3 * 256) {
        p.chunk = 512;
        p.n_chunks = (int)((k_max + 511) / 512);
    }
    return p;
}
// stream: many small workgroups - with ragged sequence lengths whole chunks fall away and few large
// workgroups leave a long tail (measured: 1024 rows per workgroup wherever the 256-chunk limit allows;
// with ragged lengths 2048 is 4 % slower)
DecodePlan plan_stream(const Shape& s, int64_t max_seqlen) {
    return plan_rows(max_seqlen, s.B * s.Hkv, 32 * kTargetBlocks, 1024, 256, tuning(KASCADE_TUNE_STREAM_CHUNK));
}

// Workgroups per segment of the decode selection.  One is the single-workgroup kernel; more pay two extra
// launches, so the split is used only when segments are few (the chip would idle) and long.
int plan_topk_parts(const Shape& s, int64_t max_seqlen) {
    if (const int v = tuning(KASCADE_TUNE_TOPK_PARTS)) return v > kTopkMaxParts ? kTopkMaxParts : v;
    const int64_t segments = (int64_t)s.B * s.Hkv;
    if (segments > 128 || max_seqlen < 65536) return 1;          // measured: no gain below 64k scores per segment
    int64_t parts = 256 / segments;                               // about one workgroup per compute unit in total
    const int64_t by_len = max_seqlen / 4096;                     // at least 4096 scores per part
    if (parts > by_len) parts = by_len;
    if (parts > kTopkMaxParts) parts = kTopkMaxParts;
    return parts < 2 ? 1 : (int)parts;
}

struct Carver {
    char* base; size_t used;
    explicit Carver(void* p) : base(static_cast<char*>(p)), used(0) {}
    template <typename T> T* take(size_t count) {
        T* r = base ? reinterpret_cast<T*>(base + used) : nullptr;
        used = align_up(used + count * sizeof(T), kAlign);
        return r;
    }
};

struct DecodeReuseWs { float* part_ml; float* part_acc; size_t bytes; };
DecodeReuseWs carve_decode_reuse(const Shape& s, const DecodePlan& plan, void* ws, size_t offset = 0) {
    Carver c(ws); c.used = offset;
    DecodeReuseWs r;
    const size_t rows = (size_t)s.B * s.Hq * plan.n_chunks;
    r.part_ml = c.take<float>(rows * 2);
    r.part_acc = c.take<float>(rows * s.D);
    r.bytes = c.used;
    return r;
}

struct DecodeAnchorWs {
    float* logits; float* pooled; float* st_ml; float* st_acc; uint32_t* hist11; int32_t* zero_map; int64_t pitch;
    void* qbar;   // [B, Hkv, D] pooled queries (Pre-Softmax pooling), 4 bytes per element reserved
    uint32_t* topk_cand; uint32_t* topk_seg; uint32_t* topk_part; int topk_parts;
    DecodeReuseWs gather; size_t bytes;
};
DecodeAnchorWs carve_decode_anchor(const Shape& s, const DecodePlan& stream, const DecodePlan& gather,
                                   int64_t max_seqlen, void* ws) {
    Carver c(ws);
    DecodeAnchorWs r;
    r.pitch = round_up_i(max_seqlen, 4);
    r.logits = c.take<float>((size_t)s.B * s.Hq * r.pitch);
    r.pooled = c.take<float>((size_t)s.B * s.Hkv * r.pitch);
    const size_t rows = (size_t)s.B * s.Hq * stream.n_chunks;
    r.st_ml = c.take<float>(rows * 2);
    r.st_acc = c.take<float>(rows * s.D);
    r.hist11 = c.take<uint32_t>((size_t)s.B * s.Hkv * 2048);
    r.zero_map = c.take<int32_t>((size_t)s.Hkv);
    r.qbar = c.take<float>((size_t)s.B * s.Hkv * s.D);
    r.topk_parts = plan_topk_parts(s, max_seqlen);
    r.topk_cand = r.topk_seg = r.topk_part = nullptr;
    if (r.topk_parts > 1) {
        const size_t segs = (size_t)s.B * s.Hkv;
        r.topk_cand = c.take<uint32_t>(segs * kTopkCandCap);
        r.topk_seg = c.take<uint32_t>(segs * 8);
        r.topk_part = c.take<uint32_t>(segs * kTopkMaxParts * 2);
    }
    r.gather = carve_decode_reuse(s, gather, ws, c.used);
    r.bytes = r.gather.bytes;
    return r;
}

struct PrefillWs { float* stats; float* pooled; int32_t* zero_map; int64_t pooled_pitch; size_t bytes; };
PrefillWs carve_prefill_anchor(const Shape& s, int64_t S, int T, void* ws) {
    Carver c(ws);
    PrefillWs r;
    const int64_t n_tiles = (S + T - 1) / T;
    r.pooled_pitch = round_up_i((int64_t)T * n_tiles * (n_tiles - 1) / 2 + 4, 4);
    r.stats = c.take<float>((size_t)s.Hq * S * 2);
    r.pooled = c.take<float>((size_t)s.Hkv * r.pooled_pitch);
    r.zero_map = c.take<int32_t>((size_t)s.Hkv);
    r.bytes = c.used;
    return r;
}

// The shape the decode kernels see when pooled queries stand in for the group's heads: one query head
// per key head, rows [unit, Hkv, D] packed.
Shape pooled_query_shape(const Shape& s, int units) {
    Shape p = s;
    p.B = units; p.Hq = s.Hkv; p.G = 1;
    p.q_stride[0] = (int64_t)s.Hkv * s.D; p.q_stride[1] = 0; p.q_stride[2] = s.D;
    return p;
}

// Pre-Softmax pooling of prefill tiles runs on the decode kernels: tile t is a "sequence" whose query is
// the tile's pooled query and whose cache is the first t*T keys of the prompt (batch stride 0).
struct PrefillPreWs {
    void* qbar; int32_t* tile_lens; float* logits; float* pooled; float* st_ml; uint32_t* hist11;
    int64_t pitch; int64_t max_len; Shape ds; DecodePlan sp; size_t bytes;
};
PrefillPreWs carve_prefill_presoftmax(const Shape& s, int64_t S, int T, void* ws) {
    Carver c(ws);
    PrefillPreWs r;
    const int64_t n_tiles = (S + T - 1) / T;
    r.max_len = (n_tiles - 1) * T > 0 ? (n_tiles - 1) * T : 1;
    r.ds = pooled_query_shape(s, (int)n_tiles);
    r.ds.kv_stride[0] = 0;
    r.sp = plan_stream(r.ds, r.max_len);
    r.pitch = round_up_i(r.max_len, 4);
    r.qbar = c.take<float>((size_t)n_tiles * s.Hkv * s.D);
    r.tile_lens = c.take<int32_t>((size_t)n_tiles);
    r.logits = c.take<float>((size_t)n_tiles * s.Hkv * r.pitch);
    r.pooled = c.take<float>((size_t)n_tiles * s.Hkv * r.pitch);
    r.st_ml = c.take<float>((size_t)n_tiles * s.Hkv * r.sp.n_chunks * 2);
    r.hist11 = c.take<uint32_t>((size_t)n_tiles * s.Hkv * 2048);
    r.bytes = c.used;
    return r;
}

int hip_status(hipError_t e) { return e == hipSuccess ? KASCADE_OK : KASCADE_HIP_ERROR; }

// Which family runs the decode row passes.  The arithmetic of the vector-ALU row kernels grows with the number of
// heads per key head, that of the matrix-unit kernels does not; both stage rows through registers in the same
// way.  The matrix-unit kernels are ahead from four heads on (batch 8 x 32768, 128-wide heads, four heads: gather
// 19.5 -> 15.6 us, key sweep 101 -> 96 us, sweep with dense output 191 -> 184 us; eight heads: 34.5 -> 18 us,
// 161 -> 101 us, 385 -> 194 us; 64-wide heads, four heads: gather 10.9 -> 8.2 us) and equal or a little behind
// below that.  kascade_tuning_set(KASCADE_TUNE_DECODE_FAMILY, 1 / 2) forces one or the other (tests).
bool use_matrix_unit(const Shape& s) {
    if (s.dtype == 0 || s.G > 16) return false;
    if (s.dtype == 2) return true;   // fp16 exists on the matrix unit only
    if (s.G != 1 && s.G != 2 && s.G != 4 && s.G != 8) return true;   // the only kernels for these groups
    const int forced = tuning(KASCADE_TUNE_DECODE_FAMILY);
    return forced ? forced == 2 : s.G >= 4;
}
// Attention over a gathered index list.
hipError_t launch_gather(const Shape& s, const DecodePlan& plan, const DecodeRowsArgs& a, hipStream_t st) {
    if (use_matrix_unit(s)) return launch_decode_gather_mfma(s, plan, a, st);
    return launch_decode_rows(s, plan, a, true, true, false, st);
}
// The anchor's sweep over every key (logits stored), with the same choice of kernel.
hipError_t launch_stream(const Shape& s, const DecodePlan& plan, const DecodeRowsArgs& a, bool with_v, hipStream_t st) {
    if (use_matrix_unit(s)) return launch_decode_stream_mfma(s, plan, a, with_v, st);
    return launch_decode_rows(s, plan, a, false, with_v, true, st);
}

// ---- optional per-kernel timing (measurement aid, off by default) -----------------
// When enabled, every kernel dispatch carries its own start and stop event (hipExtLaunchKernelGGL): both
// events are bound to the dispatch itself, so their difference is the dispatch's begin-to-end time on the
// device - the figure a kernel trace of the same run reports - and not the time between two markers around
// it.  Events are created on demand and kept until profiling is disabled; with profiling off the library
// creates nothing and launches plainly.
enum KernelId { K_STREAM = 0, K_STREAM_V, K_GATHER, K_MERGE, K_POOL, K_TOPK, K_PF_SWEEP1, K_PF_SWEEP1_V, K_PF_SWEEP2,
                K_PF_TOPK, K_PF_SPARSE, K_SIMILARITY, K_HEAD_MAP, K_IMPORTANCE, K_POOL_HEADS, K_POOL_QUERIES, K_COUNT };
const char* const kKernelNames[K_COUNT] = {
    "decode_stream", "decode_stream_v", "decode_gather", "decode_merge", "decode_pool", "decode_topk",
    "prefill_sweep1", "prefill_sweep1_v", "prefill_sweep2", "prefill_topk", "prefill_sparse",
    "similarity", "head_map", "layer_importance", "pool_heads", "pool_queries"};

struct ProfRec { int kid; hipEvent_t start, stop; };
struct Profiler {
    std::atomic<bool> on{false};
    std::vector<ProfRec> recs;
    std::vector<hipEvent_t> free_events;
    int64_t calls[K_COUNT] = {};
    std::mutex mu;
    hipEvent_t get() {
        if (!free_events.empty()) { hipEvent_t e = free_events.back(); free_events.pop_back(); return e; }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }
} g_prof;
thread_local int t_current_kernel = -1;   // the step a launch on this thread belongs to, set by timed()

template <typename F>
int timed(int kid, hipStream_t st, F&& launch) {
    (void)st;
    if (!g_prof.on.load(std::memory_order_relaxed)) return hip_status(launch());
    { std::lock_guard<std::mutex> lock(g_prof.mu); g_prof.calls[kid] += 1; }
    t_current_kernel = kid;
    const int rc = hip_status(launch());
    t_current_kernel = -1;
    return rc;
}

}  // namespace

// called by KASCADE_LAUNCH before every dispatch
kascade::LaunchEvents kascade::next_launch_events() {
    LaunchEvents ev = {nullptr, nullptr};
    if (t_current_kernel < 0 || !g_prof.on.load(std::memory_order_relaxed)) return ev;
    std::lock_guard<std::mutex> lock(g_prof.mu);
    ProfRec r{t_current_kernel, g_prof.get(), g_prof.get()};
    if (!r.start || !r.stop) return ev;
    g_prof.recs.push_back(r);
    ev.start = r.start; ev.stop = r.stop;
    return ev;
}

namespace {

}  // namespace

extern "C" {

const char* kascade_version(void) { return "0.1"; }

int kascade_tuning_set(int32_t knob, int32_t value) {
    if (knob < 0 || knob >= KASCADE_TUNE_COUNT || value < 0) return KASCADE_INVALID_ARG;
    if (knob == KASCADE_TUNE_DECODE_FAMILY && value > 2) return KASCADE_INVALID_ARG;
    g_tuning[knob].store(value, std::memory_order_relaxed);
    return KASCADE_OK;
}

int32_t kascade_tuning_get(int32_t knob) {
    if (knob < 0 || knob >= KASCADE_TUNE_COUNT) return KASCADE_INVALID_ARG;
    return tuning(knob);
}

int kascade_profile_enable(int32_t on) {
    std::lock_guard<std::mutex> lock(g_prof.mu);
    g_prof.on.store(on != 0, std::memory_order_relaxed);
    if (!on) {
        for (auto& r : g_prof.recs) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
        for (auto e : g_prof.free_events) (void)hipEventDestroy(e);
        g_prof.recs.clear();
        g_prof.free_events.clear();
        for (auto& c : g_prof.calls) c = 0;
    }
    return KASCADE_OK;
}

int kascade_profile_reset(void) {
    std::lock_guard<std::mutex> lock(g_prof.mu);
    for (auto& r : g_prof.recs) { g_prof.free_events.push_back(r.start); g_prof.free_events.push_back(r.stop); }
    g_prof.recs.clear();
    for (auto& c : g_prof.calls) c = 0;
    return KASCADE_OK;
}

int32_t kascade_profile_kernels(void) { return K_COUNT; }

int kascade_profile_read(int32_t kernel, const char** name, double* total_ms, int64_t* launches) {
    if (kernel < 0 || kernel >= K_COUNT || !name || !total_ms || !launches) return KASCADE_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_prof.mu);
    *name = kKernelNames[kernel];
    *total_ms = 0.0;
    *launches = g_prof.calls[kernel];
    for (auto& r : g_prof.recs) {
        if (r.kid != kernel) continue;
        if (hipEventSynchronize(r.stop) != hipSuccess) return KASCADE_HIP_ERROR;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) return KASCADE_HIP_ERROR;
        *total_ms += ms;
    }
    return KASCADE_OK;
}

const char* kascade_status_string(int32_t status) {
    switch (status) {
        case KASCADE_OK: return "ok";
        case KASCADE_INVALID_ARG: return "invalid argument";
        case KASCADE_UNSUPPORTED: return "unsupported head_dim, dtype, group size or tile size";
        case KASCADE_MISALIGNED: return "pointer or stride breaks 16-byte row alignment";
        case KASCADE_WORKSPACE_TOO_SMALL: return "workspace too small";
        case KASCADE_HIP_ERROR: return "HIP launch error";
    }
    return "unknown status";
}

size_t kascade_workspace_bytes(int32_t op, const kascade_desc* desc, int64_t max_seqlen, int64_t k_or_idx_total,
                               int32_t q_tile_tokens) {
    const bool prefill = op == KASCADE_OP_PREFILL_ANCHOR || op == KASCADE_OP_PREFILL_REUSE || op == KASCADE_OP_PREFILL_ANCHOR_PRESOFTMAX;
    if (check_desc(desc, prefill) != KASCADE_OK || max_seqlen <= 0 || k_or_idx_total < 0) return 0;
    const Shape s = make_shape(desc);
    switch (op) {
        case KASCADE_OP_PREFILL_ANCHOR:
            if (q_tile_tokens <= 0) return 0;
            return carve_prefill_anchor(s, max_seqlen, q_tile_tokens, nullptr).bytes;
        case KASCADE_OP_PREFILL_REUSE:
            return 0;
        case KASCADE_OP_DECODE_REUSE:
            return carve_decode_reuse(s, plan_gather(s, k_or_idx_total), nullptr).bytes;
        case KASCADE_OP_DECODE_ANCHOR:
            return carve_decode_anchor(s, plan_stream(s, max_seqlen), plan_gather(s, k_or_idx_total), max_seqlen, nullptr).bytes;
        case KASCADE_OP_DECODE_POOLED:
            return carve_decode_anchor(s, plan_stream(s, max_seqlen), plan_gather(s, 1), max_seqlen, nullptr).bytes;
        case KASCADE_OP_PREFILL_ANCHOR_PRESOFTMAX:
            if (q_tile_tokens <= 0) return 0;
            return carve_prefill_presoftmax(s, max_seqlen, q_tile_tokens, nullptr).bytes;
        default:
            return 0;
    }
}

static int decode_reuse_impl(const kascade_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                             const int32_t* seqlens, const int32_t* k_per_seq, int32_t k_max, const int32_t* idx_in,
                             int32_t n_anchor_heads, const int32_t* head_map, void* out, void* workspace,
                             size_t workspace_bytes, void* hip_stream) {
    int st = check_desc(desc, false);
    if (st != KASCADE_OK) return st;
    if (!q || !k_cache || !v_cache || !seqlens || !k_per_seq || !idx_in || !out) return KASCADE_INVALID_ARG;
    if (k_max <= 0 || n_anchor_heads <= 0) return KASCADE_INVALID_ARG;
    if (!head_map && n_anchor_heads != desc->n_kv_heads) return KASCADE_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache)) return KASCADE_MISALIGNED;
    const Shape s = make_shape(desc);
    const DecodePlan plan = plan_gather(s, k_max);
    const DecodeReuseWs ws = carve_decode_reuse(s, plan, workspace);
    if (ws.bytes > 0 && (!workspace || workspace_bytes < ws.bytes)) return KASCADE_WORKSPACE_TOO_SMALL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    DecodeRowsArgs a = {};
    a.q = q; a.k = k_cache; a.v = v_cache; a.seqlens = seqlens; a.k_per_seq = k_per_seq;
    a.idx = idx_in; a.head_map = head_map; a.k_max = k_max; a.n_src_heads = n_anchor_heads;
    a.part_ml = ws.part_ml; a.part_acc = ws.part_acc; a.out = out;
    st = timed(K_GATHER, stream, [&] { return launch_gather(s, plan, a, stream); });
    if (st != KASCADE_OK) return st;
    if (plan.n_chunks > 1)
        st = timed(K_MERGE, stream, [&] { return launch_decode_merge(s, plan.n_chunks, ws.part_ml, ws.part_acc, out, stream); });
    return st;
}

int kascade_decode_reuse(const kascade_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                         const int32_t* seqlens, const int32_t* k_per_seq, int32_t k_max, const int32_t* idx_in,
                         int32_t n_anchor_heads, const int32_t* head_map, void* out, void* workspace,
                         size_t workspace_bytes, void* hip_stream) {
    return decode_reuse_impl(desc, q, k_cache, v_cache, seqlens, k_per_seq, k_max, idx_in, n_anchor_heads, head_map, out,
                             workspace, workspace_bytes, hip_stream);
}

// ---- the reuse layer for callers that cannot allocate ---------------------------------------------
// The partial results of the gather (per chunk: max, sum, accumulator) live in a fixed array in device
// memory that is part of the library's code object; every GPU the library runs on holds its own copy
// until the process ends.  In host code the array's name is only a handle: the device address comes
// from hipGetSymbolAddress, once per device, and that address is what the kernels receive.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mu;

static int scratch_of_current_device(void** ptr) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return KASCADE_HIP_ERROR;
    if (dev < 0 || dev >= kMaxDevices) return KASCADE_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return KASCADE_HIP_ERROR;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return KASCADE_OK;
}

size_t kascade_decode_reuse_static_capacity(void) { return kStaticScratchBytes; }

int kascade_decode_reuse_static(const kascade_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                                const int32_t* seqlens, const int32_t* k_per_seq, int32_t k_max, const int32_t* idx_in,
                                int32_t n_anchor_heads, const int32_t* head_map, void* out, void* hip_stream) {
    // sizes first: a shape whose partial results do not fit the fixed array is refused before anything else
    if (check_desc(desc, false) == KASCADE_OK && k_max > 0) {
        const Shape s = make_shape(desc);
        if (carve_decode_reuse(s, plan_gather(s, k_max), nullptr).bytes > kStaticScratchBytes) return KASCADE_WORKSPACE_TOO_SMALL;
    }
    void* ptr = nullptr;
    const int st = scratch_of_current_device(&ptr);
    if (st != KASCADE_OK) return st;
    return decode_reuse_impl(desc, q, k_cache, v_cache, seqlens, k_per_seq, k_max, idx_in, n_anchor_heads, head_map, out,
                             ptr, kStaticScratchBytes, hip_stream);
}

static int decode_anchor_impl(const kascade_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                              const int32_t* seqlens, const int32_t* k_per_seq, int32_t max_seqlen, int32_t k_max,
                              int32_t recent_window, int32_t out_mode, int32_t* idx_out, void* out, void* workspace,
                              size_t workspace_bytes, void* hip_stream, int variant) {
    const bool shared = variant == kSharedSets, presoftmax = variant == kPreSoftmax;
    int st = check_desc(desc, false);
    if (st != KASCADE_OK) return st;
    if (!q || !k_cache || !v_cache || !seqlens || !k_per_seq || !idx_out || !out) return KASCADE_INVALID_ARG;
    if (max_seqlen <= 0 || k_max <= 0 || k_max > max_seqlen || recent_window < 0 || recent_window > k_max)
        return KASCADE_INVALID_ARG;
    if (out_mode != KASCADE_OUT_DENSE && out_mode != KASCADE_OUT_SPARSE) return KASCADE_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache)) return KASCADE_MISALIGNED;
    const Shape s = make_shape(desc);
    const DecodePlan sp = plan_stream(s, max_seqlen);
    const DecodePlan gp = plan_gather(s, k_max);
    const DecodeAnchorWs ws = carve_decode_anchor(s, sp, gp, max_seqlen, workspace);
    if (!workspace || workspace_bytes < ws.bytes) return KASCADE_WORKSPACE_TOO_SMALL;
    if (!aligned16(workspace)) return KASCADE_MISALIGNED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool dense = out_mode == KASCADE_OUT_DENSE;

    // pass 1: logits of every key + per-chunk softmax statistics (dense: also P.V)
    DecodeRowsArgs a = {};
    a.q = q; a.k = k_cache; a.v = v_cache; a.seqlens = seqlens; a.max_seqlen = max_seqlen;
    a.logits = ws.logits; a.logit_pitch = ws.pitch;
    a.part_ml = ws.st_ml; a.part_acc = ws.st_acc; a.out = out; a.hist11 = ws.hist11;
    // the shape passes 1-2 run on: the layer's own, or (Pre-Softmax pooling) one pooled query per key head
    Shape sel = s;
    if (presoftmax) {
        // the dense output still needs every head's own query against every key: a pass of its own, whose
        // logits and statistics are overwritten below
        if (dense) {
            st = timed(K_STREAM_V, stream, [&] { return launch_stream(s, sp, a, true, stream); });
            if (st != KASCADE_OK) return st;
            if (sp.n_chunks > 1) {
                st = timed(K_MERGE, stream, [&] { return launch_decode_merge(s, sp.n_chunks, ws.st_ml, ws.st_acc, out, stream); });
                if (st != KASCADE_OK) return st;
            }
        }
        st = timed(K_POOL_QUERIES, stream, [&] {
            return launch_pool_queries(s.dtype, q, s.q_stride[0], 0, s.q_stride[2], s.G, 1, 1, s.B, ws.qbar, s.Hkv, s.D, nullptr, stream);
        });
        if (st != KASCADE_OK) return st;
        sel = pooled_query_shape(s, s.B);
        a.q = ws.qbar;
    }
    const bool with_v = dense && !presoftmax;
    st = timed(with_v ? K_STREAM_V : K_STREAM, stream, [&] { return launch_stream(sel, sp, a, with_v, stream); });
    if (st != KASCADE_OK) return st;
    if (with_v && sp.n_chunks > 1) {
        st = timed(K_MERGE, stream, [&] { return launch_decode_merge(s, sp.n_chunks, ws.st_ml, ws.st_acc, out, stream); });
        if (st != KASCADE_OK) return st;
    }
    // pass 2: softmax + mean over the GQA group
    DecodePoolArgs pa = {};
    pa.seqlens = seqlens; pa.k_per_seq = k_per_seq; pa.k_max = k_max; pa.recent_window = recent_window;
    pa.logits = ws.logits; pa.logit_pitch = ws.pitch; pa.part_ml = ws.st_ml; pa.pooled = ws.pooled;
    pa.pooled_pitch = ws.pitch; pa.hist11 = ws.hist11; pa.max_seqlen = max_seqlen;
    const bool split = ws.topk_parts > 1 && !shared;
    pa.seg_info = split ? ws.topk_seg : nullptr;
    st = timed(K_POOL, stream, [&] { return launch_decode_pool(sel, sp.n_chunks, pa, stream); });
    if (st != KASCADE_OK) return st;
    // shared variant: one distribution per sequence = mean over the key heads (written over head 0's row)
    if (shared) {
        st = timed(K_POOL_HEADS, stream, [&] {
            return launch_pool_heads(ws.pooled, (int64_t)s.Hkv * ws.pitch, ws.pitch, s.Hkv, s.B, max_seqlen, seqlens,
                                     ws.zero_map, stream);
        });
        if (st != KASCADE_OK) return st;
    }
    // pass 3: Top-k per (sequence, key head); shared: per sequence, without the per-head histograms
    Shape ts = s;
    TopkArgs t = {};
    t.scores = ws.pooled; t.hist11 = ws.hist11; t.idx_out = idx_out; t.seqlens = seqlens; t.k_per_seq = k_per_seq;
    t.pitch = ws.pitch; t.k_max = k_max; t.recent_window = recent_window; t.max_seqlen = max_seqlen;
    if (shared) { ts.Hkv = 1; t.hist11 = nullptr; t.pitch = (int64_t)s.Hkv * ws.pitch; }
    if (split) {
        t.cand = ws.topk_cand; t.seg_info = ws.topk_seg; t.part_info = ws.topk_part; t.n_parts = ws.topk_parts;
        st = timed(K_TOPK, stream, [&] { return launch_topk_decode_split(ts, t, stream); });
    } else {
        st = timed(K_TOPK, stream, [&] { return launch_topk_decode(ts, t, stream); });
    }
    if (st != KASCADE_OK || dense) return st;
    // pass 4: attention over the fresh index set
    DecodeRowsArgs g = {};
    g.q = q; g.k = k_cache; g.v = v_cache; g.seqlens = seqlens; g.max_seqlen = max_seqlen; g.k_per_seq = k_per_seq;
    g.idx = idx_out; g.head_map = shared ? ws.zero_map : nullptr; g.k_max = k_max; g.n_src_heads = shared ? 1 : s.Hkv;
    g.part_ml = ws.gather.part_ml; g.part_acc = ws.gather.part_acc; g.out = out;
    st = timed(K_GATHER, stream, [&] { return launch_gather(s, gp, g, stream); });
    if (st != KASCADE_OK) return st;
    if (gp.n_chunks > 1)
        st = timed(K_MERGE, stream, [&] { return launch_decode_merge(s, gp.n_chunks, ws.gather.part_ml, ws.gather.part_acc, out, stream); });
    return st;
}

int kascade_decode_anchor(const kascade_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                          const int32_t* seqlens, const int32_t* k_per_seq, int32_t max_seqlen, int32_t k_max,
                          int32_t recent_window, int32_t out_mode, int32_t* idx_out, void* out, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
    return decode_anchor_impl(desc, q, k_cache, v_cache, seqlens, k_per_seq, max_seqlen, k_max, recent_window, out_mode,
                              idx_out, out, workspace, workspace_bytes, hip_stream, kPerHeadSets);
}

int kascade_decode_anchor_shared(const kascade_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                                 const int32_t* seqlens, const int32_t* k_per_seq, int32_t max_seqlen, int32_t k_max,
                                 int32_t recent_window, int32_t out_mode, int32_t* idx_out, void* out,
                                 void* workspace, size_t workspace_bytes, void* hip_stream) {
    return decode_anchor_impl(desc, q, k_cache, v_cache, seqlens, k_per_seq, max_seqlen, k_max, recent_window, out_mode,
                              idx_out, out, workspace, workspace_bytes, hip_stream, kSharedSets);
}

int kascade_decode_anchor_presoftmax(const kascade_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                                     const int32_t* seqlens, const int32_t* k_per_seq, int32_t max_seqlen, int32_t k_max,
                                     int32_t recent_window, int32_t out_mode, int32_t* idx_out, void* out,
                                     void* workspace, size_t workspace_bytes, void* hip_stream) {
    return decode_anchor_impl(desc, q, k_cache, v_cache, seqlens, k_per_seq, max_seqlen, k_max, recent_window, out_mode,
                              idx_out, out, workspace, workspace_bytes, hip_stream, kPreSoftmax);
}

}  // extern "C"

namespace {

int check_prefill(const kascade_desc* desc, const void* q, const void* k, const void* v, int32_t seqlen,
                  int32_t T, const int32_t* k_per_tile, const int64_t* idx_offsets, int64_t idx_total,
                  const void* idx, const void* out) {
    int st = check_desc(desc, true);
    if (st != KASCADE_OK) return st;
    if (!q || !k || !v || !k_per_tile || !idx_offsets || !out) return KASCADE_INVALID_ARG;
    if (seqlen <= 0 || T <= 0 || idx_total < 0) return KASCADE_INVALID_ARG;
    if (idx_total > 0 && !idx) return KASCADE_INVALID_ARG;
    if (desc->dtype != KASCADE_BF16 && desc->dtype != KASCADE_F16) return KASCADE_UNSUPPORTED;
    // a query tile is T tokens times the G heads of a key head; a workgroup owns 128 of those
    // (token, head) rows, so a tile is one or several whole workgroups
    if (((int64_t)T * (desc->n_q_heads / desc->n_kv_heads)) % 128 != 0) return KASCADE_UNSUPPORTED;
    // the kernels address the rows of one key head with 32-bit byte offsets
    if ((int64_t)seqlen * desc->kv_stride[2] * 2 >= ((int64_t)1 << 32)) return KASCADE_UNSUPPORTED;
    if ((desc->o_stride[1] * 2) % 8 || (desc->o_stride[2] * 2) % 8) return KASCADE_MISALIGNED;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || (reinterpret_cast<uintptr_t>(out) & 7u)) return KASCADE_MISALIGNED;
    return KASCADE_OK;
}

PrefillArgs prefill_args(const Shape& s, const void* q, const void* k, const void* v, void* out, int32_t seqlen, int32_t T,
                         const int32_t* k_per_tile, const int64_t* idx_offsets, int64_t idx_total) {
    PrefillArgs a = {};
    a.q = q; a.k = k; a.v = v; a.out = out; a.seqlen = seqlen; a.tile_tokens = T;
    a.n_tiles = (seqlen + T - 1) / T;
    a.sub_tokens = 128 / s.G;
    a.n_sub = (seqlen + a.sub_tokens - 1) / a.sub_tokens;
    a.k_per_tile = k_per_tile; a.idx_offsets = idx_offsets; a.idx_total = idx_total;
    return a;
}

}  // namespace

extern "C" {

static int prefill_anchor_impl(const kascade_desc* desc, const void* q, const void* k, const void* v, int32_t seqlen,
                               int32_t q_tile_tokens, const int32_t* k_per_tile, const int64_t* idx_offsets,
                               int64_t idx_total, int32_t out_mode, int32_t* idx_out, void* out, void* workspace,
                               size_t workspace_bytes, void* hip_stream, bool shared) {
    int st = check_prefill(desc, q, k, v, seqlen, q_tile_tokens, k_per_tile, idx_offsets, idx_total, idx_out, out);
    if (st != KASCADE_OK) return st;
    if (out_mode != KASCADE_OUT_DENSE && out_mode != KASCADE_OUT_SPARSE) return KASCADE_INVALID_ARG;
    const Shape s = make_shape(desc);
    const PrefillWs ws = carve_prefill_anchor(s, seqlen, q_tile_tokens, workspace);
    if (!workspace || workspace_bytes < ws.bytes) return KASCADE_WORKSPACE_TOO_SMALL;
    if (!aligned16(workspace)) return KASCADE_MISALIGNED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool dense = out_mode == KASCADE_OUT_DENSE;

    PrefillArgs a = prefill_args(s, q, k, v, out, seqlen, q_tile_tokens, k_per_tile, idx_offsets, idx_total);
    a.stats = ws.stats; a.pooled = ws.pooled; a.pooled_pitch = ws.pooled_pitch;
    // pass 1: causal scores -> row statistics (layer 0: plus the dense output)
    st = timed(dense ? K_PF_SWEEP1_V : K_PF_SWEEP1, stream, [&] { return launch_prefill_attend(s, a, false, dense, stream); });
    if (st != KASCADE_OK) return st;
    // pass 2: recompute scores over the prefix, normalise, pool the tile's rows; per-head sets are
    // selected by the same workgroups (pass 3), shared sets need the mean over the heads first
    a.topk_out = shared ? nullptr : idx_out;
    st = timed(K_PF_SWEEP2, stream, [&] { return launch_prefill_pool(s, a, stream); });
    a.topk_out = nullptr;
    if (st != KASCADE_OK) return st;
    // shared variant: one distribution per tile = mean over the key heads (written over head 0's row)
    if (shared) {
        st = timed(K_POOL_HEADS, stream, [&] {
            return launch_pool_heads(ws.pooled, 0, ws.pooled_pitch, s.Hkv, 1, ws.pooled_pitch, nullptr, ws.zero_map, stream);
        });
        if (st != KASCADE_OK) return st;
    }
    // pass 3: Top-k per (tile, key head); shared: per tile
    Shape ts = s;
    if (shared) ts.Hkv = 1;
    TopkArgs t = {};
    t.scores = ws.pooled; t.idx_out = idx_out; t.k_per_tile = k_per_tile; t.idx_offsets = idx_offsets;
    t.idx_total = idx_total; t.pooled_pitch = ws.pooled_pitch; t.tile_tokens = q_tile_tokens; t.n_tiles = a.n_tiles;
    if (shared) st = timed(K_PF_TOPK, stream, [&] { return launch_topk_prefill(ts, t, stream); });
    if (st != KASCADE_OK || dense) return st;
    // pass 4: sparse attention over the fresh sets
    a.stats = nullptr; a.idx = idx_out; a.head_map = shared ? ws.zero_map : nullptr; a.n_src_heads = shared ? 1 : s.Hkv;
    return timed(K_PF_SPARSE, stream, [&] { return launch_prefill_attend(s, a, true, true, stream); });
}

int kascade_prefill_anchor(const kascade_desc* desc, const void* q, const void* k, const void* v, int32_t seqlen,
                           int32_t q_tile_tokens, const int32_t* k_per_tile, const int64_t* idx_offsets,
                           int64_t idx_total, int32_t out_mode, int32_t* idx_out, void* out, void* workspace,
                           size_t workspace_bytes, void* hip_stream) {
    return prefill_anchor_impl(desc, q, k, v, seqlen, q_tile_tokens, k_per_tile, idx_offsets, idx_total, out_mode, idx_out,
                               out, workspace, workspace_bytes, hip_stream, false);
}

int kascade_prefill_anchor_shared(const kascade_desc* desc, const void* q, const void* k, const void* v, int32_t seqlen,
                                  int32_t q_tile_tokens, const int32_t* k_per_tile, const int64_t* idx_offsets,
                                  int64_t idx_total, int32_t out_mode, int32_t* idx_out, void* out, void* workspace,
                                  size_t workspace_bytes, void* hip_stream) {
    return prefill_anchor_impl(desc, q, k, v, seqlen, q_tile_tokens, k_per_tile, idx_offsets, idx_total, out_mode, idx_out,
                               out, workspace, workspace_bytes, hip_stream, true);
}

int kascade_prefill_anchor_presoftmax(const kascade_desc* desc, const void* q, const void* k, const void* v,
                                      int32_t seqlen, int32_t q_tile_tokens, const int32_t* k_per_tile,
                                      const int64_t* idx_offsets, int64_t idx_total, int32_t out_mode, int32_t* idx_out,
                                      void* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    int st = check_prefill(desc, q, k, v, seqlen, q_tile_tokens, k_per_tile, idx_offsets, idx_total, idx_out, out);
    if (st != KASCADE_OK) return st;
    if (out_mode != KASCADE_OUT_DENSE && out_mode != KASCADE_OUT_SPARSE) return KASCADE_INVALID_ARG;
    const Shape s = make_shape(desc);
    const PrefillPreWs ws = carve_prefill_presoftmax(s, seqlen, q_tile_tokens, workspace);
    if (!workspace || workspace_bytes < ws.bytes) return KASCADE_WORKSPACE_TOO_SMALL;
    if (!aligned16(workspace)) return KASCADE_MISALIGNED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool dense = out_mode == KASCADE_OUT_DENSE;
    PrefillArgs a = prefill_args(s, q, k, v, out, seqlen, q_tile_tokens, k_per_tile, idx_offsets, idx_total);
    if (a.n_tiles > 65535) return KASCADE_UNSUPPORTED;   // one grid row per tile in the decode kernels

    // layer 0: plain causal attention for the output; it plays no part in the selection
    if (dense) {
        st = timed(K_PF_SWEEP1_V, stream, [&] { return launch_prefill_attend(s, a, false, true, stream); });
        if (st != KASCADE_OK) return st;
    }
    // one pooled query per (tile, key head); tile_lens[t] = t*T keys precede tile t
    st = timed(K_POOL_QUERIES, stream, [&] {
        return launch_pool_queries(s.dtype, q, 0, s.q_stride[1], s.q_stride[2], s.G, q_tile_tokens, seqlen, a.n_tiles, ws.qbar,
                                   s.Hkv, s.D, ws.tile_lens, stream);
    });
    if (st != KASCADE_OK) return st;
    // passes 1-3 of the decode anchor with tiles as sequences over one shared cache
    DecodeRowsArgs r = {};
    r.q = ws.qbar; r.k = k; r.v = nullptr; r.seqlens = ws.tile_lens;
    r.logits = ws.logits; r.logit_pitch = ws.pitch; r.part_ml = ws.st_ml; r.part_acc = nullptr; r.hist11 = ws.hist11;
    st = timed(K_STREAM, stream, [&] { return launch_stream(ws.ds, ws.sp, r, false, stream); });
    if (st != KASCADE_OK) return st;
    DecodePoolArgs pa = {};
    pa.seqlens = ws.tile_lens; pa.k_per_seq = k_per_tile; pa.k_max = INT_MAX; pa.recent_window = 0;
    pa.logits = ws.logits; pa.logit_pitch = ws.pitch; pa.part_ml = ws.st_ml; pa.pooled = ws.pooled;
    pa.pooled_pitch = ws.pitch; pa.hist11 = ws.hist11; pa.max_seqlen = (int)ws.max_len;
    st = timed(K_POOL, stream, [&] { return launch_decode_pool(ws.ds, ws.sp.n_chunks, pa, stream); });
    if (st != KASCADE_OK) return st;
    TopkArgs t = {};
    t.scores = ws.pooled; t.hist11 = ws.hist11; t.idx_out = idx_out; t.seqlens = ws.tile_lens; t.k_per_seq = k_per_tile;
    t.pitch = ws.pitch; t.k_max = INT_MAX; t.recent_window = 0;
    t.out_offsets = idx_offsets; t.out_head_pitch = idx_total;
    st = timed(K_TOPK, stream, [&] { return launch_topk_decode(ws.ds, t, stream); });
    if (st != KASCADE_OK || dense) return st;
    // pass 4: sparse attention over the fresh sets
    a.idx = idx_out; a.head_map = nullptr; a.n_src_heads = s.Hkv;
    return timed(K_PF_SPARSE, stream, [&] { return launch_prefill_attend(s, a, true, true, stream); });
}

int kascade_prefill_reuse(const kascade_desc* desc, const void* q, const void* k, const void* v, int32_t seqlen,
                          int32_t q_tile_tokens, const int32_t* k_per_tile, const int64_t* idx_offsets,
                          int64_t idx_total, const int32_t* idx_in, int32_t n_anchor_heads, const int32_t* head_map,
                          void* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    (void)workspace; (void)workspace_bytes;   // this op needs no scratch memory
    int st = check_prefill(desc, q, k, v, seqlen, q_tile_tokens, k_per_tile, idx_offsets, idx_total, idx_in, out);
    if (st != KASCADE_OK) return st;
    if (n_anchor_heads <= 0) return KASCADE_INVALID_ARG;
    if (!head_map && n_anchor_heads != desc->n_kv_heads) return KASCADE_INVALID_ARG;
    const Shape s = make_shape(desc);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    PrefillArgs a = prefill_args(s, q, k, v, out, seqlen, q_tile_tokens, k_per_tile, idx_offsets, idx_total);
    a.idx = idx_in; a.head_map = head_map; a.n_src_heads = n_anchor_heads;
    return timed(K_PF_SPARSE, stream, [&] { return launch_prefill_attend(s, a, true, true, stream); });
}

// ---- calibration path (Sec. 3.3): pooled distributions, set similarity, anchor selection ----

int kascade_decode_pooled(const kascade_desc* desc, const void* q, const void* k_cache, const int32_t* seqlens,
                          int32_t max_seqlen, float* pooled_out, int64_t pooled_pitch, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
    int st = check_desc(desc, false);
    if (st != KASCADE_OK) return st;
    if (!q || !k_cache || !seqlens || !pooled_out) return KASCADE_INVALID_ARG;
    if (max_seqlen <= 0 || pooled_pitch < max_seqlen) return KASCADE_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(pooled_out) || pooled_pitch % 4) return KASCADE_MISALIGNED;
    const Shape s = make_shape(desc);
    const DecodePlan sp = plan_stream(s, max_seqlen);
    const DecodeAnchorWs ws = carve_decode_anchor(s, sp, plan_gather(s, 1), max_seqlen, workspace);
    if (!workspace || workspace_bytes < ws.bytes) return KASCADE_WORKSPACE_TOO_SMALL;
    if (!aligned16(workspace)) return KASCADE_MISALIGNED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    DecodeRowsArgs a = {};
    a.q = q; a.k = k_cache; a.v = nullptr; a.seqlens = seqlens; a.max_seqlen = max_seqlen;
    a.logits = ws.logits; a.logit_pitch = ws.pitch;
    a.part_ml = ws.st_ml; a.part_acc = ws.st_acc; a.out = nullptr; a.hist11 = ws.hist11;
    st = timed(K_STREAM, stream, [&] { return launch_stream(s, sp, a, false, stream); });
    if (st != KASCADE_OK) return st;
    DecodePoolArgs pa = {};
    pa.seqlens = seqlens; pa.k_per_seq = seqlens; pa.k_max = max_seqlen; pa.recent_window = 0;
    pa.logits = ws.logits; pa.logit_pitch = ws.pitch; pa.part_ml = ws.st_ml; pa.pooled = pooled_out;
    pa.pooled_pitch = pooled_pitch; pa.hist11 = ws.hist11; pa.max_seqlen = max_seqlen;
    return timed(K_POOL, stream, [&] { return launch_decode_pool(s, sp.n_chunks, pa, stream); });
}

int kascade_topk_similarity(int32_t batch, int32_t n_kv_heads, const float* pooled_b, int64_t pooled_pitch,
                            const int32_t* seqlens, const int32_t* k_per_seq, int32_t k_max, const int32_t* idx_a,
                            int32_t n_heads_a, const int32_t* head_map, const int32_t* idx_b, float* sim_out,
                            float* sim_min, void* hip_stream) {
    if (batch <= 0 || n_kv_heads <= 0 || n_heads_a <= 0 || k_max <= 0 || pooled_pitch <= 0) return KASCADE_INVALID_ARG;
    if (batch > 65535) return KASCADE_INVALID_ARG;
    if (!pooled_b || !seqlens || !k_per_seq || !idx_a || !idx_b) return KASCADE_INVALID_ARG;
    if (!sim_out && !sim_min) return KASCADE_INVALID_ARG;
    if (!head_map && n_heads_a != n_kv_heads) return KASCADE_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    SimilarityArgs a = {};
    a.B = batch; a.Hkv = n_kv_heads; a.pooled = pooled_b; a.pitch = pooled_pitch; a.seqlens = seqlens;
    a.k_per_seq = k_per_seq; a.k_max = k_max; a.idx_a = idx_a; a.n_heads_a = n_heads_a; a.head_map = head_map;
    a.idx_b = idx_b; a.sim_out = sim_out; a.sim_min = sim_min;
    return timed(K_SIMILARITY, stream, [&] { return launch_similarity(a, stream); });
}

int kascade_head_similarity(int32_t batch, int32_t n_kv_heads, const float* pooled_b, int64_t pooled_pitch,
                            const int32_t* seqlens, const int32_t* k_per_seq, int32_t k_max, const int32_t* idx_a,
                            int32_t n_heads_a, const int32_t* idx_b, float* sim_out, void* hip_stream) {
    if (batch <= 0 || n_kv_heads <= 0 || n_heads_a <= 0 || k_max <= 0 || pooled_pitch <= 0) return KASCADE_INVALID_ARG;
    if (batch > 65535 || n_heads_a > 65535) return KASCADE_INVALID_ARG;
    if (!pooled_b || !seqlens || !k_per_seq || !idx_a || !idx_b || !sim_out) return KASCADE_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    SimilarityArgs a = {};
    a.B = batch; a.Hkv = n_kv_heads; a.pooled = pooled_b; a.pitch = pooled_pitch; a.seqlens = seqlens;
    a.k_per_seq = k_per_seq; a.k_max = k_max; a.idx_a = idx_a; a.n_heads_a = n_heads_a; a.head_map = nullptr;
    a.idx_b = idx_b; a.sim_out = sim_out; a.sim_min = nullptr; a.all_pairs = 1;
    return timed(K_SIMILARITY, stream, [&] { return launch_similarity(a, stream); });
}

int kascade_head_map(int32_t n_samples, int32_t n_kv_heads, int32_t n_heads_a, const float* sim, float* mean_out,
                     int32_t* head_map_out, void* hip_stream) {
    if (n_samples <= 0 || n_kv_heads <= 0 || n_heads_a <= 0 || !sim || !head_map_out) return KASCADE_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    return timed(K_HEAD_MAP, stream, [&] {
        return launch_head_map(n_samples, n_kv_heads, n_heads_a, sim, mean_out, head_map_out, stream);
    });
}

int kascade_layer_importance(const void* x, const void* y, int64_t n_rows, int32_t n_cols, int32_t dtype,
                             int64_t x_row_stride, int64_t y_row_stride, float* w_out, void* hip_stream) {
    if (!x || !y || !w_out || n_rows <= 0 || n_cols <= 0) return KASCADE_INVALID_ARG;
    if (n_rows > (int64_t)0x7fffffff * 4) return KASCADE_INVALID_ARG;
    if (x_row_stride < n_cols || y_row_stride < n_cols) return KASCADE_INVALID_ARG;
    if (dtype != KASCADE_F32 && dtype != KASCADE_BF16 && dtype != KASCADE_F16) return KASCADE_UNSUPPORTED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    return timed(K_IMPORTANCE, stream, [&] {
        return launch_importance(dtype, x, y, n_rows, n_cols, x_row_stride, y_row_stride, w_out, stream);
    });
}

int kascade_select_anchor_layers(const float* similarity, const float* layer_weights, int32_t n_layers,
                                 int32_t n_anchors, int32_t* anchors_out, double* objective_out) {
    if (!similarity || !anchors_out) return KASCADE_INVALID_ARG;
    if (n_layers <= 0 || n_layers > 4096 || n_anchors <= 0 || n_anchors > n_layers) return KASCADE_INVALID_ARG;
    const int L = n_layers, M = n_anchors;
    for (int64_t i = 0; i < (int64_t)L * L; ++i)
        if (!(similarity[i] == similarity[i])) return KASCADE_INVALID_ARG;   // NaN
    for (int i = 0; layer_weights && i < L; ++i)
        if (!(layer_weights[i] == layer_weights[i])) return KASCADE_INVALID_ARG;
    // serve[i*(L+1) + j]: total similarity of the layers i..j-1 when anchor i serves them
    std::vector<double> serve((size_t)L * (L + 1), 0.0);
    for (int i = 0; i < L; ++i) {
        double run = 0.0;
        for (int j = i; j < L; ++j) {
            run += (double)similarity[(size_t)i * L + j] * (layer_weights ? (double)layer_weights[j] : 1.0);
            serve[(size_t)i * (L + 1) + j + 1] = run;
        }
    }
    // best[m*(L+1) + j]: best total with m anchors placed, the next segment starting at layer j
    // (j = L: every layer served).  The first anchor is layer 0.
    const double kNone = -INFINITY;
    std::vector<double> best((size_t)(M + 1) * (L + 1), kNone);
    std::vector<int32_t> from((size_t)(M + 1) * (L + 1), -1);
    for (int j = 1; j <= L; ++j) { best[(size_t)1 * (L + 1) + j] = serve[j]; from[(size_t)1 * (L + 1) + j] = 0; }
    for (int m = 2; m <= M; ++m) {
        for (int j = m; j <= L; ++j) {
            double top = kNone; int arg = -1;
            for (int i = m - 1; i < j; ++i) {               // i = layer of the m-th anchor
                const double prev = best[(size_t)(m - 1) * (L + 1) + i];
                if (prev == kNone) continue;
                const double val = prev + serve[(size_t)i * (L + 1) + j];
                if (val > top) { top = val; arg = i; }      // ties keep the lowest layer
            }
            best[(size_t)m * (L + 1) + j] = top; from[(size_t)m * (L + 1) + j] = arg;
        }
    }
    int j = L;
    for (int m = M; m >= 1; --m) {
        const int i = from[(size_t)m * (L + 1) + j];
        if (i < 0) return KASCADE_INVALID_ARG;
        anchors_out[m - 1] = i;
        j = i;
    }
    if (objective_out) *objective_out = best[(size_t)M * (L + 1) + L];
    return KASCADE_OK;
}

}  // extern "C"
