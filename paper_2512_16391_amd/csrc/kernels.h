// Host-side launch interface between the C ABI (api.hip) and the kernel files.
// Everything here is internal to the library.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

namespace kascade {

// Every kernel of the library is launched through KASCADE_LAUNCH.  When the per-kernel timing aid of the
// C ABI is switched on, next_launch_events() hands out a start and a stop event that are bound to the
// dispatch itself; otherwise both are null and the launch is a plain one.
struct LaunchEvents { hipEvent_t start, stop; };
LaunchEvents next_launch_events();
#define KASCADE_LAUNCH(kernel_, grid_, block_, shmem_, stream_, ...)                                            \
    do {                                                                                                        \
        const ::kascade::LaunchEvents ev_ = ::kascade::next_launch_events();                                    \
        if (ev_.start) hipExtLaunchKernelGGL(kernel_, grid_, block_, shmem_, stream_, ev_.start, ev_.stop, 0, __VA_ARGS__); \
        else hipLaunchKernelGGL(kernel_, grid_, block_, shmem_, stream_, __VA_ARGS__);                          \
    } while (0)

struct Shape {
    int B, Hq, Hkv, D, G;
    int dtype;              // 0 fp32, 1 bf16, 2 fp16 (matrix-unit kernels only)
    float scale_log2;       // softmax scale * log2(e): all softmax arithmetic is base 2
    int64_t q_stride[3];
    int64_t kv_stride[3];
    int64_t o_stride[3];
};

// ---- decode ------------------------------------------------------------------
// One launch plan for the row-streaming kernel: `chunk` rows per workgroup,
// `n_chunks` workgroups per (sequence, key head).
struct DecodePlan {
    int chunk;
    int n_chunks;
};

constexpr int kMaxChunks = 256;   // chunks per (sequence, head) a plan may ask for; the merge keeps their statistics in registers

struct DecodeRowsArgs {
    const void* q;
    const void* k;
    const void* v;
    const int32_t* seqlens;
    int32_t max_seqlen;           // lengths above this host bound are treated as the bound (it sized the buffers); 0 = none
    const int32_t* k_per_seq;     // gather mode: rows per (b, hk); null in stream mode
    const int32_t* idx;           // gather mode: [B, n_src_heads, k_max]
    const int32_t* head_map;      // gather mode: [Hkv] or null
    int32_t k_max;
    int32_t n_src_heads;
    float* logits;                // stream mode: [B, Hq, logit_pitch] base-2 scaled logits
    int64_t logit_pitch;
    float* part_ml;               // [B, Hq, n_chunks, 2]  (max, sum of 2^(s-max)) per chunk
    float* part_acc;              // [B, Hq, n_chunks, D]  sum of 2^(s-max) * V, or null (no V)
    void* out;                    // final output, written directly when n_chunks == 1 and V is read
    uint32_t* hist11;             // stream mode: [B, Hkv, 2048] Top-k histogram, zeroed here for pass 2
};

// gather = true: rows come from the index list (reuse layer); false: rows 0..L-1 (anchor pass 1)
hipError_t launch_decode_rows(const Shape& s, const DecodePlan& plan, const DecodeRowsArgs& a,
                              bool gather, bool with_v, bool store_logits, hipStream_t st);

// Gather mode on the matrix unit (bf16, head dimension 64 or 128, up to 16 heads per key head): same plan,
// arguments and partial-result format as launch_decode_rows(gather = true).
hipError_t launch_decode_gather_mfma(const Shape& s, const DecodePlan& plan, const DecodeRowsArgs& a, hipStream_t st);
// Stream mode with stored logits on the matrix unit, same restrictions; same plan, arguments and results as
// launch_decode_rows(gather = false, store_logits = true).
hipError_t launch_decode_stream_mfma(const Shape& s, const DecodePlan& plan, const DecodeRowsArgs& a, bool with_v, hipStream_t st);

// Merge the per-chunk partial results into the final output [B, Hq, D].
hipError_t launch_decode_merge(const Shape& s, int n_chunks, const float* part_ml,
                               const float* part_acc, void* out, hipStream_t st);

// Anchor pass 2: softmax from the logits and per-chunk stats, mean over the GQA group.
// Also counts, per (sequence, key head), the pooled scores of the Top-k candidates by their top
// 11 value bits into hist11 [B, Hkv, 2048] (first radix round of the selection).
struct DecodePoolArgs {
    const int32_t* seqlens;
    const int32_t* k_per_seq;
    int32_t k_max;
    int32_t recent_window;
    const float* logits;
    int64_t logit_pitch;
    const float* part_ml;
    float* pooled;
    int64_t pooled_pitch;
    uint32_t* hist11;
    int max_seqlen;
    uint32_t* seg_info;           // split selection: [B, Hkv, 8] words, word 0 (candidate counter) cleared here; or null
};
hipError_t launch_decode_pool(const Shape& s, int n_chunks, const DecodePoolArgs& a, hipStream_t st);

// ---- Top-k select -------------------------------------------------------------
// Segment descriptor modes:
//   decode : segment (b, hk): scores at pooled + (b*Hkv+hk)*pitch, length seqlens[b],
//            k = k_per_seq[b], out at idx_out + (b*Hkv+hk)*k_max, padded with -1 to k_max.
//   prefill: segment (t, hk): scores at pooled + hk*pooled_pitch + seg_offsets[t], length t*T,
//            k = k_per_tile[t], out at idx_out + hk*idx_total + idx_offsets[t].
struct TopkArgs {
    const float* scores;
    const uint32_t* hist11;       // decode: precomputed first-round histogram, or null
    int32_t* idx_out;
    // decode
    const int32_t* seqlens;
    const int32_t* k_per_seq;
    int64_t pitch;
    int32_t k_max;
    int32_t recent_window;
    // decode segments written in the prefill layout (Pre-Softmax pooling of prefill tiles, one "sequence"
    // per tile): out at idx_out + hk*out_head_pitch + out_offsets[b], no padding; null = decode layout
    const int64_t* out_offsets;
    int64_t out_head_pitch;
    // decode, split selection (several workgroups per segment): null / 0 when unused
    uint32_t* cand;               // [B, Hkv, kTopkCandCap] threshold-bucket candidates: low 20 score bits | part << 20
    uint32_t* seg_info;           // [B, Hkv, 8]: candidate count, round-1 digit / rest / bucket size, THR, need_eq, fallback flag
    uint32_t* part_info;          // [B, Hkv, kTopkMaxParts, 2]: scores above the bucket per part, then output offsets
    int32_t n_parts;
    int32_t max_seqlen;
    // prefill
    const int32_t* k_per_tile;
    const int64_t* idx_offsets;
    int64_t idx_total;
    int64_t pooled_pitch;
    int32_t tile_tokens;
    int32_t n_tiles;
};
constexpr int kTopkCandCap = 8192;   // scores of the threshold bucket the selection keeps on chip
constexpr int kTopkMaxParts = 64;
hipError_t launch_topk_decode(const Shape& s, const TopkArgs& a, hipStream_t st);
// the same selection with n_parts workgroups per segment (three launches); needs the first-round histogram
hipError_t launch_topk_decode_split(const Shape& s, const TopkArgs& a, hipStream_t st);

// ---- calibration: Top-k set similarity (Eq. 3) ----------------------------------------
struct SimilarityArgs {
    int B, Hkv;
    const float* pooled;          // layer b: [B, Hkv, pitch]
    int64_t pitch;
    const int32_t* seqlens;
    const int32_t* k_per_seq;
    int32_t k_max;
    const int32_t* idx_a;         // [B, n_heads_a, k_max]
    int32_t n_heads_a;
    const int32_t* head_map;      // [Hkv] into layer a's heads, or null
    const int32_t* idx_b;         // [B, Hkv, k_max]
    float* sim_out;               // [B, Hkv] or null; all_pairs: [B, Hkv, n_heads_a]
    float* sim_min;               // one float, min-updated, or null
    int all_pairs;                // 1: every head of layer a against every head of layer b (head_map unused)
};
hipError_t launch_similarity(const SimilarityArgs& a, hipStream_t st);
hipError_t launch_head_map(int B, int Hkv, int Ha, const float* sim, float* mean_out, int32_t* head_map_out,
                           hipStream_t st);
hipError_t launch_importance(int dtype, const void* x, const void* y, int64_t n_rows, int n_cols, int64_t x_stride,
                             int64_t y_stride, float* w_out, hipStream_t st);

// ---- Pre-Softmax pooling (Sec. 3.4 alternative): pooled queries ----------------------------------
// unit = sequence (decode: tokens_per_unit = n_tokens = 1, unit_stride = batch stride, tile_lens null)
// or query tile (prefill: tokens [unit*T, min((unit+1)*T, n_tokens)), tile_lens receives unit*T).
// qbar [n_units, Hkv, D] in the tensors' type.
hipError_t launch_pool_queries(int dtype, const void* q, int64_t unit_stride, int64_t token_stride, int64_t head_stride,
                               int G, int tokens_per_unit, int n_tokens, int n_units, void* qbar, int Hkv, int D,
                               int32_t* tile_lens, hipStream_t st);

// ---- shared index sets (Sec. 3.5, all heads pooled) --------------------------------------
// rows[batch][head][j] (head_pitch apart, batch_pitch between batches): row 0 of every batch becomes
// the mean over the n_heads rows, for j < (lens ? lens[batch] : n).  Also writes n_heads zeros to
// zero_map: the head map that sends every head of a layer to index set 0.
hipError_t launch_pool_heads(float* rows, int64_t batch_pitch, int64_t head_pitch, int n_heads, int n_batches,
                             int64_t n, const int32_t* lens, int32_t* zero_map, hipStream_t st);

// ---- prefill -----------------------------------------------------------------------
struct PrefillArgs {
    const void* q;                // [S, Hq, D] per q_stride
    const void* k;                // [Hkv, S, D] per kv_stride
    const void* v;
    void* out;                    // [S, Hq, D] per o_stride (attend kernels with V)
    float* stats;                 // [Hq, S, 2] row (max, sum) in base-2 scaled units; null = not written
    float* pooled;                // pool kernel: [Hkv, pooled_pitch], tile t at T*t*(t-1)/2
    int64_t pooled_pitch;
    const int32_t* idx;           // sparse: [n_src_heads, idx_total]
    const int64_t* idx_offsets;   // [n_tiles + 1]
    const int32_t* k_per_tile;    // [n_tiles]
    const int32_t* head_map;      // [Hkv] or null
    int64_t idx_total;
    int32_t n_src_heads;
    int32_t seqlen, tile_tokens, n_tiles;   // a tile: tile_tokens tokens x G heads = a multiple of 128 rows
    int32_t sub_tokens, n_sub;              // a workgroup's share: 128 / G tokens (x G heads = 128 rows); ceil(seqlen / sub_tokens)
    int32_t* topk_out;            // pool kernel: [Hkv, idx_total] receives the per-(tile, head) Top-k sets; null = pooled scores only
};
// sparse = false: all keys up to the diagonal (causal); with_v = false computes statistics only
hipError_t launch_prefill_attend(const Shape& s, const PrefillArgs& a, bool sparse, bool with_v, hipStream_t st);
hipError_t launch_prefill_pool(const Shape& s, const PrefillArgs& a, hipStream_t st);
hipError_t launch_topk_prefill(const Shape& s, const TopkArgs& a, hipStream_t st);

}  // namespace kascade
