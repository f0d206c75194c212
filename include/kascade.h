/*
 * kascade.h - C ABI of the Kascade sparse-attention hot path for AMD MI355X (gfx950).
 *
 * Kascade (arXiv 2512.16391) computes exact post-softmax Top-k key sets in a few
 * "anchor" attention layers and re-uses them in the "reuse" layers in between
 * (Sec. 3.1-3.2).  Index sets are kept per key head (Sec. 3.5); in decode one set
 * serves the GQA group of a key head, in prefill one set serves a tile of
 * consecutive query tokens times that group (Sec. 3.4).  The four entry points
 * below are the anchor and reuse layer of Sec. 3.6 for decode and for prefill.
 *
 * Conventions shared by all calls
 *  - Every pointer is DEVICE memory owned by the caller (inputs, outputs, index
 *    buffers, workspace) except the `kascade_desc*` itself, which is HOST memory
 *    read before the call returns.  The library never allocates, frees or keeps
 *    a pointer after return.
 *  - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = the
 *    default stream) and the call returns without synchronising.
 *  - Query head h reads key head h / G, G = n_q_heads / n_kv_heads (Sec. 2.2).
 *  - Strides are in ELEMENTS; the head dimension is contiguous.  Rows (head_dim
 *    elements) of Q, K, V and O must be 16-byte aligned.
 *  - softmax is computed in fp32 on fp32-accumulated logits, scale = 1/sqrt(d)
 *    (Eq. 1) unless `softmax_scale` is non-zero.
 *  - Top-k order of preference: larger pooled score, then lower key index.  Index
 *    sets are written ascending.
 *  - Return value: KASCADE_OK or a negative status.  All argument checks happen
 *    before the first launch; on error nothing has been enqueued.
 *  - Results are deterministic: the same inputs give the same bits.
 */
#ifndef KASCADE_H
#define KASCADE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    KASCADE_OK = 0,
    KASCADE_INVALID_ARG = -1,         /* NULL pointer, non-positive size, k > L, ...          */
    KASCADE_UNSUPPORTED = -2,         /* head_dim / dtype / group size / tile size not built  */
    KASCADE_MISALIGNED = -3,          /* a base pointer or stride breaks 16-byte row alignment*/
    KASCADE_WORKSPACE_TOO_SMALL = -4, /* workspace_bytes < kascade_workspace_bytes(...)       */
    KASCADE_HIP_ERROR = -5            /* a launch failed; hipGetLastError() has the detail    */
};

enum { KASCADE_F32 = 0, KASCADE_BF16 = 1, KASCADE_F16 = 2 };

/* out_mode of the anchor calls (Sec. 3.6): layer 0 returns dense attention
 * (Sec. 3.1), every other anchor returns Top-k attention over its own fresh set. */
enum { KASCADE_OUT_DENSE = 0, KASCADE_OUT_SPARSE = 1 };

enum {
    KASCADE_OP_DECODE_ANCHOR = 0,
    KASCADE_OP_DECODE_REUSE = 1,
    KASCADE_OP_PREFILL_ANCHOR = 2,
    KASCADE_OP_PREFILL_REUSE = 3,
    KASCADE_OP_DECODE_POOLED = 4,
    KASCADE_OP_PREFILL_ANCHOR_PRESOFTMAX = 5
};

typedef struct {
    int32_t batch;          /* sequences (decode), at most 65535; must be 1 for prefill  */
    int32_t n_q_heads;      /* Hq                                                        */
    int32_t n_kv_heads;     /* Hkv, divides Hq; G = Hq/Hkv in {1,2,4,8}; 16-bit decode:  *
                             * any G <= 16                                                */
    int32_t head_dim;       /* d in {64, 128}                                            */
    int32_t dtype;          /* KASCADE_F32, KASCADE_BF16 or KASCADE_F16; Q, K, V, O share it */
    float   softmax_scale;  /* 0 -> 1/sqrt(head_dim) (Eq. 1)                             */
    int64_t q_stride[3];    /* batch, token, head   (decode ignores the token stride)    */
    int64_t kv_stride[3];   /* batch, head, token   (covers [B,Hkv,L,d] and [B,L,Hkv,d]) */
    int64_t o_stride[3];    /* batch, token, head                                        */
} kascade_desc;

/*
 * Decode, anchor layer (Sec. 3.6, passes 1-4; pooling of Sec. 3.4; Top-k of Sec. 3.5).
 * For every sequence b (context length seqlens[b], which includes the current
 * token) and key head hk: logits of the G query heads against all keys (Eq. 1),
 * softmax per head, mean over the group, then the k_per_seq[b] best keys.  The
 * last `recent_window` positions are always members and count against k.
 *   q        [B,Hq,d]           k_cache, v_cache  per kv_stride, >= seqlens[b] rows
 *   seqlens, k_per_seq  [B] int32 (device); require recent_window <= k_per_seq[b] <= seqlens[b]
 *   k_max    >= max k_per_seq (host value; row pitch of idx_out)
 *   idx_out  [B,Hkv,k_max] int32, ascending, entries past k_per_seq[b] set to -1
 *   out      [B,Hq,d]: dense attention (Eq. 2) if out_mode = KASCADE_OUT_DENSE, else
 *            attention renormalised over the fresh index set (Sec. 3.1)
 *   max_seqlen  host upper bound of seqlens (sizes the grid and the workspace); a sequence whose
 *               seqlens[b] exceeds it is processed as if it were max_seqlen long
 */
int kascade_decode_anchor(const kascade_desc* desc, const void* q, const void* k_cache,
                          const void* v_cache, const int32_t* seqlens, const int32_t* k_per_seq,
                          int32_t max_seqlen, int32_t k_max, int32_t recent_window, int32_t out_mode,
                          int32_t* idx_out, void* out, void* workspace, size_t workspace_bytes,
                          void* hip_stream);

/*
 * Decode, reuse layer (Sec. 3.6 first paragraph; head map of Sec. 3.5).
 * Key head hk of this layer attends to rows idx_in[b, head_map[hk], 0:k_per_seq[b]]
 * of its own K/V cache; softmax over exactly those rows.  Entries that are
 * negative or >= seqlens[b] are ignored.  Any order is accepted.
 *   idx_in   [B,Hkv_anchor,k_max] int32 with n_anchor_heads rows per sequence
 *   head_map [Hkv] int32 (device) with values in [0, n_anchor_heads), or NULL = identity
 */
int kascade_decode_reuse(const kascade_desc* desc, const void* q, const void* k_cache,
                         const void* v_cache, const int32_t* seqlens, const int32_t* k_per_seq,
                         int32_t k_max, const int32_t* idx_in, int32_t n_anchor_heads,
                         const int32_t* head_map, void* out, void* workspace,
                         size_t workspace_bytes, void* hip_stream);

/*
 * kascade_decode_reuse for callers that cannot allocate or pass scratch memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and bits as
 * kascade_decode_reuse, minus the workspace: the partial results of the gather live in a fixed
 * 8 MiB array in device memory that belongs to the library (each GPU the library runs on holds its own
 * copy until the process ends; its address is looked up once per device on the first call there).  The
 * call allocates nothing and frees nothing.  A shape whose partial results need more than
 * kascade_decode_reuse_static_capacity() bytes - what kascade_workspace_bytes(KASCADE_OP_DECODE_REUSE, ...)
 * reports - returns KASCADE_WORKSPACE_TOO_SMALL before anything is enqueued (the Llama-shaped
 * configurations need about 1 MiB at any batch size).  All calls on one GPU share that GPU's array: calls
 * that overlap in time on one GPU (two streams, two threads) race on it; calls on one stream do not.
 * Nothing in the array has to start at zero: every call writes all partial results it later reads.
 */
int kascade_decode_reuse_static(const kascade_desc* desc, const void* q, const void* k_cache,
                                const void* v_cache, const int32_t* seqlens, const int32_t* k_per_seq,
                                int32_t k_max, const int32_t* idx_in, int32_t n_anchor_heads,
                                const int32_t* head_map, void* out, void* hip_stream);
size_t kascade_decode_reuse_static_capacity(void);

/*
 * Prefill, anchor layer (Sec. 3.6 passes 1-4 with the score matrix recomputed in
 * pass 2; tile pooling of Sec. 3.4; rolling Top-k of Sec. 4.1).  batch = 1.
 * Tile t covers tokens [t*T, min((t+1)*T, S)), T = q_tile_tokens; its rows are those
 * tokens times the G heads of a key head.  Candidates of tile t are the keys
 * j < t*T; the pooled score of key j is the mean over the tile's rows of the causal
 * post-softmax weight (row normalisers include the diagonal keys).  k_per_tile[t]
 * <= t*T keys are selected per key head; the diagonal block t*T..i is always
 * attended on top, causally.
 *   q [S,Hq,d] per q_stride;  k, v [Hkv,S,d] per kv_stride; bf16 or fp16, T*G a multiple of 128 (the
 *   paper's tile is T*G = 128 rows), and the rows of one key head must span less than 4 GiB
 *   (S * kv_stride[2] * 2 bytes), else KASCADE_UNSUPPORTED
 *   k_per_tile  [n_tiles] int32 (device), idx_offsets [n_tiles+1] int64 (device),
 *               idx_offsets[t+1]-idx_offsets[t] = k_per_tile[t], idx_total = idx_offsets[n_tiles]
 *               (host value; a device-side offset or budget that would reach past idx_total
 *               entries is cut to what fits)
 *   idx_out  [Hkv, idx_total] int32: tile t of head hk at hk*idx_total + idx_offsets[t]
 *   out [S,Hq,d]: causal dense attention (KASCADE_OUT_DENSE) or sparse attention over the
 *       fresh sets (KASCADE_OUT_SPARSE)
 */
int kascade_prefill_anchor(const kascade_desc* desc, const void* q, const void* k, const void* v,
                           int32_t seqlen, int32_t q_tile_tokens, const int32_t* k_per_tile,
                           const int64_t* idx_offsets, int64_t idx_total, int32_t out_mode,
                           int32_t* idx_out, void* out, void* workspace, size_t workspace_bytes,
                           void* hip_stream);

/*
 * Prefill, reuse layer (Sec. 3.6 first paragraph, Sec. 4.1): every row (token i in
 * tile t, head h) attends to idx_in[head_map[h/G]] of its tile plus the keys
 * t*T..i; one softmax over the union.  Entries outside [0, t*T) are ignored.
 */
int kascade_prefill_reuse(const kascade_desc* desc, const void* q, const void* k, const void* v,
                          int32_t seqlen, int32_t q_tile_tokens, const int32_t* k_per_tile,
                          const int64_t* idx_offsets, int64_t idx_total, const int32_t* idx_in,
                          int32_t n_anchor_heads, const int32_t* head_map, void* out,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Shared index sets (Sec. 3.5, the "all heads pooled" variant): the anchor calls above with the pooled
 * distributions of all key heads averaged into one per sequence (decode) or per tile (prefill), so one
 * Top-k set serves every head of the layer.  Same arguments, checks and workspace sizes as
 * kascade_decode_anchor / kascade_prefill_anchor, except
 *   idx_out  decode: [B,1,k_max];  prefill: [1,idx_total]
 * Reuse layers consume such a set through kascade_decode_reuse / kascade_prefill_reuse with
 * n_anchor_heads = 1 and a head_map of Hkv zeros.
 */
int kascade_decode_anchor_shared(const kascade_desc* desc, const void* q, const void* k_cache,
                                 const void* v_cache, const int32_t* seqlens, const int32_t* k_per_seq,
                                 int32_t max_seqlen, int32_t k_max, int32_t recent_window,
                                 int32_t out_mode, int32_t* idx_out, void* out, void* workspace,
                                 size_t workspace_bytes, void* hip_stream);
int kascade_prefill_anchor_shared(const kascade_desc* desc, const void* q, const void* k, const void* v,
                                  int32_t seqlen, int32_t q_tile_tokens, const int32_t* k_per_tile,
                                  const int64_t* idx_offsets, int64_t idx_total, int32_t out_mode,
                                  int32_t* idx_out, void* out, void* workspace, size_t workspace_bytes,
                                  void* hip_stream);

/*
 * Pre-Softmax pooling (Sec. 3.4, the alternative the paper evaluates and rejects; here for the same
 * comparison): instead of pooling post-softmax distributions, the query vectors of a pooling unit -
 * decode: the G heads of a key head; prefill: the T tokens x G heads of a tile - are averaged into one
 * query, attention scores (Eq. 1) are computed once with it, and the Top-k of that distribution is
 * the unit's index set.  The pooled query is kept in the tensors' own type: summed in fp32 (tokens
 * ascending, heads ascending inside a token), divided by the count, rounded once (bf16: to nearest
 * even).  Same arguments, checks, outputs and out_mode meaning as kascade_decode_anchor /
 * kascade_prefill_anchor; the sets feed the ordinary reuse calls.
 *   decode   workspace: kascade_workspace_bytes(KASCADE_OP_DECODE_ANCHOR, ...), as for the anchor call.
 *   prefill  candidates of tile t are the t*T keys before it, as in kascade_prefill_anchor.  Runs on
 *            the decode kernels with tiles as sequences over one shared cache and is not tuned; it
 *            keeps fp32 logits and pooled scores of every (tile, key head) over max prefix length:
 *            kascade_workspace_bytes(KASCADE_OP_PREFILL_ANCHOR_PRESOFTMAX, desc, seqlen, idx_total, T),
 *            about 8 * n_tiles * Hkv * seqlen bytes (2.1 GB at 32768 tokens, T = 32, 8 key heads).
 *            At most 65535 tiles, else KASCADE_UNSUPPORTED.
 */
int kascade_decode_anchor_presoftmax(const kascade_desc* desc, const void* q, const void* k_cache,
                                     const void* v_cache, const int32_t* seqlens, const int32_t* k_per_seq,
                                     int32_t max_seqlen, int32_t k_max, int32_t recent_window,
                                     int32_t out_mode, int32_t* idx_out, void* out, void* workspace,
                                     size_t workspace_bytes, void* hip_stream);
int kascade_prefill_anchor_presoftmax(const kascade_desc* desc, const void* q, const void* k, const void* v,
                                      int32_t seqlen, int32_t q_tile_tokens, const int32_t* k_per_tile,
                                      const int64_t* idx_offsets, int64_t idx_total, int32_t out_mode,
                                      int32_t* idx_out, void* out, void* workspace, size_t workspace_bytes,
                                      void* hip_stream);

/*
 * Calibration path (Sec. 3.3): which layers become anchors is decided once per model from how
 * well one layer's Top-k set recovers a later layer's attention mass (Eq. 3).
 *
 * kascade_decode_pooled: passes 1-2 of the decode anchor layer only.  Writes the pooled
 * post-softmax distribution (Eq. 1 per query head, mean over each GQA group, Sec. 3.4):
 *   pooled_out [B,Hkv,pooled_pitch] fp32 (device), entries j < seqlens[b] written, the rest
 *   untouched; pooled_pitch >= max_seqlen and a multiple of 4; 16-byte aligned base.
 *   Workspace: kascade_workspace_bytes(KASCADE_OP_DECODE_POOLED, desc, max_seqlen, 0, 0).
 */
int kascade_decode_pooled(const kascade_desc* desc, const void* q, const void* k_cache,
                          const int32_t* seqlens, int32_t max_seqlen, float* pooled_out,
                          int64_t pooled_pitch, void* workspace, size_t workspace_bytes,
                          void* hip_stream);

/*
 * Similarity of layer a's Top-k sets applied to layer b (Eq. 3), per (sequence, key head):
 *   sim = sum_{j in idx_a[b, head_map[hk]]} pooled_b[b,hk,j] / sum_{j in idx_b[b,hk]} pooled_b[b,hk,j]
 * over the first k_per_seq[b] entries of each set; entries that are negative or >= seqlens[b]
 * are ignored; an empty denominator gives 1.  Sums are fp32 in a fixed order.
 *   pooled_b [B,Hkv,pooled_pitch] fp32; idx_a [B,n_heads_a,k_max], idx_b [B,Hkv,k_max] int32;
 *   head_map [Hkv] int32 into layer a's heads (Sec. 3.5) or NULL = identity (n_heads_a = Hkv)
 *   sim_out  [B,Hkv] fp32 or NULL
 *   sim_min  one fp32 or NULL: lowered to the smallest similarity of this call if that is below
 *            its current value (Sec. 3.3 takes the minimum over the tokens of a prompt; start it
 *            at 1).  All pointers are device memory.  At least one output is required.
 */
int kascade_topk_similarity(int32_t batch, int32_t n_kv_heads, const float* pooled_b,
                            int64_t pooled_pitch, const int32_t* seqlens, const int32_t* k_per_seq,
                            int32_t k_max, const int32_t* idx_a, int32_t n_heads_a,
                            const int32_t* head_map, const int32_t* idx_b, float* sim_out,
                            float* sim_min, void* hip_stream);

/*
 * Anchor-layer selection (Sec. 3.3, Algorithm 1).  HOST function, HOST pointers, no GPU work.
 * similarity [n_layers,n_layers] row-major, entry (i,j), i <= j: similarity of layer i's Top-k
 * set applied to layer j (entries below the diagonal are not read).  Chooses n_anchors layers,
 * layer 0 always among them, such that every layer is served by the closest anchor at or before
 * it and the sum of the served similarities is largest; among equal sums the earlier layer wins
 * at each step of the recurrence.  Sums are fp64.
 *   layer_weights [n_layers] or NULL: importance of each layer; entry (i,j) is multiplied by
 *                 layer_weights[j], the weight of the served layer (Sec. 3.3)
 *   anchors_out [n_anchors] int32, ascending 0-based layer numbers
 *   objective_out  the attained sum, or NULL
 * Errors: NULL pointers, n_layers outside [1,4096], n_anchors outside [1,n_layers], NaN entries.
 */
int kascade_select_anchor_layers(const float* similarity, const float* layer_weights,
                                 int32_t n_layers, int32_t n_anchors, int32_t* anchors_out,
                                 double* objective_out);

/*
 * Head-level similarity (Sec. 3.5, Eq. 3 per pair of heads): for every sequence b, every key
 * head hk of the reuse layer and every key head ha of the anchor layer,
 *   sim_out[b,hk,ha] = sum_{j in idx_a[b,ha]} pooled_b[b,hk,j] / sum_{j in idx_b[b,hk]} pooled_b[b,hk,j]
 * with the same conventions as kascade_topk_similarity.  sim_out [B,Hkv,n_heads_a] fp32 (device).
 */
int kascade_head_similarity(int32_t batch, int32_t n_kv_heads, const float* pooled_b,
                            int64_t pooled_pitch, const int32_t* seqlens, const int32_t* k_per_seq,
                            int32_t k_max, const int32_t* idx_a, int32_t n_heads_a,
                            const int32_t* idx_b, float* sim_out, void* hip_stream);

/*
 * Head map of a reuse layer (Sec. 3.5): each of its key heads takes the anchor-layer head with
 * the largest mean similarity over the samples; several heads may take the same one; equal means
 * go to the lower anchor head.  (The paper aggregates over its development set without naming the
 * statistic; the mean is this library's reading.)
 *   sim [n_samples,Hkv,n_heads_a] fp32 (device), e.g. kascade_head_similarity outputs stacked
 *   mean_out [Hkv,n_heads_a] fp32 (device) or NULL;  head_map_out [Hkv] int32 (device), the
 *   array the reuse entry points take as `head_map`.
 */
int kascade_head_map(int32_t n_samples, int32_t n_kv_heads, int32_t n_heads_a, const float* sim,
                     float* mean_out, int32_t* head_map_out, void* hip_stream);

/*
 * Layer importance (Sec. 3.3): w_out[r] = 1 - cosine similarity of row r of x (input of a
 * layer's attention block) and row r of y (its output); fp32 accumulation.  Averaging the rows
 * of a layer gives the weight passed to kascade_select_anchor_layers.
 *   x, y [n_rows,n_cols] of `dtype` (KASCADE_F32 / KASCADE_BF16 / KASCADE_F16), row strides in elements;
 *   w_out [n_rows] fp32.  All device memory.  A zero row gives NaN.
 */
int kascade_layer_importance(const void* x, const void* y, int64_t n_rows, int32_t n_cols,
                             int32_t dtype, int64_t x_row_stride, int64_t y_row_stride,
                             float* w_out, void* hip_stream);

/*
 * Bytes of workspace the given op needs (0 is a valid answer).
 *   decode ops:  max_seqlen = largest context length, k_or_idx_total = k_max
 *   prefill ops: max_seqlen = S, k_or_idx_total = idx_total, q_tile_tokens = T
 * Returns 0 for an unknown op or an invalid descriptor.
 */
size_t kascade_workspace_bytes(int32_t op, const kascade_desc* desc, int64_t max_seqlen,
                               int64_t k_or_idx_total, int32_t q_tile_tokens);

/* Static, NUL-terminated description of a status code. */
const char* kascade_status_string(int32_t status);

/*
 * Measurement aid (not part of the method): per-kernel device time.
 * kascade_profile_enable(1) makes every later kernel dispatch of the library carry a start and a
 * stop event bound to that dispatch (their difference is the dispatch's begin-to-end time on the
 * device, the figure a kernel trace reports); events are created on demand (so do not enable it
 * under stream capture) and destroyed by kascade_profile_enable(0).  kascade_profile_read waits
 * for the recorded events of step `kernel` (0 <= kernel < kascade_profile_kernels()) and returns
 * its name, the summed milliseconds of its dispatches and the number of times the step ran since
 * the last kascade_profile_reset() (a step that takes several dispatches, such as the split Top-k
 * selection, counts once).  With profiling off (the default) the library creates no events and
 * launches plainly.  Process-wide state, guarded by a mutex.
 */
int kascade_profile_enable(int32_t on);
int kascade_profile_reset(void);
int32_t kascade_profile_kernels(void);
int kascade_profile_read(int32_t kernel, const char** name, double* total_ms, int64_t* launches);

/*
 * Test and measurement aid (not part of the method): overrides of the launch plan, process-wide.
 * value 0 (the default) leaves the choice to the library.  The overrides change the number of
 * partial results and with it kascade_workspace_bytes(): the size query and the call read the same
 * process-wide value, and a call whose workspace is smaller than its plan needs returns
 * KASCADE_WORKSPACE_TOO_SMALL as always.  The library reads no environment variables.
 *   KASCADE_TUNE_DECODE_FAMILY  1 = vector-ALU decode row kernels, 2 = matrix-unit kernels (where both exist)
 *   KASCADE_TUNE_STREAM_CHUNK   key rows per workgroup of the decode anchor's sweep (rounded up to 64)
 *   KASCADE_TUNE_GATHER_CHUNK   index entries per workgroup of the decode gather (rounded up to 64)
 *   KASCADE_TUNE_TOPK_PARTS     workgroups per (sequence, key head) of the decode selection (1 = one workgroup)
 * Returns KASCADE_INVALID_ARG for an unknown knob or a negative value.
 */
enum {
    KASCADE_TUNE_DECODE_FAMILY = 0,
    KASCADE_TUNE_STREAM_CHUNK = 1,
    KASCADE_TUNE_GATHER_CHUNK = 2,
    KASCADE_TUNE_TOPK_PARTS = 3,
    KASCADE_TUNE_COUNT = 4
};
int kascade_tuning_set(int32_t knob, int32_t value);
int32_t kascade_tuning_get(int32_t knob);

/* Library version, "major.minor". */
const char* kascade_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KASCADE_H */
