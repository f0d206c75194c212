// Decode kernels of the Kascade hot path (gfx950, wave64, HBM-bound).
//
//  decode_rows_kernel   one kernel for the three row-streaming jobs of a decode step:
//      gather mode  - reuse layer / anchor pass 4 (paper Sec. 3.6): rows named by a Top-k
//                     index list are fetched from K and V and attended (Eq. 1-2 over k keys);
//      stream mode  - anchor pass 1: every key row is read once, the base-2 logits of the
//                     G query heads are written out together with per-chunk softmax statistics;
//                     with V it also accumulates dense attention (layer 0).
//  decode_merge_kernel  combines per-chunk (max, sum, acc) triples into the output.
//  decode_pool_kernel   anchor pass 2: softmax from logits + statistics, mean over the GQA
//                       group (Sec. 3.4).
//  (bf16 groups of four heads and more run both modes on the matrix unit instead:
//  decode_mfma_kernels.hip.)
//
// Data movement: a K or V row is 128..512 bytes.  LPR = row_bytes/16 adjacent lanes read one
// row with one 16-byte load each, so a wave instruction fetches 64/LPR full rows and every
// fetched byte is used.  Each lane group keeps U rows of K and of V in flight and owns a
// private online-softmax stream (m, l, acc); streams are merged once per workgroup in LDS.
#include "device_utils.h"
#include "kernels.h"

namespace kascade {

namespace {

constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / kWave;

__device__ __forceinline__ int rows_per_chunk(int n_rows, int n_chunks) {
    const int c = (n_rows + n_chunks - 1) / n_chunks;
    return (c + 63) & ~63;
}

// Workgroup-level merge of NS online-softmax streams (one per lane group) through LDS, then
// either the final output (single chunk) or this chunk's partial (max, sum, acc) triple.
template <typename T, int D, int G, int NS, int EPL, bool WITH_V>
__device__ __forceinline__ void merge_streams(const Shape& s, const DecodeRowsArgs& a, int n_chunks, int chunk_id, int b,
                                              int hk, int sid, int c, const float (&m)[G], const float (&l)[G],
                                              const float (&acc)[WITH_V ? G : 1][EPL]) {
    constexpr int GB = (G > 4) ? 4 : G;     // heads merged per LDS round
    __shared__ float sm_m[NS][G];
    __shared__ float sm_l[NS][G];
    __shared__ float sm_acc[WITH_V ? NS : 1][GB][WITH_V ? D : 1];
    if (c == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) { sm_m[sid][g] = m[g]; sm_l[sid][g] = l[g]; }
    }
#pragma unroll
    for (int gb = 0; gb < G; gb += GB) {
        if constexpr (WITH_V) {
            if (gb > 0) __syncthreads();
#pragma unroll
            for (int g = 0; g < GB; ++g)
#pragma unroll
                for (int e = 0; e < EPL; ++e) sm_acc[sid][g][c * EPL + e] = acc[gb + g][e];
        }
        __syncthreads();
        constexpr int NE = WITH_V ? GB * D : GB;
        for (int e = threadIdx.x; e < NE; e += kBlock) {
            const int g = WITH_V ? e / D : e;
            const int col = WITH_V ? e % D : 0;
            float M = -INFINITY;
#pragma unroll
            for (int t = 0; t < NS; ++t) M = fmaxf(M, sm_m[t][gb + g]);
            const float Ms = (M == -INFINITY) ? 0.f : M;
            float lsum = 0.f, val = 0.f;
#pragma unroll
            for (int t = 0; t < NS; ++t) {
                const float wgt = __builtin_amdgcn_exp2f(sm_m[t][gb + g] - Ms);
                lsum = fmaf(wgt, sm_l[t][gb + g], lsum);
                if constexpr (WITH_V) val = fmaf(wgt, sm_acc[t][g][col], val);
            }
            const int h = hk * G + gb + g;
            const int64_t pidx = ((int64_t)(b * s.Hq + h)) * n_chunks + chunk_id;
            if (WITH_V && n_chunks == 1) {
                const float o = lsum > 0.f ? val / lsum : 0.f;
                T* op = reinterpret_cast<T*>(a.out) + b * s.o_stride[0] + (int64_t)h * s.o_stride[2] + col;
                *op = narrow<T>(o);
            } else if constexpr (WITH_V) {
                a.part_acc[pidx * D + col] = val;
            }
            if (col == 0) {
                a.part_ml[pidx * 2 + 0] = M;
                a.part_ml[pidx * 2 + 1] = lsum;
            }
        }
    }
}

// An empty chunk: mark it for the merge / pooling passes (and define the output of an empty set).
template <typename T, int D, int G, bool WITH_V>
__device__ __forceinline__ void write_empty_chunk(const Shape& s, const DecodeRowsArgs& a, int n_chunks, int chunk_id, int b, int hk) {
    const int64_t part_base = ((int64_t)(b * s.Hq + hk * G)) * n_chunks + chunk_id;
    if (threadIdx.x < G) {
        float* ml = a.part_ml + (part_base + (int64_t)threadIdx.x * n_chunks) * 2;
        ml[0] = -INFINITY;
        ml[1] = 0.f;
    }
    if (WITH_V && n_chunks == 1) {
        for (int e = threadIdx.x; e < G * D; e += kBlock) {
            const int g = e / D, col = e % D;
            T* o = reinterpret_cast<T*>(a.out) + b * s.o_stride[0] + (int64_t)(hk * G + g) * s.o_stride[2] + col;
            if constexpr (sizeof(T) == 4) *o = 0.f; else *o = 0;
        }
    }
}

template <typename T, int D, int G, bool GATHER, bool WITH_V, bool STORE>
__global__ __launch_bounds__(kBlock) void decode_rows_kernel(Shape s, DecodePlan plan, DecodeRowsArgs a) {
    constexpr int EPL = Elem<T>::EPL;
    constexpr int LPR = D / EPL;            // lanes per row
    constexpr int RPW = kWave / LPR;        // row groups per wave
    constexpr int U = 8;                    // rows in flight per row group (LPR is 8, 16 or 32)
    constexpr int NS = kWavesPerBlock * RPW;  // softmax streams per workgroup
    static_assert(LPR % U == 0, "row group must hold a whole number of load batches");

    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x >> 6;
    const int c = lane % LPR;
    const int r = lane / LPR;
    const int b = blockIdx.z, hk = blockIdx.y, chunk_id = blockIdx.x;
    const int n_chunks = plan.n_chunks;

    const int L = bounded_len(a.seqlens[b], a.max_seqlen);
    int n_rows = L;
    if constexpr (GATHER) {
        int kb = a.k_per_seq[b];
        n_rows = kb < a.k_max ? kb : a.k_max;
        if (L <= 0) n_rows = 0;
    }
    // gather: the rows of this (sequence, head) are split evenly over the n_chunks workgroups;
    // stream: fixed chunk length (short sequences leave their last workgroups empty, which is cheaper
    // than many small workgroups)
    const int chunk = GATHER ? rows_per_chunk(n_rows, n_chunks) : plan.chunk;
    const int begin = chunk_id * chunk;
    const int end = (begin + chunk < n_rows) ? begin + chunk : n_rows;

    if constexpr (!GATHER) {   // pass 2 accumulates the Top-k histogram of this (b, hk): clear it here
        if (chunk_id == 0 && a.hist11) {
            uint32_t* h = a.hist11 + ((int64_t)b * s.Hkv + hk) * 2048;
            for (int i = threadIdx.x; i < 2048; i += kBlock) h[i] = 0u;
        }
    }

    if (begin >= end) {   // nothing to do
        write_empty_chunk<T, D, G, WITH_V>(s, a, n_chunks, chunk_id, b, hk);
        return;
    }

    const T* Kb = reinterpret_cast<const T*>(a.k) + b * s.kv_stride[0] + hk * s.kv_stride[1] + c * EPL;
    const T* Vb = reinterpret_cast<const T*>(a.v) + b * s.kv_stride[0] + hk * s.kv_stride[1] + c * EPL;
    const int64_t row_stride = s.kv_stride[2];

    const int32_t* idx = nullptr;
    if constexpr (GATHER) {
        int src = a.head_map ? a.head_map[hk] : hk;
        src = src < 0 ? 0 : (src >= a.n_src_heads ? a.n_src_heads - 1 : src);
        idx = a.idx + ((int64_t)b * a.n_src_heads + src) * a.k_max;
    }

    // queries of the group, pre-multiplied by scale*log2(e)
    float qf[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const T* qp = reinterpret_cast<const T*>(a.q) + b * s.q_stride[0] + (int64_t)(hk * G + g) * s.q_stride[2] + c * EPL;
        uint4 raw = *reinterpret_cast<const uint4*>(qp);
        Elem<T>::widen(raw, qf[g]);
#pragma unroll
        for (int e = 0; e < EPL; ++e) qf[g][e] *= s.scale_log2;
    }

    float m[G], l[G];
    float acc[WITH_V ? G : 1][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) { m[g] = -INFINITY; l[g] = 0.f; }
#pragma unroll
    for (int g = 0; g < (WITH_V ? G : 1); ++g)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;

    for (int j0 = begin + w * kWave; j0 < end; j0 += kWavesPerBlock * kWave) {
        int my_row = -1;
        if constexpr (GATHER) {
            int i = j0 + lane;
            if (i < end) my_row = idx[i];
            if (my_row >= L) my_row = -1;
        }
        float keep[STORE ? G : 1];
#pragma unroll
        for (int u0 = 0; u0 < LPR; u0 += U) {
            if (j0 + u0 < end) {   // wave-uniform: the smallest row of this batch is in range
                uint4 kr[U], vr[WITH_V ? U : 1];
                bool ok[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int slot = r * LPR + u0 + u;
                    int row;
                    if constexpr (GATHER) {
                        row = __shfl(my_row, slot);
                        ok[u] = row >= 0;
                    } else {
                        row = j0 + slot;
                        ok[u] = row < end;
                    }
                    row = ok[u] ? row : 0;
                    kr[u] = *reinterpret_cast<const uint4*>(Kb + (int64_t)row * row_stride);
                    if constexpr (WITH_V) vr[u] = *reinterpret_cast<const uint4*>(Vb + (int64_t)row * row_stride);
                }
                float sc[U][G];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    float kf[EPL];
                    Elem<T>::widen(kr[u], kf);
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        float d = 0.f;
#pragma unroll
                        for (int e = 0; e < EPL; ++e) d = fmaf(qf[g][e], kf[e], d);
                        d = group_sum<LPR>(d);
                        sc[u][g] = ok[u] ? d : -INFINITY;
                    }
                }
                if constexpr (STORE) {
#pragma unroll
                    for (int u = 0; u < U; ++u)
#pragma unroll
                        for (int g = 0; g < G; ++g)
                            if (c == u0 + u) keep[g] = sc[u][g];
                }
                // online softmax (base 2) of this lane group's stream
                float alpha[G];
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    float mx = sc[0][g];
#pragma unroll
                    for (int u = 1; u < U; ++u) mx = fmaxf(mx, sc[u][g]);
                    const float mnew = fmaxf(m[g], mx);
                    const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
                    alpha[g] = __builtin_amdgcn_exp2f(m[g] - msafe);
                    float psum = 0.f;
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        sc[u][g] = __builtin_amdgcn_exp2f(sc[u][g] - msafe);
                        psum += sc[u][g];
                    }
                    l[g] = fmaf(l[g], alpha[g], psum);
                    m[g] = mnew;
                }
                if constexpr (WITH_V) {
#pragma unroll
                    for (int g = 0; g < G; ++g)
#pragma unroll
                        for (int e = 0; e < EPL; ++e) acc[g][e] *= alpha[g];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        float vf[EPL];
                        Elem<T>::widen(vr[u], vf);
#pragma unroll
                        for (int g = 0; g < G; ++g)
#pragma unroll
                            for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(sc[u][g], vf[e], acc[g][e]);
                    }
                }
            }
        }
        if constexpr (STORE) {
            const int j = j0 + lane;
            if (j < end) {
#pragma unroll
                for (int g = 0; g < G; ++g)
                    a.logits[((int64_t)b * s.Hq + hk * G + g) * a.logit_pitch + j] = keep[g];
            }
        }
    }

    merge_streams<T, D, G, NS, EPL, WITH_V>(s, a, n_chunks, chunk_id, b, hk, w * RPW + r, c, m, l, acc);
}

// ---- bf16 row kernel: reuse-layer gather and anchor pass 1 (paper Sec. 3.6) -------------------
// Same data movement and modes as decode_rows_kernel, tuned for the HBM-bound bf16 case:
//  * two register buffers of U = 4 K rows (+ 4 V rows) per lane group: the loads of the next
//    batch are issued before the current batch is consumed, so a wave always has requests in flight;
//  * q.k through v_dot2c_f32_bf16 on the raw bf16 pairs (no widening), P.V through the same
//    instruction on (row u, row u+1) pairs interleaved with v_perm_b32, P rounded to bf16;
//  * the running maximum is updated lazily: accumulators are rescaled only in batches where
//    some stream's maximum actually moved.
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

__device__ __forceinline__ float dot2_bf16(uint32_t x, uint32_t y, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, x), __builtin_bit_cast(bf16x2_t, y), acc, false);
}
__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {
    bf16x2_t r;
    r[0] = (__bf16)lo; r[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, r);
}

template <int D, int G, bool GATHER, bool WITH_V, bool STORE, bool PIPE, int U = 4>
__global__ __launch_bounds__(kBlock, ((PIPE || U > 4) ? 2 : 4)) void decode_rows_bf16_kernel(Shape s, DecodePlan plan, DecodeRowsArgs a) {
    constexpr int EPL = 8;
    constexpr int LPR = D / EPL;
    constexpr int RPW = kWave / LPR;
    constexpr int NB = LPR / U;               // batches per 64-row group
    constexpr int NS = kWavesPerBlock * RPW;
    static_assert(LPR % U == 0 && U % 2 == 0, "a batch is a whole number of row pairs");
    static_assert(!PIPE || NB % 2 == 0, "double buffering walks the batches in pairs");

    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x >> 6;
    const int c = lane % LPR;
    const int r = lane / LPR;
    const int b = blockIdx.z, hk = blockIdx.y, chunk_id = blockIdx.x;
    const int n_chunks = plan.n_chunks;

    const int L = bounded_len(a.seqlens[b], a.max_seqlen);
    int n_rows = L;
    if constexpr (GATHER) {
        n_rows = a.k_per_seq[b];
        n_rows = n_rows < a.k_max ? n_rows : a.k_max;
        if (L <= 0) n_rows = 0;
    } else {
        if (chunk_id == 0 && a.hist11) {   // pass 2 accumulates the Top-k histogram of this (b, hk): clear it here
            uint32_t* hg = a.hist11 + ((int64_t)b * s.Hkv + hk) * 2048;
            for (int i = threadIdx.x; i < 2048; i += kBlock) hg[i] = 0u;
        }
    }
    // gather: the rows of this (sequence, head) are split evenly over the n_chunks workgroups;
    // stream: fixed chunk length (short sequences leave their last workgroups empty, which is cheaper
    // than many small workgroups)
    const int chunk = GATHER ? rows_per_chunk(n_rows, n_chunks) : plan.chunk;
    const int begin = chunk_id * chunk;
    const int end = (begin + chunk < n_rows) ? begin + chunk : n_rows;
    if (begin >= end) {
        write_empty_chunk<bf16_t, D, G, WITH_V>(s, a, n_chunks, chunk_id, b, hk);
        return;
    }

    const unsigned char* Kb = reinterpret_cast<const unsigned char*>(reinterpret_cast<const bf16_t*>(a.k) + b * s.kv_stride[0] + hk * s.kv_stride[1]);
    const unsigned char* Vb = reinterpret_cast<const unsigned char*>(reinterpret_cast<const bf16_t*>(a.v) + b * s.kv_stride[0] + hk * s.kv_stride[1]);
    const uint32_t row_bytes = (uint32_t)s.kv_stride[2] * 2u;
    const uint32_t lane_off = c * 16;

    const int32_t* idx = nullptr;
    if constexpr (GATHER) {
        int src = a.head_map ? a.head_map[hk] : hk;
        src = src < 0 ? 0 : (src >= a.n_src_heads ? a.n_src_heads - 1 : src);
        idx = a.idx + ((int64_t)b * a.n_src_heads + src) * a.k_max;
    }

    // raw bf16 pairs of the group's queries (this lane's 8 elements); the scale is applied to the dot
    uint32_t q2[G][4];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const bf16_t* qp = reinterpret_cast<const bf16_t*>(a.q) + b * s.q_stride[0] + (int64_t)(hk * G + g) * s.q_stride[2] + c * EPL;
        const u32x4_t raw = *reinterpret_cast<const u32x4_t*>(qp);
        q2[g][0] = raw.x; q2[g][1] = raw.y; q2[g][2] = raw.z; q2[g][3] = raw.w;
    }
    const float scale = s.scale_log2;

    float m[G], l[G], acc[WITH_V ? G : 1][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) { m[g] = -INFINITY; l[g] = 0.f; }
#pragma unroll
    for (int g = 0; g < (WITH_V ? G : 1); ++g)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;

    u32x4_t kA[U], vA[WITH_V ? U : 1], kB[U], vB[WITH_V ? U : 1];
    uint32_t okA = 0, okB = 0;
    float keep[STORE ? G : 1];

    auto fetch_idx = [&](int j0) -> int {
        if constexpr (GATHER) {
            const int i = j0 + lane;
            int row = (i < end) ? idx[i] : -1;
            return row >= L ? -1 : row;
        } else {
            return j0;   // stream mode: rows are j0 + slot
        }
    };
#define KASCADE_ISSUE(kbuf, vbuf, okv, rows_, u0_)                                                     \
    {                                                                                                  \
        okv = 0;                                                                                       \
        _Pragma("unroll") for (int u = 0; u < U; ++u) {                                                \
            int row_;                                                                                  \
            bool valid_;                                                                               \
            if constexpr (GATHER) { row_ = __shfl(rows_, r * LPR + (u0_) + u); valid_ = row_ >= 0; }   \
            else { row_ = (rows_) + r * LPR + (u0_) + u; valid_ = row_ < end; }                        \
            okv |= (valid_ ? 1u : 0u) << u;                                                            \
            const uint64_t off_ = (uint64_t)(valid_ ? row_ : 0) * row_bytes + lane_off;                \
            /* every row is touched once per call: non-temporal loads do not allocate cache lines, so  */ \
            /* they neither evict the logits / partials nor wait for dirty lines to be written back    */ \
            kbuf[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(Kb + off_));         \
            if constexpr (WITH_V) vbuf[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(Vb + off_)); \
        }                                                                                              \
    }
#define KASCADE_COMPUTE(kbuf, vbuf, okv, u0_)                                                          \
    {                                                                                                  \
        float sc[U][G];                                                                                \
        _Pragma("unroll") for (int u = 0; u < U; ++u) {                                                \
            _Pragma("unroll") for (int g = 0; g < G; ++g) {                                            \
                float d_ = dot2_bf16(kbuf[u].x, q2[g][0], 0.f);                                        \
                d_ = dot2_bf16(kbuf[u].y, q2[g][1], d_);                                               \
                d_ = dot2_bf16(kbuf[u].z, q2[g][2], d_);                                               \
                d_ = dot2_bf16(kbuf[u].w, q2[g][3], d_);                                               \
                d_ = group_sum<LPR>(d_);                                                               \
                sc[u][g] = ((okv >> u) & 1u) ? d_ * scale : -INFINITY;                                 \
                if constexpr (STORE) { if (c == (u0_) + u) keep[g] = sc[u][g]; }                       \
            }                                                                                          \
        }                                                                                              \
        float mnew[G];                                                                                 \
        bool moved_ = false;                                                                           \
        _Pragma("unroll") for (int g = 0; g < G; ++g) {                                                \
            float mx_ = fmaxf(sc[0][g], sc[1][g]);                                                     \
            _Pragma("unroll") for (int u = 2; u < U; u += 2) mx_ = fmaxf(mx_, fmaxf(sc[u][g], sc[u + 1][g])); \
            mnew[g] = fmaxf(m[g], mx_);                                                                \
            moved_ |= mnew[g] != m[g];                                                                 \
        }                                                                                              \
        if (__any(moved_)) {                                                                           \
            _Pragma("unroll") for (int g = 0; g < G; ++g) {                                            \
                const float ms_ = (mnew[g] == -INFINITY) ? 0.f : mnew[g];                              \
                const float al_ = __builtin_amdgcn_exp2f(m[g] - ms_);                                  \
                l[g] *= al_;                                                                           \
                if constexpr (WITH_V) { _Pragma("unroll") for (int e = 0; e < EPL; ++e) acc[g][e] *= al_; } \
                m[g] = mnew[g];                                                                        \
            }                                                                                          \
        }                                                                                              \
        _Pragma("unroll") for (int g = 0; g < G; ++g) {                                                \
            const float ms_ = (m[g] == -INFINITY) ? 0.f : m[g];                                        \
            _Pragma("unroll") for (int u = 0; u < U; ++u) {                                            \
                sc[u][g] = __builtin_amdgcn_exp2f(sc[u][g] - ms_);                                     \
                l[g] += sc[u][g];                                                                      \
            }                                                                                          \
        }                                                                                              \
        if constexpr (WITH_V) {                                                                        \
            _Pragma("unroll") for (int u = 0; u < U; u += 2) {                                         \
                uint32_t vp_[EPL];                                                                     \
                vp_[0] = __builtin_amdgcn_perm(vbuf[u + 1].x, vbuf[u].x, 0x05040100u);                 \
                vp_[1] = __builtin_amdgcn_perm(vbuf[u + 1].x, vbuf[u].x, 0x07060302u);                 \
                vp_[2] = __builtin_amdgcn_perm(vbuf[u + 1].y, vbuf[u].y, 0x05040100u);                 \
                vp_[3] = __builtin_amdgcn_perm(vbuf[u + 1].y, vbuf[u].y, 0x07060302u);                 \
                vp_[4] = __builtin_amdgcn_perm(vbuf[u + 1].z, vbuf[u].z, 0x05040100u);                 \
                vp_[5] = __builtin_amdgcn_perm(vbuf[u + 1].z, vbuf[u].z, 0x07060302u);                 \
                vp_[6] = __builtin_amdgcn_perm(vbuf[u + 1].w, vbuf[u].w, 0x05040100u);                 \
                vp_[7] = __builtin_amdgcn_perm(vbuf[u + 1].w, vbuf[u].w, 0x07060302u);                 \
                _Pragma("unroll") for (int g = 0; g < G; ++g) {                                        \
                    const uint32_t pp_ = pack2_bf16(sc[u][g], sc[u + 1][g]);                           \
                    _Pragma("unroll") for (int e = 0; e < EPL; ++e) acc[g][e] = dot2_bf16(vp_[e], pp_, acc[g][e]); \
                }                                                                                      \
            }                                                                                          \
        }                                                                                              \
    }

    int j0 = begin + w * kWave;
    if constexpr (PIPE) {
        int rows_cur = -1;
        if (j0 < end) {
            rows_cur = fetch_idx(j0);
            KASCADE_ISSUE(kA, vA, okA, rows_cur, 0)
        }
        for (; j0 < end; j0 += kWavesPerBlock * kWave) {
            const int j0n = j0 + kWavesPerBlock * kWave;
            int rows_next = -1;
            if (j0n < end) rows_next = fetch_idx(j0n);
#pragma unroll
            for (int bi = 0; bi < NB; bi += 2) {
                const bool haveB = j0 + (bi + 1) * U < end;           // wave-uniform
                if (haveB) KASCADE_ISSUE(kB, vB, okB, rows_cur, (bi + 1) * U)
                KASCADE_COMPUTE(kA, vA, okA, bi * U)                   // batch bi always has its first row in range
                if (bi + 2 < NB) {
                    if (j0 + (bi + 2) * U < end) KASCADE_ISSUE(kA, vA, okA, rows_cur, (bi + 2) * U)
                    else okA = 0;
                } else if (j0n < end) {
                    KASCADE_ISSUE(kA, vA, okA, rows_next, 0)
                }
                if (haveB) KASCADE_COMPUTE(kB, vB, okB, (bi + 1) * U)
                if (bi + 2 < NB && j0 + (bi + 2) * U >= end) break;   // nothing left in this 64-row group
            }
            if constexpr (STORE) {
                const int j = j0 + lane;
                if (j < end) {
#pragma unroll
                    for (int g = 0; g < G; ++g)
                        a.logits[((int64_t)b * s.Hq + hk * G + g) * a.logit_pitch + j] = keep[g];
                }
            }
            rows_cur = rows_next;
        }
    } else {
        // small problems: one register buffer, twice the resident workgroups - every workgroup of the
        // grid is on the chip at once and latency is hidden across workgroups instead of inside a wave
        (void)kB; (void)vB; (void)okB;
        for (; j0 < end; j0 += kWavesPerBlock * kWave) {
            const int rows_cur = fetch_idx(j0);
#pragma unroll
            for (int bi = 0; bi < NB; ++bi) {
                if (j0 + bi * U < end) {
                    KASCADE_ISSUE(kA, vA, okA, rows_cur, bi * U)
                    KASCADE_COMPUTE(kA, vA, okA, bi * U)
                }
            }
            if constexpr (STORE) {
                const int j = j0 + lane;
                if (j < end) {
#pragma unroll
                    for (int g = 0; g < G; ++g)
                        a.logits[((int64_t)b * s.Hq + hk * G + g) * a.logit_pitch + j] = keep[g];
                }
            }
        }
    }
#undef KASCADE_ISSUE
#undef KASCADE_COMPUTE
    merge_streams<bf16_t, D, G, NS, EPL, WITH_V>(s, a, n_chunks, chunk_id, b, hk, w * RPW + r, c, m, l, acc);
}

// grid (Hq, B), one wave per (sequence, query head):
//   out[b,h,:] = sum_c 2^(m_c - M) acc_c / sum_c 2^(m_c - M) l_c,   M = max_c m_c.
// The wave is latency-bound, so everything is requested in one round: the statistics (chunk c in
// lane c mod 64, at most kMaxChunks/64 per lane) together with the accumulators of the first
// kMergeAhead chunks (each lane owns D/64 output columns).  Chunks are added in ascending order.
constexpr int kMergeAhead = 16;
template <typename T, int D>
__global__ __launch_bounds__(kWave) void decode_merge_kernel(Shape s, int n_chunks, const float* __restrict__ part_ml,
                                                             const float* __restrict__ part_acc, void* out) {
    constexpr int CPL = D / kWave;                 // columns per lane (1 or 2)
    constexpr int SPL = kMaxChunks / kWave;        // statistics per lane
    const int h = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
    const int64_t base = ((int64_t)(b * s.Hq + h)) * n_chunks;
    float x0[kMergeAhead][CPL];
#pragma unroll
    for (int u = 0; u < kMergeAhead; ++u) {
        const int c = u < n_chunks ? u : n_chunks - 1;
#pragma unroll
        for (int e = 0; e < CPL; ++e) x0[u][e] = part_acc[(base + c) * D + e * kWave + lane];
    }
    float mloc[SPL], lloc[SPL];
#pragma unroll
    for (int i = 0; i < SPL; ++i) {
        const int c = lane + i * kWave;
        mloc[i] = -INFINITY; lloc[i] = 0.f;
        if (c < n_chunks) {
            mloc[i] = part_ml[(base + c) * 2];
            lloc[i] = part_ml[(base + c) * 2 + 1];
        }
    }
    float M = mloc[0];
#pragma unroll
    for (int i = 1; i < SPL; ++i) M = fmaxf(M, mloc[i]);
    M = wave_max(M);
    float lsum = 0.f;
    float val[CPL];
#pragma unroll
    for (int e = 0; e < CPL; ++e) val[e] = 0.f;
    if (M != -INFINITY) {
#pragma unroll
        for (int i = 0; i < SPL; ++i)
            if (mloc[i] != -INFINITY) lsum = fmaf(__builtin_amdgcn_exp2f(mloc[i] - M), lloc[i], lsum);
        lsum = wave_sum(lsum);
#pragma unroll
        for (int u = 0; u < kMergeAhead; ++u) {
            const float mc = __shfl(mloc[0], u);   // kMergeAhead <= 64: the chunk's statistics sit in lane u
            if (u < n_chunks && mc != -INFINITY) {
                const float wgt = __builtin_amdgcn_exp2f(mc - M);
#pragma unroll
                for (int e = 0; e < CPL; ++e) val[e] = fmaf(wgt, x0[u][e], val[e]);
            }
        }
        for (int c0 = kMergeAhead; c0 < n_chunks; c0 += 8) {
            float mc[8], x[8][CPL];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int c = c0 + u < n_chunks ? c0 + u : n_chunks - 1;
                mc[u] = c0 + u < n_chunks ? part_ml[(base + c) * 2] : -INFINITY;
#pragma unroll
                for (int e = 0; e < CPL; ++e) x[u][e] = part_acc[(base + c) * D + e * kWave + lane];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (mc[u] != -INFINITY) {
                    const float wgt = __builtin_amdgcn_exp2f(mc[u] - M);
#pragma unroll
                    for (int e = 0; e < CPL; ++e) val[e] = fmaf(wgt, x[u][e], val[e]);
                }
            }
        }
    }
    T* op = reinterpret_cast<T*>(out) + b * s.o_stride[0] + (int64_t)h * s.o_stride[2];
#pragma unroll
    for (int e = 0; e < CPL; ++e) {
        const float o = lsum > 0.f ? val[e] / lsum : 0.f;
        op[e * kWave + lane] = narrow<T>(o);
    }
}

// grid (ceil(max_seqlen/1024), Hkv, B), block 256: four consecutive keys per thread.
// Writes the pooled scores and counts the Top-k candidates (positions before the forced
// recent window) by the top 11 value bits of their score.
// G = 0: the group size is read from the shape (up to 16 heads per key head).
template <int G_>
__global__ __launch_bounds__(kBlock) void decode_pool_kernel(Shape s, int n_chunks, DecodePoolArgs a) {
    const int G = G_ ? G_ : s.G;
    // sequences in descending order: the sweep wrote the logits of the last sequences last, and what of them
    // is still in L2 / the memory-side cache is read before this pass's own traffic evicts it
    const int b = (int)gridDim.z - 1 - (int)blockIdx.z, hk = blockIdx.y;
    const int L = bounded_len(a.seqlens[b], a.max_seqlen);
    if (blockIdx.x == 0 && threadIdx.x == 0 && a.seg_info) a.seg_info[((int64_t)b * s.Hkv + hk) * 8] = 0u;
    if (blockIdx.x * kBlock * 4 >= L) return;   // uniform per workgroup
    int k = a.k_per_seq[b];
    k = k < 0 ? 0 : (k > L ? L : k);
    k = k > a.k_max ? a.k_max : k;
    const int n_cand = L - (a.recent_window < k ? a.recent_window : k);
    const int j = (blockIdx.x * kBlock + threadIdx.x) * 4;
    __shared__ float sh_M[G_ ? G_ : 16], sh_inv[G_ ? G_ : 16];
    __shared__ uint32_t lh[2048];
    for (int i = threadIdx.x; i < 2048; i += kBlock) lh[i] = 0u;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    for (int g = w; g < G; g += kWavesPerBlock) {
        const float* ml = a.part_ml + ((int64_t)(b * s.Hq + hk * G + g)) * n_chunks * 2;
        float M = -INFINITY;
        for (int c = lane; c < n_chunks; c += kWave) M = fmaxf(M, ml[c * 2]);
        M = wave_max(M);
        float lsum = 0.f;
        for (int c = lane; c < n_chunks; c += kWave) {
            const float mc = ml[c * 2];
            if (mc != -INFINITY) lsum = fmaf(__builtin_amdgcn_exp2f(mc - M), ml[c * 2 + 1], lsum);
        }
        lsum = wave_sum(lsum);
        if (lane == 0) { sh_M[g] = M; sh_inv[g] = 1.f / (lsum * (float)G); }
    }
    __syncthreads();
    float p[4] = {0.f, 0.f, 0.f, 0.f};
    if (j < L) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float4 sv = *reinterpret_cast<const float4*>(a.logits + ((int64_t)b * s.Hq + hk * G + g) * a.logit_pitch + j);
            const float M = sh_M[g], inv = sh_inv[g];
            p[0] = fmaf(__builtin_amdgcn_exp2f(sv.x - M), inv, p[0]);
            p[1] = fmaf(__builtin_amdgcn_exp2f(sv.y - M), inv, p[1]);
            p[2] = fmaf(__builtin_amdgcn_exp2f(sv.z - M), inv, p[2]);
            p[3] = fmaf(__builtin_amdgcn_exp2f(sv.w - M), inv, p[3]);
        }
        float* dst = a.pooled + ((int64_t)b * s.Hkv + hk) * a.pooled_pitch + j;
        if (j + 3 < L) {
            *reinterpret_cast<float4*>(dst) = make_float4(p[0], p[1], p[2], p[3]);
        } else {
            dst[0] = p[0];
            if (j + 1 < L) dst[1] = p[1];
            if (j + 2 < L) dst[2] = p[2];
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) hist_add(lh, (__float_as_uint(p[e]) >> 20) & 2047u, j + e < n_cand);
    __syncthreads();
    uint32_t* gh = a.hist11 + ((int64_t)b * s.Hkv + hk) * 2048;
    for (int i = threadIdx.x; i < 2048; i += kBlock) {
        const uint32_t c = lh[i];
        if (c) atomicAdd(&gh[i], c);
    }
}

template <typename T, int D, int G>
hipError_t launch_rows_tdg(const Shape& s, const DecodePlan& plan, const DecodeRowsArgs& a, bool gather,
                           bool with_v, bool store, hipStream_t st) {
    dim3 grid(plan.n_chunks, s.Hkv, s.B), block(kBlock);
    if (gather) {
        KASCADE_LAUNCH((decode_rows_kernel<T, D, G, true, true, false>), grid, block, 0, st, s, plan, a);
    } else if (with_v) {
        KASCADE_LAUNCH((decode_rows_kernel<T, D, G, false, true, true>), grid, block, 0, st, s, plan, a);
    } else {
        KASCADE_LAUNCH((decode_rows_kernel<T, D, G, false, false, true>), grid, block, 0, st, s, plan, a);
    }
    (void)store;
    return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_rows_td(const Shape& s, const DecodePlan& plan, const DecodeRowsArgs& a, bool gather,
                          bool with_v, bool store, hipStream_t st) {
    switch (s.G) {
        case 1: return launch_rows_tdg<T, D, 1>(s, plan, a, gather, with_v, store, st);
        case 2: return launch_rows_tdg<T, D, 2>(s, plan, a, gather, with_v, store, st);
        case 4: return launch_rows_tdg<T, D, 4>(s, plan, a, gather, with_v, store, st);
        case 8: return launch_rows_tdg<T, D, 8>(s, plan, a, gather, with_v, store, st);
    }
    return hipErrorInvalidValue;
}

template <int D, int G>
hipError_t launch_rows_bf16_dg(const Shape& s, const DecodePlan& plan, const DecodeRowsArgs& a, bool gather, bool with_v,
                               hipStream_t st) {
    dim3 grid(plan.n_chunks, s.Hkv, s.B), block(kBlock);
    // a gather grid that fits on the chip at four workgroups per compute unit runs the unpipelined form;
    // one that fits at two per compute unit keeps a wave's whole 64-row group in flight at once (16 row
    // pairs instead of 4): the kernel is then a few long-latency round trips per wave, and fewer, larger
    // ones shorten the tail in which the memory system is no longer saturated (config 2: 20.2 -> 18.3 us)
    const int64_t wgs = (int64_t)plan.n_chunks * s.Hkv * s.B;
    const bool small = gather && G <= 4 && wgs <= 4 * 256;
    if constexpr (D == 128 && G <= 4) {
        if (small && wgs <= 2 * 256) {
            KASCADE_LAUNCH((decode_rows_bf16_kernel<D, G, true, true, false, false, 16>), grid, block, 0, st, s, plan, a);
            return hipGetLastError();
        }
    }
    if (gather && small) KASCADE_LAUNCH((decode_rows_bf16_kernel<D, G, true, true, false, false>), grid, block, 0, st, s, plan, a);
    else if (gather) KASCADE_LAUNCH((decode_rows_bf16_kernel<D, G, true, true, false, true>), grid, block, 0, st, s, plan, a);
    else if (with_v) KASCADE_LAUNCH((decode_rows_bf16_kernel<D, G, false, true, true, true>), grid, block, 0, st, s, plan, a);
    else {
        // the K stream without V has registers to spare: 8 rows per batch halve a wave's round trips, which
        // shortens the tail of the launch (2 % at batch 64; no difference at batch 8)
        constexpr int US = (D == 128 && G <= 4) ? 8 : 4;
        KASCADE_LAUNCH((decode_rows_bf16_kernel<D, G, false, false, true, true, US>), grid, block, 0, st, s, plan, a);
    }
    return hipGetLastError();
}

template <int D>
hipError_t launch_rows_bf16(const Shape& s, const DecodePlan& plan, const DecodeRowsArgs& a, bool gather, bool with_v,
                            hipStream_t st) {
    switch (s.G) {
        case 1: return launch_rows_bf16_dg<D, 1>(s, plan, a, gather, with_v, st);
        case 2: return launch_rows_bf16_dg<D, 2>(s, plan, a, gather, with_v, st);
        case 4: return launch_rows_bf16_dg<D, 4>(s, plan, a, gather, with_v, st);
        case 8: return launch_rows_bf16_dg<D, 8>(s, plan, a, gather, with_v, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_decode_rows(const Shape& s, const DecodePlan& plan, const DecodeRowsArgs& a, bool gather,
                              bool with_v, bool store_logits, hipStream_t st) {
    if (s.dtype == 1) {
        if (s.D == 64) return launch_rows_bf16<64>(s, plan, a, gather, with_v, st);
        if (s.D == 128) return launch_rows_bf16<128>(s, plan, a, gather, with_v, st);
    }
    if (s.dtype == 0) {
        if (s.D == 64) return launch_rows_td<float, 64>(s, plan, a, gather, with_v, store_logits, st);
        if (s.D == 128) return launch_rows_td<float, 128>(s, plan, a, gather, with_v, store_logits, st);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_decode_merge(const Shape& s, int n_chunks, const float* part_ml, const float* part_acc,
                               void* out, hipStream_t st) {
    dim3 grid(s.Hq, s.B);
    if (s.dtype == 0 && s.D == 64) KASCADE_LAUNCH((decode_merge_kernel<float, 64>), grid, dim3(kWave), 0, st, s, n_chunks, part_ml, part_acc, out);
    else if (s.dtype == 0 && s.D == 128) KASCADE_LAUNCH((decode_merge_kernel<float, 128>), grid, dim3(kWave), 0, st, s, n_chunks, part_ml, part_acc, out);
    else if (s.dtype == 1 && s.D == 64) KASCADE_LAUNCH((decode_merge_kernel<bf16_t, 64>), grid, dim3(kWave), 0, st, s, n_chunks, part_ml, part_acc, out);
    else if (s.dtype == 1 && s.D == 128) KASCADE_LAUNCH((decode_merge_kernel<bf16_t, 128>), grid, dim3(kWave), 0, st, s, n_chunks, part_ml, part_acc, out);
    else if (s.dtype == 2 && s.D == 64) KASCADE_LAUNCH((decode_merge_kernel<f16_t, 64>), grid, dim3(kWave), 0, st, s, n_chunks, part_ml, part_acc, out);
    else if (s.dtype == 2 && s.D == 128) KASCADE_LAUNCH((decode_merge_kernel<f16_t, 128>), grid, dim3(kWave), 0, st, s, n_chunks, part_ml, part_acc, out);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_decode_pool(const Shape& s, int n_chunks, const DecodePoolArgs& a, hipStream_t st) {
    dim3 grid((a.max_seqlen + kBlock * 4 - 1) / (kBlock * 4), s.Hkv, s.B), block(kBlock);
    switch (s.G) {
        case 1: KASCADE_LAUNCH((decode_pool_kernel<1>), grid, block, 0, st, s, n_chunks, a); break;
        case 2: KASCADE_LAUNCH((decode_pool_kernel<2>), grid, block, 0, st, s, n_chunks, a); break;
        case 4: KASCADE_LAUNCH((decode_pool_kernel<4>), grid, block, 0, st, s, n_chunks, a); break;
        case 8: KASCADE_LAUNCH((decode_pool_kernel<8>), grid, block, 0, st, s, n_chunks, a); break;
        default:
            if (s.G > 16) return hipErrorInvalidValue;
            KASCADE_LAUNCH((decode_pool_kernel<0>), grid, block, 0, st, s, n_chunks, a);
            break;
    }
    return hipGetLastError();
}

}  // namespace kascade
