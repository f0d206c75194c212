// Top-k selection kernels (paper Sec. 3.6, pass 3): one workgroup of 1024 threads per segment
// (decode: per sequence and key head; prefill: per tile and key head, used by the shared-set variant -
// the per-head prefill selection runs inside the pooling kernel), and the split form for few long
// decode segments.  The selection itself is in topk_select.h.
#include "topk_select.h"

namespace kascade {

namespace {

constexpr int kTopkBlock = 1024;
constexpr int kTopkWaves = kTopkBlock / kWave;

__global__ __launch_bounds__(kTopkBlock) void topk_decode_kernel(Shape s, TopkArgs a) {
    const int hk = blockIdx.x, b = blockIdx.y;
    const int L = bounded_len(a.seqlens[b], a.max_seqlen);
    int k = a.k_per_seq[b];
    k = k < 0 ? 0 : (k > L ? L : k);
    k = k > a.k_max ? a.k_max : k;
    int W = a.recent_window < k ? a.recent_window : k;
    Segment sg;
    sg.scores = a.scores + ((int64_t)b * s.Hkv + hk) * a.pitch;
    sg.out = a.idx_out + ((int64_t)b * s.Hkv + hk) * a.k_max;
    sg.hist11 = a.hist11 ? a.hist11 + ((int64_t)b * s.Hkv + hk) * 2048 : nullptr;
    sg.n = L - W;
    sg.k_sel = k - W;
    sg.forced = W;
    sg.pad_to = a.k_max;
    if (a.out_offsets) {
        const TileSlot slot = bounded_tile_slot(k, a.out_offsets[b], L, a.out_head_pitch);
        sg.out = a.idx_out + hk * a.out_head_pitch + slot.off;
        sg.k_sel = slot.k - W;
        sg.pad_to = slot.k;
    }
    __shared__ SelectShared<kTopkBlock> sm;
    select_segment<kTopkBlock>(sg, sm);
}

__global__ __launch_bounds__(kTopkBlock) void topk_prefill_kernel(Shape s, TopkArgs a) {
    // long segments first (the last workgroups to start are then the shortest), key head = block mod
    // Hkv as in the attention kernels, so a head's pooled scores are swept by the XCD that wrote them
    const int hk = blockIdx.x % s.Hkv;
    const int t = a.n_tiles - 1 - blockIdx.x / s.Hkv;
    const int64_t prefix = (int64_t)t * a.tile_tokens;
    const TileSlot slot = bounded_tile_slot(a.k_per_tile[t], a.idx_offsets[t], prefix, a.idx_total);
    const int k = slot.k;
    // pooled scores of tile t start after those of tiles 0..t-1: sum_{u<t} u*T = T*t*(t-1)/2
    const int64_t seg_off = (int64_t)a.tile_tokens * t * (t - 1) / 2;
    Segment sg;
    sg.scores = a.scores + hk * a.pooled_pitch + seg_off;
    sg.out = a.idx_out + hk * a.idx_total + slot.off;
    sg.hist11 = nullptr;
    sg.n = (int)prefix;
    sg.k_sel = k;
    sg.forced = 0;
    sg.pad_to = k;
    __shared__ SelectShared<kTopkBlock> sm;
    select_segment<kTopkBlock>(sg, sm);
}


// ---- split selection: several workgroups per segment -------------------------------------------
// With few long segments (one request, 128k tokens: eight segments) one workgroup per segment leaves
// the chip idle and pays two full sweeps of the segment at one workgroup's bandwidth.  Here a
// segment is cut into n_parts contiguous parts:
//   collect    every part finds the threshold bucket d1 from the precomputed first-round histogram,
//              counts its scores above the bucket and appends its scores inside the bucket (low 20
//              bits, tagged with the part) to the segment's candidate list in memory;
//   threshold  one workgroup per segment runs rounds 2-3 on the candidates (as the single-workgroup
//              path does in LDS), then counts per part how many candidates lie above / at THR and
//              turns the counts into each part's output offsets;
//   compact    every part writes its selected positions in order at its offset.
// A threshold bucket with more than kCandCap scores falls back to select_segment in `threshold`.
struct DecodeSeg {
    int n, k_sel, forced;
};
__device__ __forceinline__ DecodeSeg decode_segment(const TopkArgs& a, int b) {
    const int L = bounded_len(a.seqlens[b], a.max_seqlen);
    int k = a.k_per_seq[b];
    k = k < 0 ? 0 : (k > L ? L : k);
    k = k > a.k_max ? a.k_max : k;
    const int W = a.recent_window < k ? a.recent_window : k;
    DecodeSeg d;
    d.n = L - W; d.k_sel = k - W; d.forced = W;
    return d;
}
// scores per part: a multiple of 16 so that every part starts on a 64-byte boundary of its segment
__device__ __forceinline__ int part_length(int n, int n_parts) {
    return (((n + n_parts - 1) / n_parts) + 15) & ~15;
}

__global__ __launch_bounds__(kTopkBlock) void topk_split_collect_kernel(Shape s, TopkArgs a) {
    __shared__ uint32_t hist[2048];
    __shared__ uint32_t wave_tot[kTopkWaves];
    __shared__ uint32_t sh3[3];
    const int p = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
    const int64_t seg = (int64_t)b * s.Hkv + hk;
    const DecodeSeg d = decode_segment(a, b);
    if (d.k_sel <= 0) return;
    const int tid = threadIdx.x, lane = tid & 63;
    // first radix round from the precomputed histogram (every part computes the same values)
    for (int i = tid; i < 2048; i += kTopkBlock) hist[i] = a.hist11[seg * 2048 + i];
    __syncthreads();
    uint32_t d1, cnt1, rem = (uint32_t)d.k_sel;
    find_digit<kTopkBlock, 2048>(hist, wave_tot, &sh3[0], &sh3[1], &sh3[2], rem, d1, cnt1);
    uint32_t* info = a.seg_info + seg * 8;
    if (p == 0 && tid == 0) { info[1] = d1; info[2] = rem; info[3] = cnt1; }
    if (cnt1 > (uint32_t)kCandCap) return;   // the threshold kernel takes the whole segment

    const uint32_t* bits = reinterpret_cast<const uint32_t*>(a.scores + seg * a.pitch);
    const bool aligned = (reinterpret_cast<uintptr_t>(bits) & 15u) == 0;
    const int plen = part_length(d.n, a.n_parts);
    const int begin = p * plen;
    const int end = begin + plen < d.n ? begin + plen : d.n;
    uint32_t* cand = a.cand + seg * kCandCap;
    uint32_t above = 0;
    for (int base = begin; base < end; base += kTopkBlock * kEPT) {
        const int i0 = base + tid * kEPT;
        uint32_t u[kEPT];
        load16(bits, end, i0, aligned, u);
        uint32_t cm = 0;   // which of this lane's kEPT scores lie in the threshold bucket
#pragma unroll
        for (int e = 0; e < kEPT; ++e) {
            const bool in = i0 + e < end;
            const uint32_t dg = (u[e] >> 20) & 2047u;
            above += (in && dg > d1) ? 1u : 0u;
            cm |= (uint32_t)(in && dg == d1) << e;
        }
        // one memory atomic per wave and sweep step: lanes reserve consecutive slots by a prefix sum
        const uint32_t mine = (uint32_t)__popc(cm);
        uint32_t inc = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t y = __shfl_up(inc, o);
            if (lane >= o) inc += y;
        }
        const uint32_t wave_total = __shfl(inc, 63);
        if (wave_total) {
            uint32_t at = 0;
            if (lane == 63) at = atomicAdd(&info[0], wave_total);
            uint32_t slot = __shfl(at, 63) + inc - mine;
#pragma unroll
            for (int e = 0; e < kEPT; ++e) {
                if ((cm >> e) & 1u) {
                    if (slot < (uint32_t)kCandCap) cand[slot] = (u[e] & 0xfffffu) | ((uint32_t)p << 20);
                    ++slot;
                }
            }
        }
    }
    uint32_t tot;
    (void)block_exclusive_scan<kTopkBlock>(above, wave_tot, &tot);
    if (tid == 0) a.part_info[(seg * kTopkMaxParts + p) * 2] = tot;
}

__global__ __launch_bounds__(kTopkBlock) void topk_split_threshold_kernel(Shape s, TopkArgs a) {
    __shared__ SelectShared<kTopkBlock> sm;
    __shared__ unsigned char cpart[kCandCap];
    __shared__ uint32_t pgt[kTopkMaxParts], peq[kTopkMaxParts];
    uint32_t* const cand = sm.cand;
    const int hk = blockIdx.x, b = blockIdx.y;
    const int64_t seg = (int64_t)b * s.Hkv + hk;
    const DecodeSeg d = decode_segment(a, b);
    uint32_t* info = a.seg_info + seg * 8;
    const int tid = threadIdx.x;
    if (d.k_sel <= 0) {
        if (tid == 0) info[6] = 0u;
        return;
    }
    const uint32_t d1 = info[1], cnt1 = info[3];
    uint32_t rem = info[2];
    if (cnt1 > (uint32_t)kCandCap) {
        // very many scores share the threshold bucket: the single-workgroup path does the whole segment
        if (tid == 0) info[6] = 1u;
        Segment sg;
        sg.scores = a.scores + seg * a.pitch;
        sg.out = a.idx_out + seg * a.k_max;
        sg.hist11 = a.hist11 + seg * 2048;
        sg.n = d.n; sg.k_sel = d.k_sel; sg.forced = d.forced; sg.pad_to = a.k_max;
        select_segment<kTopkBlock>(sg, sm);
        return;
    }
    const uint32_t cnt = info[0] < (uint32_t)kCandCap ? info[0] : (uint32_t)kCandCap;
    const uint32_t* cg = a.cand + seg * kCandCap;
    for (uint32_t i = tid; i < cnt; i += kTopkBlock) {
        const uint32_t v = cg[i];
        cand[i] = v & 0xfffffu;
        cpart[i] = (unsigned char)(v >> 20);
    }
    if (tid < kTopkMaxParts) { pgt[tid] = 0u; peq[tid] = 0u; }
    __syncthreads();
    const uint32_t d2 = lds_round<kTopkBlock>(cand, cnt, 10, false, 0u, sm, rem);
    const uint32_t d3 = lds_round<kTopkBlock>(cand, cnt, 0, true, d2, sm, rem);
    const uint32_t thr20 = (d2 << 10) | d3;
    for (uint32_t i = tid; i < cnt; i += kTopkBlock) {
        const uint32_t v = cand[i];
        if (v > thr20) atomicAdd(&pgt[cpart[i]], 1u);
        else if (v == thr20) atomicAdd(&peq[cpart[i]], 1u);
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t gt_off = 0, eq_before = 0;
        uint32_t* pi = a.part_info + seg * kTopkMaxParts * 2;
        for (int p = 0; p < a.n_parts; ++p) {
            const uint32_t above = pi[p * 2];
            pi[p * 2] = gt_off;
            pi[p * 2 + 1] = eq_before;
            gt_off += above + pgt[p];
            eq_before += peq[p];
        }
        info[4] = (d1 << 20) | thr20;
        info[5] = rem;      // scores equal to THR that still belong to the set (lowest positions first)
        info[6] = 0u;
    }
}

__global__ __launch_bounds__(kTopkBlock) void topk_split_compact_kernel(Shape s, TopkArgs a) {
    __shared__ uint32_t wave_tot[kTopkWaves];
    const int p = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
    const int64_t seg = (int64_t)b * s.Hkv + hk;
    const DecodeSeg d = decode_segment(a, b);
    const uint32_t* info = a.seg_info + seg * 8;
    if (info[6] != 0u) return;   // handled by the fallback
    const int tid = threadIdx.x;
    int32_t* out = a.idx_out + seg * a.k_max;
    if (d.k_sel > 0) {
        const uint32_t thr = info[4], need_eq = info[5];
        const uint32_t* bits = reinterpret_cast<const uint32_t*>(a.scores + seg * a.pitch);
        const bool aligned = (reinterpret_cast<uintptr_t>(bits) & 15u) == 0;
        const int plen = part_length(d.n, a.n_parts);
        const int begin = p * plen;
        const int end = begin + plen < d.n ? begin + plen : d.n;
        const uint32_t* pi = a.part_info + (seg * kTopkMaxParts + p) * 2;
        compact_range<kTopkBlock>(bits, begin, end, aligned, thr, need_eq, pi[0], pi[1], out, wave_tot);
    }
    if (p == 0) {
        for (int t = tid; t < d.forced; t += kTopkBlock) out[d.k_sel + t] = d.n + t;
        for (int t = d.k_sel + d.forced + tid; t < a.k_max; t += kTopkBlock) out[t] = -1;
    }
}

}  // namespace

hipError_t launch_topk_decode_split(const Shape& s, const TopkArgs& a, hipStream_t st) {
    if (!a.hist11 || !a.cand || !a.seg_info || !a.part_info || a.n_parts < 2 || a.n_parts > kTopkMaxParts)
        return hipErrorInvalidValue;
    KASCADE_LAUNCH(topk_split_collect_kernel, dim3(a.n_parts, s.Hkv, s.B), dim3(kTopkBlock), 0, st, s, a);
    KASCADE_LAUNCH(topk_split_threshold_kernel, dim3(s.Hkv, s.B), dim3(kTopkBlock), 0, st, s, a);
    KASCADE_LAUNCH(topk_split_compact_kernel, dim3(a.n_parts, s.Hkv, s.B), dim3(kTopkBlock), 0, st, s, a);
    return hipGetLastError();
}

hipError_t launch_topk_decode(const Shape& s, const TopkArgs& a, hipStream_t st) {
    KASCADE_LAUNCH(topk_decode_kernel, dim3(s.Hkv, s.B), dim3(kTopkBlock), 0, st, s, a);
    return hipGetLastError();
}

hipError_t launch_topk_prefill(const Shape& s, const TopkArgs& a, hipStream_t st) {
    KASCADE_LAUNCH(topk_prefill_kernel, dim3(a.n_tiles * s.Hkv), dim3(kTopkBlock), 0, st, s, a);
    return hipGetLastError();
}

}  // namespace kascade
