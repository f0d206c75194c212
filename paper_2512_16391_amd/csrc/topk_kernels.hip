// Exact Top-k selection over pooled post-softmax scores (paper Sec. 3.6, pass 3; sets are per
// key head, Sec. 3.5).  Scores are non-negative fp32, so their bit patterns order like the
// values.  One workgroup per segment:
//   1. radix select in three rounds (11 + 10 + 10 bits from the top) with LDS histograms: finds
//      the bit pattern THR of the k-th largest score and how many scores equal to THR still
//      belong to the set.  The first-round histogram can be handed in precomputed (the decode
//      pooling pass builds it while it writes the scores).  After round 1 the scores of the
//      threshold bucket (a few thousand at most, unless many scores are equal) are copied to
//      LDS in one sweep and rounds 2-3 run there; memory is swept again only in the fallback.
//   2. ordered compaction by position: keeps every score > THR and the first `need_eq`
//      scores == THR, which gives ascending output and "lower index wins" among ties.
#include "device_utils.h"
#include "kernels.h"

namespace kascade {

namespace {

constexpr int kTopkBlock = 1024;
constexpr int kTopkWaves = kTopkBlock / kWave;

struct Segment {
    const float* scores;       // candidates 0..n-1
    int32_t* out;              // receives k_sel selected, then `forced` forced positions, then padding
    const uint32_t* hist11;    // optional: counts of (bits >> 20) over the candidates, 2048 bins
    int n;                     // candidates
    int k_sel;                 // to select among candidates
    int forced;                // positions n..n+forced-1 appended
    int pad_to;                // total slots to fill (-1 beyond the set)
};

// Inclusive scan across the wave, then exclusive offset across the workgroup.
// Returns the exclusive prefix of `x` in thread order; *total receives the workgroup sum.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t x, uint32_t* wave_tot /*LDS [kTopkWaves]*/,
                                                         uint32_t* total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint32_t inc = x;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t y = __shfl_up(inc, o);
        if (lane >= o) inc += y;
    }
    if (lane == 63) wave_tot[w] = inc;
    __syncthreads();
    uint32_t before = 0, tot = 0;
#pragma unroll
    for (int t = 0; t < kTopkWaves; ++t) {
        const uint32_t v = wave_tot[t];
        if (t < w) before += v;
        tot += v;
    }
    __syncthreads();   // wave_tot may be reused by the caller
    *total = tot;
    return before + inc - x;
}

constexpr int kEPT = 16;            // consecutive scores per thread per sweep step (four 16-byte loads)
constexpr int kCandCap = kTopkCandCap;   // scores of the threshold bucket kept in LDS for rounds 2 and 3
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

// Sixteen consecutive scores starting at i0 (zero beyond n).
__device__ __forceinline__ void load16(const uint32_t* bits, int n, int i0, bool aligned, uint32_t (&u)[kEPT]) {
    if (aligned && i0 + kEPT <= n) {
        const u32x4_t* p = reinterpret_cast<const u32x4_t*>(bits + i0);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const u32x4_t v = p[q];
            u[4 * q + 0] = v.x; u[4 * q + 1] = v.y; u[4 * q + 2] = v.z; u[4 * q + 3] = v.w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < kEPT; ++e) u[e] = (i0 + e < n) ? bits[i0 + e] : 0u;
    }
}

// One radix round over `cnt` values held in LDS: finds the digit (bits shift+9..shift of the
// values whose higher bits equal `want_hi`) that holds the rem-th largest, updates rem.
__device__ __forceinline__ uint32_t lds_round(const uint32_t* cand, uint32_t cnt, int shift, bool check_hi, uint32_t want_hi,
                                              uint32_t* hist, uint32_t* wave_tot, uint32_t* sh_digit, uint32_t* sh_rem,
                                              uint32_t& rem) {
    const int tid = threadIdx.x;
    hist[tid] = 0;
    __syncthreads();
    for (uint32_t base = 0; base < cnt; base += kTopkBlock) {
        const uint32_t i = base + tid;
        const uint32_t v = i < cnt ? cand[i] : 0u;
        hist_add(hist, (v >> shift) & 1023u, i < cnt && (!check_hi || (v >> 10) == want_hi));
    }
    __syncthreads();
    const uint32_t here = hist[1023 - tid];
    uint32_t tot;
    const uint32_t above = block_exclusive_scan(here, wave_tot, &tot);
    if (above < rem && above + here >= rem) { *sh_digit = 1023 - tid; *sh_rem = rem - above; }
    __syncthreads();
    rem = *sh_rem;
    return *sh_digit;
}

__device__ __forceinline__ void select_segment(const Segment& sg) {
    __shared__ uint32_t hist[2048];
    __shared__ uint32_t cand[kCandCap];
    __shared__ uint32_t wave_tot[kTopkWaves];
    __shared__ uint32_t sh_digit, sh_rem, sh_cnt, cand_n;

    const int tid = threadIdx.x, lane = tid & 63;
    const uint32_t* bits = reinterpret_cast<const uint32_t*>(sg.scores);
    const int n = sg.n;
    const bool aligned = (reinterpret_cast<uintptr_t>(bits) & 15u) == 0;
    const uint64_t lt = (1ull << lane) - 1ull;

    if (sg.k_sel > 0) {
        uint32_t rem = (uint32_t)sg.k_sel;
        // ---- round 1: bits 30..20 (bit 31 is the sign, always 0) ---------------------
        if (sg.hist11) {
            hist[tid] = sg.hist11[tid];
            hist[tid + 1024] = sg.hist11[tid + 1024];
        } else {
            hist[tid] = 0; hist[tid + 1024] = 0;
            __syncthreads();
            for (int base = 0; base < n; base += kTopkBlock * kEPT) {
                const int i0 = base + tid * kEPT;
                uint32_t u[kEPT];
                load16(bits, n, i0, aligned, u);
#pragma unroll
                for (int e = 0; e < kEPT; ++e) hist_add(hist, (u[e] >> 20) & 2047u, i0 + e < n);
            }
        }
        if (tid == 0) cand_n = 0;
        __syncthreads();
        {
            // thread t owns bins 2047-2t and 2046-2t; prefix in thread order = count above
            const uint32_t hi = hist[2047 - 2 * tid], lo = hist[2046 - 2 * tid];
            uint32_t tot;
            const uint32_t above = block_exclusive_scan(hi + lo, wave_tot, &tot);
            if (above < rem && above + hi >= rem) { sh_digit = 2047 - 2 * tid; sh_rem = rem - above; sh_cnt = hi; }
            else if (above + hi < rem && above + hi + lo >= rem) { sh_digit = 2046 - 2 * tid; sh_rem = rem - above - hi; sh_cnt = lo; }
        }
        __syncthreads();
        const uint32_t d1 = sh_digit;
        const uint32_t cnt1 = sh_cnt;
        rem = sh_rem;
        uint32_t thr;
        if (cnt1 <= (uint32_t)kCandCap) {
            // ---- gather the threshold bucket's low 20 bits into LDS (one sweep), rounds 2-3 there ----
            for (int base = 0; base < n; base += kTopkBlock * kEPT) {
                const int i0 = base + tid * kEPT;
                uint32_t u[kEPT];
                load16(bits, n, i0, aligned, u);
#pragma unroll
                for (int e = 0; e < kEPT; ++e) {
                    const bool is_c = i0 + e < n && ((u[e] >> 20) & 2047u) == d1;
                    const uint64_t mk = __ballot(is_c);
                    if (mk) {
                        const int first = __ffsll((unsigned long long)mk) - 1;
                        uint32_t at = 0;
                        if (lane == first) at = atomicAdd(&cand_n, (uint32_t)__popcll(mk));
                        at = __shfl(at, first);
                        const uint32_t slot = at + (uint32_t)__popcll(mk & lt);
                        if (is_c && slot < (uint32_t)kCandCap) cand[slot] = u[e] & 0xfffffu;
                    }
                }
            }
            __syncthreads();
            const uint32_t cnt = cand_n < (uint32_t)kCandCap ? cand_n : (uint32_t)kCandCap;
            const uint32_t d2 = lds_round(cand, cnt, 10, false, 0u, hist, wave_tot, &sh_digit, &sh_rem, rem);
            const uint32_t d3 = lds_round(cand, cnt, 0, true, d2, hist, wave_tot, &sh_digit, &sh_rem, rem);
            thr = (d1 << 20) | (d2 << 10) | d3;
        } else {
            // ---- very many scores share the threshold bucket (e.g. thousands of zeros): sweep memory ----
            uint32_t prefix = d1 << 20, mask = 0x7ffu << 20;
#pragma unroll
            for (int shift = 10; shift >= 0; shift -= 10) {
                hist[tid] = 0;
                __syncthreads();
                for (int base = 0; base < n; base += kTopkBlock * kEPT) {
                    const int i0 = base + tid * kEPT;
                    uint32_t u[kEPT];
                    load16(bits, n, i0, aligned, u);
#pragma unroll
                    for (int e = 0; e < kEPT; ++e) hist_add(hist, (u[e] >> shift) & 1023u, i0 + e < n && (u[e] & mask) == prefix);
                }
                __syncthreads();
                const uint32_t here = hist[1023 - tid];
                uint32_t tot;
                const uint32_t above = block_exclusive_scan(here, wave_tot, &tot);
                if (above < rem && above + here >= rem) { sh_digit = 1023 - tid; sh_rem = rem - above; }
                __syncthreads();
                prefix |= sh_digit << shift; mask |= 1023u << shift; rem = sh_rem;
            }
            thr = prefix;
        }
        const uint32_t need_eq = rem;   // >= 1

        // ---- ordered compaction: sixteen consecutive positions per thread -----------
        uint32_t run_gt = 0, run_eq = 0;
        for (int base = 0; base < n; base += kTopkBlock * kEPT) {
            const int i0 = base + tid * kEPT;
            uint32_t u[kEPT];
            load16(bits, n, i0, aligned, u);
            uint32_t gtm = 0, eqm = 0;
#pragma unroll
            for (int e = 0; e < kEPT; ++e) {
                const bool in = i0 + e < n;
                gtm |= (uint32_t)(in && u[e] > thr) << e;
                eqm |= (uint32_t)(in && u[e] == thr) << e;
            }
            // counts per step are at most 16384 each: pack both into one scan
            uint32_t tot;
            const uint32_t ex = block_exclusive_scan((uint32_t)__popc(gtm) | ((uint32_t)__popc(eqm) << 16), wave_tot, &tot);
            uint32_t gt_before = run_gt + (ex & 0xffffu), eq_before = run_eq + (ex >> 16);
            if ((gtm | eqm) != 0 && (gtm != 0 || eq_before < need_eq)) {
#pragma unroll
                for (int e = 0; e < kEPT; ++e) {
                    const bool gt = (gtm >> e) & 1u, eq = (eqm >> e) & 1u;
                    if (gt || (eq && eq_before < need_eq)) {
                        const uint32_t pos = gt_before + (eq_before < need_eq ? eq_before : need_eq);
                        sg.out[pos] = i0 + e;
                    }
                    gt_before += gt; eq_before += eq;
                }
            }
            run_gt += tot & 0xffffu; run_eq += tot >> 16;
        }
    }
    for (int t = tid; t < sg.forced; t += kTopkBlock) sg.out[sg.k_sel + t] = n + t;
    for (int t = sg.k_sel + sg.forced + tid; t < sg.pad_to; t += kTopkBlock) sg.out[t] = -1;
}

__global__ __launch_bounds__(kTopkBlock) void topk_decode_kernel(Shape s, TopkArgs a) {
    const int hk = blockIdx.x, b = blockIdx.y;
    int L = a.seqlens[b];
    L = L < 0 ? 0 : L;
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
    select_segment(sg);
}

__global__ __launch_bounds__(kTopkBlock) void topk_prefill_kernel(Shape s, TopkArgs a) {
    // long segments first (the last workgroups to start are then the shortest), key head = block mod
    // Hkv as in the attention kernels, so a head's pooled scores are swept by the XCD that wrote them
    const int hk = blockIdx.x % s.Hkv;
    const int t = a.n_tiles - 1 - blockIdx.x / s.Hkv;
    const int64_t prefix = (int64_t)t * a.tile_tokens;
    int k = a.k_per_tile[t];
    k = k < 0 ? 0 : (k > prefix ? (int)prefix : k);
    // pooled scores of tile t start after those of tiles 0..t-1: sum_{u<t} u*T = T*t*(t-1)/2
    const int64_t seg_off = (int64_t)a.tile_tokens * t * (t - 1) / 2;
    Segment sg;
    sg.scores = a.scores + hk * a.pooled_pitch + seg_off;
    sg.out = a.idx_out + hk * a.idx_total + a.idx_offsets[t];
    sg.hist11 = nullptr;
    sg.n = (int)prefix;
    sg.k_sel = k;
    sg.forced = 0;
    sg.pad_to = k;
    select_segment(sg);
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
    int L = a.seqlens[b];
    L = L < 0 ? 0 : L;
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

// First radix round from the precomputed histogram: digit of the threshold bucket, how many of the
// k_sel still have to come from it, and its size.  Every thread returns the same values.
__device__ __forceinline__ void round1_from_hist(const uint32_t* hist11, uint32_t k_sel, uint32_t* hist, uint32_t* wave_tot,
                                                 uint32_t* sh3, uint32_t& d1, uint32_t& rem, uint32_t& cnt1) {
    const int tid = threadIdx.x;
    hist[tid] = hist11[tid];
    hist[tid + 1024] = hist11[tid + 1024];
    __syncthreads();
    const uint32_t hi = hist[2047 - 2 * tid], lo = hist[2046 - 2 * tid];
    uint32_t tot;
    const uint32_t above = block_exclusive_scan(hi + lo, wave_tot, &tot);
    if (above < k_sel && above + hi >= k_sel) { sh3[0] = 2047 - 2 * tid; sh3[1] = k_sel - above; sh3[2] = hi; }
    else if (above + hi < k_sel && above + hi + lo >= k_sel) { sh3[0] = 2046 - 2 * tid; sh3[1] = k_sel - above - hi; sh3[2] = lo; }
    __syncthreads();
    d1 = sh3[0]; rem = sh3[1]; cnt1 = sh3[2];
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
    uint32_t d1, rem, cnt1;
    round1_from_hist(a.hist11 + seg * 2048, (uint32_t)d.k_sel, hist, wave_tot, sh3, d1, rem, cnt1);
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
        uint32_t cm = 0;   // which of this lane's sixteen scores lie in the threshold bucket
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
    (void)block_exclusive_scan(above, wave_tot, &tot);
    if (tid == 0) a.part_info[(seg * kTopkMaxParts + p) * 2] = tot;
}

__global__ __launch_bounds__(kTopkBlock) void topk_split_threshold_kernel(Shape s, TopkArgs a) {
    __shared__ uint32_t hist[1024];
    __shared__ uint32_t cand[kCandCap];
    __shared__ unsigned char cpart[kCandCap];
    __shared__ uint32_t wave_tot[kTopkWaves];
    __shared__ uint32_t sh_digit, sh_rem;
    __shared__ uint32_t pgt[kTopkMaxParts], peq[kTopkMaxParts];
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
        select_segment(sg);
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
    const uint32_t d2 = lds_round(cand, cnt, 10, false, 0u, hist, wave_tot, &sh_digit, &sh_rem, rem);
    const uint32_t d3 = lds_round(cand, cnt, 0, true, d2, hist, wave_tot, &sh_digit, &sh_rem, rem);
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
        uint32_t run_gt = pi[0], run_eq = pi[1];
        for (int base = begin; base < end; base += kTopkBlock * kEPT) {
            const int i0 = base + tid * kEPT;
            uint32_t u[kEPT];
            load16(bits, end, i0, aligned, u);
            uint32_t gtm = 0, eqm = 0;
#pragma unroll
            for (int e = 0; e < kEPT; ++e) {
                const bool in = i0 + e < end;
                gtm |= (uint32_t)(in && u[e] > thr) << e;
                eqm |= (uint32_t)(in && u[e] == thr) << e;
            }
            uint32_t tot;
            const uint32_t ex = block_exclusive_scan((uint32_t)__popc(gtm) | ((uint32_t)__popc(eqm) << 16), wave_tot, &tot);
            uint32_t gt_before = run_gt + (ex & 0xffffu), eq_before = run_eq + (ex >> 16);
            if ((gtm | eqm) != 0 && (gtm != 0 || eq_before < need_eq)) {
#pragma unroll
                for (int e = 0; e < kEPT; ++e) {
                    const bool gt = (gtm >> e) & 1u, eq = (eqm >> e) & 1u;
                    if (gt || (eq && eq_before < need_eq)) {
                        const uint32_t pos = gt_before + (eq_before < need_eq ? eq_before : need_eq);
                        out[pos] = i0 + e;
                    }
                    gt_before += gt; eq_before += eq;
                }
            }
            run_gt += tot & 0xffffu; run_eq += tot >> 16;
        }
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
    hipLaunchKernelGGL(topk_split_collect_kernel, dim3(a.n_parts, s.Hkv, s.B), dim3(kTopkBlock), 0, st, s, a);
    hipLaunchKernelGGL(topk_split_threshold_kernel, dim3(s.Hkv, s.B), dim3(kTopkBlock), 0, st, s, a);
    hipLaunchKernelGGL(topk_split_compact_kernel, dim3(a.n_parts, s.Hkv, s.B), dim3(kTopkBlock), 0, st, s, a);
    return hipGetLastError();
}

hipError_t launch_topk_decode(const Shape& s, const TopkArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(topk_decode_kernel, dim3(s.Hkv, s.B), dim3(kTopkBlock), 0, st, s, a);
    return hipGetLastError();
}

hipError_t launch_topk_prefill(const Shape& s, const TopkArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(topk_prefill_kernel, dim3(a.n_tiles * s.Hkv), dim3(kTopkBlock), 0, st, s, a);
    return hipGetLastError();
}

}  // namespace kascade
