// Exact Top-k selection of one segment of non-negative fp32 scores by one workgroup of NT threads
// (paper Sec. 3.6, pass 3; sets are per key head, Sec. 3.5).  The bit patterns of non-negative
// floats order like the values, so the selection is a radix select on the patterns:
//   1. three rounds (11 + 10 + 10 bits from the top) with LDS histograms find the bit pattern THR of
//      the k-th largest score and how many scores equal to THR still belong to the set.  The
//      first-round histogram can be handed in precomputed.  After round 1 the scores of the threshold
//      bucket (a few thousand at most, unless many scores are equal) are copied to LDS in one sweep
//      and rounds 2-3 run there; memory is swept again only in the fallback.
//   2. ordered compaction by position keeps every score > THR and the first `need_eq` scores == THR,
//      which gives ascending output and "lower index wins" among ties.
// Shared by the selection kernels (NT = 1024) and the prefill pooling kernel (NT = 256), which runs
// the selection of its own tile right after writing the tile's pooled scores.
#pragma once
#include "device_utils.h"
#include "kernels.h"

namespace kascade {

struct Segment {
    const float* scores;       // candidates 0..n-1
    int32_t* out;              // receives k_sel selected, then `forced` forced positions, then padding
    const uint32_t* hist11;    // optional: counts of (bits >> 20) over the candidates, 2048 bins
    int n;                     // candidates
    int k_sel;                 // to select among candidates
    int forced;                // positions n..n+forced-1 appended
    int pad_to;                // total slots to fill (-1 beyond the set)
};

constexpr int kEPT = 16;                 // consecutive scores per thread per sweep step (four 16-byte loads; 8 and 32 measured slower)
constexpr int kCandCap = kTopkCandCap;   // scores of the threshold bucket kept in LDS for rounds 2 and 3
typedef __attribute__((ext_vector_type(4))) uint32_t topk_u32x4_t;

template <int NT>
struct SelectShared {
    uint32_t hist[2048];
    uint32_t cand[kCandCap];
    uint32_t wave_tot[NT / kWave];
    uint32_t sh_digit, sh_rem, sh_cnt, cand_n;
};

// Inclusive scan across the wave, then exclusive offset across the workgroup.
// Returns the exclusive prefix of `x` in thread order; *total receives the workgroup sum.
template <int NT>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t x, uint32_t* wave_tot /*LDS [NT / 64]*/, uint32_t* total) {
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
    for (int t = 0; t < NT / kWave; ++t) {
        const uint32_t v = wave_tot[t];
        if (t < w) before += v;
        tot += v;
    }
    __syncthreads();   // wave_tot may be reused by the caller
    *total = tot;
    return before + inc - x;
}

// kEPT consecutive scores starting at i0 (zero beyond n).
__device__ __forceinline__ void load16(const uint32_t* bits, int n, int i0, bool aligned, uint32_t (&u)[kEPT]) {
    if (aligned && i0 + kEPT <= n) {
        const topk_u32x4_t* p = reinterpret_cast<const topk_u32x4_t*>(bits + i0);
#pragma unroll
        for (int q = 0; q < kEPT / 4; ++q) {
            const topk_u32x4_t v = p[q];
            u[4 * q + 0] = v.x; u[4 * q + 1] = v.y; u[4 * q + 2] = v.z; u[4 * q + 3] = v.w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < kEPT; ++e) u[e] = (i0 + e < n) ? bits[i0 + e] : 0u;
    }
}

// Given a histogram of NBINS bins in LDS (bin = digit, larger digit = larger score), finds the digit
// that holds the rem-th largest element: thread t owns the BPT = NBINS / NT consecutive bins
// NBINS-1 - t*BPT - j (j = 0..BPT-1), so thread order is descending digit order.  Publishes digit,
// the rank inside that digit and the digit's count through LDS; every thread returns them.
template <int NT, int NBINS>
__device__ __forceinline__ void find_digit(const uint32_t* hist, uint32_t* wave_tot, uint32_t* sh_digit, uint32_t* sh_rem,
                                           uint32_t* sh_cnt, uint32_t& rem, uint32_t& digit, uint32_t& count) {
    constexpr int BPT = NBINS / NT;
    static_assert(BPT >= 1 && BPT * NT == NBINS, "bins must divide evenly over the threads");
    const int tid = threadIdx.x;
    uint32_t local[BPT], sum = 0;
#pragma unroll
    for (int j = 0; j < BPT; ++j) { local[j] = hist[NBINS - 1 - tid * BPT - j]; sum += local[j]; }
    uint32_t tot;
    uint32_t run = block_exclusive_scan<NT>(sum, wave_tot, &tot);
#pragma unroll
    for (int j = 0; j < BPT; ++j) {
        if (run < rem && run + local[j] >= rem) {
            *sh_digit = (uint32_t)(NBINS - 1 - tid * BPT - j);
            *sh_rem = rem - run;
            *sh_cnt = local[j];
        }
        run += local[j];
    }
    __syncthreads();
    digit = *sh_digit; rem = *sh_rem; count = *sh_cnt;
}

// One radix round over `cnt` values held in LDS: finds the digit (bits shift+9..shift of the
// values whose higher bits equal `want_hi`) that holds the rem-th largest, updates rem.
template <int NT>
__device__ __forceinline__ uint32_t lds_round(const uint32_t* cand, uint32_t cnt, int shift, bool check_hi, uint32_t want_hi,
                                              SelectShared<NT>& sm, uint32_t& rem) {
    const int tid = threadIdx.x;
    for (int i = tid; i < 1024; i += NT) sm.hist[i] = 0;
    __syncthreads();
    for (uint32_t base = 0; base < cnt; base += NT) {
        const uint32_t i = base + tid;
        const uint32_t v = i < cnt ? cand[i] : 0u;
        hist_add(sm.hist, (v >> shift) & 1023u, i < cnt && (!check_hi || (v >> 10) == want_hi));
    }
    __syncthreads();
    uint32_t digit, count;
    find_digit<NT, 1024>(sm.hist, sm.wave_tot, &sm.sh_digit, &sm.sh_rem, &sm.sh_cnt, rem, digit, count);
    __syncthreads();   // the shared result words may be rewritten by the next round
    return digit;
}

// Ordered compaction of positions [begin, end) of one segment: keeps scores > thr and, while fewer than
// need_eq equal scores have been kept (run_eq counts all equal scores seen so far), scores == thr.
// run_gt / run_eq: scores > thr / == thr at positions before `begin`.
template <int NT>
__device__ __forceinline__ void compact_range(const uint32_t* bits, int begin, int end, bool aligned, uint32_t thr,
                                              uint32_t need_eq, uint32_t run_gt, uint32_t run_eq, int32_t* out,
                                              uint32_t* wave_tot) {
    const int tid = threadIdx.x;
    for (int base = begin; base < end; base += NT * kEPT) {
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
        // counts per step are at most kEPT * NT <= 32768 each: pack both into one scan
        uint32_t tot;
        const uint32_t ex = block_exclusive_scan<NT>((uint32_t)__popc(gtm) | ((uint32_t)__popc(eqm) << 16), wave_tot, &tot);
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

template <int NT>
__device__ __forceinline__ void select_segment(const Segment& sg, SelectShared<NT>& sm) {
    static_assert(NT % kWave == 0 && 2048 % NT == 0 && NT <= 1024, "workgroup size");
    static_assert(kEPT <= 32 && kEPT * 1024 < 65536, "per-thread masks are 32 bits wide, packed scan counts 16");
    const int tid = threadIdx.x, lane = tid & 63;
    const uint32_t* bits = reinterpret_cast<const uint32_t*>(sg.scores);
    const int n = sg.n;
    const bool aligned = (reinterpret_cast<uintptr_t>(bits) & 15u) == 0;

    if (sg.k_sel > 0) {
        uint32_t rem = (uint32_t)sg.k_sel;
        // ---- round 1: bits 30..20 (bit 31 is the sign, always 0) ---------------------
        if (!sg.hist11) {
            for (int i = tid; i < 2048; i += NT) sm.hist[i] = 0;
            __syncthreads();
            for (int base = 0; base < n; base += NT * kEPT) {
                const int i0 = base + tid * kEPT;
                uint32_t u[kEPT];
                load16(bits, n, i0, aligned, u);
#pragma unroll
                for (int e = 0; e < kEPT; ++e) hist_add(sm.hist, (u[e] >> 20) & 2047u, i0 + e < n);
            }
        }
        if (tid == 0) sm.cand_n = 0;
        __syncthreads();
        uint32_t d1, cnt1;
        find_digit<NT, 2048>(sg.hist11 ? sg.hist11 : sm.hist, sm.wave_tot, &sm.sh_digit, &sm.sh_rem, &sm.sh_cnt, rem, d1, cnt1);
        __syncthreads();
        uint32_t thr;
        if (cnt1 <= (uint32_t)kCandCap) {
            // ---- gather the threshold bucket's low 20 bits into LDS (one sweep), rounds 2-3 there ----
            for (int base = 0; base < n; base += NT * kEPT) {
                const int i0 = base + tid * kEPT;
                uint32_t u[kEPT];
                load16(bits, n, i0, aligned, u);
                uint32_t cm = 0;
#pragma unroll
                for (int e = 0; e < kEPT; ++e) cm |= (uint32_t)(i0 + e < n && ((u[e] >> 20) & 2047u) == d1) << e;
                // one reservation per wave and step: prefix of the lanes' counts, the last lane claims the range
                uint32_t inc = (uint32_t)__popc(cm);
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) {
                    const uint32_t y = __shfl_up(inc, o);
                    if (lane >= o) inc += y;
                }
                uint32_t at = 0;
                if (lane == 63 && inc) at = atomicAdd(&sm.cand_n, inc);
                uint32_t slot = __shfl(at, 63) + inc - (uint32_t)__popc(cm);
#pragma unroll
                for (int e = 0; e < kEPT; ++e) {
                    if ((cm >> e) & 1u) {
                        if (slot < (uint32_t)kCandCap) sm.cand[slot] = u[e] & 0xfffffu;
                        ++slot;
                    }
                }
            }
            __syncthreads();
            const uint32_t cnt = sm.cand_n < (uint32_t)kCandCap ? sm.cand_n : (uint32_t)kCandCap;
            const uint32_t d2 = lds_round<NT>(sm.cand, cnt, 10, false, 0u, sm, rem);
            const uint32_t d3 = lds_round<NT>(sm.cand, cnt, 0, true, d2, sm, rem);
            thr = (d1 << 20) | (d2 << 10) | d3;
        } else {
            // ---- very many scores share the threshold bucket (e.g. thousands of zeros): sweep memory ----
            uint32_t prefix = d1 << 20, mask = 0x7ffu << 20;
#pragma unroll
            for (int shift = 10; shift >= 0; shift -= 10) {
                for (int i = tid; i < 1024; i += NT) sm.hist[i] = 0;
                __syncthreads();
                for (int base = 0; base < n; base += NT * kEPT) {
                    const int i0 = base + tid * kEPT;
                    uint32_t u[kEPT];
                    load16(bits, n, i0, aligned, u);
#pragma unroll
                    for (int e = 0; e < kEPT; ++e) hist_add(sm.hist, (u[e] >> shift) & 1023u, i0 + e < n && (u[e] & mask) == prefix);
                }
                __syncthreads();
                uint32_t digit, count;
                find_digit<NT, 1024>(sm.hist, sm.wave_tot, &sm.sh_digit, &sm.sh_rem, &sm.sh_cnt, rem, digit, count);
                __syncthreads();
                prefix |= digit << shift; mask |= 1023u << shift;
            }
            thr = prefix;
        }
        // rem >= 1: scores equal to THR that still belong to the set, lowest positions first
        compact_range<NT>(bits, 0, n, aligned, thr, rem, 0u, 0u, sg.out, sm.wave_tot);
    }
    for (int t = tid; t < sg.forced; t += NT) sg.out[sg.k_sel + t] = n + t;
    for (int t = sg.k_sel + sg.forced + tid; t < sg.pad_to; t += NT) sg.out[t] = -1;
}

}  // namespace kascade
