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
constexpr int kCandCap = 8192;      // scores of the threshold bucket kept in LDS for rounds 2 and 3
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

}  // namespace

hipError_t launch_topk_decode(const Shape& s, const TopkArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(topk_decode_kernel, dim3(s.Hkv, s.B), dim3(kTopkBlock), 0, st, s, a);
    return hipGetLastError();
}

hipError_t launch_topk_prefill(const Shape& s, const TopkArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(topk_prefill_kernel, dim3(a.n_tiles * s.Hkv), dim3(kTopkBlock), 0, st, s, a);
    return hipGetLastError();
}

}  // namespace kascade
