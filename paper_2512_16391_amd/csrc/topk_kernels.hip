// Exact Top-k selection over pooled post-softmax scores (paper Sec. 3.6, pass 3; sets are per
// key head, Sec. 3.5).  Scores are non-negative fp32, so their bit patterns order like the
// values.  One workgroup per segment:
//   1. radix select in three rounds (11 + 10 + 10 bits from the top) with LDS histograms: finds
//      the bit pattern THR of the k-th largest score and how many scores equal to THR still
//      belong to the set.  The first-round histogram can be handed in precomputed (the decode
//      pooling pass builds it while it writes the scores).
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

__device__ __forceinline__ void select_segment(const Segment& sg) {
    __shared__ uint32_t hist[2048];
    __shared__ uint32_t wave_tot[kTopkWaves];
    __shared__ uint32_t sh_digit, sh_rem;

    const int tid = threadIdx.x;
    const uint32_t* bits = reinterpret_cast<const uint32_t*>(sg.scores);
    const int n = sg.n;

    if (sg.k_sel > 0) {
        uint32_t rem = (uint32_t)sg.k_sel;
        uint32_t prefix = 0, mask = 0;
        // ---- round 1: bits 30..20 (bit 31 is the sign, always 0) ---------------------
        if (sg.hist11) {
            hist[tid] = sg.hist11[tid];
            hist[tid + 1024] = sg.hist11[tid + 1024];
        } else {
            hist[tid] = 0; hist[tid + 1024] = 0;
            __syncthreads();
            for (int base = 0; base < n; base += kTopkBlock * 4) {
                uint32_t u[4]; bool in[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) { const int i = base + e * kTopkBlock + tid; in[e] = i < n; u[e] = in[e] ? bits[i] : 0u; }
#pragma unroll
                for (int e = 0; e < 4; ++e) hist_add(hist, (u[e] >> 20) & 2047u, in[e]);
            }
        }
        __syncthreads();
        {
            // thread t owns bins 2047-2t and 2046-2t; prefix in thread order = count above
            const uint32_t hi = hist[2047 - 2 * tid], lo = hist[2046 - 2 * tid];
            uint32_t tot;
            const uint32_t above = block_exclusive_scan(hi + lo, wave_tot, &tot);
            if (above < rem && above + hi >= rem) { sh_digit = 2047 - 2 * tid; sh_rem = rem - above; }
            else if (above + hi < rem && above + hi + lo >= rem) { sh_digit = 2046 - 2 * tid; sh_rem = rem - above - hi; }
        }
        __syncthreads();
        prefix = sh_digit << 20; mask = 0x7ffu << 20; rem = sh_rem;
        // ---- rounds 2 and 3: bits 19..10, then 9..0 ------------------------------------
#pragma unroll
        for (int shift = 10; shift >= 0; shift -= 10) {
            hist[tid] = 0;
            __syncthreads();
            for (int base = 0; base < n; base += kTopkBlock * 4) {
                uint32_t u[4]; bool in[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) { const int i = base + e * kTopkBlock + tid; in[e] = i < n; u[e] = in[e] ? bits[i] : 0u; }
#pragma unroll
                for (int e = 0; e < 4; ++e) hist_add(hist, (u[e] >> shift) & 1023u, in[e] && (u[e] & mask) == prefix);
            }
            __syncthreads();
            const uint32_t here = hist[1023 - tid];
            uint32_t tot;
            const uint32_t above = block_exclusive_scan(here, wave_tot, &tot);
            if (above < rem && above + here >= rem) { sh_digit = 1023 - tid; sh_rem = rem - above; }
            __syncthreads();
            prefix |= sh_digit << shift; mask |= 1023u << shift; rem = sh_rem;
        }
        const uint32_t thr = prefix;
        const uint32_t need_eq = rem;   // >= 1

        // ---- ordered compaction: four consecutive positions per thread ---------------
        uint32_t run_gt = 0, run_eq = 0;
        for (int base = 0; base < n; base += kTopkBlock * 4) {
            const int i0 = base + tid * 4;
            uint32_t u[4]; bool in[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) { in[e] = i0 + e < n; u[e] = in[e] ? bits[i0 + e] : 0u; }
            uint32_t cg = 0, ce = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) { cg += (in[e] && u[e] > thr); ce += (in[e] && u[e] == thr); }
            // counts per iteration are at most 4096 each: pack both into one scan
            uint32_t tot;
            const uint32_t ex = block_exclusive_scan(cg | (ce << 16), wave_tot, &tot);
            uint32_t gt_before = run_gt + (ex & 0xffffu), eq_before = run_eq + (ex >> 16);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool gt = in[e] && u[e] > thr, eq = in[e] && u[e] == thr;
                if (gt || (eq && eq_before < need_eq)) {
                    const uint32_t pos = gt_before + (eq_before < need_eq ? eq_before : need_eq);
                    sg.out[pos] = i0 + e;
                }
                gt_before += gt; eq_before += eq;
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
    const int t = blockIdx.x, hk = blockIdx.y;
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
    hipLaunchKernelGGL(topk_prefill_kernel, dim3(a.n_tiles, s.Hkv), dim3(kTopkBlock), 0, st, s, a);
    return hipGetLastError();
}

}  // namespace kascade
