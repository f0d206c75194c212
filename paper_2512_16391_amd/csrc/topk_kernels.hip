// Exact Top-k selection over pooled post-softmax scores (paper Sec. 3.6, pass 3; sets are per
// key head, Sec. 3.5).  Scores are non-negative fp32, so their bit patterns order like the
// values.  One workgroup per segment:
//   1. radix select, 4 rounds of 8 bits from the top, LDS histograms: finds the bit pattern
//      THR of the k-th largest score and how many scores equal to THR still belong to the set;
//   2. ordered compaction by position: keeps every score > THR and the first `need_eq`
//      scores == THR, which gives ascending output and "lower index wins" among ties.
#include "device_utils.h"
#include "kernels.h"

namespace kascade {

namespace {

constexpr int kTopkBlock = 1024;
constexpr int kTopkWaves = kTopkBlock / kWave;

struct Segment {
    const float* scores;   // candidates 0..n-1
    int32_t* out;          // receives k_sel selected, then `forced` forced positions, then padding
    int n;                 // candidates
    int k_sel;             // to select among candidates
    int forced;            // positions n..n+forced-1 appended
    int pad_to;            // total slots to fill (-1 beyond the set)
};

__device__ __forceinline__ void select_segment(const Segment& sg) {
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sh_digit, sh_rem;
    __shared__ uint32_t wave_gt[kTopkWaves], wave_eq[kTopkWaves];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const uint32_t* bits = reinterpret_cast<const uint32_t*>(sg.scores);
    const int n = sg.n;

    if (sg.k_sel > 0) {
        uint32_t prefix = 0, mask = 0, rem = (uint32_t)sg.k_sel;
        for (int shift = 24; shift >= 0; shift -= 8) {
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            for (int i = tid; i < n; i += kTopkBlock) {
                const uint32_t u = bits[i];
                if ((u & mask) == prefix) atomicAdd(&hist[(u >> shift) & 255u], 1u);
            }
            __syncthreads();
            if (tid < 256) {
                // above = number of matching scores whose digit is larger than tid
                uint32_t above = 0;
                for (int d = tid + 1; d < 256; ++d) above += hist[d];
                const uint32_t here = hist[tid];
                if (above < rem && above + here >= rem) { sh_digit = (uint32_t)tid; sh_rem = rem - above; }
            }
            __syncthreads();
            prefix |= sh_digit << shift;
            mask |= 255u << shift;
            rem = sh_rem;
            __syncthreads();
        }
        const uint32_t thr = prefix;
        const uint32_t need_eq = rem;   // >= 1

        uint32_t run_gt = 0, run_eq = 0;
        for (int base = 0; base < n; base += kTopkBlock) {
            const int i = base + tid;
            const bool in = i < n;
            const uint32_t u = in ? bits[i] : 0u;
            const bool gt = in && u > thr;
            const bool eq = in && u == thr;
            const uint64_t bg = __ballot(gt), be = __ballot(eq);
            if (lane == 0) { wave_gt[w] = __popcll(bg); wave_eq[w] = __popcll(be); }
            __syncthreads();
            uint32_t gt_before = run_gt, eq_before = run_eq, tot_gt = 0, tot_eq = 0;
#pragma unroll
            for (int t = 0; t < kTopkWaves; ++t) {
                const uint32_t g = wave_gt[t], e = wave_eq[t];
                if (t < w) { gt_before += g; eq_before += e; }
                tot_gt += g; tot_eq += e;
            }
            const uint64_t lt = (1ull << lane) - 1ull;
            gt_before += __popcll(bg & lt);
            eq_before += __popcll(be & lt);
            if (gt || (eq && eq_before < need_eq)) {
                const uint32_t pos = gt_before + (eq_before < need_eq ? eq_before : need_eq);
                sg.out[pos] = i;
            }
            run_gt += tot_gt;
            run_eq += tot_eq;
            __syncthreads();
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
