// Calibration-time kernels: similarity of two layers' Top-k sets (Eq. 3), head map from the
// head-level similarity (Sec. 3.5), layer importance (Sec. 3.3); and the mean over heads behind the
// shared (all heads pooled) index sets of Sec. 3.5; and the pooled query of Pre-Softmax pooling
// (the alternative of Sec. 3.4).
//
// For one (sequence, key head) segment the similarity of layer a's set applied to layer b is
// the pooled attention mass of layer b that a's set recovers, over the mass b's own set
// recovers.  Both sums are gathers of k floats out of one pooled row, so the kernel is bound
// by scattered 4-byte reads; one workgroup per segment, a fixed reduction tree (bit-stable).
#include "device_utils.h"
#include "kernels.h"

namespace kascade {

namespace {

constexpr int kSimBlock = 256;

__device__ __forceinline__ float block_sum(float x, float* sm) {
    x = wave_sum(x);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (lane == 0) sm[w] = x;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < kSimBlock / kWave; ++i) t += sm[i];
    __syncthreads();
    return t;
}

__global__ __launch_bounds__(kSimBlock) void similarity_kernel(SimilarityArgs a) {
    // all_pairs: blockIdx.z walks layer a's heads and the output is [B, Hkv, n_heads_a]
    const int hk = blockIdx.x, b = blockIdx.y;
    const int L = a.seqlens[b];
    int k = a.k_per_seq[b];
    k = k < 0 ? 0 : (k > a.k_max ? a.k_max : k);
    int src = a.all_pairs ? (int)blockIdx.z : (a.head_map ? a.head_map[hk] : hk);
    src = src < 0 ? 0 : (src >= a.n_heads_a ? a.n_heads_a - 1 : src);   // a map entry out of range is held to the range, as in the gather kernels
    const float* row = a.pooled + ((int64_t)b * a.Hkv + hk) * a.pitch;
    const int32_t* ia = a.idx_a + ((int64_t)b * a.n_heads_a + src) * a.k_max;
    const int32_t* ib = a.idx_b + ((int64_t)b * a.Hkv + hk) * a.k_max;
    float num = 0.f, den = 0.f;
    for (int i = threadIdx.x; i < k; i += kSimBlock) {
        const int ja = ia[i], jb = ib[i];
        if (ja >= 0 && ja < L) num += row[ja];
        if (jb >= 0 && jb < L) den += row[jb];
    }
    __shared__ float sm[kSimBlock / kWave];
    num = block_sum(num, sm);
    den = block_sum(den, sm);
    if (threadIdx.x == 0) {
        const float sim = den > 0.f ? num / den : 1.f;
        if (a.sim_out) a.sim_out[a.all_pairs ? (b * a.Hkv + hk) * a.n_heads_a + src : b * a.Hkv + hk] = sim;
        // similarities are non-negative, so their bit patterns order like the values
        if (a.sim_min) atomicMin(reinterpret_cast<unsigned int*>(a.sim_min), __float_as_uint(fmaxf(sim, 0.f)));
    }
}

// One wave per head of the reuse layer: mean over the samples of sim[b, hk, ha] for every anchor
// head ha (each lane sums a strided share in order, then a fixed butterfly), then the arg-max;
// equal means keep the lower anchor head.
__global__ __launch_bounds__(kWave) void head_map_kernel(int B, int Hkv, int Ha, const float* sim, float* mean_out,
                                                         int32_t* head_map_out) {
    const int hk = blockIdx.x, lane = threadIdx.x;
    float best = -INFINITY;
    int arg = 0;
    for (int ha = 0; ha < Ha; ++ha) {
        float t = 0.f;
        for (int b = lane; b < B; b += kWave) t += sim[((int64_t)b * Hkv + hk) * Ha + ha];
        t = wave_sum(t) / (float)B;
        if (mean_out && lane == 0) mean_out[hk * Ha + ha] = t;
        if (t > best) { best = t; arg = ha; }
    }
    if (lane == 0) head_map_out[hk] = arg;
}


// One wave per row: 1 - <x, y> / (|x| |y|), fp32 accumulation.
template <typename T>
__global__ __launch_bounds__(kSimBlock) void importance_kernel(const T* x, const T* y, int64_t n_rows, int n_cols,
                                                               int64_t x_stride, int64_t y_stride, float* w_out) {
    const int64_t row = (int64_t)blockIdx.x * (kSimBlock / kWave) + (threadIdx.x >> 6);
    if (row >= n_rows) return;
    const int lane = threadIdx.x & 63;
    const T* xr = x + row * x_stride;
    const T* yr = y + row * y_stride;
    float xy = 0.f, xx = 0.f, yy = 0.f;
    for (int c = lane; c < n_cols; c += kWave) {
        const float a = widen1(xr[c]), b = widen1(yr[c]);
        xy = fmaf(a, b, xy); xx = fmaf(a, a, xx); yy = fmaf(b, b, yy);
    }
    xy = wave_sum(xy); xx = wave_sum(xx); yy = wave_sum(yy);
    if (lane == 0) w_out[row] = 1.f - xy / (sqrtf(xx) * sqrtf(yy));
}

// grid (ceil(n / 1024), n_batches), 256 threads, four consecutive values per thread; heads are added
// in ascending order (bit-stable) and the mean overwrites head 0's row
__global__ __launch_bounds__(kSimBlock) void pool_heads_kernel(float* rows, int64_t batch_pitch, int64_t head_pitch,
                                                               int n_heads, int64_t n, const int32_t* lens,
                                                               int32_t* zero_map) {
    const int b = blockIdx.y;
    if (blockIdx.x == 0 && b == 0 && threadIdx.x < n_heads) zero_map[threadIdx.x] = 0;
    const int64_t len = lens ? (int64_t)bounded_len(lens[b], n > 0x7fffffff ? 0 : (int)n) : n;
    const int64_t j = ((int64_t)blockIdx.x * kSimBlock + threadIdx.x) * 4;
    if (j >= len) return;
    float* base = rows + b * batch_pitch + j;
    const float inv = 1.f / (float)n_heads;
    if (j + 3 < len) {
        float4 acc = *reinterpret_cast<const float4*>(base);
        for (int h = 1; h < n_heads; ++h) {
            const float4 v = *reinterpret_cast<const float4*>(base + h * head_pitch);
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
        *reinterpret_cast<float4*>(base) = make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
    } else {
        for (int e = 0; j + e < len; ++e) {
            float acc = base[e];
            for (int h = 1; h < n_heads; ++h) acc += base[h * head_pitch + e];
            base[e] = acc * inv;
        }
    }
}

// One rounding, to nearest with ties to even, from fp64 to the storage type T.  Going through fp32 first
// would round twice (a mean a hair above a tie of T can land on the tie in fp32), so the 16-bit types are
// rounded here: the value is divided by the spacing of T at its magnitude (a power of two, exact), rounded
// to an integer by rint (ties to even), and multiplied back (exact); the result is representable in T and
// in fp32, so the conversions that follow do not round.  SIG = significant bits, EMIN = exponent of the
// smallest normal value (below it the spacing stays that of the smallest normals).
template <int SIG, int EMIN>
__device__ __forceinline__ float round_once(double x) {
    if (x == 0.0) return (float)x;
    int e = ilogb(x);                      // floor(log2 |x|)
    e = (e < EMIN ? EMIN : e) - (SIG - 1);
    return (float)scalbn(rint(scalbn(x, -e)), e);
}
template <typename T> __device__ __forceinline__ T narrow_once(double x);
template <> __device__ __forceinline__ float narrow_once<float>(double x) { return (float)x; }   // one rounding by definition
template <> __device__ __forceinline__ bf16_t narrow_once<bf16_t>(double x) { return narrow<bf16_t>(round_once<8, -126>(x)); }
template <> __device__ __forceinline__ f16_t narrow_once<f16_t>(double x) { return narrow<f16_t>(round_once<11, -14>(x)); }

// Pre-Softmax pooling (Sec. 3.4): the query vectors of one pooling unit - decode: the G heads of key
// head hk for sequence `unit`; prefill: tokens [unit*T, min((unit+1)*T, S)) times those G heads - are
// averaged into one query of the tensors' own type.  grid (Hkv, units), one thread per dimension.  The
// sum runs in fp64, where sums of 16- or 32-bit values are exact for any realistic tile, so the order of
// the additions does not matter; then one fp64 division and ONE rounding to the storage type.
// tile_lens (prefill): receives unit*T, the number of keys before the tile, for unit < n_units.
template <typename T>
__global__ void pool_queries_kernel(const T* q, int64_t unit_stride, int64_t token_stride, int64_t head_stride, int G,
                                    int tokens_per_unit, int n_tokens, T* qbar, int Hkv, int D, int32_t* tile_lens) {
    const int hk = blockIdx.x, unit = blockIdx.y, c = threadIdx.x;
    const bool tiles = tile_lens != nullptr;     // else: one token per unit, units unit_stride apart
    const int lo = tiles ? unit * tokens_per_unit : 0;
    int hi = tiles ? lo + tokens_per_unit : 1;
    if (tiles && hi > n_tokens) hi = n_tokens;
    if (tiles && hk == 0 && c == 0) tile_lens[unit] = lo;
    double acc = 0.0;
    for (int i = lo; i < hi; ++i) {
        const T* row = q + (tiles ? 0 : unit * unit_stride) + (int64_t)i * token_stride + (int64_t)hk * G * head_stride + c;
        for (int g = 0; g < G; ++g) acc += (double)widen1(row[g * head_stride]);
    }
    const double mean = acc / (double)((hi - lo) * G);
    T* dst = qbar + ((int64_t)unit * Hkv + hk) * D + c;
    *dst = narrow_once<T>(mean);
}

}  // namespace

hipError_t launch_pool_queries(int dtype, const void* q, int64_t unit_stride, int64_t token_stride, int64_t head_stride,
                               int G, int tokens_per_unit, int n_tokens, int n_units, void* qbar, int Hkv, int D,
                               int32_t* tile_lens, hipStream_t st) {
    const dim3 grid(Hkv, n_units), block(D);
    if (dtype == 0)
        KASCADE_LAUNCH(pool_queries_kernel<float>, grid, block, 0, st, (const float*)q, unit_stride, token_stride,
                           head_stride, G, tokens_per_unit, n_tokens, (float*)qbar, Hkv, D, tile_lens);
    else if (dtype == 1)
        KASCADE_LAUNCH(pool_queries_kernel<bf16_t>, grid, block, 0, st, (const bf16_t*)q, unit_stride, token_stride,
                           head_stride, G, tokens_per_unit, n_tokens, (bf16_t*)qbar, Hkv, D, tile_lens);
    else
        KASCADE_LAUNCH(pool_queries_kernel<f16_t>, grid, block, 0, st, (const f16_t*)q, unit_stride, token_stride,
                           head_stride, G, tokens_per_unit, n_tokens, (f16_t*)qbar, Hkv, D, tile_lens);
    return hipGetLastError();
}

hipError_t launch_pool_heads(float* rows, int64_t batch_pitch, int64_t head_pitch, int n_heads, int n_batches, int64_t n,
                             const int32_t* lens, int32_t* zero_map, hipStream_t st) {
    const dim3 grid((unsigned)((n + kSimBlock * 4 - 1) / (kSimBlock * 4)), n_batches);
    KASCADE_LAUNCH(pool_heads_kernel, grid, dim3(kSimBlock), 0, st, rows, batch_pitch, head_pitch, n_heads, n, lens,
                       zero_map);
    return hipGetLastError();
}

hipError_t launch_similarity(const SimilarityArgs& a, hipStream_t st) {
    KASCADE_LAUNCH(similarity_kernel, dim3(a.Hkv, a.B, a.all_pairs ? a.n_heads_a : 1), dim3(kSimBlock), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_head_map(int B, int Hkv, int Ha, const float* sim, float* mean_out, int32_t* head_map_out,
                           hipStream_t st) {
    KASCADE_LAUNCH(head_map_kernel, dim3(Hkv), dim3(kWave), 0, st, B, Hkv, Ha, sim, mean_out, head_map_out);
    return hipGetLastError();
}

hipError_t launch_importance(int dtype, const void* x, const void* y, int64_t n_rows, int n_cols, int64_t x_stride,
                             int64_t y_stride, float* w_out, hipStream_t st) {
    const dim3 grid((unsigned)((n_rows + kSimBlock / kWave - 1) / (kSimBlock / kWave))), block(kSimBlock);
    if (dtype == 0)
        KASCADE_LAUNCH(importance_kernel<float>, grid, block, 0, st, (const float*)x, (const float*)y, n_rows, n_cols,
                           x_stride, y_stride, w_out);
    else if (dtype == 1)
        KASCADE_LAUNCH(importance_kernel<bf16_t>, grid, block, 0, st, (const bf16_t*)x, (const bf16_t*)y, n_rows,
                           n_cols, x_stride, y_stride, w_out);
    else
        KASCADE_LAUNCH(importance_kernel<f16_t>, grid, block, 0, st, (const f16_t*)x, (const f16_t*)y, n_rows,
                           n_cols, x_stride, y_stride, w_out);
    return hipGetLastError();
}

}  // namespace kascade
