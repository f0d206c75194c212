// Calibration-time kernel: similarity of two layers' Top-k sets (Eq. 3).
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
    const int hk = blockIdx.x, b = blockIdx.y;
    const int L = a.seqlens[b];
    int k = a.k_per_seq[b];
    k = k < 0 ? 0 : (k > a.k_max ? a.k_max : k);
    const int src = a.head_map ? a.head_map[hk] : hk;
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
        if (a.sim_out) a.sim_out[b * a.Hkv + hk] = sim;
        // similarities are non-negative, so their bit patterns order like the values
        if (a.sim_min) atomicMin(reinterpret_cast<unsigned int*>(a.sim_min), __float_as_uint(fmaxf(sim, 0.f)));
    }
}

}  // namespace

hipError_t launch_similarity(const SimilarityArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(similarity_kernel, dim3(a.Hkv, a.B), dim3(kSimBlock), 0, st, a);
    return hipGetLastError();
}

}  // namespace kascade
