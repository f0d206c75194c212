// Device-side helpers shared by the Kascade kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kascade {

constexpr int kWave = 64;

typedef uint16_t bf16_t;   // storage only; arithmetic is fp32
typedef _Float16 f16_t;    // the other 16-bit storage type (matrix-unit kernels only)

// A sequence length read from device memory, held to the host-side bound that sized the grid and the
// buffers (bound <= 0: none): a length beyond it must not become a write beyond them.
__device__ __forceinline__ int bounded_len(int len, int bound) {
    len = len < 0 ? 0 : len;
    return (bound > 0 && len > bound) ? bound : len;
}
// The same for a prefill tile's budget and its offset into the index arrays (idx_total entries per head):
// at most `prefix` candidates, and never a slot beyond the arrays.
struct TileSlot {
    int k;
    int64_t off;
};
__device__ __forceinline__ TileSlot bounded_tile_slot(int k, int64_t off, int64_t prefix, int64_t idx_total) {
    TileSlot r;
    r.off = off < 0 ? 0 : (off > idx_total ? idx_total : off);
    int64_t kk = k < 0 ? 0 : k;
    kk = kk > prefix ? prefix : kk;
    kk = kk > idx_total - r.off ? idx_total - r.off : kk;
    r.k = (int)kk;
    return r;
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// round-to-nearest-even fp32 -> bf16 (NaN stays NaN)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
// fp32 -> storage type T (float, bf16_t, f16_t), round to nearest even; and back
template <typename T> __device__ __forceinline__ T narrow(float f);
template <> __device__ __forceinline__ float narrow<float>(float f) { return f; }
template <> __device__ __forceinline__ bf16_t narrow<bf16_t>(float f) { return (bf16_t)f32_to_bf16_bits(f); }
template <> __device__ __forceinline__ f16_t narrow<f16_t>(float f) { return (f16_t)f; }
__device__ __forceinline__ float widen1(float v) { return v; }
__device__ __forceinline__ float widen1(bf16_t v) { return __uint_as_float((uint32_t)v << 16); }
__device__ __forceinline__ float widen1(f16_t v) { return (float)v; }

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// One 16-byte piece of a row, widened to fp32.  EPL = elements per 16 bytes.
template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int EPL = 4;
    __device__ static __forceinline__ void widen(const uint4& r, float* f) {
        f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
        f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
    }
    __device__ static __forceinline__ void store(float* dst, const float* f) {   // EPL values
        *reinterpret_cast<float4*>(dst) = make_float4(f[0], f[1], f[2], f[3]);
    }
};
template <> struct Elem<bf16_t> {
    static constexpr int EPL = 8;
    __device__ static __forceinline__ void widen(const uint4& r, float* f) {
        f[0] = bf16_lo(r.x); f[1] = bf16_hi(r.x); f[2] = bf16_lo(r.y); f[3] = bf16_hi(r.y);
        f[4] = bf16_lo(r.z); f[5] = bf16_hi(r.z); f[6] = bf16_lo(r.w); f[7] = bf16_hi(r.w);
    }
    __device__ static __forceinline__ void store(bf16_t* dst, const float* f) {  // EPL values
        uint4 r;
        r.x = pack_bf16(f[0], f[1]); r.y = pack_bf16(f[2], f[3]);
        r.z = pack_bf16(f[4], f[5]); r.w = pack_bf16(f[6], f[7]);
        *reinterpret_cast<uint4*>(dst) = r;
    }
};

// ---- cross-lane data movement inside a wave --------------------------------
// DPP controls: quad_perm[1,0,3,2] = 0xB1, quad_perm[2,3,0,1] = 0x4E,
// row_half_mirror = 0x141 (lane i <-> 7-i of each 8), row_mirror = 0x140 (i <-> 15-i of each 16).
template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}

// Sum over aligned groups of NL lanes (NL in {8,16,32,64}); every lane of the group gets the total.
template <int NL>
__device__ __forceinline__ float group_sum(float x) {
    x += dpp_f<0xB1>(x);
    x += dpp_f<0x4E>(x);
    x += dpp_f<0x141>(x);
    if constexpr (NL >= 16) x += dpp_f<0x140>(x);
    if constexpr (NL >= 32) x += __shfl_xor(x, 16);
    if constexpr (NL >= 64) x += __shfl_xor(x, 32);
    return x;
}
template <int NL>
__device__ __forceinline__ float group_max(float x) {
    x = fmaxf(x, dpp_f<0xB1>(x));
    x = fmaxf(x, dpp_f<0x4E>(x));
    x = fmaxf(x, dpp_f<0x141>(x));
    if constexpr (NL >= 16) x = fmaxf(x, dpp_f<0x140>(x));
    if constexpr (NL >= 32) x = fmaxf(x, __shfl_xor(x, 16));
    if constexpr (NL >= 64) x = fmaxf(x, __shfl_xor(x, 32));
    return x;
}

__device__ __forceinline__ float wave_sum(float x) { return group_sum<64>(x); }
__device__ __forceinline__ float wave_max(float x) { return group_max<64>(x); }

// hist[digit] += 1 for active lanes; lanes that share the first active lane's digit are
// combined into one LDS atomic (guards against thousands of equal scores hitting one bin).
__device__ __forceinline__ void hist_add(uint32_t* hist, uint32_t digit, bool active) {
    const uint64_t act = __ballot(active);
    if (act == 0) return;
    const int lane = threadIdx.x & 63;
    const int leader = __ffsll((unsigned long long)act) - 1;
    const uint32_t d0 = __shfl(digit, leader);
    const uint64_t same = __ballot(active && digit == d0);
    if (lane == leader) atomicAdd(&hist[d0], (uint32_t)__popcll(same));
    if (active && digit != d0) atomicAdd(&hist[digit], 1u);
}

// exp(x) through the hardware exp2
__device__ __forceinline__ float fast_exp(float x) { return __builtin_amdgcn_exp2f(x * 1.4426950408889634f); }

}  // namespace kascade
