// Operand layouts shared by the kernels that run attention products on the matrix unit
// (v_mfma_f32_32x32x16_bf16, wave64): LDS tile addressing with bank swizzles, fragment reads,
// direct global-to-LDS staging, and the half-wave reductions of the 32x32 output layout.
#pragma once
#include "device_utils.h"

namespace kascade {
namespace mfma {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((address_space(1))) const void* gmem_ptr_t;
typedef __attribute__((address_space(3))) void* lds_ptr_t;

// MFMA 32x32x16 output: lane (col = lane%32, half = lane/32), register r holds row
// (r/4)*8 + half*4 + r%4.  perm_key maps an operand row/col index rho to the key slot that
// makes register r of half h hold key slot (r/8)*16 + h*8 + r%8, i.e. eight consecutive keys
// per group of eight registers - the order the P^T operand of the second MFMA needs.
__device__ __forceinline__ int perm_key(int rho) {
    const int r = (rho >> 3) * 4 + (rho & 3);
    const int h = (rho >> 2) & 1;
    return (r >> 3) * 16 + h * 8 + (r & 7);
}

// K tile: [keys][D] bf16 row-major, the 16-byte chunks of a row XOR-swizzled by the key index so
// that the 16 lanes served together by one LDS read (16 different keys, same chunk) fall into 16
// different 16-byte slots of the 256-byte bank window (64 banks x 4 bytes).
template <int D>
__device__ __forceinline__ int k_off(int key, int chunk) {
    const int f = (D == 128) ? (key & 15) : ((key >> 1) & 7);   // D = 64: two rows share a window
    return key * (D * 2) + ((chunk ^ f) << 4);
}
// V tile: [keys][D] bf16 row-major like K.  The MFMA needs V^T fragments (for one d, eight
// consecutive keys); ds_read_b64_tr_b16 delivers them from the row-major tile: within each group
// of 16 lanes, lane j points at four consecutive elements of one row, and lane i receives element
// i%4 of the segments named by lanes i/4, i/4+4, i/4+8, i/4+12.  The 64-byte groups of a row are
// XOR-swizzled by key%4 so that the four rows one read touches fall into different banks.
template <int D>
__device__ __forceinline__ int v_off(int key, int d) {
    const int f = (D == 128) ? ((key & 3) << 2) : (((key >> 1) & 1) << 2);
    return key * (D * 2) + ((((d >> 3) ^ f)) << 4) + ((d & 7) << 1);
}
typedef short s16x4_t __attribute__((ext_vector_type(4)));
// V^T fragment for MFMA row (lane%32) = d index dblk*32 + lane%32, keys key0 + (lane/32)*8 + 0..7
template <int D>
__device__ __forceinline__ bf16x8_t vt_frag(const unsigned char* smV, int dblk, int key0) {
    const int lane = threadIdx.x & 63;
    const int g = lane >> 4, a = lane & 3, e = (lane >> 2) & 3;
    const int key = key0 + (g >> 1) * 8 + e;
    const int d0 = dblk * 32 + (g & 1) * 16 + 4 * a;
    typedef s16x4_t __attribute__((address_space(3))) * lds_v4;
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(smV + v_off<D>(key, d0)));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(smV + v_off<D>(key + 4, d0)));
    struct { s16x4_t lo, hi; } both = {lo, hi};
    return __builtin_bit_cast(bf16x8_t, both);
}

// max / sum across the two half-waves (lanes i and i+32) on the vector ALU: v_permlane32_swap
// exchanges the upper half of its first operand with the lower half of the second
__device__ __forceinline__ float half_swap_max(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_swap_sum(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ bf16x8_t lds_frag(const unsigned char* p) {
    return __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(p));
}

__device__ __forceinline__ bf16x8_t pack_p(const f32x16_t& s, int base) {
    bf16x8_t r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = (__bf16)s[base + e];
    return r;
}

__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0f70); }   // vmcnt(0) only

// The two 16-bit storage types share every operand layout; what differs is the MFMA opcode and the
// rounding of fp32 values to the storage type.  Fragments travel as bf16x8_t (8 x 16 raw bits) either way.
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
template <bool F16> struct Mma {
    static __device__ __forceinline__ f32x16_t mma32(bf16x8_t a, bf16x8_t b, f32x16_t c) {
        if constexpr (F16)
            return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
        else
            return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x4_t mma16(bf16x8_t a, bf16x8_t b, f32x4_t c) {
        if constexpr (F16)
            return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
        else
            return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
    // eight fp32 values rounded to nearest even in the storage type
    static __device__ __forceinline__ bf16x8_t pack8(const float* p) {
        if constexpr (F16) {   // as one vector conversion: four v_cvt_pk_f16_f32
            typedef __attribute__((ext_vector_type(8))) float f32x8_t;
            f32x8_t v;
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = p[e];
            return __builtin_bit_cast(bf16x8_t, __builtin_convertvector(v, f16x8_t));
        } else {
            bf16x8_t r;
#pragma unroll
            for (int e = 0; e < 8; ++e) r[e] = (__bf16)p[e];
            return r;
        }
    }
    // registers base .. base+7 of a 32x32 accumulator tile as one operand fragment
    static __device__ __forceinline__ bf16x8_t pack_tile(const f32x16_t& t, int base) {
        float p[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) p[e] = t[base + e];
        return pack8(p);
    }
    static __device__ __forceinline__ uint32_t bits(float x) {
        if constexpr (F16) return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)x);
        else return f32_to_bf16_bits(x);
    }
};

}  // namespace mfma
}  // namespace kascade
