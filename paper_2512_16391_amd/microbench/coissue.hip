// Measurement aid, not part of the library: how much vector-ALU work fits beside matrix instructions on one
// SIMD of a gfx950 compute unit?  Registers only (no memory traffic), one tiny store at the end.
// Every step issues one v_mfma_f32_32x32x16_bf16 (or two 16x16x32, the same work) and NV independent vector
// operations, EXPS of them v_exp_f32; waves per SIMD 1 and 3.
// build: hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops coissue.hip -o coissue
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("err %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
// SHAPE 0: 32x32x16 (one per step), 1: 16x16x32 (two per step = same flops); NV = vector ops per step; EXPS of them are exp2
template <int SHAPE, int NV, int EXPS, bool MFMA>
__global__ __launch_bounds__(64) void k(float* out, int iters, float seed) {
    bf16x8_t a, b;
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(seed + threadIdx.x); b[e] = (__bf16)(seed * 0.5f); }
    f32x16_t c0, c1;
    f32x4_t d0, d1, d2, d3;
    for (int r = 0; r < 16; ++r) { c0[r] = 0.f; c1[r] = 0.f; }
    for (int r = 0; r < 4; ++r) { d0[r] = d1[r] = d2[r] = d3[r] = 0.f; }
    float v[16];
    for (int j = 0; j < 16; ++j) v[j] = seed + j + threadIdx.x;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (MFMA) {
                if (SHAPE == 0) {
                    if (i & 1) c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
                    else c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
                } else {
                    if (i & 1) { d2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, d2, 0, 0, 0); d3 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, d3, 0, 0, 0); }
                    else { d0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, d0, 0, 0, 0); d1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, d1, 0, 0, 0); }
                }
            }
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                if (j < EXPS) v[j] = __builtin_amdgcn_exp2f(v[j]);
                else v[j] = fmaf(v[j], 1.0001f, 0.5f);
            }
            if (NV > 0) asm volatile("" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]),
                                          "+v"(v[8]), "+v"(v[9]), "+v"(v[10]), "+v"(v[11]));
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    float s = 0.f;
    for (int r = 0; r < 16; ++r) s += c0[r] + c1[r];
    for (int r = 0; r < 4; ++r) s += d0[r] + d1[r] + d2[r] + d3[r];
    for (int j = 0; j < 16; ++j) s += v[j];
    if (s == 12345.678f) out[0] = s;
}
template <int SHAPE, int NV, int EXPS, bool MFMA> void run(const char* name, int wps, float* out) {
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const int iters = 2000, grid = 256 * 4 * wps;
    for (int rep = 0; rep < 2; ++rep) {
        CK(hipEventRecord(e0)); k<SHAPE, NV, EXPS, MFMA><<<grid, 64>>>(out, iters, 1.0f); CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
        float ms; CK(hipEventElapsedTime(&ms, e0, e1));
        if (rep) printf("%-44s waves/SIMD %d: %7.3f ms -> %6.1f ns per step per SIMD-wave\n", name, wps, ms, ms * 1e6 / (iters * 16.0) / wps);
    }
}
int main() {
    float* out; CK(hipMalloc(&out, 4));
    for (int w : {1, 3}) {
#define R(S, NV, EX, M, name) if (w == 1) run<S, NV, EX, M>(name, 1, out); else run<S, NV, EX, M>(name, 3, out);
        R(0, 0, 0, true, "32x32x16 only")
        R(1, 0, 0, true, "2 x 16x16x32 only")
        R(0, 4, 0, true, "32x32x16 + 4 fma")
        R(0, 6, 0, true, "32x32x16 + 6 fma")
        R(0, 8, 0, true, "32x32x16 + 8 fma")
        R(0, 12, 0, true, "32x32x16 + 12 fma")
        R(1, 4, 0, true, "2 x 16x16x32 + 4 fma")
        R(1, 6, 0, true, "2 x 16x16x32 + 6 fma")
        R(1, 8, 0, true, "2 x 16x16x32 + 8 fma")
        R(1, 12, 0, true, "2 x 16x16x32 + 12 fma")
        R(0, 6, 2, true, "32x32x16 + 4 fma + 2 exp")
        R(1, 6, 2, true, "2 x 16x16x32 + 4 fma + 2 exp")
        R(0, 6, 2, false, "4 fma + 2 exp only")
        R(0, 8, 0, false, "8 fma only")
        R(0, 12, 0, false, "12 fma only")
    }
    return 0;
}
