// The decode row passes on the matrix unit, for bf16 and fp16 caches (head dimension 64 or 128): attention over the
// K/V rows named by a Top-k index list (paper Sec. 3.6, reuse layers and anchor pass 4) and the
// anchor's sweep over every key (Sec. 3.6 pass 1: logits and softmax statistics, with P.V when the
// layer's output is dense).
//
// The vector-ALU row kernels spend arithmetic in proportion to the number of query heads per key
// head; from four heads up that arithmetic, not HBM, sets their speed.  Here the G query heads of
// a key head are the columns of one MFMA operand (zero padded), so q.k and P.V cost the same for any
// G up to 16, and rows are staged the way the vector-ALU kernels stage them: every wave streams on its
// own, with coalesced 16-byte loads into register buffers (the next batch in flight while the current
// one is used), and a wave-private LDS tile turns a batch of 32 rows into MFMA fragments.  No
// workgroup barrier in the loops.  One workgroup = one chunk of a (sequence, key head) row list, as
// in the row kernels; its four waves take 32-row batches in turn and merge their online-softmax
// states through LDS at the end, leaving either the output or this chunk's partial (max, sum, acc)
// triple for decode_merge_kernel.
//   decode_sweep_mfma_kernel     the sweep without P.V (logits + statistics), 32-wide MFMA tiles
//   decode_rows_mfma16_kernel    attention with P.V (gather, and the sweep with dense output), 16-wide tiles
#include "device_utils.h"
#include "kernels.h"
#include "mfma_tiles.h"

namespace kascade {

namespace {

using namespace mfma;

constexpr int kMB = 256;              // threads per workgroup
constexpr int kMW = kMB / kWave;      // waves
constexpr int kWaveKeys = 32;         // keys per wave and pass

__device__ __forceinline__ int mfma_rows_per_chunk(int n_rows, int n_chunks) {
    const int c = (n_rows + n_chunks - 1) / n_chunks;
    return (c + 63) & ~63;
}

// ---------------------------------------------------------------------------------------------------
// The anchor's sweep over every key without P.V (Sec. 3.6 pass 1: logits and softmax statistics).
//   S^T[32 keys x 32 heads] = K[32 keys x d] Q^T[d x 32 heads]   (d/16 x v_mfma_f32_32x32x16_bf16 per batch)
// A wave loads 32 key rows into one of two register buffers, copies them into its LDS tile in the swizzled
// operand layout of the prefill kernels, reads the A fragments back and multiplies.  The vector ALU only
// sees 16 scores per lane and batch and the matrix unit is idle most of the time: the kernel is as
// memory-bound as the vector-ALU sweep with one head per key head.  (Staging through LDS tiles filled by
// direct global-to-LDS loads, as the prefill kernels do, was 10 % slower here: a compute unit's LDS holds
// fewer bytes in flight than its registers, and the waves of a workgroup wait for each other.)
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

template <int D, bool F16>
__global__ __launch_bounds__(kMB, 3) void decode_sweep_mfma_kernel(Shape s, DecodePlan plan, DecodeRowsArgs a) {
    constexpr int KSTEPS = D / 16;
    constexpr int LPR = D / 8;                 // lanes (16-byte pieces) per row
    constexpr int RPI = kWave / LPR;           // rows per load instruction
    constexpr int NI = kWaveKeys / RPI;        // load instructions per batch of 32 keys
    __shared__ __align__(16) unsigned char smK[kMW][kWaveKeys * D * 2];
    __shared__ float sm_m[kMW][32], sm_l[kMW][32];

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int q = lane & 31, h = lane >> 5;
    const int b = blockIdx.z, hk = blockIdx.y, chunk_id = blockIdx.x;
    const int n_chunks = plan.n_chunks, G = s.G;

    const int L = bounded_len(a.seqlens[b], a.max_seqlen);
    if (chunk_id == 0 && a.hist11) {   // pass 2 accumulates the Top-k histogram of this (b, hk): clear it here
        uint32_t* hg = a.hist11 + ((int64_t)b * s.Hkv + hk) * 2048;
        for (int i = threadIdx.x; i < 2048; i += kMB) hg[i] = 0u;
    }
    const int begin = chunk_id * plan.chunk;
    const int end = (begin + plan.chunk < L) ? begin + plan.chunk : L;
    const int64_t part_base = ((int64_t)(b * s.Hq + hk * G)) * n_chunks + chunk_id;
    if (begin >= end) {
        if ((int)threadIdx.x < G) {
            float* ml = a.part_ml + (part_base + (int64_t)threadIdx.x * n_chunks) * 2;
            ml[0] = -INFINITY;
            ml[1] = 0.f;
        }
        return;
    }

    const unsigned char* Kb = reinterpret_cast<const unsigned char*>(reinterpret_cast<const bf16_t*>(a.k) + b * s.kv_stride[0] + hk * s.kv_stride[1]);
    const uint64_t row_bytes = (uint64_t)s.kv_stride[2] * 2u;
    bf16x8_t qf[KSTEPS];
    {
        const bf16_t* qp = reinterpret_cast<const bf16_t*>(a.q) + b * s.q_stride[0] + (int64_t)(hk * G + q) * s.q_stride[2];
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (q < G) raw = *reinterpret_cast<const uint4*>(qp + kk * 16 + h * 8);
            qf[kk] = __builtin_bit_cast(bf16x8_t, raw);
        }
    }
    const float c = s.scale_log2;
    float m_run = -INFINITY, l_run = 0.f;
    float* lg0 = a.logits + ((int64_t)b * s.Hq + hk * G) * a.logit_pitch;

    unsigned char* tile = smK[w];
    const int lr = lane / LPR, lc = lane % LPR;
    const int frag_key = perm_key(q);

    u32x4_t kA[NI], kB[NI];
    // rows j0 .. j0 + 31 of the sequence into a register buffer; rows past the end re-read row `begin`
    auto issue = [&](u32x4_t* buf, int j0) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int row = j0 + i * RPI + lr;
            const uint64_t off = (uint64_t)(row < end ? row : begin) * row_bytes + (uint32_t)(lc * 16);
            buf[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(Kb + off));
        }
    };
    auto attend = [&](const u32x4_t* buf, int j0) {
#pragma unroll
        for (int i = 0; i < NI; ++i)
            *reinterpret_cast<u32x4_t*>(tile + k_off<D>(i * RPI + lr, lc)) = buf[i];
        f32x16_t s0;
#pragma unroll
        for (int r = 0; r < 16; ++r) s0[r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk)
            s0 = Mma<F16>::mma32(lds_frag(tile + k_off<D>(frag_key, kk * 2 + h)), qf[kk], s0);
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int j = j0 + (r >> 3) * 16 + h * 8 + (r & 7);
            s0[r] = j < end ? s0[r] * c : -INFINITY;
            mx = fmaxf(mx, s0[r]);
        }
        // logits out: a lane holds two runs of eight keys of its head; through the tile (its fragments have
        // been read) they become one 128-byte line per head, written by eight lanes of one instruction
        float* sc = reinterpret_cast<float*>(tile);
        if (q < G) {
#pragma unroll
            for (int r8 = 0; r8 < 16; r8 += 8) {
                float* dst = sc + q * kWaveKeys + (r8 >> 3) * 16 + h * 8;
                *reinterpret_cast<float4*>(dst) = make_float4(s0[r8], s0[r8 + 1], s0[r8 + 2], s0[r8 + 3]);
                *reinterpret_cast<float4*>(dst + 4) = make_float4(s0[r8 + 4], s0[r8 + 5], s0[r8 + 6], s0[r8 + 7]);
            }
        }
        for (int e = lane; e < G * (kWaveKeys / 4); e += kWave) {
            const int g = e >> 3, piece = (e & 7) * 4;
            const float4 val = *reinterpret_cast<const float4*>(sc + g * kWaveKeys + piece);
            float* lgp = lg0 + (int64_t)g * a.logit_pitch + j0 + piece;
            if (j0 + piece + 4 <= end) {
                *reinterpret_cast<float4*>(lgp) = val;
            } else {
                if (j0 + piece < end) lgp[0] = val.x;
                if (j0 + piece + 1 < end) lgp[1] = val.y;
                if (j0 + piece + 2 < end) lgp[2] = val.z;
            }
        }
        mx = half_swap_max(mx);
        const float m_new = fmaxf(m_run, mx);
        const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        l_run *= __builtin_amdgcn_exp2f(m_run - m_safe);   // 0 while m_run is -inf
        m_run = m_new;
        float rs = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) rs += __builtin_amdgcn_exp2f(s0[r] - m_safe);
        l_run += half_swap_sum(rs);
    };

    // the workgroup walks its chunk 128 rows at a time, 32 per wave
    constexpr int kStep = kMW * kWaveKeys;
    int j0 = begin + w * kWaveKeys;
    if (j0 < end) issue(kA, j0);
    for (; j0 < end; j0 += 2 * kStep) {
        const int j1 = j0 + kStep;
        if (j1 < end) issue(kB, j1);
        attend(kA, j0);
        if (j1 + kStep < end) issue(kA, j1 + kStep);
        if (j1 < end) attend(kB, j1);
    }

    // ---- merge the four waves' statistics, fixed order
    if (h == 0) { sm_m[w][q] = m_run; sm_l[w][q] = l_run; }
    __syncthreads();
    if ((int)threadIdx.x < G) {
        const int g = threadIdx.x;
        float M = -INFINITY;
#pragma unroll
        for (int t = 0; t < kMW; ++t) M = fmaxf(M, sm_m[t][g]);
        const float Ms = (M == -INFINITY) ? 0.f : M;
        float lsum = 0.f;
#pragma unroll
        for (int t = 0; t < kMW; ++t) lsum = fmaf(__builtin_amdgcn_exp2f(sm_m[t][g] - Ms), sm_l[t][g], lsum);
        float* ml = a.part_ml + (part_base + (int64_t)g * n_chunks) * 2;
        ml[0] = M;
        ml[1] = lsum;
    }
}

// ---------------------------------------------------------------------------------------------------
// Attention with P.V: gather mode (reuse layers, anchor pass 4) and the sweep over every key with dense
// output.  32 K rows and 32 V rows per batch in registers (two buffers for K, one for V).  To fit the
// buffers (96 registers for 128-wide heads) the products use the 16-wide tile, v_mfma_f32_16x16x32_bf16:
// the heads of the group are padded to 16 columns instead of 32, so the output accumulators take 32
// registers instead of 64 and the query fragments 16 instead of 32:
//   S^T[16 keys x 16 heads] = K[16 keys x 32 d] Q^T[32 d x 16 heads]        (4 per tile, 2 tiles per batch)
//   O^T[16 d x 16 heads]   += V^T[16 d x 32 keys] P^T[32 keys x 16 heads]   (one per 16 d)
// Output layout of the 16x16 tile: lane (col = lane%16, rg = lane/16), register r holds row rg*4 + r.
// Operands: lane (row or col = lane%16, kg = lane/16) holds the 8 consecutive k of group kg.  The key
// slot behind row rho of S tile t is sigma(t, rho) = (rho/4)*8 + t*4 + rho%4, so that the eight scores a
// lane holds (two tiles x four registers) are the key slots rg*8 .. rg*8+7: exactly its part of the
// P^T operand.  The one LDS tile of a wave holds the K rows first and the V rows after the S tiles are
// computed (LDS operations of a wave execute in order).

// K rows in the tile: 16-byte chunks XOR-swizzled by the S-tile row rho of the slot, so that the 16 rows one
// fragment read touches (same chunk) fall into different banks: 16 chunk positions for 256-byte rows; for
// 128-byte rows rho/2 picks one of 8 positions and the rows rho, rho+1 lie in different halves of a 256-byte window
template <int D>
__device__ __forceinline__ int k16_off(int slot, int chunk) {
    const int rho = ((slot >> 3) << 2) | (slot & 3);
    const int f = (D == 128) ? rho : (rho >> 1);
    return slot * (D * 2) + ((chunk ^ f) << 4);
}
// V rows in the tile: 32-byte pieces (16 d) XOR-swizzled so that the 16 rows one transposing read touches
// (slots g*8 + m, g = 0..3, m = 0..3, same piece) spread evenly over the eight piece positions of a
// 256-byte window
template <int D>
__device__ __forceinline__ int v16_swz(int slot) {
    return (D == 128) ? ((slot & 3) | (((slot >> 3) & 1) << 2)) : ((slot ^ (slot >> 3)) & 3);
}
template <int D>
__device__ __forceinline__ int v16_off(int slot, int d) {
    return slot * (D * 2) + ((((d >> 4) ^ v16_swz<D>(slot))) << 5) + ((d & 15) << 1);
}
// V^T fragment: row = d index dt*16 + lane%16, keys (lane/16)*8 + 0..7 (see vt_frag in mfma_tiles.h)
template <int D>
__device__ __forceinline__ bf16x8_t vt16_frag(const unsigned char* tile, int dt) {
    const int lane = threadIdx.x & 63;
    const int g = lane >> 4, cb = lane & 3, m = (lane >> 2) & 3;
    typedef s16x4_t __attribute__((address_space(3))) * lds_v4;
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(tile + v16_off<D>(g * 8 + m, dt * 16 + cb * 4)));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(tile + v16_off<D>(g * 8 + 4 + m, dt * 16 + cb * 4)));
    struct { s16x4_t lo, hi; } both = {lo, hi};
    return __builtin_bit_cast(bf16x8_t, both);
}
__device__ __forceinline__ float quad_rows_max(float x) {   // over the four lanes l, l+16, l+32, l+48
    x = fmaxf(x, __shfl_xor(x, 16));
    return fmaxf(x, __shfl_xor(x, 32));
}
__device__ __forceinline__ float quad_rows_sum(float x) {
    x += __shfl_xor(x, 16);
    return x + __shfl_xor(x, 32);
}

// GATHER: rows from the index list; otherwise rows begin .. end of a fixed-length chunk, logits stored (the sweep
// with dense output).
template <int D, bool GATHER, bool F16>
__global__ __launch_bounds__(kMB, 2) void decode_rows_mfma16_kernel(Shape s, DecodePlan plan, DecodeRowsArgs a) {
    constexpr int KS = D / 32, DT = D / 16;
    constexpr int LPR = D / 8;                 // lanes (16-byte pieces) per row
    constexpr int RPI = kWave / LPR;           // rows per load instruction
    constexpr int NI = kWaveKeys / RPI;        // load instructions per batch of 32 keys
    __shared__ __align__(16) unsigned char smT[kMW][kWaveKeys * D * 2];
    __shared__ float sm_m[kMW][16], sm_l[kMW][16];

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int hd = lane & 15, rg = lane >> 4;
    const int b = blockIdx.z, hk = blockIdx.y, chunk_id = blockIdx.x;
    const int n_chunks = plan.n_chunks, G = s.G;

    const int L = bounded_len(a.seqlens[b], a.max_seqlen);
    int n_rows = L;
    if constexpr (GATHER) {
        n_rows = a.k_per_seq[b];
        n_rows = n_rows < a.k_max ? n_rows : a.k_max;
        if (L <= 0 || n_rows < 0) n_rows = 0;
    } else {
        if (chunk_id == 0 && a.hist11) {   // pass 2 accumulates the Top-k histogram of this (b, hk): clear it here
            uint32_t* hg = a.hist11 + ((int64_t)b * s.Hkv + hk) * 2048;
            for (int i = threadIdx.x; i < 2048; i += kMB) hg[i] = 0u;
        }
    }
    const int chunk = GATHER ? mfma_rows_per_chunk(n_rows, n_chunks) : plan.chunk;
    const int begin = chunk_id * chunk;
    const int end = (begin + chunk < n_rows) ? begin + chunk : n_rows;
    const int64_t part_base = ((int64_t)(b * s.Hq + hk * G)) * n_chunks + chunk_id;
    if (begin >= end) {   // an empty chunk: mark it for the merge (and define the output of an empty set)
        if ((int)threadIdx.x < G) {
            float* ml = a.part_ml + (part_base + (int64_t)threadIdx.x * n_chunks) * 2;
            ml[0] = -INFINITY;
            ml[1] = 0.f;
        }
        if (n_chunks == 1) {
            for (int e = threadIdx.x; e < G * D; e += kMB) {
                bf16_t* o = reinterpret_cast<bf16_t*>(a.out) + b * s.o_stride[0] + (int64_t)(hk * G + e / D) * s.o_stride[2] + e % D;
                *o = 0;
            }
        }
        return;
    }

    const unsigned char* Kb = reinterpret_cast<const unsigned char*>(reinterpret_cast<const bf16_t*>(a.k) + b * s.kv_stride[0] + hk * s.kv_stride[1]);
    const unsigned char* Vb = reinterpret_cast<const unsigned char*>(reinterpret_cast<const bf16_t*>(a.v) + b * s.kv_stride[0] + hk * s.kv_stride[1]);
    const uint64_t row_bytes = (uint64_t)s.kv_stride[2] * 2u;
    const int32_t* idx = nullptr;
    if constexpr (GATHER) {
        int src = a.head_map ? a.head_map[hk] : hk;
        src = src < 0 ? 0 : (src >= a.n_src_heads ? a.n_src_heads - 1 : src);
        idx = a.idx + ((int64_t)b * a.n_src_heads + src) * a.k_max;
    }
    float* lg = GATHER ? nullptr : a.logits + ((int64_t)b * s.Hq + hk * G + (hd < G ? hd : 0)) * a.logit_pitch;

    bf16x8_t qf[KS];
    {
        const bf16_t* qp = reinterpret_cast<const bf16_t*>(a.q) + b * s.q_stride[0] + (int64_t)(hk * G + hd) * s.q_stride[2];
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (hd < G) raw = *reinterpret_cast<const uint4*>(qp + kk * 32 + rg * 8);
            qf[kk] = __builtin_bit_cast(bf16x8_t, raw);
        }
    }
    const float c = s.scale_log2;
    float m_run = -INFINITY, l_run = 0.f;
    f32x4_t acc[DT];
#pragma unroll
    for (int i = 0; i < DT; ++i) acc[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    unsigned char* tile = smT[w];
    const int lr = lane / LPR, lc = lane % LPR;   // row within a load instruction, 16-byte piece of the row
    const int v_piece = lc >> 1, v_half = (lc & 1) << 4;

    // list entries j0 .. j0+31 of this wave's batch (lanes 32..63 repeat them); -1 = nothing to attend to
    auto fetch_idx = [&](int j0) -> int {
        const int j = j0 + (lane & 31);
        if constexpr (GATHER) {
            const int row = j < end ? idx[j] : -1;
            return (row >= 0 && row < L) ? row : -1;
        } else {
            return j < end ? j : -1;
        }
    };
    // two register buffers for K rows, one for V rows: the V rows of the next batch are requested as soon as
    // this batch's have moved into the tile
    u32x4_t kA[NI], kB[NI], vb[NI];
    auto issue = [&](u32x4_t* buf, const unsigned char* base, int rows) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int row = __shfl(rows, i * RPI + lr);
            const uint64_t off = (uint64_t)(row < 0 ? 0 : row) * row_bytes + (uint32_t)(lc * 16);
            buf[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(base + off));
        }
    };
    auto attend = [&](const u32x4_t* kb, int rows, int next_rows, bool have_next, int j0) {
        const uint32_t ok = (uint32_t)__builtin_amdgcn_ballot_w64(rows >= 0);   // bit = key slot (lanes 0..31)
#pragma unroll
        for (int i = 0; i < NI; ++i) *reinterpret_cast<u32x4_t*>(tile + k16_off<D>(i * RPI + lr, lc)) = kb[i];
        f32x4_t st[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            st[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            const int slot = ((hd >> 2) << 3) + t * 4 + (hd & 3);   // sigma(t, rho = hd)
#pragma unroll
            for (int kk = 0; kk < KS; ++kk)
                st[t] = Mma<F16>::mma16(lds_frag(tile + k16_off<D>(slot, kk * 4 + rg)), qf[kk], st[t]);
        }
        float p[8];
        float mx = -INFINITY;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const bool valid = (ok >> (rg * 8 + e)) & 1u;
            p[e] = valid ? st[e >> 2][e & 3] * c : -INFINITY;
            mx = fmaxf(mx, p[e]);
        }
        if constexpr (!GATHER) {   // a lane holds eight consecutive keys of its head
            if (hd < G) {
                const int j = j0 + rg * 8;
                if (j + 8 <= end) {
                    *reinterpret_cast<float4*>(lg + j) = make_float4(p[0], p[1], p[2], p[3]);
                    *reinterpret_cast<float4*>(lg + j + 4) = make_float4(p[4], p[5], p[6], p[7]);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (j + e < end) lg[j + e] = p[e];
                }
            }
        }
        mx = quad_rows_max(mx);
        const float m_new = fmaxf(m_run, mx);
        const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        if (__builtin_amdgcn_ballot_w64(m_new != m_run) != 0) {   // wave-uniform: rescale only when a maximum moved
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);   // 0 while m_run is -inf
            l_run *= alpha;
#pragma unroll
            for (int i = 0; i < DT; ++i) acc[i] *= alpha;
            m_run = m_new;
        }
        float rs = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            p[e] = __builtin_amdgcn_exp2f(p[e] - m_safe);
            rs += p[e];
        }
        l_run += quad_rows_sum(rs);
        const bf16x8_t pf = Mma<F16>::pack8(p);
        // the K fragments have been read: the tile takes the V rows
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int slot = i * RPI + lr;
            *reinterpret_cast<u32x4_t*>(tile + slot * (D * 2) + ((v_piece ^ v16_swz<D>(slot)) << 5) + v_half) = vb[i];
        }
        if (have_next) issue(vb, Vb, next_rows);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
            acc[dt] = Mma<F16>::mma16(vt16_frag<D>(tile, dt), pf, acc[dt]);
    };

    // the workgroup walks its chunk 128 list entries at a time, 32 per wave; index entries are fetched two
    // batches ahead of their rows so that waiting for them never waits for rows in flight
    constexpr int kStep = kMW * kWaveKeys;
    int j0 = begin + w * kWaveKeys;
    int r0 = fetch_idx(j0), r1 = fetch_idx(j0 + kStep);
    if (j0 < end) {
        issue(kA, Kb, r0);
        issue(vb, Vb, r0);
    }
    for (; j0 < end; j0 += 2 * kStep) {
        const int r2 = fetch_idx(j0 + 2 * kStep);
        if (j0 + kStep < end) issue(kB, Kb, r1);
        attend(kA, r0, r1, j0 + kStep < end, j0);
        const int r3 = fetch_idx(j0 + 3 * kStep);
        if (j0 + 2 * kStep < end) issue(kA, Kb, r2);
        if (j0 + kStep < end) attend(kB, r1, r2, j0 + 2 * kStep < end, j0 + kStep);
        r0 = r2;
        r1 = r3;
    }

    // ---- merge the four waves' states through LDS (the tiles are free after the barrier), fixed order
    __syncthreads();
    float* sm_acc = reinterpret_cast<float*>(&smT[0][0]);   // [kMW][G][D]: 4 * 16 * 128 floats = the four tiles
    if (rg == 0) { sm_m[w][hd] = m_run; sm_l[w][hd] = l_run; }
    if (hd < G) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 4; ++r) sm_acc[(w * G + hd) * D + dt * 16 + rg * 4 + r] = acc[dt][r];
    }
    __syncthreads();
    for (int e = threadIdx.x; e < G * D; e += kMB) {
        const int g = e / D, col = e % D;
        float M = -INFINITY;
#pragma unroll
        for (int t = 0; t < kMW; ++t) M = fmaxf(M, sm_m[t][g]);
        const float Ms = (M == -INFINITY) ? 0.f : M;
        float lsum = 0.f, val = 0.f;
#pragma unroll
        for (int t = 0; t < kMW; ++t) {
            const float wgt = __builtin_amdgcn_exp2f(sm_m[t][g] - Ms);
            lsum = fmaf(wgt, sm_l[t][g], lsum);
            val = fmaf(wgt, sm_acc[(t * G + g) * D + col], val);
        }
        const int hq = hk * G + g;
        const int64_t pidx = ((int64_t)(b * s.Hq + hq)) * n_chunks + chunk_id;
        if (n_chunks == 1) {
            const float o = lsum > 0.f ? val / lsum : 0.f;
            bf16_t* op = reinterpret_cast<bf16_t*>(a.out) + b * s.o_stride[0] + (int64_t)hq * s.o_stride[2] + col;
            *op = (bf16_t)Mma<F16>::bits(o);
        } else {
            a.part_acc[pidx * D + col] = val;
        }
        if (col == 0) {
            a.part_ml[pidx * 2 + 0] = M;
            a.part_ml[pidx * 2 + 1] = lsum;
        }
    }
}

}  // namespace

// Gather-mode attention for 16-bit caches (dtype 1 = bf16, 2 = fp16), groups of up to 16 heads.
hipError_t launch_decode_gather_mfma(const Shape& s, const DecodePlan& plan, const DecodeRowsArgs& a, hipStream_t st) {
    if ((s.dtype != 1 && s.dtype != 2) || (s.D != 128 && s.D != 64) || s.G > 16) return hipErrorInvalidValue;
    dim3 grid(plan.n_chunks, s.Hkv, s.B), block(kMB);
    const bool f16 = s.dtype == 2;
    if (s.D == 128 && !f16) KASCADE_LAUNCH((decode_rows_mfma16_kernel<128, true, false>), grid, block, 0, st, s, plan, a);
    else if (s.D == 128) KASCADE_LAUNCH((decode_rows_mfma16_kernel<128, true, true>), grid, block, 0, st, s, plan, a);
    else if (!f16) KASCADE_LAUNCH((decode_rows_mfma16_kernel<64, true, false>), grid, block, 0, st, s, plan, a);
    else KASCADE_LAUNCH((decode_rows_mfma16_kernel<64, true, true>), grid, block, 0, st, s, plan, a);
    return hipGetLastError();
}

// Stream mode (every row of a sequence, logits stored), same restrictions; the logit rows must be
// 16-byte aligned (pitch a multiple of 4 floats) and the chunk length a multiple of 8.
hipError_t launch_decode_stream_mfma(const Shape& s, const DecodePlan& plan, const DecodeRowsArgs& a, bool with_v, hipStream_t st) {
    if ((s.dtype != 1 && s.dtype != 2) || (s.D != 128 && s.D != 64) || s.G > 16) return hipErrorInvalidValue;
    if ((a.logit_pitch & 3) || (reinterpret_cast<uintptr_t>(a.logits) & 15) || (plan.chunk & 7)) return hipErrorInvalidValue;
    dim3 grid(plan.n_chunks, s.Hkv, s.B), block(kMB);
    const bool f16 = s.dtype == 2;
#define KASCADE_LAUNCH_SWEEP(D_, F_)                                                                                   \
    {                                                                                                                  \
        if (with_v) KASCADE_LAUNCH((decode_rows_mfma16_kernel<D_, false, F_>), grid, block, 0, st, s, plan, a);     \
        else KASCADE_LAUNCH((decode_sweep_mfma_kernel<D_, F_>), grid, block, 0, st, s, plan, a);                   \
    }
    if (s.D == 128 && !f16) KASCADE_LAUNCH_SWEEP(128, false)
    else if (s.D == 128) KASCADE_LAUNCH_SWEEP(128, true)
    else if (!f16) KASCADE_LAUNCH_SWEEP(64, false)
    else KASCADE_LAUNCH_SWEEP(64, true)
#undef KASCADE_LAUNCH_SWEEP
    return hipGetLastError();
}

}  // namespace kascade
