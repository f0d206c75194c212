// Prefill kernels of the Kascade hot path (gfx950, bf16 MFMA 32x32x16, fp32 softmax).
//
// A query tile is T consecutive tokens times the G query heads of one key head (paper Sec. 3.4):
// 128 rows in the paper's configuration, any multiple of 128 here.  One workgroup of four waves owns
// 128 rows = Ts = 128/G consecutive tokens times the G heads (a whole tile, or one of its R = T/Ts
// parts); wave w owns rows 32w..32w+31, row rho = g*Ts + token_in_part.  Index sets, their budget
// and the Top-k candidates (the keys before the tile) belong to the tile; the causal diagonal of a
// part runs from the tile's first token to the part's last.  Keys are processed in blocks of 64 held in LDS,
// K and V row-major and XOR-swizzled against bank conflicts; V^T operand fragments come from the
// transposing LDS read (ds_read_b64_tr_b16).  Tiles are double buffered and filled by direct
// global-to-LDS loads, so block kb+1 streams in while block kb is multiplied and a block costs one
// barrier.  The running softmax keeps a reference exponent that may lag the true maximum and looks
// at a block's maximum only when a term would exceed 2^30.
//
//  prefill_attend_kernel  flash-style attention over a key list:
//      dense  - all keys up to the diagonal, causal, with the dense output (anchor pass 1 of layer 0, Sec. 3.6);
//      sparse - the tile's Top-k index list plus its diagonal block (reuse layers / pass 4).
//      Scores are computed transposed (S^T = K Q^T) so that a lane owns one query row and the
//      row max / row sum are in-lane reductions; O^T = V^T P^T accumulates in the same layout.
//  prefill_stats_kernel   anchor pass 1 when only the row statistics (max, sum) are wanted: the same causal
//      sweep without V, 64 rows per wave, the products of one key block issued between the exponentials of
//      the block before.
//  prefill_pool2_kernel   anchor pass 2 for 128-row tiles: recomputes S = Q K^T over the strict prefix,
//      normalises with the known statistics and sums the tile's rows per key (post-softmax pooling,
//      Sec. 3.4); a lane owns one key column, so the column sum is in-lane.  Same product order as the
//      statistics kernel; then pass 3 (per-tile Top-k) in the same workgroup.
//  prefill_pool_kernel    the same for tiles of more than 128 rows, swept in 128-row parts.
#include <limits.h>

#include "device_utils.h"
#include "kernels.h"
#include "mfma_tiles.h"
#include "topk_select.h"

namespace kascade {

namespace {

constexpr int kPB = 256;          // threads per workgroup
constexpr int kPW = kPB / kWave;  // waves
constexpr int BK = 64;            // keys per block
constexpr int kTileRows = 128;

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;   // one 16-byte piece in flight
using namespace mfma;

struct RowMap {   // which (token, head) a tile row is
    int token, head;
    bool ok;
};
__device__ __forceinline__ RowMap map_row(int rho, int t, int T, int hk, int G, int S) {
    RowMap m;
    m.token = t * T + rho % T;
    m.head = hk * G + rho / T;
    m.ok = m.token < S;
    return m;
}

// ---- direct global -> LDS staging ---------------------------------------------------------
// global_load_lds_dwordx4 writes lane i's 16 bytes to (wave-uniform LDS base) + 16 i, so the LDS
// side is linear in the thread index and the XOR swizzle is applied on the source side: the
// thread that fills chunk position pp of a row fetches logical chunk pp ^ f(row).  The resulting
// LDS image is the one k_off<D> addresses.  No staging registers, no LDS write instructions.

template <int D> struct Dma {
    static constexpr int PPR = D / 8, RPP = kPB / PPR, PASSES = BK / RPP;
    // byte offset inside a row of the chunk this thread fetches (same for all its passes)
    static __device__ __forceinline__ uint32_t chunk_off() {
        const int r0 = threadIdx.x / PPR, pp = threadIdx.x % PPR;
        const int f = (D == 128) ? (r0 & 15) : ((r0 >> 1) & 7);
        return (uint32_t)((pp ^ f) << 4);
    }
};

// stage key rows row_first + slot (slot = 0..63), rows clamped to row_last, into `tile`
template <int D>
__device__ __forceinline__ void dma_rows_seq(unsigned char* tile, const unsigned char* base, uint32_t row_bytes,
                                             int row_first, int row_last, uint32_t coff, int w) {
    const int r0 = threadIdx.x / Dma<D>::PPR;
    if (row_first + BK - 1 <= row_last) {   // every row exists: uniform block/pass offset + a constant per-thread part
        const uint32_t tofs = (uint32_t)r0 * row_bytes + coff;
#pragma unroll
        for (int i = 0; i < Dma<D>::PASSES; ++i) {
            const unsigned char* src = base + (size_t)(row_first + i * Dma<D>::RPP) * row_bytes + (size_t)tofs;
            __builtin_amdgcn_global_load_lds((gmem_ptr_t)src, (lds_ptr_t)(tile + (i * kPB + w * kWave) * 16), 16, 0, 0);
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < Dma<D>::PASSES; ++i) {
        int row = row_first + i * Dma<D>::RPP + r0;
        row = row < row_last ? row : row_last;
        const unsigned char* src = base + (size_t)((uint32_t)row * row_bytes + coff);
        __builtin_amdgcn_global_load_lds((gmem_ptr_t)src, (lds_ptr_t)(tile + (i * kPB + w * kWave) * 16), 16, 0, 0);
    }
}


// Flash-style attention over a key list with both tiles (K and V) double
// buffered in LDS and filled by direct loads: block kb+1 streams in while block kb is multiplied,
// one barrier per block.  BUF is the LDS buffer of this block; it is a template constant so that all
// LDS addresses of a block differ from the other buffer's only by an immediate offset.
template <int D, bool SPARSE, bool F16>
__global__ __launch_bounds__(kPB, 2) void prefill_attend_kernel(Shape s, PrefillArgs a) {
    constexpr int KSTEPS = D / 16, DBLK = D / 32, TILE = BK * D * 2;
    constexpr int PASSES = Dma<D>::PASSES, RPP = Dma<D>::RPP, PPR = Dma<D>::PPR;
    __shared__ __align__(16) unsigned char smK[2 * TILE];
    __shared__ __align__(16) unsigned char smV[2 * TILE];
    __shared__ int smPos[2][BK];
    __shared__ int smFlag[3];   // "block holds a slot without a key", rotating over three blocks

    const int hk = blockIdx.x % s.Hkv;
    const int u = a.n_sub - 1 - blockIdx.x / s.Hkv;     // this workgroup's 128 rows; long ones first
    const int Ts = a.sub_tokens, S = a.seqlen;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave index, held in a scalar register
    const int q = lane & 31, h = lane >> 5;
    const RowMap rm = map_row(w * 32 + q, u, Ts, hk, s.G, S);
    const int q_token = rm.ok ? rm.token : INT_MAX - 1;
    const float c = s.scale_log2;
    // a block's weights are rescaled once a lane's block sum exceeds this: far below the largest value of the
    // type the weights are rounded to for the second product (bf16: 2^127, fp16: 65504)
    constexpr float kRescaleAbove = F16 ? 32768.f : 1073741824.f;

    // sparse: the tile these rows belong to owns the index list and the candidates end where it starts;
    // dense: plain causal attention, everything before the rows' own first token is unmasked
    const int own = u * Ts;
    const int t = own / a.tile_tokens;
    const int prefix = SPARSE ? t * a.tile_tokens : own;
    const int diag_end = (own + Ts < S) ? own + Ts : S;
    int n_sparse = 0, nb_gather = 0, n_blocks;
    const int32_t* idx = nullptr;
    if constexpr (SPARSE) {
        const TileSlot slot = bounded_tile_slot(a.k_per_tile[t], a.idx_offsets[t], prefix, a.idx_total);
        n_sparse = slot.k;
        nb_gather = (n_sparse + BK - 1) / BK;
        n_blocks = nb_gather + (diag_end - prefix + BK - 1) / BK;
        int src = a.head_map ? a.head_map[hk] : hk;
        src = src < 0 ? 0 : (src >= a.n_src_heads ? a.n_src_heads - 1 : src);
        idx = a.idx + (int64_t)src * a.idx_total + slot.off;
    } else {
        n_blocks = (diag_end + BK - 1) / BK;
    }
    const int n_seq = SPARSE ? 0 : prefix / BK;   // dense: blocks entirely before the tile, every slot a key

    const unsigned char* Kb = reinterpret_cast<const unsigned char*>(reinterpret_cast<const bf16_t*>(a.k) + hk * s.kv_stride[1]);
    const unsigned char* Vb = reinterpret_cast<const unsigned char*>(reinterpret_cast<const bf16_t*>(a.v) + hk * s.kv_stride[1]);
    const uint32_t row_bytes = (uint32_t)s.kv_stride[2] * 2u;
    const int r0 = threadIdx.x / PPR, pp = threadIdx.x % PPR;
    const uint32_t koff = Dma<D>::chunk_off();
    const uint32_t voff = (uint32_t)((pp ^ ((D == 128) ? ((r0 & 3) << 2) : (((r0 >> 1) & 1) << 2))) << 4);
    const uint32_t seq_k = (uint32_t)r0 * row_bytes + koff, seq_v = (uint32_t)r0 * row_bytes + voff;

    // Key position of this thread's staging slots in block kb (-1 = no key).  Gathered blocks take
    // two steps so that nothing waits on the index load when it is issued: KASCADE_BLOCK_RAW fetches
    // the list entries a block early (clamped subscript, value untouched), KASCADE_BLOCK_POS turns
    // them into positions when the block is staged.
#define KASCADE_BLOCK_RAW(kb_, pos_)                                                        \
    if (SPARSE && (kb_) < nb_gather) {                                                       \
        _Pragma("unroll") for (int i_ = 0; i_ < PASSES; ++i_) {                              \
            const int j_ = (kb_) * BK + i_ * RPP + r0;                                       \
            pos_[i_] = idx[j_ < n_sparse ? j_ : n_sparse - 1];                               \
        }                                                                                    \
    }
#define KASCADE_BLOCK_POS(kb_, pos_)                                                        \
    _Pragma("unroll") for (int i_ = 0; i_ < PASSES; ++i_) {                                  \
        const int slot_ = i_ * RPP + r0;                                                     \
        int p_;                                                                              \
        if (SPARSE && (kb_) < nb_gather) {                                                   \
            p_ = ((kb_) * BK + slot_ < n_sparse && pos_[i_] < prefix) ? pos_[i_] : -1;       \
        } else {                                                                             \
            p_ = (SPARSE ? prefix + ((kb_) - nb_gather) * BK : (kb_) * BK) + slot_;          \
            if (p_ >= diag_end) p_ = -1;                                                     \
        }                                                                                    \
        pos_[i_] = p_;                                                                       \
    }
    // direct loads of the rows pos_[] into buffer buf_; records the positions for the masks
#define KASCADE_STAGE(buf_, pos_, flag_)                                                                     \
    {                                                                                                        \
        bool bad_ = false;                                                                                   \
        _Pragma("unroll") for (int i_ = 0; i_ < PASSES; ++i_) {                                               \
            const uint32_t off_ = (uint32_t)(pos_[i_] < 0 ? 0 : pos_[i_]) * row_bytes;                       \
            unsigned char* dk_ = smK + (buf_) * TILE + (i_ * kPB + w * kWave) * 16;                           \
            __builtin_amdgcn_global_load_lds((gmem_ptr_t)(Kb + (size_t)(off_ + koff)), (lds_ptr_t)dk_, 16, 0, 0); \
            unsigned char* dv_ = smV + (buf_) * TILE + (i_ * kPB + w * kWave) * 16;                           \
            __builtin_amdgcn_global_load_lds((gmem_ptr_t)(Vb + (size_t)(off_ + voff)), (lds_ptr_t)dv_, 16, 0, 0); \
            if (pp == 0) smPos[buf_][i_ * RPP + r0] = pos_[i_] < 0 ? INT_MAX : pos_[i_];                     \
            bad_ |= pos_[i_] < 0;                                                                            \
        }                                                                                                    \
        if (bad_) smFlag[flag_] = 1;                                                                         \
    }
    // the same for a block of consecutive keys that all exist (no masks, no bookkeeping): the block
    // and pass offsets are uniform (scalar base), the per-thread part never changes
#define KASCADE_STAGE_SEQ(buf_, kb_)                                                                         \
    {                                                                                                        \
        _Pragma("unroll") for (int i_ = 0; i_ < PASSES; ++i_) {                                               \
            const size_t blk_ = (size_t)((kb_) * BK + i_ * RPP) * row_bytes;                                  \
            unsigned char* dk_ = smK + (buf_) * TILE + (i_ * kPB + w * kWave) * 16;                           \
            __builtin_amdgcn_global_load_lds((gmem_ptr_t)(Kb + blk_ + (size_t)seq_k), (lds_ptr_t)dk_, 16, 0, 0); \
            unsigned char* dv_ = smV + (buf_) * TILE + (i_ * kPB + w * kWave) * 16;                           \
            __builtin_amdgcn_global_load_lds((gmem_ptr_t)(Vb + blk_ + (size_t)seq_v), (lds_ptr_t)dv_, 16, 0, 0); \
        }                                                                                                    \
    }

    // query fragments (B operand of S^T = K Q^T): row q of this wave, 8 elements per k-step
    bf16x8_t qf[KSTEPS];
    {
        const bf16_t* qp = reinterpret_cast<const bf16_t*>(a.q) + (int64_t)rm.token * s.q_stride[1] + (int64_t)rm.head * s.q_stride[2];
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (rm.ok) raw = *reinterpret_cast<const uint4*>(qp + kk * 16 + h * 8);
            qf[kk] = __builtin_bit_cast(bf16x8_t, raw);
        }
    }

    // (m_run, l_run): reference exponent and the sum of 2^(s c - m_run) over the keys seen so far;
    // neg_ref = -m_run once a finite reference exists, +inf before (forces the exact path)
    float m_run = -INFINITY, l_run = 0.f, neg_ref = INFINITY;
    f32x16_t acc_o[DBLK];
#pragma unroll
    for (int i = 0; i < DBLK; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[i][r] = 0.f;

    if (threadIdx.x < 3) smFlag[threadIdx.x] = 0;
    __syncthreads();
    int pos[PASSES];
    if (0 < n_seq) {
        KASCADE_STAGE_SEQ(0, 0)
    } else {
        KASCADE_BLOCK_RAW(0, pos)
        KASCADE_BLOCK_POS(0, pos)
        KASCADE_STAGE(0, pos, 0)
    }
    KASCADE_BLOCK_RAW(1, pos)

    const int key0 = perm_key(q), key1 = 32 + key0;
    int f_cur = 0, f_next = 1, f_free = 2;   // smFlag slots of block kb, kb+1 and the one to clear for kb+2

    // S^T block: rows = 64 keys (two MFMA tiles), cols = this wave's 32 queries; then the masks:
    // causal inside / beyond the diagonal, and slots without a key.  Fragment reads run four k-steps
    // ahead of the products that use them.
#define KASCADE_SCORES(tK_, buf_, kb_)                                                                       \
    {                                                                                                        \
        _Pragma("unroll") for (int r = 0; r < 16; ++r) { s0[r] = 0.f; s1[r] = 0.f; }                          \
        bf16x8_t fa_[KSTEPS], fb_[KSTEPS];                                                                   \
        _Pragma("unroll") for (int kk = 0; kk < KSTEPS; ++kk) {                                               \
            fa_[kk] = lds_frag(tK_ + k_off<D>(key0, kk * 2 + h));                                            \
            fb_[kk] = lds_frag(tK_ + k_off<D>(key1, kk * 2 + h));                                            \
        }                                                                                                    \
        _Pragma("unroll") for (int kk = 0; kk < KSTEPS; ++kk) {                                               \
            s0 = Mma<F16>::mma32(fa_[kk], qf[kk], s0);                                                       \
            s1 = Mma<F16>::mma32(fb_[kk], qf[kk], s1);                                                       \
        }                                                                                                    \
        __builtin_amdgcn_sched_group_barrier(0x100, KSTEPS >= 4 ? 8 : 2 * KSTEPS, 0);                        \
        _Pragma("unroll") for (int kk = 0; kk + 4 < KSTEPS; ++kk) {                                           \
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                                               \
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);                                               \
        }                                                                                                    \
        __builtin_amdgcn_sched_group_barrier(0x008, KSTEPS >= 4 ? 8 : 2 * KSTEPS, 0);                        \
        bool need_mask = smFlag[f_cur] != 0;                                                                 \
        if constexpr (SPARSE) need_mask |= (kb_) >= nb_gather;                                               \
        else need_mask |= ((kb_) + 1) * BK > prefix;                                                         \
        if (need_mask) {                                                                                     \
            _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                                  \
                const int slot = (r >> 3) * 16 + h * 8 + (r & 7);                                            \
                if (smPos[buf_][slot] > q_token) s0[r] = -INFINITY;                                          \
                if (smPos[buf_][32 + slot] > q_token) s1[r] = -INFINITY;                                     \
            }                                                                                                \
        }                                                                                                    \
    }

    // one block; buf_ is a literal
#define KASCADE_ATTEND_BLOCK(kb_, buf_)                                                                       \
    {                                                                                                        \
        wait_vmem();                                                                                         \
        __syncthreads();   /* tile kb_ has landed; nobody reads the other buffer any more */                 \
        if (threadIdx.x == 0) smFlag[f_free] = 0;                                                            \
        const unsigned char* tK_ = smK + (buf_) * TILE;                                                      \
        f32x16_t s0, s1;                                                                                     \
        KASCADE_SCORES(tK_, buf_, kb_)                                                                       \
        /* The loads of the next block are issued here, behind this block's score products, not right   */ \
        /* after the barrier: there every wave of the compute unit would issue its loads at once and     */ \
        /* queue behind the others while its matrix work waits.                                          */ \
        if ((kb_) + 1 < n_seq) {                                                                             \
            KASCADE_STAGE_SEQ(1 - (buf_), (kb_) + 1)                                                         \
        } else if ((kb_) + 1 < n_blocks) {                                                                   \
            KASCADE_BLOCK_POS((kb_) + 1, pos)                                                                \
            KASCADE_STAGE(1 - (buf_), pos, f_next)                                                           \
            KASCADE_BLOCK_RAW((kb_) + 2, pos)                                                                \
        }                                                                                                    \
        /* Online softmax, base 2; this lane owns query row q (the other half-wave holds the other keys   */ \
        /* of the same row).  The exponentials are taken against a reference that may lag the true running */ \
        /* maximum: any reference gives the same quotient acc / l as long as nothing overflows, so the     */ \
        /* block maximum is only looked at when a term exceeds 2^30 (or is not finite, which is how the    */ \
        /* first block gets its reference).  That rare path is wave-uniform and recomputes the scores.     */ \
        float rs = 0.f;                                                                                      \
        _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                                      \
            s0[r] = __builtin_amdgcn_exp2f(fmaf(s0[r], c, neg_ref));                                         \
            s1[r] = __builtin_amdgcn_exp2f(fmaf(s1[r], c, neg_ref));                                         \
            rs += s0[r] + s1[r];                                                                             \
        }                                                                                                    \
        if (__builtin_amdgcn_ballot_w64(!(rs <= kRescaleAbove)) != 0) {                                      \
            KASCADE_SCORES(tK_, buf_, kb_)                                                                   \
            float mx = s0[0];                                                                                \
            _Pragma("unroll") for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s0[r]);                             \
            _Pragma("unroll") for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s1[r]);                             \
            mx *= c;                                                                                         \
            mx = half_swap_max(mx);                                                                          \
            const float m_new = fmaxf(m_run, mx);                                                            \
            const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;                                         \
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);   /* 0 while m_run is -inf */        \
            rs = 0.f;                                                                                        \
            _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                                  \
                s0[r] = __builtin_amdgcn_exp2f(fmaf(s0[r], c, -m_safe));                                     \
                s1[r] = __builtin_amdgcn_exp2f(fmaf(s1[r], c, -m_safe));                                     \
                rs += s0[r] + s1[r];                                                                         \
            }                                                                                                \
            l_run *= alpha;                                                                                  \
            _Pragma("unroll") for (int i = 0; i < DBLK; ++i)                                                  \
                _Pragma("unroll") for (int r = 0; r < 16; ++r) acc_o[i][r] *= alpha;                          \
            m_run = m_new;                                                                                   \
            /* no key seen yet (every slot so far masked or ignored): keep forcing the exact path, so    */ \
            /* that the first block with a live key sets the reference                                    */ \
            neg_ref = (m_new == -INFINITY) ? INFINITY : -m_safe;                                             \
        }                                                                                                    \
        rs = half_swap_sum(rs);                                                                              \
        l_run += rs;                                                                                         \
        {                                                                                                    \
            const unsigned char* tV_ = smV + (buf_) * TILE;                                                  \
            bf16x8_t pf[4];                                                                                  \
            pf[0] = Mma<F16>::pack_tile(s0, 0); pf[1] = Mma<F16>::pack_tile(s0, 8);                          \
            pf[2] = Mma<F16>::pack_tile(s1, 0); pf[3] = Mma<F16>::pack_tile(s1, 8);                          \
            _Pragma("unroll") for (int i = 0; i < DBLK; ++i) {                                                \
                _Pragma("unroll") for (int st = 0; st < 4; ++st) {                                            \
                    const bf16x8_t va = vt_frag<D>(tV_, i, st * 16);                                         \
                    acc_o[i] = Mma<F16>::mma32(va, pf[st], acc_o[i]);                                        \
                }                                                                                            \
            }                                                                                                \
        }                                                                                                    \
        { const int f_ = f_cur; f_cur = f_next; f_next = f_free; f_free = f_; }                              \
    }

    int kb = 0;
    for (; kb + 1 < n_blocks; kb += 2) {
        KASCADE_ATTEND_BLOCK(kb, 0)
        KASCADE_ATTEND_BLOCK(kb + 1, 1)
    }
    if (kb < n_blocks) { KASCADE_ATTEND_BLOCK(kb, 0) }
#undef KASCADE_ATTEND_BLOCK
#undef KASCADE_SCORES
#undef KASCADE_STAGE_SEQ
#undef KASCADE_STAGE
#undef KASCADE_BLOCK_POS
#undef KASCADE_BLOCK_RAW

    if (!rm.ok) return;
    if (a.stats && h == 0) {
        float* st = a.stats + ((int64_t)rm.head * S + rm.token) * 2;
        st[0] = m_run;
        st[1] = l_run;
    }
    {
        const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
        bf16_t* op = reinterpret_cast<bf16_t*>(a.out) + (int64_t)rm.token * s.o_stride[1] + (int64_t)rm.head * s.o_stride[2];
#pragma unroll
        for (int i = 0; i < DBLK; ++i) {
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int d0 = i * 32 + r4 * 8 + h * 4;
                uint2 pk;
                pk.x = Mma<F16>::bits(acc_o[i][r4 * 4 + 0] * inv) | (Mma<F16>::bits(acc_o[i][r4 * 4 + 1] * inv) << 16);
                pk.y = Mma<F16>::bits(acc_o[i][r4 * 4 + 2] * inv) | (Mma<F16>::bits(acc_o[i][r4 * 4 + 3] * inv) << 16);
                *reinterpret_cast<uint2*>(op + d0) = pk;
            }
        }
    }
}

// Anchor pass 1 when only the row statistics are wanted (anchors other than layer 0, Sec. 3.6): the causal
// Q K^T sweep of prefill_attend_kernel without V and without an output.  Same tiles, same direct loads,
// same transposed product (a lane owns a query row).  What differs is the order of the work inside a
// wave: over the blocks that lie entirely before the workgroup's own tokens (no mask, every key exists)
// the matrix products of block kb+1 are issued between the exponentials of block kb - one product, then
// six vector operations - with two sets of score registers, so that a single wave keeps the matrix pipe
// and the vector ALU busy at the same time instead of alternating between a phase of sixteen products
// and a phase of a hundred vector operations.  (With phases, the four waves of a SIMD fall into step:
// counters show the matrix pipe and the vector ALU busy together for only a quarter of the time.)
// The reference exponent of that stretch is the row maximum of block 0 and is not looked at again; a row
// whose sum overflows fp32 (a logit more than 2^127 above block 0's maximum) sends the whole workgroup
// through the careful loop from the start.  The last blocks (causal mask, ragged end) always take the
// careful loop, which continues from the state the fast stretch leaves.
template <int D, bool F16>
__global__ __launch_bounds__(kPB, 2) void prefill_stats_kernel(Shape s, PrefillArgs a) {
    constexpr int KSTEPS = D / 16, TILE = BK * D * 2;
    constexpr int PF = 4;   // fragment reads issued ahead of the products that use them
    // two tiles as two arrays: the compiler then knows that a fragment read from one cannot see a direct
    // load into the other, and does not wait for the loads in flight before every read
    __shared__ __align__(16) unsigned char smK0[TILE];
    __shared__ __align__(16) unsigned char smK1[TILE];

    // A workgroup owns two consecutive 128-row units (256 rows); wave w owns 64 rows of unit u0 + w/2: rows
    // 64 (w%2) + q and 64 (w%2) + 32 + q of that unit for lane q - every K fragment read from LDS feeds two products.
    const int hk = blockIdx.x % s.Hkv;
    const int n_pairs = (a.n_sub + 1) / 2;
    const int u0 = 2 * (n_pairs - 1 - blockIdx.x / s.Hkv);     // long ones first
    const int Ts = a.sub_tokens, S = a.seqlen;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int q = lane & 31, h = lane >> 5;
    const int u = u0 + (w >> 1);
    const RowMap rmA = map_row((w & 1) * 64 + q, u, Ts, hk, s.G, S);
    const RowMap rmB = map_row((w & 1) * 64 + 32 + q, u, Ts, hk, s.G, S);
    const int tokA = rmA.ok ? rmA.token : INT_MAX - 1, tokB = rmB.ok ? rmB.token : INT_MAX - 1;
    const float c = s.scale_log2;
    const int own = u0 * Ts;                                    // first token of the workgroup's rows
    const int diag_end = (own + 2 * Ts < S) ? own + 2 * Ts : S;
    const int n_blocks = (diag_end + BK - 1) / BK;
    const int n_full = own / BK;                                // blocks whose keys all precede every row here

    const unsigned char* Kb = reinterpret_cast<const unsigned char*>(reinterpret_cast<const bf16_t*>(a.k) + hk * s.kv_stride[1]);
    const uint32_t row_bytes = (uint32_t)s.kv_stride[2] * 2u;
    const uint32_t coff = Dma<D>::chunk_off();
    // a whole block of existing rows: uniform block/pass offset + a constant per-thread part, no clamping
    const uint32_t tofs = (uint32_t)(threadIdx.x / Dma<D>::PPR) * row_bytes + coff;
#define KASCADE_DMA_FULL(tile_, kb_)                                                                        \
    _Pragma("unroll") for (int i_ = 0; i_ < Dma<D>::PASSES; ++i_) {                                          \
        const unsigned char* src_ = Kb + (size_t)((kb_) * BK + i_ * Dma<D>::RPP) * row_bytes + (size_t)tofs; \
        __builtin_amdgcn_global_load_lds((gmem_ptr_t)src_, (lds_ptr_t)((tile_) + (i_ * kPB + w * kWave) * 16), 16, 0, 0); \
    }

    bf16x8_t qa[KSTEPS], qb[KSTEPS];
    {
        const bf16_t* pa = reinterpret_cast<const bf16_t*>(a.q) + (int64_t)rmA.token * s.q_stride[1] + (int64_t)rmA.head * s.q_stride[2];
        const bf16_t* pb = reinterpret_cast<const bf16_t*>(a.q) + (int64_t)rmB.token * s.q_stride[1] + (int64_t)rmB.head * s.q_stride[2];
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            uint4 ra = make_uint4(0, 0, 0, 0), rb = make_uint4(0, 0, 0, 0);
            if (rmA.ok) ra = *reinterpret_cast<const uint4*>(pa + kk * 16 + h * 8);
            if (rmB.ok) rb = *reinterpret_cast<const uint4*>(pb + kk * 16 + h * 8);
            qa[kk] = __builtin_bit_cast(bf16x8_t, ra);
            qb[kk] = __builtin_bit_cast(bf16x8_t, rb);
        }
    }
    // LDS byte offsets of this lane's K fragments (key slot perm_key(q), k-step kk); the second 32 keys of a
    // block are a constant offset from them
    const int key0 = perm_key(q);
    int fo[KSTEPS];
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) fo[kk] = k_off<D>(key0, kk * 2 + h);
    constexpr int KEY1 = 32 * D * 2;

    // this lane's share of its two rows' sums, against the rows' reference exponents (the other half-wave holds
    // the other keys of the same rows); two chains per row so that the additions do not wait for each other
    float mA = -INFINITY, mB = -INFINITY, nrA = INFINITY, nrB = INFINITY;
    float la0 = 0.f, la1 = 0.f, lb0 = 0.f, lb1 = 0.f;
    f32x16_t zero;
#pragma unroll
    for (int r = 0; r < 16; ++r) zero[r] = 0.f;

    // S^T of one block: (xa0, xa1) = keys 0-31 / 32-63 against row A, (xb0, xb1) against row B; plain order
#define KASCADE_STATS_SCORES(tK_, xa0_, xa1_, xb0_, xb1_)                                    \
    {                                                                                        \
        _Pragma("unroll") for (int kk = 0; kk < KSTEPS; ++kk) {                               \
            const bf16x8_t f0_ = lds_frag((tK_) + fo[kk]);                                   \
            const bf16x8_t f1_ = lds_frag((tK_) + fo[kk] + KEY1);                            \
            xa0_ = Mma<F16>::mma32(f0_, qa[kk], kk == 0 ? zero : xa0_);                      \
            xb0_ = Mma<F16>::mma32(f0_, qb[kk], kk == 0 ? zero : xb0_);                      \
            xa1_ = Mma<F16>::mma32(f1_, qa[kk], kk == 0 ? zero : xa1_);                      \
            xb1_ = Mma<F16>::mma32(f1_, qb[kk], kk == 0 ? zero : xb1_);                      \
        }                                                                                    \
    }
    // the exponentials of one block's scores into the four chains
#define KASCADE_STATS_EXPS(ca0_, ca1_, cb0_, cb1_)                                           \
    _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                          \
        la0 += __builtin_amdgcn_exp2f(fmaf(ca0_[r], c, nrA));                                \
        lb0 += __builtin_amdgcn_exp2f(fmaf(cb0_[r], c, nrB));                                \
        la1 += __builtin_amdgcn_exp2f(fmaf(ca1_[r], c, nrA));                                \
        lb1 += __builtin_amdgcn_exp2f(fmaf(cb1_[r], c, nrB));                                \
    }
    // products of the block in tile tN_ into the n registers interleaved with the exponentials of the block
    // whose scores are in the c registers, in an order written out step by step and fenced so that the compiler
    // keeps it: per product two scale-and-shift, two exp2 and the two additions of the step before (an exp2
    // result is never used by the next instruction), per two products one fragment read, issued PF reads
    // ahead.  The empty asm statement pins the results to this point of the program: without it the compiler
    // moves the arithmetic of one block across the barrier into the next.
#define KASCADE_STATS_PIPE(tN_, na0_, na1_, nb0_, nb1_, ca0_, ca1_, cb0_, cb1_)              \
    {                                                                                        \
        constexpr int PPS_ = 32 / (4 * KSTEPS);   /* (row A, row B) score pairs per product */ \
        __builtin_amdgcn_sched_barrier(0);                                                   \
        bf16x8_t fr_[2 * KSTEPS];                                                            \
        _Pragma("unroll") for (int j_ = 0; j_ < PF; ++j_)                                     \
            fr_[j_] = lds_frag((tN_) + fo[j_ >> 1] + ((j_ & 1) ? KEY1 : 0));                 \
        float pea_[PPS_], peb_[PPS_];   /* the exponentials of the step before */            \
        _Pragma("unroll") for (int i_ = 0; i_ < 4 * KSTEPS; ++i_) {                           \
            const int kk_ = i_ >> 2;                                                         \
            if ((i_ & 1) == 0 && (i_ >> 1) + PF < 2 * KSTEPS) {                              \
                const int j_ = (i_ >> 1) + PF;                                               \
                fr_[j_] = lds_frag((tN_) + fo[j_ >> 1] + ((j_ & 1) ? KEY1 : 0));             \
            }                                                                                \
            if ((i_ & 3) == 0) na0_ = Mma<F16>::mma32(fr_[2 * kk_], qa[kk_], kk_ == 0 ? zero : na0_);          \
            else if ((i_ & 3) == 1) nb0_ = Mma<F16>::mma32(fr_[2 * kk_], qb[kk_], kk_ == 0 ? zero : nb0_);     \
            else if ((i_ & 3) == 2) na1_ = Mma<F16>::mma32(fr_[2 * kk_ + 1], qa[kk_], kk_ == 0 ? zero : na1_); \
            else nb1_ = Mma<F16>::mma32(fr_[2 * kk_ + 1], qb[kk_], kk_ == 0 ? zero : nb1_);                    \
            _Pragma("unroll") for (int p_ = 0; p_ < PPS_; ++p_) {                             \
                const int P_ = i_ * PPS_ + p_, r_ = P_ >> 1;   /* pair P_: key half P_ & 1, register r_ */ \
                const float xa_ = fmaf((P_ & 1) ? ca1_[r_] : ca0_[r_], c, nrA);              \
                const float xb_ = fmaf((P_ & 1) ? cb1_[r_] : cb0_[r_], c, nrB);              \
                if (i_ > 0) { if ((P_ - PPS_) & 1) { la1 += pea_[p_]; lb1 += peb_[p_]; } else { la0 += pea_[p_]; lb0 += peb_[p_]; } } \
                pea_[p_] = __builtin_amdgcn_exp2f(xa_);                                      \
                peb_[p_] = __builtin_amdgcn_exp2f(xb_);                                      \
            }                                                                                \
            __builtin_amdgcn_sched_barrier(0);                                               \
        }                                                                                    \
        _Pragma("unroll") for (int p_ = 0; p_ < PPS_; ++p_) {                                 \
            if ((32 - PPS_ + p_) & 1) { la1 += pea_[p_]; lb1 += peb_[p_]; } else { la0 += pea_[p_]; lb0 += peb_[p_]; } \
        }                                                                                    \
        asm volatile("" : "+v"(na0_), "+v"(na1_), "+v"(nb0_), "+v"(nb1_), "+v"(la0), "+v"(la1), "+v"(lb0), "+v"(lb1)); \
        __builtin_amdgcn_sched_barrier(0);                                                   \
    }
#define KASCADE_ROW_MAX(x0_, x1_, out_)                                                      \
    {                                                                                        \
        float mx_ = x0_[0];                                                                  \
        _Pragma("unroll") for (int r = 1; r < 16; ++r) mx_ = fmaxf(mx_, x0_[r]);              \
        _Pragma("unroll") for (int r = 0; r < 16; ++r) mx_ = fmaxf(mx_, x1_[r]);              \
        out_ = half_swap_max(mx_ * c);                                                       \
    }

    int kb_start = 0;
    if (n_full >= 3) {
        // ---- the fast stretch: blocks 0 .. n_full-1 ----
        f32x16_t sa0, sa1, sb0, sb1, ta0, ta1, tb0, tb1;
        KASCADE_DMA_FULL(smK0, 0)
        wait_vmem();
        __syncthreads();
        KASCADE_DMA_FULL(smK1, 1)
        KASCADE_STATS_SCORES(smK0, sa0, sa1, sb0, sb1)
        // reference exponents: the row maxima of block 0
        KASCADE_ROW_MAX(sa0, sa1, mA)
        KASCADE_ROW_MAX(sb0, sb1, mB)
        nrA = -mA; nrB = -mB;
        // iteration kb: tile kb has landed in buffer kb & 1; its products run between the exponentials of
        // block kb-1; tile kb+1 streams into the other buffer meanwhile
        int kb = 1;
        for (; kb + 1 < n_full; kb += 2) {
            wait_vmem();
            __syncthreads();
            KASCADE_DMA_FULL(smK0, kb + 1)
            KASCADE_STATS_PIPE(smK1, ta0, ta1, tb0, tb1, sa0, sa1, sb0, sb1)
            wait_vmem();
            __syncthreads();
            if (kb + 2 < n_full) { KASCADE_DMA_FULL(smK1, kb + 2) }
            KASCADE_STATS_PIPE(smK0, sa0, sa1, sb0, sb1, ta0, ta1, tb0, tb1)
        }
        if (kb < n_full) {      // one block left for the products (odd count): its scores end up in the t registers
            wait_vmem();
            __syncthreads();
            KASCADE_STATS_PIPE(smK1, ta0, ta1, tb0, tb1, sa0, sa1, sb0, sb1)
#pragma unroll
            for (int r = 0; r < 16; ++r) { sa0[r] = ta0[r]; sa1[r] = ta1[r]; sb0[r] = tb0[r]; sb1[r] = tb1[r]; }
        }
        // the exponentials of the last block
        KASCADE_STATS_EXPS(sa0, sa1, sb0, sb1)
        const float partA = la0 + la1, partB = lb0 + lb1;
        const int overflowed = __syncthreads_or(!(partA <= 3.0e38f) || !(partB <= 3.0e38f));   // also the barrier that frees the tiles
        if (overflowed) {
            mA = mB = -INFINITY; nrA = nrB = INFINITY;
            la0 = la1 = lb0 = lb1 = 0.f;
        } else {
            la0 = partA; lb0 = partB; la1 = lb1 = 0.f;
            kb_start = n_full;
        }
    }
#undef KASCADE_STATS_PIPE
#undef KASCADE_DMA_FULL

    // ---- the careful loop: blocks kb_start .. n_blocks-1, two at a time so that the tile is a constant ----
    // exp2 against the lagging reference; a block whose share of a row's sum is not a modest finite number
    // (the first block: the reference is still +inf) renews that row's reference from the scores, which are
    // still in registers.  Masks where the block reaches the workgroup's own tokens: key position > row's token.
#define KASCADE_STATS_ROW(x0_, x1_, tok_, m_, nr_, l_, kb_)                                                    \
    {                                                                                                          \
        if (((kb_) + 1) * BK > own) {                                                                          \
            _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                                    \
                const int slot = (kb_) * BK + (r >> 3) * 16 + h * 8 + (r & 7);                                 \
                if (slot > tok_) x0_[r] = -INFINITY;                                                           \
                if (slot + 32 > tok_) x1_[r] = -INFINITY;                                                      \
            }                                                                                                  \
        }                                                                                                      \
        float rs = 0.f;                                                                                        \
        _Pragma("unroll") for (int r = 0; r < 16; ++r)                                                          \
            rs += __builtin_amdgcn_exp2f(fmaf(x0_[r], c, nr_)) + __builtin_amdgcn_exp2f(fmaf(x1_[r], c, nr_)); \
        if (__builtin_amdgcn_ballot_w64(!(rs <= 1073741824.f)) != 0) {                                         \
            float mx;                                                                                          \
            KASCADE_ROW_MAX(x0_, x1_, mx)                                                                      \
            const float m_new = fmaxf(m_, mx);                                                                 \
            const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;                                           \
            const float alpha = __builtin_amdgcn_exp2f(m_ - m_safe);   /* 0 while m_ is -inf */                \
            rs = 0.f;                                                                                          \
            _Pragma("unroll") for (int r = 0; r < 16; ++r)                                                      \
                rs += __builtin_amdgcn_exp2f(fmaf(x0_[r], c, -m_safe)) + __builtin_amdgcn_exp2f(fmaf(x1_[r], c, -m_safe)); \
            l_ *= alpha;                                                                                       \
            m_ = m_new;                                                                                        \
            nr_ = (m_new == -INFINITY) ? INFINITY : -m_safe;                                                   \
        }                                                                                                      \
        l_ += rs;                                                                                              \
    }
#define KASCADE_STATS_CAREFUL(tK_, tNext_, kb_)                                                                \
    {                                                                                                          \
        wait_vmem();                                                                                           \
        __syncthreads();                                                                                       \
        f32x16_t xa0, xa1, xb0, xb1;                                                                           \
        KASCADE_STATS_SCORES(tK_, xa0, xa1, xb0, xb1)                                                          \
        if ((kb_) + 1 < n_blocks) dma_rows_seq<D>(tNext_, Kb, row_bytes, ((kb_) + 1) * BK, diag_end - 1, coff, w); \
        KASCADE_STATS_ROW(xa0, xa1, tokA, mA, nrA, la0, kb_)                                                   \
        KASCADE_STATS_ROW(xb0, xb1, tokB, mB, nrB, lb0, kb_)                                                   \
    }
    if (kb_start < n_blocks) dma_rows_seq<D>(smK0, Kb, row_bytes, kb_start * BK, diag_end - 1, coff, w);
    {
        int kb = kb_start;
        for (; kb + 1 < n_blocks; kb += 2) {
            KASCADE_STATS_CAREFUL(smK0, smK1, kb)
            KASCADE_STATS_CAREFUL(smK1, smK0, kb + 1)
        }
        if (kb < n_blocks) { KASCADE_STATS_CAREFUL(smK0, smK1, kb) }
    }
#undef KASCADE_STATS_CAREFUL
#undef KASCADE_STATS_ROW
#undef KASCADE_ROW_MAX
#undef KASCADE_STATS_EXPS
#undef KASCADE_STATS_SCORES

    const float lA = half_swap_sum(la0), lB = half_swap_sum(lb0);
    if (a.stats && h == 0) {
        if (rmA.ok) {
            float* st = a.stats + ((int64_t)rmA.head * S + rmA.token) * 2;
            st[0] = mA; st[1] = lA;
        }
        if (rmB.ok) {
            float* st = a.stats + ((int64_t)rmB.head * S + rmB.token) * 2;
            st[0] = mB; st[1] = lB;
        }
    }
}

// One 64-key block of anchor pass 2 for this wave: S = Q K^T from the staged tile, pooled
// weights 2^(s c - e_r), column sums over the wave's 32 rows into part[w][key].
template <int D, bool F16>
__device__ __forceinline__ void pool_block(const unsigned char* tile, float (*part)[BK], const bf16x8_t (&qf)[D / 16],
                                           const float (&e_r)[16], float c, int key0, int key1, int h, int w) {
    constexpr int KSTEPS = D / 16;
    f32x16_t s0, s1;
#pragma unroll
    for (int r = 0; r < 16; ++r) { s0[r] = 0.f; s1[r] = 0.f; }
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
        const bf16x8_t b0 = lds_frag(tile + k_off<D>(key0, kk * 2 + h));
        const bf16x8_t b1 = lds_frag(tile + k_off<D>(key1, kk * 2 + h));
        s0 = Mma<F16>::mma32(qf[kk], b0, s0);
        s1 = Mma<F16>::mma32(qf[kk], b1, s1);
    }
    float c0 = 0.f, c1 = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        c0 += __builtin_amdgcn_exp2f(fmaf(s0[r], c, -e_r[r]));
        c1 += __builtin_amdgcn_exp2f(fmaf(s1[r], c, -e_r[r]));
    }
    c0 = half_swap_sum(c0);
    c1 = half_swap_sum(c1);
    if (h == 0) { part[w][key0] = c0; part[w][key1] = c1; }
}

// Anchor pass 2 with two K tiles in LDS filled by direct loads: block kb+1 streams in while block
// kb is multiplied; one barrier per block.  The cross-wave sum of block kb's column partials is
// taken after the next barrier (two partial buffers), so it needs no barrier of its own.
// For tiles of more than 128 rows, which are swept in parts of 128 (128-row tiles go to prefill_pool2_kernel).
template <int D, bool F16>
__global__ __launch_bounds__(kPB, 2) void prefill_pool_kernel(Shape s, PrefillArgs a) {
    constexpr int KSTEPS = D / 16, TILE = BK * D * 2;
    constexpr int PART = kPW * BK * (int)sizeof(float);
    // two K tiles and two buffers of column partials during the sweep; afterwards the same memory
    // holds the selection's histogram and candidate list
    constexpr int kSmem = (2 * TILE + 2 * PART) > (int)sizeof(SelectShared<kPB>) ? (2 * TILE + 2 * PART) : (int)sizeof(SelectShared<kPB>);
    __shared__ __align__(16) unsigned char smem[kSmem];
    unsigned char* const smK0 = smem;
    unsigned char* const smK1 = smem + TILE;
    float (*const smPart0)[BK] = reinterpret_cast<float (*)[BK]>(smem + 2 * TILE);
    float (*const smPart1)[BK] = reinterpret_cast<float (*)[BK]>(smem + 2 * TILE + PART);

    const int hk = blockIdx.x % s.Hkv;
    const int t = a.n_tiles - 1 - blockIdx.x / s.Hkv;
    const int T = a.tile_tokens, Ts = a.sub_tokens, S = a.seqlen;
    const int prefix = t * T;
    if (prefix == 0) return;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave index, held in a scalar register
    const int q = lane & 31, h = lane >> 5;
    const float c = s.scale_log2;
    const int tile_end = (prefix + T < S) ? prefix + T : S;
    const float inv_rows = 1.f / (float)((tile_end - prefix) * s.G);
    const int n_blocks = (prefix + BK - 1) / BK;
    const int n_parts = (tile_end - prefix + Ts - 1) / Ts;   // 128 rows at a time

    const unsigned char* Kb = reinterpret_cast<const unsigned char*>(reinterpret_cast<const bf16_t*>(a.k) + hk * s.kv_stride[1]);
    const uint32_t row_bytes = (uint32_t)s.kv_stride[2] * 2u;
    const uint32_t coff = Dma<D>::chunk_off();
    const int key0 = perm_key(q), key1 = 32 + key0;
    float* dst = a.pooled + hk * a.pooled_pitch + (int64_t)T * t * (t - 1) / 2;

    // Every part sweeps the tile's whole prefix with its own 128 rows; the first writes the column
    // sums, the others add theirs to what is there (same thread, same address: program order).
    for (int part = 0; part < n_parts; ++part) {
        const int u = prefix / Ts + part;
        dma_rows_seq<D>(smK0, Kb, row_bytes, 0, prefix - 1, coff, w);

        const RowMap rm = map_row(w * 32 + q, u, Ts, hk, s.G, S);
        bf16x8_t qf[KSTEPS];
        {
            const bf16_t* qp = reinterpret_cast<const bf16_t*>(a.q) + (int64_t)rm.token * s.q_stride[1] + (int64_t)rm.head * s.q_stride[2];
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk) {
                uint4 raw = make_uint4(0, 0, 0, 0);
                if (rm.ok) raw = *reinterpret_cast<const uint4*>(qp + kk * 16 + h * 8);
                qf[kk] = __builtin_bit_cast(bf16x8_t, raw);
            }
        }
        // e_r = m + log2(l * rows) of the query rows whose scores land in this lane's registers;
        // rows beyond the sequence get weight 0
        float e_r[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const RowMap rr = map_row(w * 32 + (r >> 2) * 8 + h * 4 + (r & 3), u, Ts, hk, s.G, S);
            e_r[r] = INFINITY;
            if (rr.ok) {
                const float* st = a.stats + ((int64_t)rr.head * S + rr.token) * 2;
                e_r[r] = st[0] + __builtin_amdgcn_logf(st[1] / inv_rows);
            }
        }

#define KASCADE_POOL_STORE(part_, kb_)                                                                         \
        if (threadIdx.x < BK) {                                                                                \
            const int j_ = (kb_) * BK + threadIdx.x;                                                           \
            if (j_ < prefix) {                                                                                 \
                const float sum_ = (part_[0][threadIdx.x] + part_[1][threadIdx.x]) +                           \
                                   (part_[2][threadIdx.x] + part_[3][threadIdx.x]);                            \
                dst[j_] = part == 0 ? sum_ : dst[j_] + sum_;                                                   \
            }                                                                                                  \
        }
#define KASCADE_POOL_STEP(kb_, cur_, nxt_, part_cur_, part_prev_)                                              \
        {                                                                                                      \
            wait_vmem();                                                                                       \
            __syncthreads();                                                                                   \
            if ((kb_) + 1 < n_blocks) dma_rows_seq<D>(nxt_, Kb, row_bytes, ((kb_) + 1) * BK, prefix - 1, coff, w); \
            if ((kb_) > 0) KASCADE_POOL_STORE(part_prev_, (kb_) - 1)                                           \
            pool_block<D, F16>(cur_, part_cur_, qf, e_r, c, key0, key1, h, w);                                      \
        }
        int kb = 0;
        for (; kb + 1 < n_blocks; kb += 2) {
            KASCADE_POOL_STEP(kb, smK0, smK1, smPart0, smPart1)
            KASCADE_POOL_STEP(kb + 1, smK1, smK0, smPart1, smPart0)
        }
        if (kb < n_blocks) {
            KASCADE_POOL_STEP(kb, smK0, smK1, smPart0, smPart1)
            ++kb;
        }
        __syncthreads();   // the last block's partials are complete; every read of the K tiles is done
        {
            float (*last)[BK] = (kb & 1) ? smPart0 : smPart1;
            KASCADE_POOL_STORE(last, kb - 1)
        }
#undef KASCADE_POOL_STEP
#undef KASCADE_POOL_STORE
    }
    // anchor pass 3 for this (tile, key head): the pooled scores of the tile were all written by this
    // workgroup, so it selects right away - while it does, the other workgroups of the compute unit keep
    // the matrix pipes busy, and no separate selection launch (one workgroup per compute unit, latency
    // bound) is needed
    if (a.topk_out) {
        __syncthreads();   // the pooled scores are visible to the whole workgroup; LDS is free
        const TileSlot slot = bounded_tile_slot(a.k_per_tile[t], a.idx_offsets[t], prefix, a.idx_total);
        Segment sg;
        sg.scores = dst;
        sg.out = a.topk_out + hk * a.idx_total + slot.off;
        sg.hist11 = nullptr;
        sg.n = prefix; sg.k_sel = slot.k; sg.forced = 0; sg.pad_to = slot.k;
        select_segment<kPB>(sg, *reinterpret_cast<SelectShared<kPB>*>(smem));
    }
}

// Anchor pass 2 for tiles of exactly 128 rows (the paper's configuration), with the product order of
// prefill_stats_kernel: a workgroup owns two consecutive tiles of one key head (256 rows), a wave 64 rows of
// one of them, so that every K fragment read from LDS feeds two products; and the products of one half block
// (32 keys) are issued between the exponentials of the half block before it.  S = Q K^T is not transposed
// here - a lane owns a key column, the registers are rows - so the tile's column sums are in-lane additions;
// two sets of score registers take turns (products into one while the vector ALU empties the other).
// Column partials of the four waves meet in LDS (three rotating buffers: a block's second half is pooled
// one barrier later than its first) and leave as coalesced stores two barriers after the block's products.
// Both tiles sweep the longer prefix (T more keys than the first tile's); what a tile computes beyond its
// own prefix is not stored.  Pass 3 (per-tile Top-k) follows in the same workgroup, one tile after the other.
template <int D, bool F16>
__global__ __launch_bounds__(kPB, 2) void prefill_pool2_kernel(Shape s, PrefillArgs a) {
    constexpr int KSTEPS = D / 16, TILE = BK * D * 2;
    constexpr int PF = 4;
    constexpr int PARTSZ = kPW * BK;   // floats per buffer of column partials
    // The two tiles, the partials and the selection's state are separate arrays: the compiler then knows that
    // a read from one cannot see a direct load into another, and does not wait for the loads in flight first.
    __shared__ __align__(16) unsigned char smK0[TILE];
    __shared__ __align__(16) unsigned char smK1[TILE];
    __shared__ __align__(16) float smPart[3 * PARTSZ];
    __shared__ SelectShared<kPB> smSel;

    const int hk = blockIdx.x % s.Hkv;
    const int n_pairs = (a.n_tiles + 1) / 2;
    const int tA = 2 * (n_pairs - 1 - blockIdx.x / s.Hkv);      // long ones first
    const int T = a.tile_tokens, S = a.seqlen;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int q = lane & 31, h = lane >> 5;
    const int tw = tA + (w >> 1);                                 // this wave's tile
    const bool tileB = tA + 1 < a.n_tiles;
    const int prefixA = tA * T, prefixB = tileB ? prefixA + T : 0;
    const int sweep = tileB ? prefixB : prefixA;                  // keys 0 .. sweep-1 are swept
    if (sweep == 0) return;
    const float c = s.scale_log2;
    const int n_blocks = (sweep + BK - 1) / BK;

    const unsigned char* Kb = reinterpret_cast<const unsigned char*>(reinterpret_cast<const bf16_t*>(a.k) + hk * s.kv_stride[1]);
    const uint32_t row_bytes = (uint32_t)s.kv_stride[2] * 2u;
    const uint32_t coff = Dma<D>::chunk_off();
    const uint32_t tofs = (uint32_t)(threadIdx.x / Dma<D>::PPR) * row_bytes + coff;
    // stage block kb_: whole blocks by uniform offsets, the ragged last one with clamped rows
#define KASCADE_POOL_STAGE(tile_, kb_)                                                                          \
    if (((kb_) + 1) * BK <= sweep) {                                                                            \
        _Pragma("unroll") for (int i_ = 0; i_ < Dma<D>::PASSES; ++i_) {                                          \
            const unsigned char* src_ = Kb + (size_t)((kb_) * BK + i_ * Dma<D>::RPP) * row_bytes + (size_t)tofs; \
            __builtin_amdgcn_global_load_lds((gmem_ptr_t)src_, (lds_ptr_t)((tile_) + (i_ * kPB + w * kWave) * 16), 16, 0, 0); \
        }                                                                                                       \
    } else {                                                                                                    \
        dma_rows_seq<D>(tile_, Kb, row_bytes, (kb_) * BK, sweep - 1, coff, w);                                  \
    }

    // rows of this wave: 64 (w%2) + q (block A) and + 32 (block B) of tile tw; row rho of a tile is head rho / T,
    // token rho % T
    const RowMap rmA = map_row((w & 1) * 64 + q, tw, T, hk, s.G, S);
    const RowMap rmB = map_row((w & 1) * 64 + 32 + q, tw, T, hk, s.G, S);
    bf16x8_t qa[KSTEPS], qb[KSTEPS];
    {
        const bf16_t* pa = reinterpret_cast<const bf16_t*>(a.q) + (int64_t)rmA.token * s.q_stride[1] + (int64_t)rmA.head * s.q_stride[2];
        const bf16_t* pb = reinterpret_cast<const bf16_t*>(a.q) + (int64_t)rmB.token * s.q_stride[1] + (int64_t)rmB.head * s.q_stride[2];
        const bool live = tw < a.n_tiles;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            uint4 ra = make_uint4(0, 0, 0, 0), rb = make_uint4(0, 0, 0, 0);
            if (live && rmA.ok) ra = *reinterpret_cast<const uint4*>(pa + kk * 16 + h * 8);
            if (live && rmB.ok) rb = *reinterpret_cast<const uint4*>(pb + kk * 16 + h * 8);
            qa[kk] = __builtin_bit_cast(bf16x8_t, ra);
            qb[kk] = __builtin_bit_cast(bf16x8_t, rb);
        }
    }
    // exponent offsets e = m + log2(l * rows of the tile) of the query rows whose scores land in this lane's
    // registers; rows beyond the sequence (and a missing second tile) get weight 0
    float ea[16], eb[16];
    {
        const int tile_end = ((tw + 1) * T < S) ? (tw + 1) * T : S;
        const float rows = (float)((tile_end - tw * T) * s.G);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int rho = (w & 1) * 64 + (r >> 2) * 8 + h * 4 + (r & 3);
            const RowMap ra_ = map_row(rho, tw, T, hk, s.G, S), rb_ = map_row(rho + 32, tw, T, hk, s.G, S);
            ea[r] = INFINITY; eb[r] = INFINITY;
            if (tw < a.n_tiles && ra_.ok) {
                const float* st = a.stats + ((int64_t)ra_.head * S + ra_.token) * 2;
                ea[r] = st[0] + __builtin_amdgcn_logf(st[1] * rows);
            }
            if (tw < a.n_tiles && rb_.ok) {
                const float* st = a.stats + ((int64_t)rb_.head * S + rb_.token) * 2;
                eb[r] = st[0] + __builtin_amdgcn_logf(st[1] * rows);
            }
        }
    }
    // LDS byte offsets of this lane's K fragments: key column q of a half block, k-step kk
    int fo[KSTEPS];
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) fo[kk] = k_off<D>(q, kk * 2 + h);
    constexpr int KEY1 = 32 * D * 2;
    f32x16_t zero;
#pragma unroll
    for (int r = 0; r < 16; ++r) zero[r] = 0.f;
    float* const dstA = a.pooled + hk * a.pooled_pitch + (int64_t)T * tA * (tA - 1) / 2;
    float* const dstB = a.pooled + hk * a.pooled_pitch + (int64_t)T * (tA + 1) * tA / 2;

    // products of one half block: keys KOFF_ .. KOFF_+31 of tile tK_ against both row blocks
#define KASCADE_POOL_MMA(tK_, KOFF_, xa_, xb_)                                               \
    _Pragma("unroll") for (int kk = 0; kk < KSTEPS; ++kk) {                                   \
        const bf16x8_t f_ = lds_frag((tK_) + fo[kk] + (KOFF_));                              \
        xa_ = Mma<F16>::mma32(qa[kk], f_, kk == 0 ? zero : xa_);                             \
        xb_ = Mma<F16>::mma32(qb[kk], f_, kk == 0 ? zero : xb_);                             \
    }
    // pooled weights of one half block, summed over this wave's 64 rows for the lane's key column
#define KASCADE_POOL_SUM(xa_, xb_, out_)                                                     \
    {                                                                                        \
        float c0_ = 0.f, c1_ = 0.f, c2_ = 0.f, c3_ = 0.f;   /* four chains: the additions do not wait for each other */ \
        _Pragma("unroll") for (int r = 0; r < 16; r += 2) {                                   \
            c0_ += __builtin_amdgcn_exp2f(fmaf(xa_[r], c, -ea[r]));                          \
            c1_ += __builtin_amdgcn_exp2f(fmaf(xb_[r], c, -eb[r]));                          \
            c2_ += __builtin_amdgcn_exp2f(fmaf(xa_[r + 1], c, -ea[r + 1]));                  \
            c3_ += __builtin_amdgcn_exp2f(fmaf(xb_[r + 1], c, -eb[r + 1]));                  \
        }                                                                                    \
        out_ = (c0_ + c1_) + (c2_ + c3_);                                                    \
    }
    // one pipeline step: products of a half block into (na_, nb_) between the exponentials of the half block in
    // (ca_, cb_), whose column sums go to pdst_[q]; the order is written out product by product and fenced so
    // that the compiler keeps it (per product two scale-and-shift, two exp2, and the two additions of the
    // product before; per two products one fragment read, PF reads ahead)
#define KASCADE_POOL_PIPE(tK_, KOFF_, na_, nb_, ca_, cb_, pdst_)                             \
    {                                                                                        \
        constexpr int PPS_ = 16 / (2 * KSTEPS);   /* (row block A, row block B) score pairs per product */ \
        __builtin_amdgcn_sched_barrier(0);                                                   \
        bf16x8_t fr_[KSTEPS];                                                                \
        _Pragma("unroll") for (int j_ = 0; j_ < (PF < KSTEPS ? PF : KSTEPS); ++j_) fr_[j_] = lds_frag((tK_) + fo[j_] + (KOFF_)); \
        float pea_[PPS_], peb_[PPS_], c0_ = 0.f, c1_ = 0.f, c2_ = 0.f, c3_ = 0.f;            \
        _Pragma("unroll") for (int i_ = 0; i_ < 2 * KSTEPS; ++i_) {                           \
            const int kk_ = i_ >> 1;                                                         \
            if ((i_ & 1) == 0 && kk_ + PF < KSTEPS) fr_[kk_ + PF] = lds_frag((tK_) + fo[kk_ + PF] + (KOFF_)); \
            if ((i_ & 1) == 0) na_ = Mma<F16>::mma32(qa[kk_], fr_[kk_], kk_ == 0 ? zero : na_); \
            else nb_ = Mma<F16>::mma32(qb[kk_], fr_[kk_], kk_ == 0 ? zero : nb_);            \
            _Pragma("unroll") for (int p_ = 0; p_ < PPS_; ++p_) {                             \
                const int r_ = i_ * PPS_ + p_;                                               \
                const float xa_ = fmaf(ca_[r_], c, -ea[r_]);                                 \
                const float xb_ = fmaf(cb_[r_], c, -eb[r_]);                                 \
                if (i_ > 0) { if (i_ & 1) { c0_ += pea_[p_]; c1_ += peb_[p_]; } else { c2_ += pea_[p_]; c3_ += peb_[p_]; } } \
                pea_[p_] = __builtin_amdgcn_exp2f(xa_);                                      \
                peb_[p_] = __builtin_amdgcn_exp2f(xb_);                                      \
            }                                                                                \
            __builtin_amdgcn_sched_barrier(0);                                               \
        }                                                                                    \
        _Pragma("unroll") for (int p_ = 0; p_ < PPS_; ++p_) { c2_ += pea_[p_]; c3_ += peb_[p_]; } \
        const float cs_ = half_swap_sum((c0_ + c1_) + (c2_ + c3_));                          \
        if (h == 0) (pdst_)[q] = cs_;                                                        \
        asm volatile("" : "+v"(na_), "+v"(nb_));                                             \
        __builtin_amdgcn_sched_barrier(0);                                                   \
    }
    // the tile's column sums of block kb_: threads 0-63 the first tile, 64-127 the second
#define KASCADE_POOL_STORE(kb_)                                                              \
    if (threadIdx.x < 2 * BK) {                                                              \
        const int tl_ = threadIdx.x >> 6, j_ = (kb_) * BK + (threadIdx.x & 63);              \
        if (j_ < (tl_ ? prefixB : prefixA)) {                                                \
            const float* pp_ = smPart + ((kb_) % 3) * PARTSZ + 2 * tl_ * BK + (threadIdx.x & 63); \
            (tl_ ? dstB : dstA)[j_] = pp_[0] + pp_[BK];                                      \
        }                                                                                    \
    }

    // step s = 2 kb + half: products of step s run beside the sums of step s-1.  xs = (xa, xb) holds first
    // halves, ys second halves.
    f32x16_t xa, xb, ya, yb;
    KASCADE_POOL_STAGE(smK0, 0)
    wait_vmem();
    __syncthreads();
    if (1 < n_blocks) { KASCADE_POOL_STAGE(smK1, 1) }
    KASCADE_POOL_MMA(smK0, 0, xa, xb)                                  // step 0, nothing to sum yet
    KASCADE_POOL_PIPE(smK0, KEY1, ya, yb, xa, xb, smPart + w * BK)     // step 1: sums of block 0, first half
    int kb = 1;
    for (; kb + 1 < n_blocks; kb += 2) {
        // block kb (tile 1), then block kb+1 (tile 0)
        wait_vmem();
        __syncthreads();
        KASCADE_POOL_STAGE(smK0, kb + 1)
        if (kb >= 2) KASCADE_POOL_STORE(kb - 2)
        KASCADE_POOL_PIPE(smK1, 0, xa, xb, ya, yb, smPart + ((kb - 1) % 3) * PARTSZ + w * BK + 32)
        KASCADE_POOL_PIPE(smK1, KEY1, ya, yb, xa, xb, smPart + (kb % 3) * PARTSZ + w * BK)
        wait_vmem();
        __syncthreads();
        if (kb + 2 < n_blocks) { KASCADE_POOL_STAGE(smK1, kb + 2) }
        KASCADE_POOL_STORE(kb - 1)
        KASCADE_POOL_PIPE(smK0, 0, xa, xb, ya, yb, smPart + (kb % 3) * PARTSZ + w * BK + 32)
        KASCADE_POOL_PIPE(smK0, KEY1, ya, yb, xa, xb, smPart + ((kb + 1) % 3) * PARTSZ + w * BK)
    }
    if (kb < n_blocks) {     // one block left (tile 1)
        wait_vmem();
        __syncthreads();
        if (kb >= 2) KASCADE_POOL_STORE(kb - 2)
        KASCADE_POOL_PIPE(smK1, 0, xa, xb, ya, yb, smPart + ((kb - 1) % 3) * PARTSZ + w * BK + 32)
        KASCADE_POOL_PIPE(smK1, KEY1, ya, yb, xa, xb, smPart + (kb % 3) * PARTSZ + w * BK)
        ++kb;
    }
    // kb == n_blocks: the second half of the last block is still in (ya, yb)
    {
        float cs;
        KASCADE_POOL_SUM(ya, yb, cs)
        cs = half_swap_sum(cs);
        if (h == 0) smPart[((n_blocks - 1) % 3) * PARTSZ + w * BK + 32 + q] = cs;
    }
    __syncthreads();
    if (n_blocks >= 2) KASCADE_POOL_STORE(n_blocks - 2)
    KASCADE_POOL_STORE(n_blocks - 1)
#undef KASCADE_POOL_STORE
#undef KASCADE_POOL_PIPE
#undef KASCADE_POOL_SUM
#undef KASCADE_POOL_MMA
#undef KASCADE_POOL_STAGE

    // anchor pass 3: both tiles' pooled scores were written by this workgroup, so it selects right away, one
    // tile after the other, while the other workgroup of the compute unit keeps the matrix pipe busy
    if (a.topk_out) {
        SelectShared<kPB>& sel = smSel;
#pragma unroll 1
        for (int i = 0; i < 2; ++i) {
            const int t = tA + i, prefix = i ? prefixB : prefixA;
            if (prefix == 0) continue;
            __syncthreads();   // the pooled scores are visible to the whole workgroup; LDS is free
            const TileSlot slot = bounded_tile_slot(a.k_per_tile[t], a.idx_offsets[t], prefix, a.idx_total);
            Segment sg;
            sg.scores = i ? dstB : dstA;
            sg.out = a.topk_out + hk * a.idx_total + slot.off;
            sg.hist11 = nullptr;
            sg.n = prefix; sg.k_sel = slot.k; sg.forced = 0; sg.pad_to = slot.k;
            select_segment<kPB>(sg, sel);
        }
    }
}

}  // namespace

hipError_t launch_prefill_attend(const Shape& s, const PrefillArgs& a, bool sparse, bool with_v, hipStream_t st) {
    dim3 grid(a.n_sub * s.Hkv), block(kPB);   // one workgroup per 128 rows
    if (s.dtype != 1 && s.dtype != 2) return hipErrorInvalidValue;
    const bool f16 = s.dtype == 2;
#define KASCADE_LAUNCH_STATS(DD, FF)                                                                                   \
    {                                                                                                                  \
        const dim3 grid2(((a.n_sub + 1) / 2) * s.Hkv);   /* one workgroup per 256 rows */                              \
        KASCADE_LAUNCH((prefill_stats_kernel<DD, FF>), grid2, block, 0, st, s, a);                                     \
    }
#define KASCADE_LAUNCH_ATTEND(DD, FF)                                                                                  \
    {                                                                                                                  \
        if (sparse) KASCADE_LAUNCH((prefill_attend_kernel<DD, true, FF>), grid, block, 0, st, s, a);         \
        else if (with_v) KASCADE_LAUNCH((prefill_attend_kernel<DD, false, FF>), grid, block, 0, st, s, a);   \
        else KASCADE_LAUNCH_STATS(DD, FF)                                                                              \
    }
    if (s.D == 128 && !f16) KASCADE_LAUNCH_ATTEND(128, false)
    else if (s.D == 128) KASCADE_LAUNCH_ATTEND(128, true)
    else if (s.D == 64 && !f16) KASCADE_LAUNCH_ATTEND(64, false)
    else if (s.D == 64) KASCADE_LAUNCH_ATTEND(64, true)
    else return hipErrorInvalidValue;
#undef KASCADE_LAUNCH_ATTEND
    return hipGetLastError();
}

hipError_t launch_prefill_pool(const Shape& s, const PrefillArgs& a, hipStream_t st) {
    dim3 grid(a.n_tiles * s.Hkv), block(kPB);
    if (s.dtype != 1 && s.dtype != 2) return hipErrorInvalidValue;
    const bool multi = a.tile_tokens != a.sub_tokens, f16 = s.dtype == 2;
#define KASCADE_LAUNCH_POOL(DD, FF)                                                                              \
    {                                                                                                            \
        if (multi) KASCADE_LAUNCH((prefill_pool_kernel<DD, FF>), grid, block, 0, st, s, a);            \
        else KASCADE_LAUNCH((prefill_pool2_kernel<DD, FF>), dim3(((a.n_tiles + 1) / 2) * s.Hkv), block, 0, st, s, a); \
    }
    if (s.D == 128 && !f16) KASCADE_LAUNCH_POOL(128, false)
    else if (s.D == 128) KASCADE_LAUNCH_POOL(128, true)
    else if (s.D == 64 && !f16) KASCADE_LAUNCH_POOL(64, false)
    else if (s.D == 64) KASCADE_LAUNCH_POOL(64, true)
    else return hipErrorInvalidValue;
#undef KASCADE_LAUNCH_POOL
    return hipGetLastError();
}

}  // namespace kascade
