// Host-side exerciser of the C ABI for sanitizer builds (address + undefined behaviour, host code only).
// It calls what runs on the host before any launch: argument validation, launch planning and workspace
// sizing over many shapes, status strings, and the anchor-layer selection of Algorithm 1 (checked here
// against exhaustive search over all anchor subsets).  No GPU is needed and no kernel is launched: every
// call either is pure host code or returns from validation.  Exit code 0 = all checks passed.
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <vector>

#include "../include/kascade.h"

static int failures = 0;
#define EXPECT(cond)                                                              \
    do {                                                                          \
        if (!(cond)) { ++failures; fprintf(stderr, "line %d: %s\n", __LINE__, #cond); } \
    } while (0)

static kascade_desc make_desc(int B, int Hq, int Hkv, int d, int dtype, int64_t L) {
    kascade_desc x = {};
    x.batch = B; x.n_q_heads = Hq; x.n_kv_heads = Hkv; x.head_dim = d; x.dtype = dtype; x.softmax_scale = 0.f;
    x.q_stride[0] = (int64_t)Hq * d; x.q_stride[1] = (int64_t)Hq * d; x.q_stride[2] = d;
    x.kv_stride[0] = (int64_t)Hkv * L * d; x.kv_stride[1] = L * d; x.kv_stride[2] = d;
    x.o_stride[0] = (int64_t)Hq * d; x.o_stride[1] = (int64_t)Hq * d; x.o_stride[2] = d;
    return x;
}

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double uniform() {
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 9007199254740992.0;
}

// best total similarity over all anchor sets of size M that contain layer 0 (layer j is served by the
// nearest anchor at or before it), by enumeration
static double exhaustive(const std::vector<float>& S, const std::vector<float>* w, int L, int M, std::vector<int>* best_set) {
    double best = -1e300;
    for (uint32_t mask = 1; mask < (1u << L); mask += 2) {
        if (__builtin_popcount(mask) != M) continue;
        double tot = 0.0;
        int anchor = 0;
        for (int j = 0; j < L; ++j) {
            if (mask >> j & 1u) anchor = j;
            tot += (double)S[anchor * L + j] * (w ? (double)(*w)[j] : 1.0);
        }
        if (tot > best + 1e-12) {
            best = tot;
            best_set->clear();
            for (int j = 0; j < L; ++j) if (mask >> j & 1u) best_set->push_back(j);
        }
    }
    return best;
}

int main() {
    char* fake = reinterpret_cast<char*>(0x10000);   // never dereferenced: every call below returns from validation
    // ---- status strings
    for (int st = -8; st <= 1; ++st) EXPECT(kascade_status_string(st) != nullptr);
    EXPECT(kascade_version() != nullptr);

    // ---- workspace sizing and launch planning over many shapes (no pointers involved)
    const int groups[] = {1, 2, 4, 8};
    for (int dtype = 0; dtype < 2; ++dtype)
        for (int d : {64, 128})
            for (int G : groups)
                for (int Hkv : {1, 2, 8})
                    for (int B : {1, 3, 64, 1000})
                        for (int64_t L : {1ll, 63ll, 4096ll, 131072ll, 1048576ll}) {
                            kascade_desc x = make_desc(B, Hkv * G, Hkv, d, dtype, L);
                            const int64_t k = L / 10 + 1;
                            const size_t wa = kascade_workspace_bytes(KASCADE_OP_DECODE_ANCHOR, &x, L, k, 0);
                            const size_t wr = kascade_workspace_bytes(KASCADE_OP_DECODE_REUSE, &x, L, k, 0);
                            const size_t wp = kascade_workspace_bytes(KASCADE_OP_DECODE_POOLED, &x, L, 0, 0);
                            EXPECT(wa >= wr && wa > 0 && wp > 0 && wa % 256 == 0);
                            EXPECT(wa >= (size_t)B * Hkv * G * L * 4);          // the fp32 logits alone
                            if (B == 1) {
                                const int T = 128 / G;
                                const size_t w1 = kascade_workspace_bytes(KASCADE_OP_PREFILL_ANCHOR, &x, L, 0, T);
                                const size_t w4 = kascade_workspace_bytes(KASCADE_OP_PREFILL_ANCHOR, &x, L, 0, 4 * T);
                                EXPECT(w1 > 0 && w4 > 0 && w4 <= w1);
                                EXPECT(kascade_workspace_bytes(KASCADE_OP_PREFILL_REUSE, &x, L, 0, T) == 0);
                                if (L <= 131072)
                                    EXPECT(kascade_workspace_bytes(KASCADE_OP_PREFILL_ANCHOR_PRESOFTMAX, &x, L, 0, T) > 0);
                            }
                        }
    EXPECT(kascade_workspace_bytes(99, nullptr, 1, 1, 1) == 0);
    // an empty budget is a valid size query (k = 0): no division by a zero chunk, a finite answer
    for (int dtype = 0; dtype < 3; ++dtype)
        for (int d : {64, 128})
            for (int B : {1, 8, 64, 1000})
                for (int forced_chunk : {0, 1, 300}) {
                    EXPECT(kascade_tuning_set(KASCADE_TUNE_GATHER_CHUNK, forced_chunk) == KASCADE_OK);
                    kascade_desc x = make_desc(B, 32, 8, d, dtype, 4096);
                    const size_t wr0 = kascade_workspace_bytes(KASCADE_OP_DECODE_REUSE, &x, 4096, 0, 0);
                    const size_t wr1 = kascade_workspace_bytes(KASCADE_OP_DECODE_REUSE, &x, 4096, 1, 0);
                    const size_t wa0 = kascade_workspace_bytes(KASCADE_OP_DECODE_ANCHOR, &x, 4096, 0, 0);
                    const size_t wa1 = kascade_workspace_bytes(KASCADE_OP_DECODE_ANCHOR, &x, 4096, 1, 0);
                    EXPECT(wr0 == wr1 && wa0 == wa1 && wa0 > wr0);
                }
    EXPECT(kascade_tuning_set(KASCADE_TUNE_GATHER_CHUNK, 0) == KASCADE_OK);
    // ---- launch-plan overrides: validation, and the size query follows them
    EXPECT(kascade_tuning_set(-1, 1) == KASCADE_INVALID_ARG);
    EXPECT(kascade_tuning_set(KASCADE_TUNE_COUNT, 1) == KASCADE_INVALID_ARG);
    EXPECT(kascade_tuning_set(KASCADE_TUNE_TOPK_PARTS, -3) == KASCADE_INVALID_ARG);
    EXPECT(kascade_tuning_set(KASCADE_TUNE_DECODE_FAMILY, 3) == KASCADE_INVALID_ARG);
    EXPECT(kascade_tuning_get(KASCADE_TUNE_COUNT) == KASCADE_INVALID_ARG);
    {
        kascade_desc x = make_desc(8, 32, 8, 128, KASCADE_BF16, 32768);
        const size_t w_auto = kascade_workspace_bytes(KASCADE_OP_DECODE_REUSE, &x, 32768, 3277, 0);
        EXPECT(kascade_tuning_set(KASCADE_TUNE_GATHER_CHUNK, 64) == KASCADE_OK);
        EXPECT(kascade_tuning_get(KASCADE_TUNE_GATHER_CHUNK) == 64);
        const size_t w_small = kascade_workspace_bytes(KASCADE_OP_DECODE_REUSE, &x, 32768, 3277, 0);
        EXPECT(w_small > w_auto);                      // more chunks, more partial results
        // a workspace sized before the override is refused, not overrun
        EXPECT(kascade_decode_reuse(&x, fake, fake, fake, (int32_t*)fake, (int32_t*)fake, 3277, (int32_t*)fake, 8, nullptr,
                                    fake, fake, w_auto, nullptr) == KASCADE_WORKSPACE_TOO_SMALL);
        for (int knob = 0; knob < KASCADE_TUNE_COUNT; ++knob) {
            EXPECT(kascade_tuning_set(knob, 0) == KASCADE_OK);
            EXPECT(kascade_tuning_get(knob) == 0);
        }
    }

    // ---- argument validation (decode)
    kascade_desc good = make_desc(2, 8, 2, 128, KASCADE_BF16, 4096);
    EXPECT(kascade_decode_reuse(nullptr, fake, fake, fake, (int32_t*)fake, (int32_t*)fake, 8, (int32_t*)fake, 2, nullptr,
                                fake, fake, 1 << 20, nullptr) == KASCADE_INVALID_ARG);
    EXPECT(kascade_decode_reuse(&good, nullptr, fake, fake, (int32_t*)fake, (int32_t*)fake, 8, (int32_t*)fake, 2, nullptr,
                                fake, fake, 1 << 20, nullptr) == KASCADE_INVALID_ARG);
    EXPECT(kascade_decode_reuse(&good, fake + 2, fake, fake, (int32_t*)fake, (int32_t*)fake, 8, (int32_t*)fake, 2, nullptr,
                                fake, fake, 1 << 20, nullptr) == KASCADE_MISALIGNED);
    EXPECT(kascade_decode_reuse(&good, fake, fake, fake, (int32_t*)fake, (int32_t*)fake, 0, (int32_t*)fake, 2, nullptr,
                                fake, fake, 1 << 20, nullptr) == KASCADE_INVALID_ARG);
    EXPECT(kascade_decode_reuse(&good, fake, fake, fake, (int32_t*)fake, (int32_t*)fake, 8, (int32_t*)fake, 1, nullptr,
                                fake, fake, 1 << 20, nullptr) == KASCADE_INVALID_ARG);     // 1 anchor head without a map
    EXPECT(kascade_decode_reuse(&good, fake, fake, fake, (int32_t*)fake, (int32_t*)fake, 5000, (int32_t*)fake, 2, nullptr,
                                fake, fake, 16, nullptr) == KASCADE_WORKSPACE_TOO_SMALL);
    for (int variant = 0; variant < 3; ++variant) {
        auto call = variant == 0 ? kascade_decode_anchor : variant == 1 ? kascade_decode_anchor_shared : kascade_decode_anchor_presoftmax;
        EXPECT(call(&good, fake, fake, fake, (int32_t*)fake, (int32_t*)fake, 4096, 5000, 0, 1, (int32_t*)fake, fake, fake,
                    (size_t)1 << 40, nullptr) == KASCADE_INVALID_ARG);                      // k_max > max_seqlen
        EXPECT(call(&good, fake, fake, fake, (int32_t*)fake, (int32_t*)fake, 4096, 400, 401, 1, (int32_t*)fake, fake, fake,
                    (size_t)1 << 40, nullptr) == KASCADE_INVALID_ARG);                      // window > k
        EXPECT(call(&good, fake, fake, fake, (int32_t*)fake, (int32_t*)fake, 4096, 400, 0, 7, (int32_t*)fake, fake, fake,
                    (size_t)1 << 40, nullptr) == KASCADE_INVALID_ARG);                      // out_mode
        EXPECT(call(&good, fake, fake, fake, (int32_t*)fake, (int32_t*)fake, 4096, 400, 0, 1, (int32_t*)fake, fake, fake,
                    1024, nullptr) == KASCADE_WORKSPACE_TOO_SMALL);
    }
    kascade_desc bad = good;
    bad.n_q_heads = 6; bad.dtype = KASCADE_F32;           // G = 3 exists for bf16 only
    EXPECT(kascade_workspace_bytes(KASCADE_OP_DECODE_ANCHOR, &bad, 100, 10, 0) == 0);
    bad = good; bad.n_q_heads = 6;
    EXPECT(kascade_workspace_bytes(KASCADE_OP_DECODE_ANCHOR, &bad, 100, 10, 0) > 0);
    EXPECT(kascade_workspace_bytes(KASCADE_OP_PREFILL_ANCHOR, &bad, 4096, 1000, 128) == 0);   // and for decode only
    EXPECT(kascade_workspace_bytes(KASCADE_OP_PREFILL_ANCHOR_PRESOFTMAX, &bad, 4096, 1000, 128) == 0);
    bad = good; bad.n_q_heads = 34; bad.n_kv_heads = 2;   // G = 17
    EXPECT(kascade_decode_anchor(&bad, fake, fake, fake, (int32_t*)fake, (int32_t*)fake, 4096, 400, 0, 1, (int32_t*)fake, fake,
                                 fake, (size_t)1 << 40, nullptr) == KASCADE_UNSUPPORTED);
    bad = good; bad.batch = 70000;
    EXPECT(kascade_decode_anchor(&bad, fake, fake, fake, (int32_t*)fake, (int32_t*)fake, 4096, 400, 0, 1, (int32_t*)fake, fake,
                                 fake, (size_t)1 << 40, nullptr) == KASCADE_UNSUPPORTED);
    bad = good; bad.head_dim = 96;
    EXPECT(kascade_decode_anchor(&bad, fake, fake, fake, (int32_t*)fake, (int32_t*)fake, 4096, 400, 0, 1, (int32_t*)fake, fake,
                                 fake, (size_t)1 << 40, nullptr) == KASCADE_UNSUPPORTED);
    bad = good; bad.softmax_scale = NAN;
    EXPECT(kascade_decode_anchor(&bad, fake, fake, fake, (int32_t*)fake, (int32_t*)fake, 4096, 400, 0, 1, (int32_t*)fake, fake,
                                 fake, (size_t)1 << 40, nullptr) == KASCADE_INVALID_ARG);

    // ---- argument validation (prefill)
    kascade_desc pf = make_desc(1, 32, 8, 128, KASCADE_BF16, 4096);
    for (int variant = 0; variant < 3; ++variant) {
        auto call = variant == 0 ? kascade_prefill_anchor : variant == 1 ? kascade_prefill_anchor_shared : kascade_prefill_anchor_presoftmax;
        EXPECT(call(&pf, fake, fake, fake, 4096, 16, (int32_t*)fake, (int64_t*)fake, 10, 1, (int32_t*)fake, fake, fake,
                    (size_t)1 << 40, nullptr) == KASCADE_UNSUPPORTED);                      // 64 rows per tile
        EXPECT(call(&pf, fake, fake, fake, 0, 32, (int32_t*)fake, (int64_t*)fake, 10, 1, (int32_t*)fake, fake, fake,
                    (size_t)1 << 40, nullptr) == KASCADE_INVALID_ARG);
        EXPECT(call(&pf, fake, fake, fake, 4096, 32, (int32_t*)fake, (int64_t*)fake, 10, 1, (int32_t*)fake, fake, fake,
                    64, nullptr) == KASCADE_WORKSPACE_TOO_SMALL);
        EXPECT(call(&pf, fake, fake, fake, 4096, 128, (int32_t*)fake, (int64_t*)fake, 10, 3, (int32_t*)fake, fake, fake,
                    (size_t)1 << 40, nullptr) == KASCADE_INVALID_ARG);                      // out_mode
    }
    kascade_desc pf32 = pf; pf32.dtype = KASCADE_F32;
    EXPECT(kascade_prefill_reuse(&pf32, fake, fake, fake, 4096, 32, (int32_t*)fake, (int64_t*)fake, 10, (int32_t*)fake, 8,
                                 nullptr, fake, nullptr, 0, nullptr) == KASCADE_UNSUPPORTED);

    // ---- Algorithm 1 on the host against exhaustive search
    for (int trial = 0; trial < 60; ++trial) {
        const int L = 2 + (int)(uniform() * 13);            // 2..14 layers
        const int M = 1 + (int)(uniform() * L);
        std::vector<float> S((size_t)L * L), w(L);
        for (auto& v : S) v = (float)uniform();
        for (auto& v : w) v = (float)(0.1 + uniform());
        const bool weighted = trial % 2;
        std::vector<int32_t> anchors(M);
        double objective = 0.0;
        EXPECT(kascade_select_anchor_layers(S.data(), weighted ? w.data() : nullptr, L, M, anchors.data(), &objective) == KASCADE_OK);
        std::vector<int> best_set;
        const double best = exhaustive(S, weighted ? &w : nullptr, L, M, &best_set);
        EXPECT(fabs(best - objective) <= 1e-9 * (1.0 + fabs(best)));
        EXPECT(anchors[0] == 0);
        for (int i = 1; i < M; ++i) EXPECT(anchors[i] > anchors[i - 1] && anchors[i] < L);
    }
    int32_t one;
    double obj;
    float s1 = 0.5f;
    EXPECT(kascade_select_anchor_layers(&s1, nullptr, 1, 1, &one, &obj) == KASCADE_OK && one == 0);
    EXPECT(kascade_select_anchor_layers(&s1, nullptr, 1, 2, &one, &obj) == KASCADE_INVALID_ARG);
    EXPECT(kascade_select_anchor_layers(nullptr, nullptr, 4, 2, &one, &obj) == KASCADE_INVALID_ARG);

    if (failures) { fprintf(stderr, "%d host check(s) failed\n", failures); return 1; }
    printf("host checks passed\n");
    return 0;
}
