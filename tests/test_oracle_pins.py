"""Pins of the CPU oracle against things it did not produce itself: a library
attention routine (torch SDPA in fp64), brute-force subset enumeration, closed
forms, invariants the method must satisfy, and numbers the paper prints."""
import itertools
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import kascade_oracle as ko

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def sdpa_decode(q, K, V, scale):
    """library attention: q [Hq,d], K/V [Hkv,L,d] -> [Hq,d] (fp64, GQA by repetition)."""
    Hq = q.shape[0]
    G = Hq // K.shape[0]
    tq = torch.from_numpy(q)[None, :, None, :]                       # [1,Hq,1,d]
    tk = torch.from_numpy(K).repeat_interleave(G, dim=0)[None]       # [1,Hq,L,d]
    tv = torch.from_numpy(V).repeat_interleave(G, dim=0)[None]
    return F.scaled_dot_product_attention(tq, tk, tv, scale=scale)[0, :, 0, :].numpy()


# ------------------------------------------------------------------ Eq. 1-2

@pytest.mark.parametrize("Hq,Hkv,d,L", [(8, 2, 64, 300), (4, 4, 16, 33), (6, 1, 32, 1), (32, 8, 128, 257)])
def test_dense_decode_matches_library_attention(Hq, Hkv, d, L):
    r = rng(L)
    q, K, V = r.standard_normal((Hq, d)), r.standard_normal((Hkv, L, d)), r.standard_normal((Hkv, L, d))
    scale = ko.default_scale(d)
    np.testing.assert_allclose(ko.dense_decode(q, K, V, scale), sdpa_decode(q, K, V, scale), atol=1e-12)
    # a non-default scale must be honoured too
    np.testing.assert_allclose(ko.dense_decode(q, K, V, 0.37), sdpa_decode(q, K, V, 0.37), atol=1e-12)


def test_probabilities_match_library_via_identity_values():
    # with V = identity (d_v = L) library attention returns p itself
    r = rng(5)
    Hq, Hkv, d, L = 6, 3, 16, 40
    q, K = r.standard_normal((Hq, d)), r.standard_normal((Hkv, L, d))
    G = Hq // Hkv
    tq = torch.from_numpy(q)[None, :, None, :]
    tk = torch.from_numpy(K).repeat_interleave(G, dim=0)[None]
    tv = torch.eye(L, dtype=torch.float64).expand(1, Hq, L, L)
    p_lib = F.scaled_dot_product_attention(tq, tk, tv, scale=0.25)[0, :, 0, :].numpy()
    p = ko.decode_probabilities(q, K, 0.25)
    np.testing.assert_allclose(p, p_lib, atol=1e-13)
    np.testing.assert_allclose(p.sum(axis=1), 1.0, atol=1e-12)
    assert (p >= 0).all()


def test_softmax_closed_forms():
    # equal logits -> uniform; two logits -> logistic
    np.testing.assert_allclose(ko.softmax_lastdim(np.full((3, 7), 2.5)), 1.0 / 7, atol=1e-15)
    x = 1.3
    p = ko.softmax_lastdim(np.array([x, 0.0]))
    np.testing.assert_allclose(p[0], 1.0 / (1.0 + np.exp(-x)), atol=1e-15)
    # shift invariance and no overflow for large logits
    np.testing.assert_allclose(ko.softmax_lastdim(np.array([1000.0, 999.0])),
                               ko.softmax_lastdim(np.array([1.0, 0.0])), atol=1e-15)


def test_default_scale():
    assert ko.default_scale(64) == 0.125
    np.testing.assert_allclose(ko.default_scale(128), 128 ** -0.5)


# ------------------------------------------------------------------ pooling

def test_pool_gqa_mean_and_group_assignment():
    r = rng(7)
    Hq, Hkv, L = 8, 2, 50
    p = ko.softmax_lastdim(r.standard_normal((Hq, L)))
    a = ko.pool_gqa(p, Hkv)
    np.testing.assert_allclose(a.sum(axis=1), 1.0, atol=1e-12)
    # heads 0..3 feed key head 0, heads 4..7 feed key head 1 (consecutive grouping)
    np.testing.assert_allclose(a[0], (p[0] + p[1] + p[2] + p[3]) / 4, atol=1e-15)
    np.testing.assert_allclose(a[1], (p[4] + p[5] + p[6] + p[7]) / 4, atol=1e-15)
    # G = 1: pooling is the identity
    np.testing.assert_allclose(ko.pool_gqa(p, Hq), p, atol=0)


# ------------------------------------------------------------------ Top-k

def brute_force_topk(a, k, W):
    """Enumerate every admissible k-subset; best = largest total score, then
    the lexicographically smallest index tuple (= lower index wins ties)."""
    L = len(a)
    forced = tuple(range(L - W, L))
    best, best_key = None, None
    for sub in itertools.combinations(range(L - W), k - W):
        cand = tuple(sorted(sub + forced))
        key = (-sum(a[j] for j in sub), cand)
        if best_key is None or key < best_key:
            best, best_key = cand, key
    return np.array(best, dtype=np.int64)


@pytest.mark.parametrize("seed", range(6))
def test_topk_brute_force_with_exact_ties(seed):
    r = rng(100 + seed)
    L = 9
    # few distinct dyadic values -> many exact ties, exact sums
    a = r.integers(0, 4, size=L).astype(np.float64) / 8.0
    for W in (0, 1, 3):
        for k in range(W, L + 1):
            got = ko.select_topk(a, k, W)
            np.testing.assert_array_equal(got, brute_force_topk(a, k, W))


def test_topk_matches_library_topk_without_ties():
    r = rng(11)
    a = r.random(5000)
    for k in (1, 17, 500, 4999, 5000):
        lib = torch.topk(torch.from_numpy(a), k).indices.sort().values.numpy()
        np.testing.assert_array_equal(ko.select_topk(a, k), lib)


def test_topk_invariants_and_window():
    r = rng(12)
    L, k, W = 1000, 100, 16
    a = np.round(r.random(L), 2)          # two-decimal scores: many ties
    I = ko.select_topk(a, k, W)
    assert I.shape == (k,) and I.dtype == np.int64
    assert (np.diff(I) > 0).all() and I[0] >= 0 and I[-1] < L
    assert set(range(L - W, L)) <= set(I.tolist())
    cand_in = [j for j in I if j < L - W]
    cand_out = [j for j in range(L - W) if j not in set(cand_in)]
    thr = min(a[cand_in])
    assert max(a[cand_out]) <= thr                       # maximality
    # among scores equal to the threshold the chosen ones are the lowest indices
    eq_in = [j for j in cand_in if a[j] == thr]
    eq_out = [j for j in cand_out if a[j] == thr]
    if eq_in and eq_out:
        assert max(eq_in) < min(eq_out)
    with pytest.raises(ValueError):
        ko.select_topk(a, L + 1)
    with pytest.raises(ValueError):
        ko.select_topk(a, 3, 4)
    assert ko.select_topk(a, 0).size == 0


def test_anchor_indices_single_head_equal_topk_of_raw_logits():
    # G = 1: softmax is monotone, so the Top-k of p is the Top-k of q.K
    r = rng(13)
    Hkv, d, L, k = 3, 32, 400, 40
    q, K = r.standard_normal((Hkv, d)), r.standard_normal((Hkv, L, d))
    idx, a = ko.decode_anchor_indices(q, K, ko.default_scale(d), k)
    for hk in range(Hkv):
        raw = torch.topk(torch.from_numpy(K[hk] @ q[hk]), k).indices.sort().values.numpy()
        np.testing.assert_array_equal(idx[hk], raw)
    np.testing.assert_allclose(a.sum(axis=1), 1.0, atol=1e-12)


def test_anchor_indices_find_planted_keys():
    # one key per key head is made overwhelmingly dominant for every head of the group
    r = rng(14)
    Hq, Hkv, d, L = 8, 2, 16, 64
    q, K = r.standard_normal((Hq, d)), 0.01 * r.standard_normal((Hkv, L, d))
    plant = [5, 41]
    for hk in range(Hkv):
        K[hk, plant[hk]] = 50.0 * q[hk * 4:(hk + 1) * 4].mean(axis=0)
    idx, _ = ko.decode_anchor_indices(q, K, 1.0, 1)
    assert idx[:, 0].tolist() == plant


# ------------------------------------------------------------------ sparse attention

def test_sparse_decode_special_cases():
    r = rng(21)
    Hq, Hkv, d, L = 8, 2, 32, 120
    q, K, V = r.standard_normal((Hq, d)), r.standard_normal((Hkv, L, d)), r.standard_normal((Hkv, L, d))
    scale = ko.default_scale(d)
    full = [np.arange(L)] * Hkv
    # k = L  =>  dense
    np.testing.assert_allclose(ko.sparse_decode(q, K, V, full, scale), ko.dense_decode(q, K, V, scale), atol=1e-13)
    # k = 1  =>  the selected value row
    one = [np.array([7]), np.array([99])]
    y1 = ko.sparse_decode(q, K, V, one, scale)
    for h in range(Hq):
        np.testing.assert_allclose(y1[h], V[h // 4, one[h // 4][0]], atol=1e-15)
    # arbitrary sets = library attention on the gathered sub-cache (per key head)
    sets = [np.sort(r.choice(L, 30, replace=False)) for _ in range(Hkv)]
    y = ko.sparse_decode(q, K, V, sets, scale)
    for hk in range(Hkv):
        ref = sdpa_decode(q[hk * 4:(hk + 1) * 4], K[hk:hk + 1, sets[hk]], V[hk:hk + 1, sets[hk]], scale)
        np.testing.assert_allclose(y[hk * 4:(hk + 1) * 4], ref, atol=1e-12)
    # order of the indices does not matter
    shuffled = [r.permutation(s) for s in sets]
    np.testing.assert_allclose(ko.sparse_decode(q, K, V, shuffled, scale), y, atol=1e-13)
    # permuting key positions together with the indices leaves the output unchanged
    perm = r.permutation(L)
    inv = np.argsort(perm)
    np.testing.assert_allclose(ko.sparse_decode(q, K[:, perm], V[:, perm], [inv[s] for s in sets], scale), y, atol=1e-13)


def test_head_map():
    r = rng(22)
    Hq, Hkv, d, L = 6, 3, 16, 50
    q, K, V = r.standard_normal((Hq, d)), r.standard_normal((Hkv, L, d)), r.standard_normal((Hkv, L, d))
    sets = [np.sort(r.choice(L, 10, replace=False)) for _ in range(Hkv)]
    y_id = ko.sparse_decode(q, K, V, sets, 0.3)
    np.testing.assert_allclose(ko.sparse_decode(q, K, V, sets, 0.3, head_map=[0, 1, 2]), y_id, atol=0)
    hm = [2, 0, 0]                                # many-to-one
    y_map = ko.sparse_decode(q, K, V, sets, 0.3, head_map=hm)
    y_ref = ko.sparse_decode(q, K, V, [sets[hm[0]], sets[hm[1]], sets[hm[2]]], 0.3)
    np.testing.assert_allclose(y_map, y_ref, atol=0)
    assert np.abs(y_map - y_id).max() > 1e-3


# ------------------------------------------------------------------ prefill

def sdpa_prefill(Q, Kp, Vp, scale, mask=None):
    """library attention over a whole prompt: returns [S, Hq, d]."""
    Hq = Q.shape[1]
    G = Hq // Kp.shape[0]
    tq = torch.from_numpy(Q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(Kp).repeat_interleave(G, dim=0)[None]
    tv = torch.from_numpy(Vp).repeat_interleave(G, dim=0)[None]
    if mask is None:
        o = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    else:
        o = F.scaled_dot_product_attention(tq, tk, tv, attn_mask=torch.from_numpy(mask)[None], scale=scale)
    return o[0].permute(1, 0, 2).numpy()


def make_prefill(seed, S, Hq, Hkv, d):
    r = rng(seed)
    return r.standard_normal((S, Hq, d)), r.standard_normal((Hkv, S, d)), r.standard_normal((Hkv, S, d))


@pytest.mark.parametrize("S,T", [(40, 8), (37, 8), (16, 1)])
def test_prefill_dense_tiles_match_library_causal_attention(S, T):
    Q, Kp, Vp = make_prefill(31, S, 4, 2, 16)
    ref = sdpa_prefill(Q, Kp, Vp, 0.25)
    for t in range((S + T - 1) // T):
        lo, hi = ko.tile_bounds(t, T, S)
        np.testing.assert_allclose(ko.prefill_dense_tile(Q, Kp, Vp, t, T, 0.25), ref[lo:hi], atol=1e-12)


def test_prefill_pooled_is_mean_of_per_row_library_probabilities():
    S, T, Hq, Hkv, d = 24, 4, 4, 2, 8
    G = Hq // Hkv
    Q, Kp, _ = make_prefill(32, S, Hq, Hkv, d)
    # causal library attention with V = identity returns the causal P matrix
    eye = np.broadcast_to(np.eye(S), (Hkv, S, S)).copy()
    P_lib = sdpa_prefill(Q, Kp, eye, 0.4)                      # [S, Hq, S]
    for t in range(S // T):
        a = ko.prefill_pooled_tile(Q, Kp, t, T, 0.4)
        assert a.shape == (Hkv, t * T)
        for hk in range(Hkv):
            rows = P_lib[t * T:(t + 1) * T, hk * G:(hk + 1) * G, : t * T]
            np.testing.assert_allclose(a[hk], rows.mean(axis=(0, 1)), atol=1e-13)
            # prefix mass + mean diagonal mass = 1
            diag = P_lib[t * T:(t + 1) * T, hk * G:(hk + 1) * G, t * T:].sum(axis=2).mean()
            np.testing.assert_allclose(a[hk].sum() + diag, 1.0, atol=1e-12)


def test_prefill_single_token_tiles_reduce_to_decode():
    # T = 1: the row of token i is a decode call at L = i + 1 on the same cache
    S, Hq, Hkv, d = 12, 4, 2, 8
    Q, Kp, Vp = make_prefill(33, S, Hq, Hkv, d)
    for i in (1, 5, 11):
        a = ko.prefill_pooled_tile(Q, Kp, i, 1, 0.5)
        p_dec = ko.pool_gqa(ko.decode_probabilities(Q[i], Kp[:, : i + 1], 0.5), Hkv)
        np.testing.assert_allclose(a, p_dec[:, :i], atol=1e-14)
        np.testing.assert_allclose(ko.prefill_dense_tile(Q, Kp, Vp, i, 1, 0.5)[0],
                                   ko.dense_decode(Q[i], Kp[:, : i + 1], Vp[:, : i + 1], 0.5), atol=1e-13)
        # sparse row: prefix indices plus the diagonal key i = a decode over that set
        I = [np.array([0, i - 1]) if i > 1 else np.array([0])] * Hkv
        y = ko.prefill_sparse_tile(Q, Kp, Vp, i, 1, I, 0.5)[0]
        I_dec = [np.concatenate([s, [i]]) for s in I]
        np.testing.assert_allclose(y, ko.sparse_decode(Q[i], Kp, Vp, I_dec, 0.5), atol=1e-13)


def test_prefill_sparse_matches_library_attention_with_explicit_mask():
    S, T, Hq, Hkv, d = 40, 8, 4, 2, 16
    G = Hq // Hkv
    r = rng(34)
    Q, Kp, Vp = make_prefill(34, S, Hq, Hkv, d)
    n_tiles = S // T
    sets = {}
    mask = np.zeros((Hq, S, S), dtype=bool)
    hm = [1, 1]                                    # both key heads use anchor head 1's sets
    for t in range(n_tiles):
        kt = min(t * T, 5)
        sets[t] = [np.sort(r.choice(t * T, kt, replace=False)) if kt else np.zeros(0, np.int64) for _ in range(Hkv)]
        for i in range(t * T, (t + 1) * T):
            for h in range(Hq):
                mask[h, i, sets[t][hm[h // G]]] = True
                mask[h, i, t * T: i + 1] = True
    ref = sdpa_prefill(Q, Kp, Vp, 0.25, mask=mask)
    for t in range(n_tiles):
        y = ko.prefill_sparse_tile(Q, Kp, Vp, t, T, sets[t], 0.25, head_map=hm)
        np.testing.assert_allclose(y, ref[t * T:(t + 1) * T], atol=1e-12)


def test_prefill_sparse_with_full_prefix_is_dense_and_tile0_is_dense():
    S, T = 30, 8                                    # ragged last tile
    Q, Kp, Vp = make_prefill(35, S, 4, 2, 8)
    for t in range(4):
        full = [np.arange(t * T)] * 2
        np.testing.assert_allclose(ko.prefill_sparse_tile(Q, Kp, Vp, t, T, full, 0.3),
                                   ko.prefill_dense_tile(Q, Kp, Vp, t, T, 0.3), atol=1e-13)
    with pytest.raises(ValueError):
        ko.prefill_sparse_tile(Q, Kp, Vp, 1, T, [np.array([8])] * 2, 0.3)


def test_prefill_anchor_indices_tile():
    S, T = 64, 8
    Q, Kp, _ = make_prefill(36, S, 8, 2, 16)
    t, kt = 6, 10
    idx, a = ko.prefill_anchor_indices_tile(Q, Kp, t, T, 0.25, kt)
    assert idx.shape == (2, kt) and a.shape == (2, t * T)
    for hk in range(2):
        lib = torch.topk(torch.from_numpy(a[hk]), kt).indices.sort().values.numpy()
        np.testing.assert_array_equal(idx[hk], lib)


# ------------------------------------------------------------------ Eq. 3

def test_similarity_bounds():
    r = rng(41)
    p = ko.softmax_lastdim(3 * r.standard_normal(200))
    Ib = ko.select_topk(p, 20)
    assert ko.topk_similarity(p, Ib, Ib) == 1.0
    for _ in range(10):
        Ia = np.sort(r.choice(200, 20, replace=False))
        s = ko.topk_similarity(p, Ia, Ib)
        assert 0.0 <= s <= 1.0
    # hand value: p = (.5,.3,.2), own top-1 = {0}, other set {1} -> 0.3/0.5
    np.testing.assert_allclose(ko.topk_similarity(np.array([.5, .3, .2]), [1], [0]), 0.6)


# ------------------------------------------------------------------ numbers the paper prints

def read_rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_k_rule_golden():
    for L, frac, kmin, k in read_rows("k_rule.txt"):
        assert ko.topk_budget(int(L), float(frac), int(kmin)) == int(k)


def test_table3_weighted_average_golden():
    for step, seqlen, pct, a0, a, r_, avg in read_rows("table3_layer_average.txt"):
        got = ko.kascade_layer_average(float(a0), float(a), float(r_))
        # printed inputs carry +-0.005 each, weights sum to 1 -> +-0.005, plus the result's own rounding
        assert abs(got - float(avg)) <= 0.0101, (step, seqlen, pct, got, avg)


# ------------------------------------------------------------------ Algorithm 1

def brute_force_anchors(S, M):
    L = S.shape[0]
    best, best_val = None, -np.inf
    for rest in itertools.combinations(range(1, L), M - 1):
        anchors = (0,) + rest
        val = sum(S[i, l] for i, nxt in zip(anchors, anchors[1:] + (L,)) for l in range(i, nxt))
        if val > best_val + 1e-12:
            best, best_val = list(anchors), val
    return best, best_val


@pytest.mark.parametrize("L,M,seed", [(6, 2, 0), (8, 3, 1), (9, 4, 2), (10, 5, 3), (7, 1, 4), (5, 5, 5),
                                      # matrices on which splitting greedily is not optimal
                                      (11, 4, 6), (7, 3, 8), (8, 3, 8), (9, 4, 10), (8, 3, 11)])
def test_anchor_selection_matches_exhaustive_search(L, M, seed):
    S = rng(200 + seed).random((L, L))
    got = ko.select_anchor_layers(S, M)
    ref, ref_val = brute_force_anchors(S, M)
    assert got == ref
    np.testing.assert_allclose(ko.segment_score(S, got), ref_val, atol=1e-12)
    assert got[0] == 0 and len(got) == M and all(b > a for a, b in zip(got, got[1:]))


def test_anchor_selection_on_block_structure():
    # three blocks of mutually similar layers: anchors must sit on the block starts
    L = 9
    S = np.full((L, L), 0.2)
    for lo, hi in ((0, 2), (2, 6), (6, 9)):
        S[lo:hi, lo:hi] = 0.99
    assert ko.select_anchor_layers(S, 3) == [0, 2, 6]
    np.testing.assert_allclose(ko.segment_score(S, [0, 2, 6]), 9 * 0.99)


def test_similarity_matrix_properties():
    r = rng(77)
    n_layers, n_seg, N, k = 4, 3, 60, 6
    pooled = [ko.softmax_lastdim(2 * r.standard_normal((n_seg, N))) for _ in range(n_layers)]
    sets = [np.stack([ko.select_topk(p[g], k) for g in range(n_seg)]) for p in pooled]
    S = ko.similarity_from_layers(pooled, sets)
    np.testing.assert_allclose(np.diag(S), 1.0)
    assert (S[np.triu_indices(n_layers)] <= 1.0 + 1e-15).all() and (S >= 0).all()
    assert (S[np.tril_indices(n_layers, -1)] == 0).all()
    # hand check of one entry
    g_vals = [pooled[2][g][sets[0][g]].sum() / pooled[2][g][sets[2][g]].sum() for g in range(n_seg)]
    np.testing.assert_allclose(S[0, 2], min(g_vals))


def test_layer_weighting_scales_the_served_layer():
    S = np.arange(16, dtype=np.float64).reshape(4, 4)
    w = np.array([1.0, 0.5, 0.25, 2.0])
    W = ko.weight_similarity(S, w)
    for i in range(4):
        for j in range(4):
            assert W[i, j] == S[i, j] * w[j]
    # weights that vanish on the late layers pull the anchors towards the early ones
    L = 8
    base = np.full((L, L), 0.5) + 0.5 * np.eye(L)
    early = np.array([1, 1, 1, 1, 1e-3, 1e-3, 1e-3, 1e-3])
    assert ko.select_anchor_layers(ko.weight_similarity(base, early), 4) == [0, 1, 2, 3]
    assert ko.select_anchor_layers(ko.weight_similarity(base, early[::-1].copy()), 5) == [0, 4, 5, 6, 7]


def test_layer_importance_closed_forms():
    x = np.array([[1.0, 0.0], [1.0, 0.0], [1.0, 1.0], [2.0, 0.0]])
    y = np.array([[3.0, 0.0], [0.0, 5.0], [1.0, 0.0], [-1.0, 0.0]])
    np.testing.assert_allclose(ko.layer_importance(x, y), [0.0, 1.0, 1.0 - 1.0 / np.sqrt(2.0), 2.0], atol=1e-15)


def test_head_map_recovers_planted_permutation_and_beats_every_other_map():
    r = rng(91)
    H, N, k, n_samples = 4, 200, 10, 3
    perm = [2, 0, 3, 1]                       # reuse head h behaves like anchor head perm[h]
    sims = []
    for _ in range(n_samples):
        pooled_a = ko.softmax_lastdim(3 * r.standard_normal((H, N)))
        pooled_b = np.stack([ko.softmax_lastdim(np.log(pooled_a[perm[h]]) + 0.1 * r.standard_normal(N)) for h in range(H)])
        sets_a = np.stack([ko.select_topk(p, k) for p in pooled_a])
        sets_b = np.stack([ko.select_topk(p, k) for p in pooled_b])
        sims.append(ko.head_similarity(pooled_b, sets_a, sets_b))
    hm, mean = ko.head_map_from_similarity(np.stack(sims))
    assert hm.tolist() == perm
    # exhaustive: no assignment of anchor heads to reuse heads has a larger total mean similarity
    best = max(itertools.product(range(H), repeat=H), key=lambda m: sum(mean[h, m[h]] for h in range(H)))
    assert list(best) == hm.tolist()
    # entry check by hand
    h, g = 1, 3
    want = pooled_b[h][sets_a[g]].sum() / pooled_b[h][sets_b[h]].sum()
    np.testing.assert_allclose(sims[-1][h, g], want)


def test_head_map_many_to_one_and_ties():
    sims = np.zeros((2, 3, 2))
    sims[:, 0] = [0.9, 0.1]
    sims[:, 1] = [0.8, 0.2]
    sims[:, 2] = [0.5, 0.5]                   # tie -> lower anchor head
    hm, _ = ko.head_map_from_similarity(sims)
    assert hm.tolist() == [0, 0, 0]


# ------------------------------------------------------------------ shared (all heads pooled) sets

def test_shared_indices_are_the_mean_of_the_per_head_pooled_scores():
    r = rng(61)
    Hq, Hkv, d, L, k = 8, 2, 16, 90, 9
    q, K = r.standard_normal((Hq, d)), r.standard_normal((Hkv, L, d))
    idx, a = ko.decode_shared_indices(q, K, 0.3, k)
    _, per_head = ko.decode_anchor_indices(q, K, 0.3, k)
    np.testing.assert_allclose(a, per_head.mean(axis=0), atol=1e-15)      # equal group sizes: mean of means
    np.testing.assert_allclose(a.sum(), 1.0, atol=1e-12)
    lib = torch.topk(torch.from_numpy(a), k).indices.sort().values.numpy()
    np.testing.assert_array_equal(idx, lib)
    # one key head: the shared set is that head's set
    idx1, _ = ko.decode_shared_indices(q[:4], K[:1], 0.3, k)
    per1, _ = ko.decode_anchor_indices(q[:4], K[:1], 0.3, k)
    np.testing.assert_array_equal(idx1, per1[0])


def test_shared_prefill_indices_match_decode_for_single_token_tiles():
    r = rng(62)
    S, Hq, Hkv, d = 12, 4, 2, 8
    Q, Kp = r.standard_normal((S, Hq, d)), r.standard_normal((Hkv, S, d))
    t, k_t = 9, 4
    idx, a = ko.prefill_shared_indices_tile(Q, Kp, t, 1, 0.5, k_t)
    # T = 1: the tile is token t; its prefix scores are the decode probabilities over keys 0..t
    p = ko.decode_probabilities(Q[t], Kp[:, : t + 1], 0.5).mean(axis=0)
    np.testing.assert_allclose(a, p[:t], atol=1e-15)
    np.testing.assert_array_equal(idx, ko.select_topk(p[:t], k_t))
    per_head = ko.prefill_pooled_tile(Q, Kp, t, 1, 0.5)
    np.testing.assert_allclose(a, per_head.mean(axis=0), atol=1e-15)


# ------------------------------------------------------------------ Sec. 3.4: Pre-Softmax pooling

def test_round_to_bf16_matches_library_conversion():
    r = rng(70)
    x = np.concatenate([r.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** r.integers(-20, 20, 20000).astype(np.float32),
                        np.array([0.0, -0.0, 1.0, -1.0, 3.0e38, 1e-40, 65504.0], dtype=np.float32)])
    # exact ties between two neighbours, with an even and with an odd kept part
    ties = (np.array([0x3F808000, 0x3F818000, 0xBF808000, 0x40FF8000, 0x00018000], dtype=np.uint32)).view(np.float32)
    x = np.concatenate([x, ties])
    lib = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(ko.round_to_bf16(x).view(np.uint32), lib.view(np.uint32))
    np.testing.assert_array_equal(ko.round_to_bf16(ties).view(np.uint32),
                                  np.array([0x3F800000, 0x3F820000, 0xBF800000, 0x41000000, 0x00020000], dtype=np.uint32))


def test_round_nearest_even_is_one_correct_rounding():
    """Pins for the single rounding from float64: library conversions that are known to round once
    (numpy float64 -> float16 / float32; torch float32 -> bfloat16 on values that are float32 already), and
    hand-built values on which rounding in two steps (float64 -> float32 -> bfloat16) gives another answer."""
    r = rng(74)
    x = r.standard_normal(20000) * 10.0 ** r.integers(-6, 5, 20000)
    np.testing.assert_array_equal(ko.round_nearest_even(x, 11, -14), x.astype(np.float16).astype(np.float64))
    np.testing.assert_array_equal(ko.round_nearest_even(x, 24, -126), x.astype(np.float32).astype(np.float64))
    x32 = x.astype(np.float32)
    lib = torch.from_numpy(x32).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(ko.round_nearest_even(x32.astype(np.float64), 8, -126), lib)
    np.testing.assert_array_equal(ko.round_nearest_even(x32.astype(np.float64), 8, -126),
                                  ko.round_to_bf16(x32).astype(np.float64))
    # subnormal range of binary16 and of bfloat16: the step stops shrinking
    tiny = np.array([2.0 ** -25, 3 * 2.0 ** -25, 2.0 ** -24, 5 * 2.0 ** -26, 0.0, -2.0 ** -25 * 1.0001])
    np.testing.assert_array_equal(ko.round_nearest_even(tiny, 11, -14),
                                  np.array([0.0, 2.0 ** -23, 2.0 ** -24, 2.0 ** -24, 0.0, -2.0 ** -24]))
    np.testing.assert_array_equal(ko.round_nearest_even(np.array([2.0 ** -134, 3 * 2.0 ** -134]), 8, -126),
                                  np.array([0.0, 2.0 ** -132]))
    # 1 + 2^-8 is the tie between the bfloat16 neighbours 1 and 1 + 2^-7; a value a hair above it must go up,
    # although its float32 rounding is the tie itself (which would then go to the even neighbour 1)
    above = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert np.float32(above) == np.float32(1.0 + 2.0 ** -8)
    assert ko.round_nearest_even(above, 8, -126) == 1.0 + 2.0 ** -7
    assert ko.round_nearest_even(1.0 + 2.0 ** -8, 8, -126) == 1.0
    assert ko.round_nearest_even(1.0 + 3 * 2.0 ** -8, 8, -126) == 1.0 + 2.0 ** -6


def test_pooled_query_is_the_rounded_mean():
    r = rng(71)
    rows = r.standard_normal((12, 16)).astype(np.float32).astype(np.float64)
    exact = rows.mean(axis=0)
    np.testing.assert_array_equal(ko.pool_query_vectors(rows, "fp32"), exact.astype(np.float32).astype(np.float64))
    pb = ko.pool_query_vectors(rows, "bf16")
    assert np.all(np.abs(pb - exact) <= np.abs(exact) * 2.0 ** -8)                  # at most half a bf16 step
    assert np.all(pb.astype(np.float32).view(np.uint32) & 0xFFFF == 0)             # representable in bf16
    # one vector, or equal vectors: the pooled query is that vector (already representable)
    v = torch.randn(16, generator=torch.Generator().manual_seed(3)).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(ko.pool_query_vectors(np.tile(v, (4, 1)), "bf16"), v)
    np.testing.assert_array_equal(ko.pool_query_vectors(v[None], "fp32"), v)


def test_pooled_query_mean_is_exact_before_the_one_rounding():
    """Hand-built bf16 rows whose exact mean lies a hair above a bf16 tie.  A float32 running sum drops the
    small addend (the sum then lands on the tie and goes to the even neighbour), and so does a mean that is
    rounded to float32 before it is rounded to bf16; the definition - exact mean, one rounding - goes up."""
    col = np.array([1.0 + 2.0 ** -5, 1.0, 1.0, 1.0, 1.0, 1.0, 2.0, 2.0 ** -30])    # every value is a bf16
    assert col.sum() == 8.0 + 2.0 ** -5 + 2.0 ** -30                               # exact in float64
    acc32 = np.float32(0.0)
    for v in col:
        acc32 = np.float32(acc32 + np.float32(v))
    assert acc32 == np.float32(8.0 + 2.0 ** -5)                                    # the small addend is gone
    rows = np.stack([col, col[::-1], -col], axis=1)                                # three components
    want = np.array([1.0 + 2.0 ** -7, 1.0 + 2.0 ** -7, -(1.0 + 2.0 ** -7)])
    np.testing.assert_array_equal(ko.pool_query_vectors(rows, "bf16"), want)
    # binary16 analogue: mean 1 + 2^-11 + 2^-33, tie between 1 and 1 + 2^-10
    col16 = np.array([1.0 + 2.0 ** -8, 1.0, 1.0, 1.0, 1.0, 1.0, 2.0, 2.0 ** -24])   # the last: smallest subnormal
    got = ko.pool_query_vectors(col16[:, None], "fp16")
    assert col16.sum() / 8 == 1.0 + 2.0 ** -11 + 2.0 ** -27
    np.testing.assert_array_equal(got, np.array([1.0 + 2.0 ** -10]))
    # fp32 storage: mean 1 + 2^-24 + 2^-50 from float32 rows, tie between 1 and 1 + 2^-23
    col32 = np.array([1.0 + 2.0 ** -21, 1.0, 1.0, 1.0, 1.0, 1.0, 2.0, 2.0 ** -47])
    assert col32.sum() / 8 == 1.0 + 2.0 ** -24 + 2.0 ** -50
    np.testing.assert_array_equal(ko.pool_query_vectors(col32[:, None], "fp32"), np.array([1.0 + 2.0 ** -23]))


def test_pooled_query_in_fp16_storage():
    """binary16: 10 fraction bits, ties to even, largest finite value 65504; expectations written out from
    the format's definition, not taken from a conversion routine."""
    one = np.zeros((1, 6))
    one[0] = [1.0 + 2.0 ** -11,            # exact tie above 1: the even neighbour is 1
              1.0 + 3.0 * 2.0 ** -11,      # tie between 1 + 2^-10 (odd) and 1 + 2^-9 (even)
              1.0 + 2.0 ** -11 + 2.0 ** -20,   # just above the tie
              -0.3333333432674408,         # float32(-1/3): below 0.5 the step is 2^-12 ... here 2^-12
              2.0 ** -25,                  # half the smallest subnormal: tie, the even neighbour is 0
              1000.4]                      # step 0.5 between 512 and 1024
    got = ko.pool_query_vectors(one, "fp16")[...]
    want = [1.0, 1.0 + 2.0 ** -9, 1.0 + 2.0 ** -10, -(1365.0 / 4096.0), 0.0, 1000.5]
    np.testing.assert_array_equal(got, np.array(want))
    # the mean of rows, then one rounding: within half a step of the exact mean, and representable
    r = rng(73)
    rows = r.standard_normal((12, 16)).astype(np.float32).astype(np.float64)
    exact = rows.mean(axis=0)
    pf = ko.pool_query_vectors(rows, "fp16")
    assert np.all(np.abs(pf - exact) <= np.abs(exact) * 2.0 ** -11 + 1e-6)
    m, e = np.frexp(pf)
    assert np.all((m * 2048.0) == np.round(m * 2048.0))        # 11 significant bits
    with pytest.raises(ValueError):
        ko.pool_query_vectors(rows, "fp8")


def test_presoftmax_decode_is_softmax_of_the_mean_logits():
    r = rng(72)
    Hq, Hkv, d, L, k = 8, 2, 16, 70, 9
    q = r.standard_normal((Hq, d)).astype(np.float32).astype(np.float64)
    K = r.standard_normal((Hkv, L, d))
    idx, a = ko.decode_presoftmax_indices(q, K, 0.3, k, "fp32")
    # the dot product is linear: the pooled query's logits are the mean of the group's logits (library softmax)
    s = ko.decode_logits(q, K, 0.3).reshape(Hkv, Hq // Hkv, L).mean(axis=1)
    lib = torch.softmax(torch.from_numpy(s), dim=-1).numpy()
    np.testing.assert_allclose(a, lib, atol=1e-6)
    np.testing.assert_allclose(a.sum(axis=1), 1.0, atol=1e-12)
    # softmax is monotone: the set is the Top-k of the mean logits themselves
    for hk in range(Hkv):
        brute = sorted(sorted(range(L), key=lambda j: (-s[hk, j], j))[:k])
        assert idx[hk].tolist() == brute
    # it is NOT the post-softmax pooling (mean of softmaxes) unless the group has one head
    _, post = ko.decode_anchor_indices(q, K, 0.3, k)
    assert np.max(np.abs(post - a)) > 1e-3
    idx1, a1 = ko.decode_presoftmax_indices(q[:2], K, 0.3, k, "fp32")           # G = 1
    idx1p, a1p = ko.decode_anchor_indices(q[:2], K, 0.3, k)
    np.testing.assert_allclose(a1, a1p, atol=1e-15)
    np.testing.assert_array_equal(idx1, idx1p)
    # recent window handled by the same selection rule
    idxw, _ = ko.decode_presoftmax_indices(q, K, 0.3, k, "fp32", recent_window=4)
    assert all(set(range(L - 4, L)) <= set(row.tolist()) for row in idxw)


def test_presoftmax_decode_equal_queries_reduce_to_post_softmax_pooling():
    r = rng(73)
    Hkv, G, d, L, k = 2, 4, 16, 50, 7
    base = torch.randn(Hkv, d, generator=torch.Generator().manual_seed(5)).to(torch.bfloat16).to(torch.float64).numpy()
    q = np.repeat(base, G, axis=0)                       # every head of a group asks the same query
    K = r.standard_normal((Hkv, L, d))
    idx, a = ko.decode_presoftmax_indices(q, K, 0.25, k, "bf16")
    idxp, ap = ko.decode_anchor_indices(q, K, 0.25, k)
    np.testing.assert_allclose(a, ap, atol=1e-15)
    np.testing.assert_array_equal(idx, idxp)


def test_presoftmax_prefill_tile_special_cases():
    r = rng(74)
    S, Hq, Hkv, d, T = 24, 4, 2, 8, 4
    Q = r.standard_normal((S, Hq, d)).astype(np.float32).astype(np.float64)
    Kp = r.standard_normal((Hkv, S, d))
    G = Hq // Hkv
    t, k_t = 4, 5
    idx, a = ko.prefill_presoftmax_indices_tile(Q, Kp, t, T, 0.4, k_t, "fp32")
    assert a.shape == (Hkv, t * T) and idx.shape == (Hkv, k_t)
    np.testing.assert_allclose(a.sum(axis=1), 1.0, atol=1e-12)
    for hk in range(Hkv):
        # mean over the tile's T*G rows of their logits on the prefix keys, then a library softmax
        s = np.mean([0.4 * (Kp[hk, : t * T] @ Q[i, hk * G + g]) for i in range(t * T, (t + 1) * T) for g in range(G)], axis=0)
        np.testing.assert_allclose(a[hk], torch.softmax(torch.from_numpy(s), dim=-1).numpy(), atol=1e-6)
        assert idx[hk].tolist() == sorted(sorted(range(t * T), key=lambda j: (-s[j], j))[:k_t])
    # tiles of one token and one head per group: the tile's distribution is that token's causal row,
    # renormalised over the keys before it; the sets agree with post-softmax pooling
    Q1, K1 = Q[:, ::G], Kp
    idx1, a1 = ko.prefill_presoftmax_indices_tile(Q1, K1, 9, 1, 0.4, 3, "fp32")
    idx1p, a1p = ko.prefill_anchor_indices_tile(Q1, K1, 9, 1, 0.4, 3)
    np.testing.assert_allclose(a1, a1p / a1p.sum(axis=1, keepdims=True), atol=1e-12)
    np.testing.assert_array_equal(idx1, idx1p)
    # a ragged last tile averages only the rows that exist
    Qr, Kr = Q[:22], Kp[:, :22]
    _, ar = ko.prefill_presoftmax_indices_tile(Qr, Kr, 5, T, 0.4, 2, "fp32")
    s = np.mean([0.4 * (Kr[0, :20] @ Qr[i, g]) for i in (20, 21) for g in range(G)], axis=0)
    np.testing.assert_allclose(ar[0], torch.softmax(torch.from_numpy(s), dim=-1).numpy(), atol=1e-6)
    # tile 0 has no candidates
    idx0, a0 = ko.prefill_presoftmax_indices_tile(Q, Kp, 0, T, 0.4, 0, "fp32")
    assert a0.shape == (Hkv, 0) and idx0.shape == (Hkv, 0)
