"""Do the pins bite?  Each case plants one plausible mistake in the CPU oracle (wrong head grouping, a
dropped scale, ties to the wrong side, a mask off by one, ...) and requires that at least one pin in
test_oracle_pins.py fails.  Everything here runs on the CPU and touches only the oracle."""
import numpy as np
import pytest

import test_oracle_pins as pins
from oracle import kascade_oracle as ko


def wrong_group_logits(q, K, scale):
    q, K = np.asarray(q, dtype=np.float64), np.asarray(K, dtype=np.float64)
    Hq, Hkv = q.shape[0], K.shape[0]
    return np.stack([scale * (K[h % Hkv] @ q[h]) for h in range(Hq)])      # interleaved instead of consecutive


def unscaled_logits(q, K, scale):
    q, K = np.asarray(q, dtype=np.float64), np.asarray(K, dtype=np.float64)
    G = q.shape[0] // K.shape[0]
    return np.stack([K[h // G] @ q[h] for h in range(q.shape[0])])


def topk_ties_high(a, k, recent_window=0):
    a = np.asarray(a, dtype=np.float64)
    L, W = a.shape[0], int(recent_window)
    if not (0 <= k <= L) or not (0 <= W <= k):
        raise ValueError
    n_cand = L - W
    order = np.argsort(-a[:n_cand][::-1], kind="stable")                   # higher index wins ties
    chosen = (n_cand - 1 - order)[: k - W]
    return np.sort(np.concatenate([chosen.astype(np.int64), np.arange(n_cand, L, dtype=np.int64)]))


def topk_no_window(a, k, recent_window=0):
    a = np.asarray(a, dtype=np.float64)
    if not (0 <= k <= a.shape[0]) or not (0 <= recent_window <= k):
        raise ValueError
    return np.sort(np.argsort(-a, kind="stable")[:k]).astype(np.int64)


def pool_wrong_groups(p, n_kv_heads):
    p = np.asarray(p, dtype=np.float64)
    Hq, L = p.shape
    return p.reshape(Hq // n_kv_heads, n_kv_heads, L).mean(axis=0)


def sparse_not_renormalised(q, K, V, idx_sets, scale, head_map=None):
    q, K, V = (np.asarray(x, dtype=np.float64) for x in (q, K, V))
    Hq, G = q.shape[0], q.shape[0] // K.shape[0]
    y = np.empty((Hq, V.shape[2]))
    for h in range(Hq):
        hk = h // G
        src = hk if head_map is None else int(head_map[hk])
        I = np.asarray(idx_sets[src], dtype=np.int64)
        p = ko.softmax_lastdim(scale * (K[hk] @ q[h]))                    # dense denominator
        y[h] = p[I] @ V[hk, I]
    return y


def sparse_ignores_head_map(q, K, V, idx_sets, scale, head_map=None):
    return ORIGINAL["sparse_decode"](q, K, V, idx_sets, scale, None)


def tile_probs_strict_causal(Q, Kp, t, T, scale):
    Q, Kp = np.asarray(Q, dtype=np.float64), np.asarray(Kp, dtype=np.float64)
    S, Hq, _ = Q.shape
    G = Hq // Kp.shape[0]
    lo, hi = ko.tile_bounds(t, T, S)
    P = np.zeros((hi - lo, Hq, hi))
    for r in range(hi - lo):
        i = lo + r
        for h in range(Hq):
            n = max(i, 1)                                                  # the token's own key is left out
            P[r, h, :n] = ko.softmax_lastdim(scale * (Kp[h // G, :n] @ Q[i, h]))
    return P


def pooled_tile_prefix_normalised(Q, Kp, t, T, scale):
    Hkv = np.asarray(Kp).shape[0]
    P = ORIGINAL["prefill_tile_probabilities"](Q, Kp, t, T, scale)
    n_tok, Hq, _ = P.shape
    prefix = t * T
    Pp = P[:, :, :prefix]
    Pp = Pp / np.maximum(Pp.sum(axis=2, keepdims=True), 1e-300)            # normaliser without the diagonal keys
    return Pp.reshape(n_tok, Hkv, Hq // Hkv, prefix).mean(axis=(0, 2))


def prefill_sparse_without_diagonal(Q, Kp, Vp, t, T, idx_sets, scale, head_map=None):
    Q, Kp, Vp = (np.asarray(x, dtype=np.float64) for x in (Q, Kp, Vp))
    S, Hq, _ = Q.shape
    G = Hq // Kp.shape[0]
    lo, hi = ko.tile_bounds(t, T, S)
    y = np.zeros((hi - lo, Hq, Vp.shape[2]))
    for r in range(hi - lo):
        for h in range(Hq):
            hk = h // G
            I = np.asarray(idx_sets[hk if head_map is None else int(head_map[hk])], dtype=np.int64)
            keys = np.concatenate([I, [lo + r]]).astype(np.int64)          # only the token itself, not lo..i
            p = ko.softmax_lastdim(scale * (Kp[hk, keys] @ Q[lo + r, h]))
            y[r, h] = p @ Vp[hk, keys]
    return y


def similarity_inverted(p_b, idx_a, idx_b):
    p_b = np.asarray(p_b, dtype=np.float64)
    return float(p_b[np.asarray(idx_b)].sum() / p_b[np.asarray(idx_a)].sum())


def budget_floor(L, fraction, k_min=0):
    return int(min(max(int(np.floor(fraction * L)), k_min), L))


def layer_average_unweighted(anchor0, anchor, reuse, n_layers=32, n_anchors=5):
    return (anchor0 + anchor + reuse) / 3.0


def anchors_greedy(S, n_anchors):
    """Greedy instead of the dynamic programme: always split the worst-served segment."""
    S = np.asarray(S, dtype=np.float64)
    L = S.shape[0]
    anchors = [0]
    while len(anchors) < n_anchors:
        best, arg = -np.inf, None
        for c in range(1, L):
            if c in anchors:
                continue
            val = ko.segment_score(S, sorted(anchors + [c]))
            if val > best:
                best, arg = val, c
        anchors = sorted(anchors + [arg])
    return anchors


def weight_by_anchor_layer(S, w):
    return np.asarray(S, dtype=np.float64) * np.asarray(w, dtype=np.float64)[:, None]


def head_map_argmin(sims):
    mean = np.asarray(sims, dtype=np.float64).mean(axis=0)
    return np.argmin(mean, axis=1).astype(np.int64), mean


def shared_indices_first_head_only(q, K, scale, k, recent_window=0):
    a = ko.decode_probabilities(q, K, scale)[0]
    return ko.select_topk(a, k, recent_window), a


ORIGINAL = {name: getattr(ko, name) for name in dir(ko) if callable(getattr(ko, name))}

P = pytest.param


def bf16_truncates(x):
    bits = np.asarray(x, dtype=np.float32).view(np.uint32)
    return (bits & np.uint32(0xFFFF0000)).view(np.float32)


def bf16_ties_away(x):
    bits = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return ((bits + np.uint64(0x8000)) & np.uint64(0xFFFF0000)).astype(np.uint32).view(np.float32)


def pooled_query_is_the_sum(rows, storage):
    acc = np.asarray(rows, dtype=np.float64).sum(axis=0)
    return ko.round_nearest_even(acc, *ko.STORAGE_FORMATS[storage])


def pooled_query_first_row(rows, storage):
    row = np.asarray(rows, dtype=np.float64)[0]
    return ko.round_nearest_even(row, *ko.STORAGE_FORMATS[storage])


def pooled_query_fp16_truncates(rows, storage):
    if storage != "fp16":
        return ORIGINAL_POOL_QUERY_VECTORS(rows, storage)
    mean = np.asarray(rows, dtype=np.float64).mean(axis=0)
    up = mean.astype(np.float16)                      # nearest; step back where that went away from zero
    away = np.abs(up.astype(np.float64)) > np.abs(mean)
    toward = np.nextafter(up, np.float16(0.0))
    return np.where(away, toward, up).astype(np.float64)


def pooled_query_fp32_running_sum(rows, storage):
    """the mean from a float32 running sum and a float32 division, then the storage rounding"""
    rows = np.asarray(rows, dtype=np.float32)
    acc = np.zeros(rows.shape[1], dtype=np.float32)
    for r in rows:
        acc = acc + r
    mean = (acc / np.float32(rows.shape[0])).astype(np.float64)
    return ko.round_nearest_even(mean, *ko.STORAGE_FORMATS[storage])


def pooled_query_rounded_twice(rows, storage):
    """exact mean, but rounded to float32 first and to the storage type after that"""
    mean = np.asarray(rows, dtype=np.float64).mean(axis=0).astype(np.float32).astype(np.float64)
    return ko.round_nearest_even(mean, *ko.STORAGE_FORMATS[storage])


def nearest_ties_away(x, sig_bits, min_exp):
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)
    step_exp = np.maximum(e - 1, min_exp) - (sig_bits - 1)
    y = np.ldexp(x, -step_exp)
    return np.ldexp(np.sign(y) * np.floor(np.abs(y) + 0.5), step_exp)


def nearest_without_subnormals(x, sig_bits, min_exp):
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)
    step_exp = (e - 1) - (sig_bits - 1)
    return np.ldexp(np.rint(np.ldexp(x, -step_exp)), step_exp)


def pooled_query_fp16_as_bf16(rows, storage):
    return ORIGINAL_POOL_QUERY_VECTORS(rows, "bf16" if storage == "fp16" else storage)


def presoftmax_wrong_groups(q, K, scale, k, storage, recent_window=0):
    q, K = np.asarray(q, dtype=np.float64), np.asarray(K, dtype=np.float64)
    Hkv = K.shape[0]
    a = np.stack([ko.softmax_lastdim(scale * (K[hk] @ ko.pool_query_vectors(q[hk::Hkv], storage))) for hk in range(Hkv)])
    return np.stack([ko.select_topk(a[hk], k, recent_window) for hk in range(Hkv)]), a


def presoftmax_tile_includes_diagonal(Q, Kp, t, T, scale, k_t, storage):
    Q, Kp = np.asarray(Q, dtype=np.float64), np.asarray(Kp, dtype=np.float64)
    S, Hq, d = Q.shape
    Hkv = Kp.shape[0]
    G = Hq // Hkv
    lo, hi = ko.tile_bounds(t, T, S)
    a = np.stack([ko.softmax_lastdim(scale * (Kp[hk, :hi] @ ko.pool_query_vectors(Q[lo:hi, hk * G:(hk + 1) * G].reshape(-1, d), storage)))[:lo]
                  for hk in range(Hkv)])
    return np.stack([ko.select_topk(a[hk], k_t, 0) for hk in range(Hkv)]), a


ORIGINAL_POOL_QUERY_VECTORS = ko.pool_query_vectors

MUTATIONS = [
    P("decode_logits", wrong_group_logits, id="heads grouped h mod Hkv"),
    P("decode_logits", unscaled_logits, id="softmax scale dropped"),
    P("default_scale", lambda d: 1.0 / d, id="scale 1/d"),
    P("select_topk", topk_ties_high, id="ties to the higher index"),
    P("select_topk", topk_no_window, id="recent window ignored"),
    P("pool_gqa", pool_wrong_groups, id="pooling over the wrong heads"),
    P("sparse_decode", sparse_not_renormalised, id="sparse softmax not renormalised"),
    P("sparse_decode", sparse_ignores_head_map, id="head map ignored"),
    P("prefill_tile_probabilities", tile_probs_strict_causal, id="causal mask excludes the token itself"),
    P("prefill_pooled_tile", pooled_tile_prefix_normalised, id="pooling normaliser without the diagonal"),
    P("prefill_sparse_tile", prefill_sparse_without_diagonal, id="diagonal block dropped"),
    P("topk_similarity", similarity_inverted, id="similarity ratio inverted"),
    P("topk_budget", budget_floor, id="k rule floors"),
    P("kascade_layer_average", layer_average_unweighted, id="layer average unweighted"),
    P("select_anchor_layers", anchors_greedy, id="greedy anchor choice"),
    P("weight_similarity", weight_by_anchor_layer, id="importance of the anchor instead of the served layer"),
    P("head_map_from_similarity", head_map_argmin, id="least similar head"),
    P("decode_shared_indices", shared_indices_first_head_only, id="shared set from one head"),
    P("round_to_bf16", bf16_truncates, id="bf16 by truncation"),
    P("round_to_bf16", bf16_ties_away, id="bf16 ties away from zero"),
    P("pool_query_vectors", pooled_query_is_the_sum, id="pooled query not divided"),
    P("pool_query_vectors", pooled_query_first_row, id="pooled query from one row"),
    P("pool_query_vectors", pooled_query_fp16_truncates, id="fp16 pooled query by truncation"),
    P("pool_query_vectors", pooled_query_fp16_as_bf16, id="fp16 pooled query rounded to bf16"),
    P("pool_query_vectors", pooled_query_fp32_running_sum, id="pooled query from a float32 running sum"),
    P("pool_query_vectors", pooled_query_rounded_twice, id="pooled query rounded twice"),
    P("round_nearest_even", nearest_ties_away, id="storage rounding ties away from zero"),
    P("round_nearest_even", nearest_without_subnormals, id="storage rounding without subnormals"),
    P("decode_presoftmax_indices", presoftmax_wrong_groups, id="pre-softmax pooling over the wrong heads"),
    P("prefill_presoftmax_indices_tile", presoftmax_tile_includes_diagonal, id="pre-softmax candidates include the tile"),
]


def all_pin_calls():
    """Every pin of test_oracle_pins.py with its parametrisations expanded by hand."""
    calls = []
    for name in dir(pins):
        fn = getattr(pins, name)
        if not name.startswith("test_") or not callable(fn):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            calls.append((name, fn, ()))
            continue
        names = [n.strip() for n in marks[0].args[0].split(",")]
        for values in marks[0].args[1]:
            values = values if isinstance(values, (tuple, list)) else (values,)
            assert len(values) == len(names)
            calls.append((name, fn, tuple(values)))
    return calls


def test_the_unmodified_oracle_passes_every_pin():
    for name, fn, args in all_pin_calls():
        fn(*args)


@pytest.mark.parametrize("target,mutant", MUTATIONS)
def test_planted_mistake_is_caught(monkeypatch, target, mutant):
    monkeypatch.setattr(ko, target, mutant)
    caught = []
    for name, fn, args in all_pin_calls():
        try:
            fn(*args)
        except Exception:          # an assertion, or the mutant tripping over its own inputs
            caught.append(name)
    assert caught, f"no pin notices a wrong {target}"
    print(f"  {target}: caught by {sorted(set(caught))}")
