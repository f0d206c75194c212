"""Anchor-layer selection (Sec. 3.3, Algorithm 1): the library's host routine against the oracle's
transcription of the recurrence and against exhaustive search.  Runs without a GPU."""
import itertools

import numpy as np
import pytest

from oracle import kascade_oracle as ko
from paper_2512_16391_amd import binding as kb


def exhaustive(S, M):
    L = S.shape[0]
    best, best_val = None, -np.inf
    for rest in itertools.combinations(range(1, L), M - 1):
        anchors = (0,) + rest
        val = sum(float(S[i, l]) for i, nxt in zip(anchors, anchors[1:] + (L,)) for l in range(i, nxt))
        if val > best_val + 1e-9:
            best, best_val = list(anchors), val
    return best, best_val


@pytest.mark.parametrize("L,M,seed", [(1, 1, 0), (6, 2, 1), (8, 3, 2), (12, 5, 3), (10, 10, 4), (9, 1, 5), (14, 4, 6)])
def test_library_selection_matches_oracle_and_exhaustive_search(L, M, seed):
    S = np.random.default_rng(seed).random((L, L)).astype(np.float32)
    got, obj = kb.kascade_select_anchor_layers(S, M)
    assert got == ko.select_anchor_layers(S.astype(np.float64), M)
    ref, ref_val = exhaustive(S.astype(np.float64), M)
    assert got == ref
    np.testing.assert_allclose(obj, ref_val, rtol=0, atol=1e-9)
    np.testing.assert_allclose(obj, ko.segment_score(S, got), rtol=0, atol=1e-9)


def test_library_selection_model_sized():
    # 36 layers, 5 anchors as in the paper's Qwen3-8B setting; 32 layers, 5 anchors as Llama-3.1-8B
    for L, M, seed in ((36, 5, 11), (32, 5, 12)):
        r = np.random.default_rng(seed)
        # similarity decays with layer distance, plus noise: a banded structure like Fig. 3
        i, j = np.meshgrid(np.arange(L), np.arange(L), indexing="ij")
        S = (np.exp(-np.abs(i - j) / 6.0) * (0.9 + 0.1 * r.random((L, L)))).astype(np.float32)
        got, obj = kb.kascade_select_anchor_layers(S, M)
        assert got == ko.select_anchor_layers(S.astype(np.float64), M)
        assert got[0] == 0 and all(b > a for a, b in zip(got, got[1:]))
        np.testing.assert_allclose(obj, ko.segment_score(S, got), atol=1e-9)


def test_library_selection_ties_keep_earliest_layer():
    S = np.ones((7, 7), dtype=np.float32)            # every choice scores the same
    got, obj = kb.kascade_select_anchor_layers(S, 3)
    assert got == ko.select_anchor_layers(S.astype(np.float64), 3)
    assert obj == 7.0


def test_library_selection_ignores_entries_below_the_diagonal():
    r = np.random.default_rng(3)
    S = r.random((9, 9)).astype(np.float32)
    T = S.copy()
    T[np.tril_indices(9, -1)] = 1e6
    assert kb.kascade_select_anchor_layers(S, 4) == kb.kascade_select_anchor_layers(T, 4)


def test_library_selection_rejects_bad_arguments():
    S = np.eye(4, dtype=np.float32)
    for M in (0, 5, -1):
        with pytest.raises(kb.KascadeError):
            kb.kascade_select_anchor_layers(S, M)
    bad = S.copy(); bad[0, 2] = np.nan
    with pytest.raises(kb.KascadeError):
        kb.kascade_select_anchor_layers(bad, 2)
    with pytest.raises(ValueError):
        kb.kascade_select_anchor_layers(np.zeros((3, 4), dtype=np.float32), 2)


def test_library_selection_with_layer_weights():
    r = np.random.default_rng(21)
    L, M = 11, 4
    S = r.random((L, L)).astype(np.float32)
    w = (1.0 / (1.0 + np.arange(L))).astype(np.float32)       # importance falling with depth
    got, obj = kb.kascade_select_anchor_layers(S, M, layer_weights=w)
    SW = ko.weight_similarity(S.astype(np.float64), w.astype(np.float64))
    assert got == ko.select_anchor_layers(SW, M)
    ref, ref_val = exhaustive(SW, M)
    assert got == ref
    np.testing.assert_allclose(obj, ref_val, atol=1e-9)
    # unit weights change nothing
    assert kb.kascade_select_anchor_layers(S, M, layer_weights=np.ones(L))[0] == kb.kascade_select_anchor_layers(S, M)[0]
    with pytest.raises(ValueError):
        kb.kascade_select_anchor_layers(S, M, layer_weights=np.ones(L + 1))


def test_config5_anchor_layers_from_planted_drift_oracle_similarity():
    """32 layers whose heavy hitters are redrawn at layers 0, 1, 4, 12, 20 and drift 5 % per layer in
    between: from the oracle's similarity matrix (Eq. 3, minimum over the key heads) both the library's
    host routine and the oracle's Algorithm 1 return exactly those layers for five anchors."""
    from paper_2512_16391_amd import workloads
    starts = workloads.CONFIG5_ANCHORS
    wl = workloads.layer_stack("cpu", n_layers=32, block_starts=starts, B=1, Hq=8, Hkv=2, d=64,
                               seqlens=(2000,), k=64, n_hitters=32, within=0.95)
    f64 = lambda t: t.double().numpy()
    ref = [ko.decode_anchor_indices(f64(l.q[0]), f64(l.k[0]), ko.default_scale(wl.d), 64) for l in wl.layers]
    n = len(ref)
    S = np.zeros((n, n))
    for a in range(n):
        for b in range(a, n):
            S[a, b] = min(ko.topk_similarity(ref[b][1][h], ref[a][0][h], ref[b][0][h]) for h in range(wl.Hkv))
    assert ko.select_anchor_layers(S, 5) == list(starts)
    got, _ = kb.kascade_select_anchor_layers(S.astype(np.float32), 5)
    assert got == list(starts)
    # inside a block the similarity decays slowly, across a redraw it collapses
    assert S[4, 11] > 0.3 and S[4, 12] < 0.1 and S[20, 31] > 0.3 and S[0, 1] < 0.1
