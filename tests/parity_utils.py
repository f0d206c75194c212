"""Comparison helpers shared by the GPU parity tests (the bars are stated here once)."""
import numpy as np
import torch

# output tolerance, max-abs against the fp64 oracle evaluated on the same input bits
# (fp16 keeps 3 more fraction bits than bf16: the bf16 bar / 8)
TOL_OUT = {torch.bfloat16: 2e-2, torch.float16: 2.5e-3, torch.float32: 1e-4}
# Top-k sets may differ from the oracle's only by swaps among keys whose pooled score lies
# within this relative distance of the k-th largest score (relative on the pooled
# probability = absolute on the logit for a single query)
TIE_REL = 1e-3


def f64(t):
    """Exact device bits widened to float64 numpy."""
    return t.detach().to("cpu").to(torch.float32).to(torch.float64).numpy()


def check_index_set(idx_gpu, idx_ref, scores, n_forced=0, where=""):
    """idx_gpu / idx_ref: 1-D int arrays of one set; scores: the oracle's pooled scores.
    Returns the number of swapped members."""
    g = np.asarray(idx_gpu, dtype=np.int64)
    r = np.asarray(idx_ref, dtype=np.int64)
    assert g.shape == r.shape, f"{where}: set size {g.shape} vs {r.shape}"
    assert (np.diff(g) > 0).all(), f"{where}: indices not strictly ascending"
    only_g = np.setdiff1d(g, r)
    only_r = np.setdiff1d(r, g)
    if only_g.size == 0:
        return 0
    n_cand = scores.shape[0] - n_forced
    picked = r[r < n_cand]
    kth = scores[picked].min()
    for j in np.concatenate([only_g, only_r]):
        assert 0 <= j < n_cand, f"{where}: index {j} outside the candidates"
        assert abs(scores[j] - kth) <= TIE_REL * kth, \
            f"{where}: index {j} score {scores[j]:.6e} is not within {TIE_REL} of the k-th score {kth:.6e}"
    # mass of the set is preserved
    assert scores[g].sum() >= (1.0 - TIE_REL) * scores[r].sum()
    return int(only_g.size)


def max_abs(a, b):
    return float(np.max(np.abs(np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64)))) if np.size(a) else 0.0
