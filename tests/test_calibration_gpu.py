"""GPU parity of the calibration path (Sec. 3.3): pooled distributions, Top-k set similarity
(Eq. 3) and the anchor layers chosen from the resulting matrix, against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import kascade_oracle as ko
from paper_2512_16391_amd import binding, workloads
from parity_utils import f64

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def i32(x):
    return torch.tensor(x, dtype=torch.int32, device=DEV)


def oracle_layer(layer, wl):
    """Per (sequence, key head) pooled distribution and Top-k set of one layer."""
    pooled, sets = [], []
    for b in range(wl.B):
        L, k = wl.seqlens[b], wl.k_per_seq[b]
        idx, a = ko.decode_anchor_indices(f64(layer.q[b]), f64(layer.k[b, :, :L]), ko.default_scale(wl.d), k)
        pooled.append(a)
        sets.append(idx)
    return pooled, sets


@pytest.mark.parametrize("dtype,tol", [(torch.float32, 2e-5), (torch.bfloat16, 2e-5)])
def test_similarity_matrix_and_anchor_choice(dtype, tol):
    print(f"case calibration stack dtype={dtype}", flush=True)
    starts = (0, 3, 5)
    wl = workloads.layer_stack("cpu", n_layers=8, block_starts=starts, dtype=dtype)
    n, B, Hkv = len(wl.layers), wl.B, wl.Hkv
    Lmax, k_max = max(wl.seqlens), max(wl.k_per_seq)
    lens, ks = i32(wl.seqlens), i32(wl.k_per_seq)

    # device: pooled distribution and fresh Top-k set of every layer
    pooled_d, idx_d = [], []
    for layer in wl.layers:
        q, k, v = layer.q.to(DEV), layer.k.to(DEV), layer.v.to(DEV)
        pooled_d.append(binding.kascade_decode_pooled(q, k, lens, Lmax))
        idx, _ = binding.kascade_decode_anchor(q, k, v, lens, ks, Lmax, k_max)
        idx_d.append(idx)
    # oracle: the same, from the definition
    ref = [oracle_layer(layer, wl) for layer in wl.layers]
    for l in range(n):
        for b in range(B):
            L = wl.seqlens[b]
            got = pooled_d[l][b, :, :L].double().cpu().numpy()
            assert np.abs(got - ref[l][0][b]).max() <= 1e-6 + 1e-4 * ref[l][0][b].max(), (l, b)

    # similarity matrix: minimum over the (sequence, key head) samples, per layer pair
    S_dev = np.zeros((n, n), dtype=np.float32)
    S_ref = np.zeros((n, n))
    for a in range(n):
        for b_ in range(a, n):
            smin = torch.ones(1, dtype=torch.float32, device=DEV)
            sim, _ = binding.kascade_topk_similarity(pooled_d[b_], lens, ks, idx_d[a], idx_d[b_], sim_min=smin)
            sim = sim.cpu().numpy()
            want = np.array([[ko.topk_similarity(ref[b_][0][s][h], ref[a][1][s][h], ref[b_][1][s][h])
                              for h in range(Hkv)] for s in range(B)])
            assert np.abs(sim - want).max() <= tol, (a, b_, np.abs(sim - want).max())
            assert float(smin.item()) == float(sim.min())
            S_dev[a, b_], S_ref[a, b_] = smin.item(), want.min()
    np.testing.assert_allclose(np.diag(S_dev), 1.0, atol=1e-6)
    # block structure of the recipe shows up: inside a block high, across blocks low
    assert S_dev[0, 2] > 0.6 and S_dev[3, 4] > 0.6 and S_dev[5, 7] > 0.6
    assert S_dev[0, 3] < 0.3 and S_dev[2, 5] < 0.3

    got, obj = binding.kascade_select_anchor_layers(S_dev, len(starts))
    want = ko.select_anchor_layers(S_ref, len(starts))
    assert got == want == list(starts)
    np.testing.assert_allclose(obj, ko.segment_score(S_ref, want), atol=n * tol)


def test_similarity_with_head_map_partial_sets_and_running_minimum():
    print("case similarity head map", flush=True)
    rs = np.random.default_rng(5)
    B, Hkv, Ha, pitch, k_max = 3, 4, 2, 1000, 96
    lens, ks = [1000, 37, 512], [96, 5, 0]
    pooled = rs.random((B, Hkv, pitch)).astype(np.float32)
    idx_a = np.full((B, Ha, k_max), -1, dtype=np.int32)
    idx_b = np.full((B, Hkv, k_max), -1, dtype=np.int32)
    for b in range(B):
        for h in range(Ha):
            idx_a[b, h, : ks[b]] = rs.choice(lens[b], ks[b], replace=False)
        for h in range(Hkv):
            idx_b[b, h, : ks[b]] = rs.choice(lens[b], ks[b], replace=False)
    idx_a[0, 1, 3] = -1          # ignored entries: negative and beyond the sequence
    idx_a[0, 0, 7] = 5000
    head_map = [1, 0, 0, 1]
    smin = torch.full((1,), 0.25, dtype=torch.float32, device=DEV)
    sim, _ = binding.kascade_topk_similarity(torch.from_numpy(pooled).to(DEV), i32(lens), i32(ks),
                                             torch.from_numpy(idx_a).to(DEV), torch.from_numpy(idx_b).to(DEV),
                                             head_map=i32(head_map), sim_min=smin)
    sim = sim.cpu().numpy()
    for b in range(B):
        for h in range(Hkv):
            ia = [j for j in idx_a[b, head_map[h], : ks[b]] if 0 <= j < lens[b]]
            ib = idx_b[b, h, : ks[b]]
            want = 1.0 if ks[b] == 0 else ko.topk_similarity(pooled[b, h].astype(np.float64), np.array(ia, dtype=np.int64), ib)
            assert abs(sim[b, h] - want) <= 1e-5 * max(1.0, want), (b, h, sim[b, h], want)
    assert smin.item() == min(0.25, float(sim.min()))


def test_calibration_entries_reject_bad_arguments():
    q = torch.zeros(1, 8, 64, device=DEV)
    k = torch.zeros(1, 2, 128, 64, device=DEV)
    lens = i32([128])
    with pytest.raises(binding.KascadeError):       # pitch shorter than the sequence bound
        binding.kascade_decode_pooled(q, k, lens, 128, pooled_out=torch.zeros(1, 2, 64, device=DEV))
    with pytest.raises(binding.KascadeError):       # workspace too small
        binding.kascade_decode_pooled(q, k, lens, 128, workspace=torch.zeros(256, dtype=torch.uint8, device=DEV))
    pooled = torch.zeros(1, 2, 128, device=DEV)
    idx = torch.zeros(1, 2, 8, dtype=torch.int32, device=DEV)
    idx3 = torch.zeros(1, 3, 8, dtype=torch.int32, device=DEV)
    with pytest.raises(binding.KascadeError):       # head counts differ and no head map
        binding.kascade_topk_similarity(pooled, lens, i32([8]), idx3, idx)


def test_head_map_from_planted_head_permutation_and_reuse_with_it():
    print("case head map calibration", flush=True)
    wl = workloads.layer_stack("cpu", n_layers=1, block_starts=(0,), B=4, Hq=16, Hkv=4, d=64,
                               seqlens=(2000, 1500, 1800, 777), k=64, n_hitters=24)
    perm = [2, 0, 3, 1]
    anchor = wl.layers[0]
    reuse = workloads.permuted_head_layer(anchor, perm, wl.Hq)
    lens, ks = i32(wl.seqlens), i32(wl.k_per_seq)
    Lmax, k_max = max(wl.seqlens), max(wl.k_per_seq)
    dev = lambda t: t.to(DEV)
    idx_a, _ = binding.kascade_decode_anchor(dev(anchor.q), dev(anchor.k), dev(anchor.v), lens, ks, Lmax, k_max)
    idx_b, _ = binding.kascade_decode_anchor(dev(reuse.q), dev(reuse.k), dev(reuse.v), lens, ks, Lmax, k_max)
    pooled_b = binding.kascade_decode_pooled(dev(reuse.q), dev(reuse.k), lens, Lmax)
    sim = binding.kascade_head_similarity(pooled_b, lens, ks, idx_a, idx_b)
    head_map, mean = binding.kascade_head_map(sim)

    # oracle: same quantities from the definitions
    ref_a = oracle_layer(anchor, wl)
    ref_b = oracle_layer(reuse, wl)
    sims = np.stack([ko.head_similarity(ref_b[0][s], ref_a[1][s], ref_b[1][s]) for s in range(wl.B)])
    hm_ref, mean_ref = ko.head_map_from_similarity(sims)
    assert np.abs(sim.cpu().numpy() - sims).max() <= 2e-5
    assert np.abs(mean.cpu().numpy() - mean_ref).max() <= 2e-5
    assert head_map.cpu().tolist() == hm_ref.tolist() == perm

    # the calibrated map drives a reuse layer: parity with the oracle under the same map
    out = binding.kascade_decode_reuse(dev(reuse.q), dev(reuse.k), dev(reuse.v), lens, ks, k_max, idx_a,
                                       head_map=head_map)
    idx_host = idx_a.cpu().numpy()
    for s in range(wl.B):
        L = wl.seqlens[s]
        sets = [idx_host[s, h, : wl.k_per_seq[s]] for h in range(wl.Hkv)]
        want = ko.sparse_decode(f64(reuse.q[s]), f64(reuse.k[s, :, :L]), f64(reuse.v[s, :, :L]), sets,
                                ko.default_scale(wl.d), perm)
        assert np.abs(out[s].double().cpu().numpy() - want).max() <= 1e-4


@pytest.mark.parametrize("dtype,tol", [(torch.float32, 1e-5), (torch.bfloat16, 1e-5)])
def test_layer_importance_matches_oracle(dtype, tol):
    print(f"case layer importance {dtype}", flush=True)
    g = torch.Generator().manual_seed(9)
    n_rows, n_cols = 1029, 4096
    x = torch.randn(n_rows, n_cols, generator=g)
    y = (x * torch.linspace(0, 1, n_rows)[:, None] + torch.randn(n_rows, n_cols, generator=g) * 0.5)
    x, y = x.to(dtype), y.to(dtype)
    y[3] = x[3] * 2          # parallel rows: importance 0
    y[4] = -x[4]             # opposite rows: importance 2
    w = binding.kascade_layer_importance(x.to(DEV), y.to(DEV)).double().cpu().numpy()
    want = ko.layer_importance(f64(x), f64(y))
    assert np.abs(w - want).max() <= tol, np.abs(w - want).max()
    assert abs(w[3]) <= tol and abs(w[4] - 2.0) <= tol
    # strided rows (a column slice of a wider tensor)
    wide = torch.randn(64, 512, generator=g).to(dtype).to(DEV)
    w2 = binding.kascade_layer_importance(wide[:, :200], wide[:, 256:456]).double().cpu().numpy()
    want2 = ko.layer_importance(f64(wide[:, :200].cpu()), f64(wide[:, 256:456].cpu()))
    assert np.abs(w2 - want2).max() <= tol


def test_config5_anchor_layers_emerge_from_planted_drift():
    """A 32-layer stack whose heavy-hitter positions are redrawn at layers 0, 1, 4, 12 and 20 and drift
    slowly (5 % per layer) in between: the similarity matrix measured on the GPU path (pooled distributions,
    Top-k sets, Eq. 3 with the minimum over the samples) makes Algorithm 1 return the configuration's anchor
    layers {0, 1, 4, 12, 20} for five anchors - from the library's host routine and from the oracle's."""
    print("case config5 anchors from planted drift", flush=True)
    starts = workloads.CONFIG5_ANCHORS
    wl = workloads.layer_stack("cpu", n_layers=32, block_starts=starts, B=1, Hq=8, Hkv=2, d=64,
                               seqlens=(2000,), k=64, n_hitters=32, within=0.95)
    n, Hkv = len(wl.layers), wl.Hkv
    Lmax, k_max = max(wl.seqlens), max(wl.k_per_seq)
    lens, ks = i32(wl.seqlens), i32(wl.k_per_seq)
    pooled_d, idx_d = [], []
    for layer in wl.layers:
        q, k, v = layer.q.to(DEV), layer.k.to(DEV), layer.v.to(DEV)
        pooled_d.append(binding.kascade_decode_pooled(q, k, lens, Lmax))
        idx_d.append(binding.kascade_decode_anchor(q, k, v, lens, ks, Lmax, k_max)[0])
    ref = [oracle_layer(layer, wl) for layer in wl.layers]
    S_dev = np.zeros((n, n), dtype=np.float32)
    S_ref = np.zeros((n, n))
    for a in range(n):
        for b_ in range(a, n):
            smin = torch.ones(1, dtype=torch.float32, device=DEV)
            binding.kascade_topk_similarity(pooled_d[b_], lens, ks, idx_d[a], idx_d[b_], sim_min=smin)
            S_dev[a, b_] = smin.item()
            S_ref[a, b_] = min(ko.topk_similarity(ref[b_][0][0][h], ref[a][1][0][h], ref[b_][1][0][h]) for h in range(Hkv))
    assert np.abs(S_dev - S_ref).max() <= 2e-5
    got, obj = binding.kascade_select_anchor_layers(S_dev, len(starts))
    want = ko.select_anchor_layers(S_ref, len(starts))
    print(f"  anchors {got}, objective {obj:.3f}", flush=True)
    assert got == want == list(starts)
