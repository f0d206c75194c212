"""Host logic of the seeded input generators: determinism, shapes, budgets, hitter drift."""
import torch

from paper_2512_16391_amd import workloads


def test_budget_rule():
    assert workloads.budget(2048, 100) == 205            # ceil(0.1 * 2048)
    assert workloads.budget(32768, 100) == 3277
    assert workloads.budget(100, 100, 128) == 100        # never above the length
    assert workloads.budget(5000, 100, 128) == 500
    assert workloads.budget(1000, 100, 128) == 128       # the floor
    assert workloads.ceil_fraction(7, 500) == 4
    kpt = workloads.prefill_budgets(300, 32, 100, 24)
    assert len(kpt) == 10 and kpt[0] == 0                # tile 0 has no prefix
    assert kpt[1] == 24 and kpt[9] == 29                 # floor, then ceil(10 % of 288)
    assert all(k <= t * 32 for t, k in enumerate(kpt))


def test_config1_is_deterministic_and_shaped():
    a, b = workloads.config1(), workloads.config1()
    assert len(a.layers) == 2 and a.B == 1 and a.Hq == 8 and a.Hkv == 2 and a.d == 64
    assert a.seqlens == [2048] and a.k_per_seq == [205]
    for la, lb in zip(a.layers, b.layers):
        assert la.q.dtype == torch.float32 and la.k.shape == (1, 2, 2048, 64)
        assert torch.equal(la.q, lb.q) and torch.equal(la.k, lb.k) and torch.equal(la.v, lb.v)
    assert not torch.equal(a.layers[0].k, a.layers[1].k)


def test_hitters_drift_by_the_requested_overlap():
    wl = workloads.make_decode_workload("t", 99, 3, 2, 8, 2, 64, torch.float32, [500, 300], [50, 30], 40,
                                        [0.0, 0.75, 0.0])
    for b in range(2):
        for h in range(2):
            h0, h1, h2 = (set(wl.layers[l].hitters[b][h].tolist()) for l in range(3))
            assert len(h0) == len(h1) == len(h2) == 40
            assert len(h0 & h1) >= 30                        # 75 % kept (redraws may hit kept positions' neighbours only)
            assert len(h1 & h2) <= 15                        # a fresh draw: overlap only by chance
            assert max(h0 | h1 | h2) < [500, 300][b]


def test_layer_stack_and_permuted_heads():
    wl = workloads.layer_stack("cpu", n_layers=4, block_starts=(0, 2), B=1, seqlens=(400,), k=32, n_hitters=16)
    assert len(wl.layers) == 4
    same = len(set(wl.layers[0].hitters[0][0].tolist()) & set(wl.layers[1].hitters[0][0].tolist()))
    fresh = len(set(wl.layers[1].hitters[0][0].tolist()) & set(wl.layers[2].hitters[0][0].tolist()))
    assert same >= 14 and fresh <= 6
    perm = [1, 0]
    other = workloads.permuted_head_layer(wl.layers[0], perm, wl.Hq, noise=0.0)
    G = wl.Hq // wl.Hkv
    assert torch.equal(other.k[:, 0], wl.layers[0].k[:, 1]) and torch.equal(other.k[:, 1], wl.layers[0].k[:, 0])
    assert torch.equal(other.q[:, :G], wl.layers[0].q[:, G:2 * G])


def test_config5_layer_kinds():
    kinds = [workloads.config5_layer_kind(l) for l in range(32)]
    assert [l for l, (kind, _) in enumerate(kinds) if kind == "anchor"] == [0, 1, 4, 12, 20]
    assert kinds[2] == ("reuse", 1) and kinds[11] == ("reuse", 4) and kinds[31] == ("reuse", 20)
    assert sum(1 for kind, _ in kinds if kind == "reuse") == 27
