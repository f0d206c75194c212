"""GPU parity of the Pre-Softmax pooling variant (the alternative of Sec. 3.4): the pooling unit's query
vectors are averaged into one query and attention is scored once with it.  Against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import kascade_oracle as ko
from paper_2512_16391_amd import binding, workloads
from parity_utils import TOL_OUT, check_index_set, f64, max_abs

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
STORAGE = {torch.float32: "fp32", torch.bfloat16: "bf16"}


def i32(x):
    return torch.tensor(x, dtype=torch.int32, device=DEV)


@pytest.mark.parametrize("dtype,d,Hq,Hkv,W", [(torch.float32, 64, 8, 2, 0), (torch.bfloat16, 128, 32, 8, 0),
                                              (torch.bfloat16, 128, 8, 4, 16), (torch.float32, 128, 4, 1, 0),
                                              (torch.bfloat16, 64, 16, 2, 0), (torch.bfloat16, 128, 4, 4, 8)])
def test_decode_presoftmax(dtype, d, Hq, Hkv, W):
    print(f"case decode pre-softmax dtype={dtype} d={d} Hq={Hq} Hkv={Hkv} W={W}", flush=True)
    lens, ks = [1500, 333, 5049], [150, 40, 505]
    wl = workloads.make_decode_workload("presoftmax", 20, 2, 3, Hq, Hkv, d, dtype, lens, ks, 48, 0.8, recent_window=W,
                                        boost=6.0, q_boost=2.0)
    a, r = wl.layers
    Lmax, k_max = max(lens), max(ks)
    dev = lambda t: t.to(DEV)
    scale = ko.default_scale(d)
    swaps = 0
    for mode in (binding.KASCADE_OUT_SPARSE, binding.KASCADE_OUT_DENSE):
        idx, out = binding.kascade_decode_anchor_presoftmax(dev(a.q), dev(a.k), dev(a.v), i32(lens), i32(ks), Lmax, k_max,
                                                            recent_window=W, out_mode=mode)
        torch.cuda.synchronize()
        assert idx.shape == (3, Hkv, k_max)
        idx_h, out_h = idx.cpu().numpy(), f64(out)
        for b in range(3):
            L, k = lens[b], ks[b]
            ref_idx, pooled = ko.decode_presoftmax_indices(f64(a.q[b]), f64(a.k[b, :, :L]), scale, k, STORAGE[dtype], W)
            for hk in range(Hkv):
                swaps += check_index_set(idx_h[b, hk, :k], ref_idx[hk], pooled[hk], n_forced=W, where=f"seq {b} head {hk}")
            assert (idx_h[b, :, k:] == -1).all()
            if mode == binding.KASCADE_OUT_DENSE:
                want = ko.dense_decode(f64(a.q[b]), f64(a.k[b, :, :L]), f64(a.v[b, :, :L]), scale)
            else:
                want = ko.sparse_decode(f64(a.q[b]), f64(a.k[b, :, :L]), f64(a.v[b, :, :L]),
                                        [idx_h[b, hk, :k] for hk in range(Hkv)], scale)
            assert max_abs(out_h[b], want) <= TOL_OUT[dtype]
    print(f"  swapped members {swaps}", flush=True)
    # the sets feed the ordinary reuse call
    out = binding.kascade_decode_reuse(dev(r.q), dev(r.k), dev(r.v), i32(lens), i32(ks), k_max, idx)
    for b in range(3):
        L, k = lens[b], ks[b]
        want = ko.sparse_decode(f64(r.q[b]), f64(r.k[b, :, :L]), f64(r.v[b, :, :L]), [idx_h[b, hk, :k] for hk in range(Hkv)], scale)
        assert max_abs(f64(out)[b], want) <= TOL_OUT[dtype]


def test_decode_presoftmax_differs_from_post_softmax_pooling_and_agrees_for_single_head_groups():
    dtype, d = torch.bfloat16, 128
    lens, ks = [4000, 2500], [400, 250]
    for Hq, Hkv, expect_same in ((8, 2, False), (4, 4, True)):
        wl = workloads.make_decode_workload("pre-vs-post", 21, 1, 2, Hq, Hkv, d, dtype, lens, ks, 64, 0.8)
        a = wl.layers[0]
        args = (a.q.to(DEV), a.k.to(DEV), a.v.to(DEV), i32(lens), i32(ks), max(lens), max(ks))
        pre, _ = binding.kascade_decode_anchor_presoftmax(*args)
        post, _ = binding.kascade_decode_anchor(*args)
        torch.cuda.synchronize()
        assert torch.equal(pre, post) == expect_same


@pytest.mark.parametrize("S,Hq,Hkv,d,T", [(300, 8, 2, 128, 32), (200, 4, 2, 64, 64), (260, 2, 2, 64, 128), (1100, 8, 2, 128, 32),
                                          (520, 8, 2, 128, 128)])
@pytest.mark.parametrize("out_mode", [0, 1])
def test_prefill_presoftmax(S, Hq, Hkv, d, T, out_mode):
    print(f"case prefill pre-softmax S={S} Hq={Hq} Hkv={Hkv} d={d} T={T} out_mode={out_mode}", flush=True)
    g = torch.Generator().manual_seed(S + 9)
    q = torch.randn(S, Hq, d, generator=g).bfloat16()
    k = torch.randn(Hkv, S, d, generator=g).bfloat16()
    v = torch.randn(Hkv, S, d, generator=g).bfloat16()
    kpt = workloads.prefill_budgets(S, T, 100, 24)
    off = [0]
    for kt in kpt:
        off.append(off[-1] + kt)
    idx, out = binding.kascade_prefill_anchor_presoftmax(q.to(DEV), k.to(DEV), v.to(DEV), T, i32(kpt),
                                                         torch.tensor(off, dtype=torch.int64, device=DEV), off[-1],
                                                         out_mode=out_mode)
    torch.cuda.synchronize()
    assert idx.shape == (Hkv, max(off[-1], 1))
    idx_h, o = idx.cpu().numpy(), f64(out)
    Q, Kp, Vp = f64(q), f64(k), f64(v)
    scale = ko.default_scale(d)
    worst, swaps = 0.0, 0
    for t, kt in enumerate(kpt):
        lo, hi = ko.tile_bounds(t, T, S)
        mine = [idx_h[hk, off[t]:off[t] + kt] for hk in range(Hkv)]
        if kt > 0:
            ref_idx, pooled = ko.prefill_presoftmax_indices_tile(Q, Kp, t, T, scale, kt, "bf16")
            for hk in range(Hkv):
                swaps += check_index_set(mine[hk], ref_idx[hk], pooled[hk], where=f"tile {t} head {hk}")
        if out_mode == binding.KASCADE_OUT_DENSE:
            ref = ko.prefill_dense_tile(Q, Kp, Vp, t, T, scale)
        else:
            ref = ko.prefill_sparse_tile(Q, Kp, Vp, t, T, mine, scale)
        worst = max(worst, max_abs(o[lo:hi], ref))
    print(f"  max-abs {worst:.3e}, swapped members {swaps}", flush=True)
    assert worst <= TOL_OUT[torch.bfloat16]


def test_prefill_presoftmax_single_tile_prompt_and_argument_checks():
    # a prompt shorter than one tile has no candidates at all: dense attention, no sets
    S, Hq, Hkv, d, T = 20, 8, 2, 128, 32
    g = torch.Generator().manual_seed(3)
    q, k, v = (torch.randn(*s, generator=g).bfloat16() for s in ((S, Hq, d), (Hkv, S, d), (Hkv, S, d)))
    idx, out = binding.kascade_prefill_anchor_presoftmax(q.to(DEV), k.to(DEV), v.to(DEV), T, i32([0]),
                                                         torch.tensor([0, 0], dtype=torch.int64, device=DEV), 0)
    torch.cuda.synchronize()
    ref = ko.prefill_dense_tile(f64(q), f64(k), f64(v), 0, T, ko.default_scale(d))
    assert max_abs(f64(out), ref) <= TOL_OUT[torch.bfloat16]
    small = torch.empty(256, dtype=torch.uint8, device=DEV)
    S = 300
    q, k, v = (torch.randn(*s, generator=g).bfloat16() for s in ((S, Hq, d), (Hkv, S, d), (Hkv, S, d)))
    kpt = workloads.prefill_budgets(S, T, 100, 24)
    off = np.concatenate([[0], np.cumsum(kpt)]).tolist()
    with pytest.raises(binding.KascadeError) as e:
        binding.kascade_prefill_anchor_presoftmax(q.to(DEV), k.to(DEV), v.to(DEV), T, i32(kpt),
                                                  torch.tensor(off, dtype=torch.int64, device=DEV), off[-1], workspace=small)
    assert e.value.status == -4      # KASCADE_WORKSPACE_TOO_SMALL


def test_prefill_presoftmax_config4_size_sampled():
    """The prefill benchmark shape (S = 32768, T = 32, 32/8 heads, d 128): sampled tiles, all heads."""
    print("case prefill pre-softmax cfg4 size", flush=True)
    wl = workloads.config4(device=DEV, n_layers=1)
    a = wl.layers[0]
    off = wl.idx_offsets
    kpt_d = torch.tensor(wl.k_per_tile, dtype=torch.int32, device=DEV)
    off_d = torch.tensor(off, dtype=torch.int64, device=DEV)
    idx_d, out = binding.kascade_prefill_anchor_presoftmax(a.q, a.k, a.v, wl.T, kpt_d, off_d, off[-1])
    torch.cuda.synchronize()
    idx = idx_d.cpu().numpy()
    Q, Kp, Vp, o = f64(a.q), f64(a.k), f64(a.v), f64(out)
    scale = ko.default_scale(wl.d)
    swaps, worst = 0, 0.0
    for t in [0, 1, 8, 80, 81, 511, wl.n_tiles - 1]:
        kt = wl.k_per_tile[t]
        lo, hi = t * wl.T, (t + 1) * wl.T
        sets = [idx[h, off[t]:off[t] + kt] for h in range(wl.Hkv)]
        if kt:
            idx_ref, pooled = ko.prefill_presoftmax_indices_tile(Q, Kp, t, wl.T, scale, kt, "bf16")
            for h in range(wl.Hkv):
                swaps += check_index_set(sets[h], idx_ref[h], pooled[h], where=f"tile {t} head {h}")
        worst = max(worst, max_abs(o[lo:hi], ko.prefill_sparse_tile(Q, Kp, Vp, t, wl.T, sets, scale)))
        print(f"  tile {t} k_t={kt}: swaps {swaps}, worst max-abs {worst:.3e}", flush=True)
    assert worst <= TOL_OUT[torch.bfloat16]
    for t in range(1, wl.n_tiles, 53):
        for h in range(wl.Hkv):
            row = idx[h, off[t]:off[t + 1]]
            assert (np.diff(row) > 0).all() and row[0] >= 0 and row[-1] < t * wl.T
