"""GPU parity of the shared (all heads pooled) index-set variant of Sec. 3.5: one Top-k set per sequence
(decode) or per tile (prefill) for every head of the layer, against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import kascade_oracle as ko
from paper_2512_16391_amd import binding, workloads
from parity_utils import TOL_OUT, check_index_set, f64, max_abs

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def i32(x):
    return torch.tensor(x, dtype=torch.int32, device=DEV)


@pytest.mark.parametrize("dtype,d,Hq,Hkv,W", [(torch.float32, 64, 8, 2, 0), (torch.bfloat16, 128, 32, 8, 0),
                                              (torch.bfloat16, 128, 8, 4, 16), (torch.float32, 128, 4, 1, 0)])
def test_decode_shared_sets(dtype, d, Hq, Hkv, W):
    print(f"case decode shared dtype={dtype} d={d} Hq={Hq} Hkv={Hkv} W={W}", flush=True)
    lens, ks = [1500, 333, 2049], [150, 40, 205]
    wl = workloads.make_decode_workload("shared", 10, 2, 3, Hq, Hkv, d, dtype, lens, ks, 48, 0.8, recent_window=W,
                                        boost=6.0, q_boost=2.0)
    a, r = wl.layers
    Lmax, k_max = max(lens), max(ks)
    dev = lambda t: t.to(DEV)
    scale = ko.default_scale(d)
    for mode in (binding.KASCADE_OUT_SPARSE, binding.KASCADE_OUT_DENSE):
        idx, out = binding.kascade_decode_anchor_shared(dev(a.q), dev(a.k), dev(a.v), i32(lens), i32(ks), Lmax, k_max,
                                                        recent_window=W, out_mode=mode)
        assert idx.shape == (3, 1, k_max)
        idx_h, out_h = idx.cpu().numpy(), f64(out)
        for b in range(3):
            L, k = lens[b], ks[b]
            ref_idx, pooled = ko.decode_shared_indices(f64(a.q[b]), f64(a.k[b, :, :L]), scale, k, W)
            check_index_set(idx_h[b, 0, :k], ref_idx, pooled, n_forced=W, where=f"seq {b}")
            assert (idx_h[b, 0, k:] == -1).all()
            if mode == binding.KASCADE_OUT_DENSE:
                want = ko.dense_decode(f64(a.q[b]), f64(a.k[b, :, :L]), f64(a.v[b, :, :L]), scale)
            else:
                want = ko.sparse_decode(f64(a.q[b]), f64(a.k[b, :, :L]), f64(a.v[b, :, :L]), [idx_h[b, 0, :k]], scale,
                                        [0] * Hkv)
            assert max_abs(out_h[b], want) <= TOL_OUT[dtype]
    # a reuse layer driven by the shared set: n_anchor_heads = 1, every head mapped to set 0
    zero_map = i32([0] * Hkv)
    out = binding.kascade_decode_reuse(dev(r.q), dev(r.k), dev(r.v), i32(lens), i32(ks), k_max, idx, head_map=zero_map)
    for b in range(3):
        L, k = lens[b], ks[b]
        want = ko.sparse_decode(f64(r.q[b]), f64(r.k[b, :, :L]), f64(r.v[b, :, :L]), [idx_h[b, 0, :k]], scale, [0] * Hkv)
        assert max_abs(f64(out)[b], want) <= TOL_OUT[dtype]


@pytest.mark.parametrize("S,Hq,Hkv,d,T", [(300, 8, 2, 128, 32), (200, 4, 2, 64, 64), (260, 2, 2, 64, 128),
                                          (520, 8, 2, 128, 128)])
@pytest.mark.parametrize("out_mode", [0, 1])
def test_prefill_shared_sets(S, Hq, Hkv, d, T, out_mode):
    print(f"case prefill shared S={S} Hq={Hq} Hkv={Hkv} d={d} T={T} out_mode={out_mode}", flush=True)
    g = torch.Generator().manual_seed(S + 5)
    q = torch.randn(S, Hq, d, generator=g).bfloat16()
    k = torch.randn(Hkv, S, d, generator=g).bfloat16()
    v = torch.randn(Hkv, S, d, generator=g).bfloat16()
    kpt = workloads.prefill_budgets(S, T, 100, 24)
    off = [0]
    for kt in kpt:
        off.append(off[-1] + kt)
    idx, out = binding.kascade_prefill_anchor_shared(q.to(DEV), k.to(DEV), v.to(DEV), T, i32(kpt),
                                                     torch.tensor(off, dtype=torch.int64, device=DEV), off[-1],
                                                     out_mode=out_mode)
    torch.cuda.synchronize()
    assert idx.shape[0] == 1
    idx_h, o = idx.cpu().numpy(), f64(out)
    Q, Kp, Vp = f64(q), f64(k), f64(v)
    scale = ko.default_scale(d)
    worst = 0.0
    for t, kt in enumerate(kpt):
        lo, hi = ko.tile_bounds(t, T, S)
        mine = idx_h[0, off[t]:off[t] + kt]
        if kt > 0:
            ref_idx, pooled = ko.prefill_shared_indices_tile(Q, Kp, t, T, scale, kt)
            check_index_set(mine, ref_idx, pooled, where=f"tile {t}")
        if out_mode == binding.KASCADE_OUT_DENSE:
            ref = ko.prefill_dense_tile(Q, Kp, Vp, t, T, scale)
        else:
            ref = ko.prefill_sparse_tile(Q, Kp, Vp, t, T, [mine], scale, [0] * Hkv)
        worst = max(worst, max_abs(o[lo:hi], ref))
    print(f"  max-abs {worst:.3e}", flush=True)
    assert worst <= TOL_OUT[torch.bfloat16]
    # reuse layer with the shared sets
    out_r = binding.kascade_prefill_reuse(q.to(DEV), k.to(DEV), v.to(DEV), T, i32(kpt),
                                          torch.tensor(off, dtype=torch.int64, device=DEV), off[-1], idx,
                                          head_map=i32([0] * Hkv), n_anchor_heads=1)
    o_r = f64(out_r)
    for t, kt in enumerate(kpt):
        lo, hi = ko.tile_bounds(t, T, S)
        ref = ko.prefill_sparse_tile(Q, Kp, Vp, t, T, [idx_h[0, off[t]:off[t] + kt]], scale, [0] * Hkv)
        assert max_abs(o_r[lo:hi], ref) <= TOL_OUT[torch.bfloat16]
