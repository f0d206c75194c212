"""GPU parity of the prefill entry points against the CPU oracle, tile by tile."""
import numpy as np
import pytest
import torch

from oracle import kascade_oracle as ko
from paper_2512_16391_amd import binding, workloads
from parity_utils import TOL_OUT, check_index_set, f64, max_abs

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
BF16 = torch.bfloat16


def dev_i32(x):
    return torch.tensor(x, dtype=torch.int32, device=DEV)


def dev_i64(x):
    return torch.tensor(x, dtype=torch.int64, device=DEV)


def random_prefill(seed, S, Hq, Hkv, d, dtype=BF16):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(S, Hq, d, generator=g).to(dtype)
    k = torch.randn(Hkv, S, d, generator=g).to(dtype)
    v = torch.randn(Hkv, S, d, generator=g).to(dtype)
    return q, k, v


def offsets(k_per_tile):
    off = [0]
    for kt in k_per_tile:
        off.append(off[-1] + kt)
    return off


def run_anchor(q, k, v, T, k_per_tile, out_mode, tiles=None, where=""):
    """Runs kascade_prefill_anchor and checks the listed tiles (all by default)."""
    S, Hq, d = q.shape
    Hkv = k.shape[0]
    off = offsets(k_per_tile)
    idx, out = binding.kascade_prefill_anchor(q.to(DEV), k.to(DEV), v.to(DEV), T, dev_i32(k_per_tile), dev_i64(off),
                                              off[-1], out_mode=out_mode)
    torch.cuda.synchronize()
    idx = idx.cpu().numpy()
    o = f64(out)
    Q, Kp, Vp = f64(q), f64(k), f64(v)
    scale = ko.default_scale(d)
    n_tiles = len(k_per_tile)
    swaps, worst = 0, 0.0
    for t in (tiles if tiles is not None else range(n_tiles)):
        kt = k_per_tile[t]
        lo, hi = ko.tile_bounds(t, T, S)
        sets = [idx[h, off[t]:off[t] + kt] for h in range(Hkv)]
        if kt > 0:
            idx_ref, a = ko.prefill_anchor_indices_tile(Q, Kp, t, T, scale, kt)
            for h in range(Hkv):
                swaps += check_index_set(sets[h], idx_ref[h], a[h], where=f"{where} tile {t} head {h}")
        if out_mode == binding.KASCADE_OUT_DENSE:
            ref = ko.prefill_dense_tile(Q, Kp, Vp, t, T, scale)
        else:
            ref = ko.prefill_sparse_tile(Q, Kp, Vp, t, T, sets, scale)
        worst = max(worst, max_abs(o[lo:hi], ref))
    print(f"  {where}: swaps {swaps}, max-abs {worst:.3e}", flush=True)
    assert worst <= TOL_OUT[q.dtype]
    return idx, out


@pytest.mark.parametrize("S,Hq,Hkv,d,T", [
    (300, 8, 2, 128, 32),      # ragged last tile (12 tokens), G = 4
    (260, 2, 2, 64, 128),      # G = 1, tiles of 128 tokens
    (200, 4, 2, 128, 64),      # G = 2
    (100, 8, 1, 64, 16),       # G = 8, tiles of 16 tokens
])
@pytest.mark.parametrize("out_mode", [0, 1])
def test_prefill_anchor_small(S, Hq, Hkv, d, T, out_mode):
    print(f"case prefill anchor S={S} Hq={Hq} Hkv={Hkv} d={d} T={T} out_mode={out_mode}", flush=True)
    q, k, v = random_prefill(S, S, Hq, Hkv, d)
    kpt = workloads.prefill_budgets(S, T, 100, 24)
    run_anchor(q, k, v, T, kpt, out_mode, where=f"S{S}")


@pytest.mark.parametrize("S,Hq,Hkv,d,T", [
    (700, 8, 2, 128, 128),     # 512 rows per tile (four workgroups), last tile 60 tokens = two parts, the second ragged
    (500, 4, 2, 128, 128),     # G = 2: 256 rows, last tile 116 tokens
    (600, 2, 2, 64, 256),      # G = 1: 256 rows, tiles of 256 tokens
    (330, 16, 2, 64, 64),      # G = 8: 512 rows, parts of 16 tokens
])
@pytest.mark.parametrize("out_mode", [0, 1])
def test_prefill_anchor_tiles_larger_than_one_workgroup(S, Hq, Hkv, d, T, out_mode):
    """Tiles of 256 and 512 (token, head) rows: one index set per tile, pooled over all of its rows,
    shared by the two or four workgroups that attend for it; then a reuse layer on the same sets."""
    print(f"case prefill large tiles S={S} Hq={Hq} Hkv={Hkv} d={d} T={T} out_mode={out_mode}", flush=True)
    q, k, v = random_prefill(S + 1, S, Hq, Hkv, d)
    kpt = workloads.prefill_budgets(S, T, 150, 40)
    idx, _ = run_anchor(q, k, v, T, kpt, out_mode, where=f"S{S} T{T}")
    q2, k2, v2 = random_prefill(S + 2, S, Hq, Hkv, d)
    off = offsets(kpt)
    out = binding.kascade_prefill_reuse(q2.to(DEV), k2.to(DEV), v2.to(DEV), T, dev_i32(kpt), dev_i64(off), off[-1],
                                        torch.from_numpy(idx).to(DEV))
    torch.cuda.synchronize()
    Q, Kp, Vp, o = f64(q2), f64(k2), f64(v2), f64(out)
    for t, kt in enumerate(kpt):
        lo, hi = ko.tile_bounds(t, T, S)
        ref = ko.prefill_sparse_tile(Q, Kp, Vp, t, T, [idx[h, off[t]:off[t] + kt] for h in range(Hkv)], ko.default_scale(d))
        assert max_abs(o[lo:hi], ref) <= TOL_OUT[BF16]


def test_prefill_anchor_tile_reduces_to_dense_when_k_covers_prefix():
    # k_t = whole prefix for every tile: the sparse output must equal dense causal attention
    S, Hq, Hkv, d, T = 256, 8, 2, 128, 32
    q, k, v = random_prefill(7, S, Hq, Hkv, d)
    kpt = [t * T for t in range(S // T)]
    off = offsets(kpt)
    idx, out = binding.kascade_prefill_anchor(q.to(DEV), k.to(DEV), v.to(DEV), T, dev_i32(kpt), dev_i64(off), off[-1],
                                              out_mode=binding.KASCADE_OUT_SPARSE)
    _, dense = binding.kascade_prefill_anchor(q.to(DEV), k.to(DEV), v.to(DEV), T, dev_i32(kpt), dev_i64(off), off[-1],
                                              out_mode=binding.KASCADE_OUT_DENSE)
    torch.cuda.synchronize()
    idx = idx.cpu().numpy()
    for t in range(S // T):
        for h in range(Hkv):
            np.testing.assert_array_equal(idx[h, off[t]:off[t + 1]], np.arange(t * T))
    Q, Kp, Vp = f64(q), f64(k), f64(v)
    for t in range(S // T):
        ref = ko.prefill_dense_tile(Q, Kp, Vp, t, T, ko.default_scale(d))
        assert max_abs(f64(out)[t * T:(t + 1) * T], ref) <= TOL_OUT[BF16]
        assert max_abs(f64(dense)[t * T:(t + 1) * T], ref) <= TOL_OUT[BF16]


def test_prefill_reuse_head_map_and_ignored_entries():
    S, Hq, Hkv, d, T = 330, 16, 4, 128, 32
    q, k, v = random_prefill(11, S, Hq, Hkv, d)
    n_tiles = (S + T - 1) // T
    rs = np.random.default_rng(12)
    n_anchor = 2
    hm = [1, 0, 0, 1]
    kpt = [min(t * T, 40) for t in range(n_tiles)]
    off = offsets(kpt)
    idx = np.full((n_anchor, max(off[-1], 1)), -1, dtype=np.int32)
    sets = {}
    for t in range(n_tiles):
        sets[t] = []
        for h in range(n_anchor):
            kt = kpt[t]
            if kt == 0:
                sets[t].append(np.zeros(0, np.int64))
                continue
            good = rs.permutation(rs.choice(t * T, kt - 2 if kt > 2 else kt, replace=False))     # unordered
            row = np.concatenate([good[:1], [-1, t * T + 5][: kt - good.size], good[1:]])           # 2 entries to ignore
            idx[h, off[t]:off[t] + kt] = row
            sets[t].append(good)
    out = binding.kascade_prefill_reuse(q.to(DEV), k.to(DEV), v.to(DEV), T, dev_i32(kpt), dev_i64(off), off[-1],
                                        torch.from_numpy(idx).to(DEV), head_map=dev_i32(hm))
    torch.cuda.synchronize()
    Q, Kp, Vp = f64(q), f64(k), f64(v)
    o = f64(out)
    worst = 0.0
    for t in range(n_tiles):
        lo, hi = ko.tile_bounds(t, T, S)
        ref = ko.prefill_sparse_tile(Q, Kp, Vp, t, T, sets[t], ko.default_scale(d), head_map=hm)
        worst = max(worst, max_abs(o[lo:hi], ref))
    print(f"  reuse max-abs {worst:.3e}", flush=True)
    assert worst <= TOL_OUT[BF16]
    # deterministic
    out2 = binding.kascade_prefill_reuse(q.to(DEV), k.to(DEV), v.to(DEV), T, dev_i32(kpt), dev_i64(off), off[-1],
                                         torch.from_numpy(idx).to(DEV), head_map=dev_i32(hm))
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


def test_prefill_config4_shape_reduced_length():
    """Config-4 recipe (32/8 heads, d 128, T = 32, 10 % with a floor of 256, planted hitters) at
    S = 4096: anchor then a reuse layer, every tile against the oracle."""
    print("case prefill cfg4 reduced", flush=True)
    wl = workloads.config4(device="cpu", n_layers=2, S=4096)
    a, r = wl.layers
    tiles = list(range(0, wl.n_tiles, 5)) + [7, 8, 9, 79, 80, 81, wl.n_tiles - 1]    # includes the k_min boundary
    idx, _ = run_anchor(a.q, a.k, a.v, wl.T, wl.k_per_tile, binding.KASCADE_OUT_SPARSE, tiles=sorted(set(tiles)),
                        where="cfg4-S4096 anchor")
    off = wl.idx_offsets
    out = binding.kascade_prefill_reuse(r.q.to(DEV), r.k.to(DEV), r.v.to(DEV), wl.T, dev_i32(wl.k_per_tile),
                                        dev_i64(off), off[-1], torch.from_numpy(idx).to(DEV))
    torch.cuda.synchronize()
    Q, Kp, Vp = f64(r.q), f64(r.k), f64(r.v)
    o = f64(out)
    worst = 0.0
    for t in sorted(set(tiles)):
        sets = [idx[h, off[t]:off[t + 1]] for h in range(wl.Hkv)]
        ref = ko.prefill_sparse_tile(Q, Kp, Vp, t, wl.T, sets, ko.default_scale(wl.d))
        worst = max(worst, max_abs(o[t * wl.T:(t + 1) * wl.T], ref))
    print(f"  cfg4-S4096 reuse max-abs {worst:.3e}", flush=True)
    assert worst <= TOL_OUT[BF16]


def test_prefill_rejects_unsupported():
    q, k, v = random_prefill(1, 64, 8, 2, 128)
    kpt, off = [0, 0], [0, 0, 0]
    with pytest.raises(binding.KascadeError) as e:      # T * G must be a multiple of 128 (here 64)
        binding.kascade_prefill_anchor(q.to(DEV), k.to(DEV), v.to(DEV), 16, dev_i32([0] * 4), dev_i64([0] * 5), 0)
    assert e.value.status == -2
    with pytest.raises(binding.KascadeError) as e:      # 192 rows
        binding.kascade_prefill_anchor(q.to(DEV), k.to(DEV), v.to(DEV), 48, dev_i32([0] * 2), dev_i64([0] * 3), 0)
    assert e.value.status == -2
    with pytest.raises(binding.KascadeError) as e:      # fp32 prefill is not built
        binding.kascade_prefill_anchor(q.float().to(DEV), k.float().to(DEV), v.float().to(DEV), 32, dev_i32(kpt),
                                       dev_i64(off), 0)
    assert e.value.status == -2


def test_prefill_config4_full_size_sampled():
    """The prefill benchmark configuration itself (S = 32768, T = 32, 32/8 heads, d 128), generated on
    the GPU as bench.py does: anchor (sparse output) then one reuse layer; sampled tiles (first
    tiles, the k_min boundary, the last tile, a few in between) against the oracle, all heads."""
    print("case prefill cfg4 full size", flush=True)
    wl = workloads.config4(device=DEV, n_layers=2)
    a, r = wl.layers
    off = wl.idx_offsets
    kpt_d, off_d = dev_i32(wl.k_per_tile), dev_i64(off)
    idx_d, out_a = binding.kascade_prefill_anchor(a.q, a.k, a.v, wl.T, kpt_d, off_d, off[-1])
    out_r = binding.kascade_prefill_reuse(r.q, r.k, r.v, wl.T, kpt_d, off_d, off[-1], idx_d)
    torch.cuda.synchronize()
    idx = idx_d.cpu().numpy()
    tiles = [0, 1, 2, 8, 79, 80, 81, 300, 511, 777, wl.n_tiles - 1]
    scale = ko.default_scale(wl.d)
    Qa, Ka, Va = f64(a.q), f64(a.k), f64(a.v)
    Qr, Kr, Vr = f64(r.q), f64(r.k), f64(r.v)
    oa, orr = f64(out_a), f64(out_r)
    swaps, worst = 0, 0.0
    for t in tiles:
        kt = wl.k_per_tile[t]
        lo, hi = t * wl.T, (t + 1) * wl.T
        sets = [idx[h, off[t]:off[t] + kt] for h in range(wl.Hkv)]
        if kt:
            idx_ref, pooled = ko.prefill_anchor_indices_tile(Qa, Ka, t, wl.T, scale, kt)
            for h in range(wl.Hkv):
                swaps += check_index_set(sets[h], idx_ref[h], pooled[h], where=f"cfg4 tile {t} head {h}")
        worst = max(worst, max_abs(oa[lo:hi], ko.prefill_sparse_tile(Qa, Ka, Va, t, wl.T, sets, scale)))
        worst = max(worst, max_abs(orr[lo:hi], ko.prefill_sparse_tile(Qr, Kr, Vr, t, wl.T, sets, scale)))
        print(f"  cfg4 tile {t} k_t={kt}: swaps {swaps}, worst max-abs {worst:.3e}", flush=True)
    assert worst <= TOL_OUT[BF16]
    # every tile: ascending, in range
    for t in range(1, wl.n_tiles, 37):
        for h in range(wl.Hkv):
            row = idx[h, off[t]:off[t + 1]]
            assert (np.diff(row) > 0).all() and row[0] >= 0 and row[-1] < t * wl.T


def test_config5_shape_prefill_131072_then_decode():
    """Largest configuration: 32/8 heads, d 128, bf16, causal prefill of 131072 tokens (k_t = 10 % of
    the prefix, 4096 tiles, 26.8 M indices per key head, 8.6 GB of pooled scores), layers 0 (dense-output
    anchor), 1 (anchor) and 2 (reuses layer 1), then two decode steps on the same caches at
    L = 131073, 131074 (k = 10 %).  Sampled tiles / all decode outputs against the oracle."""
    print("case cfg5 S=131072", flush=True)
    S, T, steps = 131072, 32, 2
    wl = workloads.config5_prefill(device=DEV, layers=(0, 1, 2), S=S, T=T, decode_steps=steps)
    off = wl.idx_offsets
    kpt_d, off_d = dev_i32(wl.k_per_tile), dev_i64(off)
    l0, l1, l2 = wl.layers
    kv = lambda layer: (layer.k[:, :S], layer.v[:, :S])
    scale = ko.default_scale(wl.d)
    tiles = [1, 2047, wl.n_tiles - 1]

    def check_tiles(layer, out, sets_of, dense, where):
        Q, Kp, Vp = f64(layer.q), f64(layer.k[:, :S]), f64(layer.v[:, :S])
        o = None
        worst = 0.0
        for t in tiles:
            lo, hi = t * T, (t + 1) * T
            ref = ko.prefill_dense_tile(Q, Kp, Vp, t, T, scale) if dense else \
                ko.prefill_sparse_tile(Q, Kp, Vp, t, T, sets_of(t), scale)
            worst = max(worst, max_abs(f64(out[lo:hi]), ref))
            print(f"  {where} tile {t}: worst max-abs {worst:.3e}", flush=True)
        assert worst <= TOL_OUT[BF16]
        return Q, Kp

    # layer 0: anchor with dense output
    k0, v0 = kv(l0)
    idx0, out0 = binding.kascade_prefill_anchor(l0.q, k0, v0, T, kpt_d, off_d, off[-1], out_mode=binding.KASCADE_OUT_DENSE)
    torch.cuda.synchronize()
    check_tiles(l0, out0, None, True, "layer0 dense")
    del idx0, out0
    # layer 1: anchor with sparse output, index sets against the oracle on the sampled tiles
    k1, v1 = kv(l1)
    idx1, out1 = binding.kascade_prefill_anchor(l1.q, k1, v1, T, kpt_d, off_d, off[-1])
    torch.cuda.synchronize()
    sets_of = lambda t: [idx1[h, off[t]:off[t + 1]].cpu().numpy() for h in range(wl.Hkv)]
    Q1, K1 = check_tiles(l1, out1, sets_of, False, "layer1 anchor")
    swaps = 0
    for t in tiles:
        idx_ref, pooled = ko.prefill_anchor_indices_tile(Q1, K1, t, T, scale, wl.k_per_tile[t])
        got = sets_of(t)
        for h in range(wl.Hkv):
            swaps += check_index_set(got[h], idx_ref[h], pooled[h], where=f"cfg5 tile {t} head {h}")
    print(f"  layer1 index sets: swaps {swaps}", flush=True)
    del Q1, K1, out1
    # layer 2: reuse of layer 1's sets
    k2, v2 = kv(l2)
    out2 = binding.kascade_prefill_reuse(l2.q, k2, v2, T, kpt_d, off_d, off[-1], idx1)
    torch.cuda.synchronize()
    check_tiles(l2, out2, sets_of, False, "layer2 reuse")
    del out2, idx1

    # decode steps appended to the same caches: layer 1 as anchor, layer 2 reusing its set
    g = torch.Generator(device=DEV).manual_seed(777)
    for step in range(steps):
        L = S + step + 1
        kk = workloads.budget(L, 100)
        newq = torch.randn(2, 1, wl.Hq, wl.d, generator=g, device=DEV).to(BF16)
        for layer in (l1, l2):
            layer.k[:, L - 1] = torch.randn(wl.Hkv, wl.d, generator=g, device=DEV).to(BF16)
            layer.v[:, L - 1] = torch.randn(wl.Hkv, wl.d, generator=g, device=DEV).to(BF16)
        sl, kp = dev_i32([L]), dev_i32([kk])
        kc1, vc1 = l1.k[None, :, :L], l1.v[None, :, :L]
        kc2, vc2 = l2.k[None, :, :L], l2.v[None, :, :L]
        idx_d, o1 = binding.kascade_decode_anchor(newq[0], kc1, vc1, sl, kp, L, kk)
        o2 = binding.kascade_decode_reuse(newq[1], kc2, vc2, sl, kp, kk, idx_d)
        torch.cuda.synchronize()
        idx_np = idx_d.cpu().numpy()
        idx_ref, pooled = ko.decode_anchor_indices(f64(newq[0, 0]), f64(kc1[0]), scale, kk)
        sw = sum(check_index_set(idx_np[0, h], idx_ref[h], pooled[h], where=f"cfg5 decode step {step} head {h}")
                 for h in range(wl.Hkv))
        sets = [idx_np[0, h] for h in range(wl.Hkv)]
        e1 = max_abs(f64(o1[0]), ko.sparse_decode(f64(newq[0, 0]), f64(kc1[0]), f64(vc1[0]), sets, scale))
        e2 = max_abs(f64(o2[0]), ko.sparse_decode(f64(newq[1, 0]), f64(kc2[0]), f64(vc2[0]), sets, scale))
        print(f"  decode step {step} L={L} k={kk}: swaps {sw}, max-abs anchor {e1:.3e} reuse {e2:.3e}", flush=True)
        assert max(e1, e2) <= TOL_OUT[BF16]


def test_config5_late_layers_prefill_131072_then_decode():
    """The far end of the 32-layer stack at full length: layer 20 (the last anchor), layer 21 (its first reuse
    layer) and layer 31 (its last, eleven layers of 15 % hitter drift away from the sets it reuses), on tiles
    the other config-5 test does not sample, then three decode steps on the same caches (anchor on layer 20,
    reuse on 21 and 31).  Reuse outputs are compared with oracle attention over the anchor's own sets."""
    print("case cfg5 late layers S=131072", flush=True)
    S, T, steps = 131072, 32, 3
    wl = workloads.config5_prefill(device=DEV, layers=(20, 21, 31), S=S, T=T, decode_steps=steps)
    off = wl.idx_offsets
    kpt_d, off_d = dev_i32(wl.k_per_tile), dev_i64(off)
    la, lr1, lr2 = wl.layers
    scale = ko.default_scale(wl.d)
    tiles = [9, 1023, 3071, wl.n_tiles - 2]

    idx_a, out_a = binding.kascade_prefill_anchor(la.q, la.k[:, :S], la.v[:, :S], T, kpt_d, off_d, off[-1])
    torch.cuda.synchronize()
    sets_of = lambda t: [idx_a[h, off[t]:off[t + 1]].cpu().numpy() for h in range(wl.Hkv)]

    def check_sparse(layer, out, where):
        Q, Kp, Vp = f64(layer.q), f64(layer.k[:, :S]), f64(layer.v[:, :S])
        worst = 0.0
        for t in tiles:
            ref = ko.prefill_sparse_tile(Q, Kp, Vp, t, T, sets_of(t), scale)
            worst = max(worst, max_abs(f64(out[t * T:(t + 1) * T]), ref))
        print(f"  {where}: worst max-abs {worst:.3e}", flush=True)
        assert worst <= TOL_OUT[BF16]
        return Q, Kp

    Qa, Ka = check_sparse(la, out_a, "layer20 anchor")
    swaps = 0
    for t in tiles:
        idx_ref, pooled = ko.prefill_anchor_indices_tile(Qa, Ka, t, T, scale, wl.k_per_tile[t])
        got = sets_of(t)
        for h in range(wl.Hkv):
            swaps += check_index_set(got[h], idx_ref[h], pooled[h], where=f"cfg5 layer20 tile {t} head {h}")
    print(f"  layer20 index sets: swaps {swaps}", flush=True)
    del Qa, Ka, out_a
    for layer, name in ((lr1, "layer21 reuse"), (lr2, "layer31 reuse")):
        out = binding.kascade_prefill_reuse(layer.q, layer.k[:, :S], layer.v[:, :S], T, kpt_d, off_d, off[-1], idx_a)
        torch.cuda.synchronize()
        check_sparse(layer, out, name)
        del out
    del idx_a

    g = torch.Generator(device=DEV).manual_seed(778)
    for step in range(steps):
        L = S + step + 1
        kk = workloads.budget(L, 100)
        newq = torch.randn(3, 1, wl.Hq, wl.d, generator=g, device=DEV).to(BF16)
        for layer in wl.layers:
            layer.k[:, L - 1] = torch.randn(wl.Hkv, wl.d, generator=g, device=DEV).to(BF16)
            layer.v[:, L - 1] = torch.randn(wl.Hkv, wl.d, generator=g, device=DEV).to(BF16)
        sl, kp = dev_i32([L]), dev_i32([kk])
        caches = [(layer.k[None, :, :L], layer.v[None, :, :L]) for layer in wl.layers]
        idx_d, o_a = binding.kascade_decode_anchor(newq[0], caches[0][0], caches[0][1], sl, kp, L, kk)
        outs = [o_a] + [binding.kascade_decode_reuse(newq[i], caches[i][0], caches[i][1], sl, kp, kk, idx_d) for i in (1, 2)]
        torch.cuda.synchronize()
        idx_np = idx_d.cpu().numpy()
        idx_ref, pooled = ko.decode_anchor_indices(f64(newq[0, 0]), f64(caches[0][0][0]), scale, kk)
        sw = sum(check_index_set(idx_np[0, h], idx_ref[h], pooled[h], where=f"cfg5 late decode step {step} head {h}")
                 for h in range(wl.Hkv))
        sets = [idx_np[0, h] for h in range(wl.Hkv)]
        errs = [max_abs(f64(outs[i][0]), ko.sparse_decode(f64(newq[i, 0]), f64(caches[i][0][0]), f64(caches[i][1][0]), sets, scale))
                for i in range(3)]
        print(f"  decode step {step} L={L} k={kk}: swaps {sw}, max-abs {['%.3e' % e for e in errs]}", flush=True)
        assert max(errs) <= TOL_OUT[BF16]


@pytest.mark.parametrize("out_mode", [0, 1])
def test_prefill_anchor_logits_rising_and_falling_along_the_keys(out_mode):
    """Keys whose logits climb by hundreds of nats along the sequence (and drop again): the running
    softmax must move its reference exponent many times and still match the oracle."""
    print(f"case prefill rising logits out_mode={out_mode}", flush=True)
    S, Hq, Hkv, d, T = 640, 8, 2, 128, 32
    g = torch.Generator().manual_seed(31)
    u = torch.randn(d, generator=g)
    u = u / u.norm()
    q = (0.3 * torch.randn(S, Hq, d, generator=g) + 4.0 * u).to(BF16)
    ramp = torch.cat([torch.linspace(0.0, 240.0, 400), torch.linspace(240.0, -40.0, S - 400)])
    k = (0.3 * torch.randn(Hkv, S, d, generator=g) + ramp[None, :, None] * u).to(BF16)
    v = torch.randn(Hkv, S, d, generator=g).to(BF16)
    # logit of key j ~ 4 * ramp[j] / sqrt(d): up to 85 nats (122 in base 2), i.e. several reference updates
    kpt = workloads.prefill_budgets(S, T, 100, 24)
    run_anchor(q, k, v, T, kpt, out_mode, where="ramp")


@pytest.mark.parametrize("seed", list(range(8)) + [8, 9, 10, 11])
def test_prefill_reuse_random_shapes(seed):
    """Seeded random shapes: both head dimensions, every group size, lengths that end inside a tile and
    inside a 64-key block, budgets around the block size, unordered lists with entries to ignore."""
    rs = np.random.default_rng(1000 + seed)
    d = [64, 128][seed % 2]
    G = [1, 2, 4, 8][(seed // 2) % 4]
    T = 128 // G
    Hkv = int(rs.integers(1, 4))
    Hq = Hkv * G
    S = int(rs.integers(T + 1, 6 * T + 40))
    n_tiles = (S + T - 1) // T
    n_anchor = int(rs.integers(1, Hkv + 1))
    hm = rs.integers(0, n_anchor, size=Hkv).tolist()
    kpt = [int(min(t * T, rs.choice([0, 1, 63, 64, 65, 100, 129]))) for t in range(n_tiles)]
    off = offsets(kpt)
    dtype = [BF16, torch.float16][(seed // 8) % 2]       # seeds 0-7 of the suite: bf16; beyond that the two alternate
    print(f"case prefill reuse random seed={seed}: {dtype} S={S} Hq={Hq} Hkv={Hkv} d={d} T={T} anchors={n_anchor} k_t={kpt}", flush=True)
    q, k, v = random_prefill(2000 + seed, S, Hq, Hkv, d, dtype)
    idx = np.full((n_anchor, max(off[-1], 1)), -1, dtype=np.int32)
    sets = {}
    for t in range(n_tiles):
        sets[t] = []
        for h in range(n_anchor):
            kt = kpt[t]
            n_bad = int(min(kt, rs.integers(0, 3)))
            good = rs.permutation(rs.choice(t * T, kt - n_bad, replace=False)) if kt - n_bad > 0 else np.zeros(0, np.int64)
            bad = rs.choice([-1, -7, t * T, t * T + 3, S + 5], size=n_bad)
            row = rs.permutation(np.concatenate([good, bad]).astype(np.int64))
            idx[h, off[t]:off[t] + kt] = row
            sets[t].append(np.asarray(good, dtype=np.int64))
    out = binding.kascade_prefill_reuse(q.to(DEV), k.to(DEV), v.to(DEV), T, dev_i32(kpt), dev_i64(off), off[-1],
                                        torch.from_numpy(idx).to(DEV), head_map=dev_i32(hm), n_anchor_heads=n_anchor)
    torch.cuda.synchronize()
    Q, Kp, Vp = f64(q), f64(k), f64(v)
    o = f64(out)
    worst = 0.0
    for t in range(n_tiles):
        lo, hi = ko.tile_bounds(t, T, S)
        ref = ko.prefill_sparse_tile(Q, Kp, Vp, t, T, sets[t], ko.default_scale(d), head_map=hm)
        worst = max(worst, max_abs(o[lo:hi], ref))
    print(f"  max-abs {worst:.3e}", flush=True)
    assert worst <= TOL_OUT[dtype]


@pytest.mark.parametrize("seed", list(range(6)) + [8, 9, 10, 11])
def test_prefill_anchor_random_shapes(seed):
    rs = np.random.default_rng(3000 + seed)
    d = [128, 64][seed % 2]
    G = [4, 1, 8, 2][(seed // 2) % 4]
    T = 128 // G
    Hkv = int(rs.integers(1, 3))
    Hq = Hkv * G
    S = int(rs.integers(2 * T + 1, 5 * T + 30))
    n_tiles = (S + T - 1) // T
    kpt = [int(min(t * T, rs.choice([1, 17, 64, 90]))) for t in range(n_tiles)]
    dtype = [BF16, torch.float16][(seed // 8) % 2]
    print(f"case prefill anchor random seed={seed}: {dtype} S={S} Hq={Hq} Hkv={Hkv} d={d} T={T} k_t={kpt}", flush=True)
    q, k, v = random_prefill(4000 + seed, S, Hq, Hkv, d, dtype)
    run_anchor(q, k, v, T, kpt, seed % 2, where=f"random {seed}")


@pytest.mark.parametrize("S", [1, 31, 32, 33, 64, 65])
def test_prefill_anchor_and_reuse_tiny_prompts(S):
    """Prompts of one token, just under / exactly / just over one tile and two tiles: tile 0 never has
    candidates, a tile with k_t = 0 attends its diagonal only."""
    print(f"case prefill tiny S={S}", flush=True)
    Hq, Hkv, d, T = 8, 2, 128, 32
    q, k, v = random_prefill(700 + S, S, Hq, Hkv, d)
    n_tiles = (S + T - 1) // T
    for kpt in ([min(t * T, 5) for t in range(n_tiles)], [0] * n_tiles):
        for mode in (0, 1):
            idx, _ = run_anchor(q, k, v, T, kpt, mode, where=f"S{S} k_t={kpt} mode{mode}")
        off = offsets(kpt)
        out = binding.kascade_prefill_reuse(q.to(DEV), k.to(DEV), v.to(DEV), T, dev_i32(kpt), dev_i64(off), off[-1],
                                            torch.from_numpy(idx).to(DEV))
        torch.cuda.synchronize()
        o = f64(out)
        for t, kt in enumerate(kpt):
            lo, hi = ko.tile_bounds(t, T, S)
            ref = ko.prefill_sparse_tile(f64(q), f64(k), f64(v), t, T, [idx[h, off[t]:off[t] + kt] for h in range(Hkv)],
                                         ko.default_scale(d))
            assert max_abs(o[lo:hi], ref) <= TOL_OUT[BF16]


@pytest.mark.parametrize("variant", ["per_head", "shared", "presoftmax"])
def test_prefill_holds_device_side_budgets_to_the_index_arrays(variant):
    """idx_total sizes the index arrays on the host; a device-side budget or offset that would reach
    past them is cut to what fits (the last tile here asks for 1000 entries more than its slot has):
    same bits as the consistent call, nothing written or read beyond the arrays."""
    print(f"case prefill budgets above the index arrays, {variant}", flush=True)
    S, Hq, Hkv, d, T = 640, 8, 2, 128, 32
    q, k, v = random_prefill(77, S, Hq, Hkv, d)
    n_tiles = S // T
    kpt = [min(t * T, 48) for t in range(n_tiles)]
    off = offsets(kpt)
    bad = list(kpt)
    bad[-1] += 1000
    call = {"per_head": binding.kascade_prefill_anchor, "shared": binding.kascade_prefill_anchor_shared,
            "presoftmax": binding.kascade_prefill_anchor_presoftmax}[variant]
    res = []
    for budgets in (bad, kpt):
        idx, out = call(q.to(DEV), k.to(DEV), v.to(DEV), T, dev_i32(budgets), dev_i64(off), off[-1],
                        out_mode=binding.KASCADE_OUT_SPARSE)
        torch.cuda.synchronize()
        res.append((idx.clone(), out.clone()))
    assert torch.equal(res[0][0], res[1][0]) and torch.equal(res[0][1], res[1][1])
    idx = res[1][0]
    n_src = idx.shape[0]
    out = binding.kascade_prefill_reuse(q.to(DEV), k.to(DEV), v.to(DEV), T, dev_i32(bad), dev_i64(off), off[-1], idx,
                                        head_map=dev_i32([0] * Hkv) if n_src == 1 else None)
    out_ok = binding.kascade_prefill_reuse(q.to(DEV), k.to(DEV), v.to(DEV), T, dev_i32(kpt), dev_i64(off), off[-1], idx,
                                           head_map=dev_i32([0] * Hkv) if n_src == 1 else None)
    torch.cuda.synchronize()
    assert torch.equal(out, out_ok)


@pytest.mark.parametrize("dtype", [BF16, torch.float16])
@pytest.mark.parametrize("out_mode", [0, 1])
def test_prefill_token_major_kv(dtype, out_mode):
    """K and V stored token major, [S, Hkv, d], and handed over through kv_stride (head stride d, token
    stride Hkv*d): anchor in both output modes, then a reuse layer with its own token-major K/V; ragged
    last tile, two key heads next to each other in memory."""
    print(f"case prefill token-major K/V dtype={dtype} out_mode={out_mode}", flush=True)
    S, Hq, Hkv, d, T = 333, 8, 2, 128, 32
    g = torch.Generator().manual_seed(91)
    q = torch.randn(S, Hq, d, generator=g).to(dtype)
    k_tm = torch.randn(S, Hkv, d, generator=g).to(dtype).to(DEV)
    v_tm = torch.randn(S, Hkv, d, generator=g).to(dtype).to(DEV)
    k, v = k_tm.permute(1, 0, 2), v_tm.permute(1, 0, 2)        # [Hkv, S, d] views of the token-major storage
    assert k.stride() == (d, Hkv * d, 1) and not k.is_contiguous()
    kpt = workloads.prefill_budgets(S, T, 250, 20)
    idx, _ = run_anchor(q, k, v, T, kpt, out_mode, where="token-major anchor")
    # the same call on a head-major copy gives the same bits (same arithmetic, other addresses)
    off = offsets(kpt)
    idx2, out2 = binding.kascade_prefill_anchor(q.to(DEV), k.contiguous(), v.contiguous(), T, dev_i32(kpt), dev_i64(off),
                                                off[-1], out_mode=out_mode)
    idx1, out1 = binding.kascade_prefill_anchor(q.to(DEV), k, v, T, dev_i32(kpt), dev_i64(off), off[-1], out_mode=out_mode)
    torch.cuda.synchronize()
    assert torch.equal(idx1, idx2) and torch.equal(out1, out2)
    # reuse layer: fresh Q/K/V, again token major
    q2 = torch.randn(S, Hq, d, generator=g).to(dtype)
    k2 = torch.randn(S, Hkv, d, generator=g).to(dtype).to(DEV).permute(1, 0, 2)
    v2 = torch.randn(S, Hkv, d, generator=g).to(dtype).to(DEV).permute(1, 0, 2)
    out = binding.kascade_prefill_reuse(q2.to(DEV), k2, v2, T, dev_i32(kpt), dev_i64(off), off[-1], torch.from_numpy(idx).to(DEV))
    torch.cuda.synchronize()
    o, worst = f64(out), 0.0
    for t, kt in enumerate(kpt):
        lo, hi = ko.tile_bounds(t, T, S)
        ref = ko.prefill_sparse_tile(f64(q2), f64(k2), f64(v2), t, T, [idx[h, off[t]:off[t] + kt] for h in range(Hkv)],
                                     ko.default_scale(d))
        worst = max(worst, max_abs(o[lo:hi], ref))
    print(f"  token-major reuse: max-abs {worst:.3e}", flush=True)
    assert worst <= TOL_OUT[dtype]


@pytest.mark.parametrize("dtype", [BF16, torch.float16])
def test_prefill_reuse_list_starts_with_ignored_entries_and_logits_far_below_zero(dtype):
    """An index list whose first 64 or more entries are all entries to ignore (negative, or not before the
    tile), so that the first key block of a tile holds no key at all, while every live logit lies far
    below zero (about -150 in base 2): the running softmax must take its reference exponent from the
    first block that holds a key, not from the empty one."""
    print(f"case prefill reuse, list begins with ignored entries, dtype={dtype}", flush=True)
    S, Hq, Hkv, d, T = 165, 8, 2, 128, 32
    g = torch.Generator().manual_seed(17)
    u = torch.randn(d, generator=g)
    u = u / u.norm()
    q = (0.2 * torch.randn(S, Hq, d, generator=g) - 40.0 * u).to(dtype)
    k = (0.2 * torch.randn(Hkv, S, d, generator=g) + 30.0 * u).to(dtype)
    v = torch.randn(Hkv, S, d, generator=g).to(dtype)
    n_tiles = (S + T - 1) // T
    kpt = [0, 0, 0, 90, 128, 128][:n_tiles]
    n_bad = [0, 0, 0, 64, 64, 100][:n_tiles]
    off = offsets(kpt)
    rs = np.random.default_rng(5)
    idx = np.full((Hkv, off[-1]), -1, dtype=np.int32)
    sets = {}
    for t in range(n_tiles):
        sets[t] = []
        for h in range(Hkv):
            good = rs.permutation(rs.choice(t * T, kpt[t] - n_bad[t], replace=False)) if kpt[t] > n_bad[t] else np.zeros(0, np.int64)
            bad = rs.choice([-1, -9, t * T, t * T + 5, S + 3], size=n_bad[t])
            idx[h, off[t]:off[t] + kpt[t]] = np.concatenate([bad, good])
            sets[t].append(np.asarray(good, dtype=np.int64))
    out = binding.kascade_prefill_reuse(q.to(DEV), k.to(DEV), v.to(DEV), T, dev_i32(kpt), dev_i64(off), off[-1],
                                        torch.from_numpy(idx).to(DEV))
    torch.cuda.synchronize()
    o, worst = f64(out), 0.0
    assert np.isfinite(o).all()
    for t in range(n_tiles):
        lo, hi = ko.tile_bounds(t, T, S)
        ref = ko.prefill_sparse_tile(f64(q), f64(k), f64(v), t, T, sets[t], ko.default_scale(d))
        worst = max(worst, max_abs(o[lo:hi], ref))
    print(f"  max-abs {worst:.3e}", flush=True)
    assert worst <= TOL_OUT[dtype]
