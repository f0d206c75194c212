"""GPU parity of every entry point on fp16 tensors (the precision the paper's own timings use), against the
CPU oracle.  fp16 runs on the matrix-unit kernels only, so these cases also cover one and two heads per key
head on those kernels."""
import numpy as np
import pytest
import torch

from oracle import kascade_oracle as ko
from paper_2512_16391_amd import binding
from parity_utils import TOL_OUT, check_index_set, f64, max_abs
from test_decode_gpu import i32, random_case, run_anchor_case
from test_prefill_gpu import dev_i32, dev_i64, offsets, run_anchor

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
F16 = torch.float16


@pytest.mark.parametrize("G,Hkv,d", [(1, 2, 128), (2, 2, 64), (4, 2, 128), (7, 1, 128), (8, 2, 64), (16, 1, 128)])
@pytest.mark.parametrize("out_mode", [0, 1])
def test_fp16_decode_anchor_and_reuse(G, Hkv, d, out_mode):
    print(f"case fp16 decode G={G} Hkv={Hkv} d={d} out_mode={out_mode}", flush=True)
    lens, ks, W = [3000, 0, 1025, 9, 130], [300, 0, 103, 9, 64], 4
    live = [b for b, L in enumerate(lens) if L > 0]
    q, k, v = random_case(300 + G, len(lens), G * Hkv, Hkv, d, F16, lens)
    sub = lambda t: t[live]
    idx, out = run_anchor_case(sub(q), sub(k), sub(v), [lens[b] for b in live], [ks[b] for b in live], W, out_mode, F16,
                               where="fp16 anchor")
    # the whole batch (with the empty sequence) gives the same rows, zeros for the empty one
    idx_all, out_all = binding.kascade_decode_anchor(q.to(DEV), k.to(DEV), v.to(DEV), i32(lens), i32(ks), max(lens), max(ks),
                                                     recent_window=W, out_mode=out_mode)
    torch.cuda.synchronize()
    assert (idx_all[1] == -1).all() and (out_all[1] == 0).all()
    assert np.array_equal(idx_all.cpu().numpy()[live], idx) and torch.equal(out_all[live], out)
    # reuse layer with its own tensors and a head map
    q2, k2, v2 = random_case(400 + G, len(lens), G * Hkv, Hkv, d, F16, lens)
    hm = [(h + 1) % Hkv for h in range(Hkv)]
    o2 = binding.kascade_decode_reuse(q2.to(DEV), k2.to(DEV), v2.to(DEV), i32(lens), i32(ks), max(ks), idx_all, head_map=i32(hm))
    torch.cuda.synchronize()
    o2 = f64(o2)
    idx_h = idx_all.cpu().numpy()
    for b in live:
        L, kb = lens[b], ks[b]
        want = ko.sparse_decode(f64(q2[b]), f64(k2[b, :, :L]), f64(v2[b, :, :L]), [idx_h[b, h, :kb] for h in range(Hkv)],
                                ko.default_scale(d), hm)
        assert max_abs(o2[b], want) <= TOL_OUT[F16], f"reuse b{b}"
    assert np.all(o2[1] == 0.0)


@pytest.mark.parametrize("variant", ["shared", "presoftmax"])
def test_fp16_decode_anchor_variants(variant):
    print(f"case fp16 decode {variant}", flush=True)
    G, Hkv, d, lens, ks, W = 4, 2, 128, [2000, 300, 64], [200, 30, 64], 2
    q, k, v = random_case(500, len(lens), G * Hkv, Hkv, d, F16, lens)
    call = {"shared": binding.kascade_decode_anchor_shared, "presoftmax": binding.kascade_decode_anchor_presoftmax}[variant]
    scale = ko.default_scale(d)
    for mode in (binding.KASCADE_OUT_SPARSE, binding.KASCADE_OUT_DENSE):
        idx, out = call(q.to(DEV), k.to(DEV), v.to(DEV), i32(lens), i32(ks), max(lens), max(ks), recent_window=W, out_mode=mode)
        torch.cuda.synchronize()
        idx_h, o = idx.cpu().numpy(), f64(out)
        n_sets = 1 if variant == "shared" else Hkv
        for b, (L, kb) in enumerate(zip(lens, ks)):
            qb, kb_, vb = f64(q[b]), f64(k[b, :, :L]), f64(v[b, :, :L])
            if variant == "presoftmax":
                ref_idx, a = ko.decode_presoftmax_indices(qb, kb_, scale, kb, "fp16", W)
            else:
                ri, aa = ko.decode_shared_indices(qb, kb_, scale, kb, W)
                ref_idx, a = ri[None], aa[None]
            for h in range(n_sets):
                check_index_set(idx_h[b, h, :kb], ref_idx[h], a[h], n_forced=W, where=f"{variant} b{b} h{h}")
            want = ko.dense_decode(qb, kb_, vb, scale) if mode == binding.KASCADE_OUT_DENSE else \
                ko.sparse_decode(qb, kb_, vb, [idx_h[b, h, :kb] for h in range(n_sets)], scale,
                                 None if variant != "shared" else [0] * Hkv)
            assert max_abs(o[b], want) <= TOL_OUT[F16]


def fp16_prefill(seed, S, Hq, Hkv, d):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(S, Hq, d, generator=g).to(F16), torch.randn(Hkv, S, d, generator=g).to(F16),
            torch.randn(Hkv, S, d, generator=g).to(F16))


@pytest.mark.parametrize("S,Hq,Hkv,d,T", [(300, 8, 2, 128, 32), (257, 8, 1, 64, 16), (520, 4, 2, 128, 64), (400, 8, 2, 128, 128)])
@pytest.mark.parametrize("out_mode", [0, 1])
def test_fp16_prefill_anchor_then_reuse(S, Hq, Hkv, d, T, out_mode):
    print(f"case fp16 prefill S={S} Hq={Hq} Hkv={Hkv} d={d} T={T} out_mode={out_mode}", flush=True)
    q, k, v = fp16_prefill(600 + S, S, Hq, Hkv, d)
    n_tiles = (S + T - 1) // T
    kpt = [min(t * T, max(8, t * T // 5)) for t in range(n_tiles)]
    idx, _ = run_anchor(q, k, v, T, kpt, out_mode, where="fp16 prefill anchor")
    off = offsets(kpt)
    q2, k2, v2 = fp16_prefill(700 + S, S, Hq, Hkv, d)
    out = binding.kascade_prefill_reuse(q2.to(DEV), k2.to(DEV), v2.to(DEV), T, dev_i32(kpt), dev_i64(off), off[-1],
                                        torch.from_numpy(idx).to(DEV))
    torch.cuda.synchronize()
    Q, Kp, Vp, o = f64(q2), f64(k2), f64(v2), f64(out)
    for t in range(n_tiles):
        lo, hi = ko.tile_bounds(t, T, S)
        sets = [idx[h, off[t]:off[t] + kpt[t]] for h in range(Hkv)]
        ref = ko.prefill_sparse_tile(Q, Kp, Vp, t, T, sets, ko.default_scale(d))
        assert max_abs(o[lo:hi], ref) <= TOL_OUT[F16], f"reuse tile {t}"


@pytest.mark.parametrize("out_mode", [0, 1])
def test_fp16_prefill_logits_far_above_the_first_reference(out_mode):
    """Scores that climb by many powers of two along the keys: the weights of a block against the lagging
    reference exponent would leave fp16's range (65504) long before they leave bf16's, so the fp16 kernels
    renew the reference earlier."""
    print(f"case fp16 prefill rising logits out_mode={out_mode}", flush=True)
    S, Hq, Hkv, d, T = 384, 8, 2, 128, 32
    g = torch.Generator().manual_seed(801)
    q = torch.randn(S, Hq, d, generator=g)
    k = torch.randn(Hkv, S, d, generator=g) * 0.05
    v = torch.randn(Hkv, S, d, generator=g)
    ramp = torch.linspace(0.0, 1.0, S)                    # key j is aligned with every query by ramp[j]
    qdir = q.mean(dim=(0, 1))
    qdir = qdir / qdir.norm()
    q = q * 0.2 + 6.0 * qdir                              # every query has a large component along qdir
    k = k + (ramp[None, :, None] * 12.0) * qdir[None, None, :]
    q, k, v = q.to(F16), k.to(F16), v.to(F16)
    n_tiles = S // T
    kpt = [min(t * T, 24) for t in range(n_tiles)]
    run_anchor(q, k, v, T, kpt, out_mode, where="fp16 rising logits")


def test_fp16_prefill_variants_and_importance():
    S, Hq, Hkv, d, T = 320, 8, 2, 128, 32
    q, k, v = fp16_prefill(900, S, Hq, Hkv, d)
    n_tiles = S // T
    kpt = [min(t * T, 20) for t in range(n_tiles)]
    off = offsets(kpt)
    scale = ko.default_scale(d)
    Q, Kp, Vp = f64(q), f64(k), f64(v)
    for variant, call in (("shared", binding.kascade_prefill_anchor_shared), ("presoftmax", binding.kascade_prefill_anchor_presoftmax)):
        idx, out = call(q.to(DEV), k.to(DEV), v.to(DEV), T, dev_i32(kpt), dev_i64(off), off[-1], out_mode=binding.KASCADE_OUT_SPARSE)
        torch.cuda.synchronize()
        idx_h, o = idx.cpu().numpy(), f64(out)
        for t in range(1, n_tiles):
            kt = kpt[t]
            if variant == "shared":
                ri, aa = ko.prefill_shared_indices_tile(Q, Kp, t, T, scale, kt)
                check_index_set(idx_h[0, off[t]:off[t] + kt], ri, aa, where=f"shared tile {t}")
                sets = [idx_h[0, off[t]:off[t] + kt]] * Hkv
            else:
                ri, aa = ko.prefill_presoftmax_indices_tile(Q, Kp, t, T, scale, kt, "fp16")
                for h in range(Hkv):
                    check_index_set(idx_h[h, off[t]:off[t] + kt], ri[h], aa[h], where=f"presoftmax tile {t} head {h}")
                sets = [idx_h[h, off[t]:off[t] + kt] for h in range(Hkv)]
            lo, hi = ko.tile_bounds(t, T, S)
            ref = ko.prefill_sparse_tile(Q, Kp, Vp, t, T, sets, scale)
            assert max_abs(o[lo:hi], ref) <= TOL_OUT[F16], f"{variant} tile {t}"
    # layer importance on fp16 activations
    g = torch.Generator().manual_seed(901)
    x = torch.randn(50, 96, generator=g).to(F16)
    y = (x.float() * 0.7 + 0.3 * torch.randn(50, 96, generator=g)).to(F16)
    w = binding.kascade_layer_importance(x.to(DEV), y.to(DEV))
    torch.cuda.synchronize()
    want = ko.layer_importance(f64(x), f64(y))
    np.testing.assert_allclose(f64(w), want, rtol=0, atol=1e-5)
