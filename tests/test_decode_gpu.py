"""GPU parity of the decode entry points against the CPU oracle, element by element, on
seeded inputs.  Everything goes through the C ABI (binding.py marshals arguments only)."""
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


def random_case(seed, B, Hq, Hkv, d, dtype, lens, Lmax=None):
    g = torch.Generator().manual_seed(seed)
    Lmax = Lmax or max(lens)
    q = torch.randn(B, Hq, d, generator=g).to(dtype)
    k = torch.randn(B, Hkv, Lmax, d, generator=g).to(dtype)
    v = torch.randn(B, Hkv, Lmax, d, generator=g).to(dtype)
    return q, k, v


def oracle_reuse(q, k, v, lens, sets, head_map=None, scale=None):
    """sets[b][h_anchor] -> index array.  Returns [B,Hq,d] float64."""
    B, Hq, d = q.shape
    scale = scale or ko.default_scale(d)
    out = np.zeros((B, Hq, d))
    for b in range(B):
        L = lens[b]
        out[b] = ko.sparse_decode(f64(q[b]), f64(k[b, :, :L]), f64(v[b, :, :L]), sets[b], scale, head_map)
    return out


# --------------------------------------------------------------------------- reuse

@pytest.mark.parametrize("dtype,d,Hq,Hkv", [
    (torch.float32, 64, 8, 2), (torch.bfloat16, 128, 32, 8), (torch.bfloat16, 64, 8, 8),
    (torch.float32, 128, 4, 2), (torch.bfloat16, 128, 8, 1), (torch.float32, 64, 2, 2),
])
def test_decode_reuse_matches_oracle(dtype, d, Hq, Hkv):
    print(f"case reuse dtype={dtype} d={d} Hq={Hq} Hkv={Hkv}", flush=True)
    B = 3
    lens = [700, 1, 389]
    ks = [70, 1, 389]            # 10 %, a single key, and k = L
    k_max = 400
    q, k, v = random_case(1, B, Hq, Hkv, d, dtype, lens)
    rs = np.random.default_rng(2)
    idx = torch.full((B, Hkv, k_max), -1, dtype=torch.int32)
    sets = []
    for b in range(B):
        sets.append([np.sort(rs.choice(lens[b], ks[b], replace=False)) for _ in range(Hkv)])
        for h in range(Hkv):
            idx[b, h, : ks[b]] = torch.from_numpy(sets[b][h]).int()
    out = binding.kascade_decode_reuse(q.to(DEV), k.to(DEV), v.to(DEV), i32(lens), i32(ks), k_max, idx.to(DEV))
    torch.cuda.synchronize()
    ref = oracle_reuse(q, k, v, lens, sets)
    err = max_abs(f64(out), ref)
    print(f"  max-abs {err:.3e}", flush=True)
    assert err <= TOL_OUT[dtype]
    # k = L case equals dense attention (the method's own invariant), against the oracle's dense path
    dense = ko.dense_decode(f64(q[2]), f64(k[2, :, :389]), f64(v[2, :, :389]), ko.default_scale(d))
    assert max_abs(f64(out[2]), dense) <= TOL_OUT[dtype]


def test_decode_reuse_head_map_unordered_and_invalid_entries():
    dtype, d, Hq, Hkv, B = torch.float32, 64, 8, 4, 2
    lens, ks, k_max = [1000, 513], [300, 257], 320
    q, k, v = random_case(3, B, Hq, Hkv, d, dtype, lens)
    rs = np.random.default_rng(4)
    n_anchor = 2
    hm = [1, 0, 1, 1]
    idx = torch.full((B, n_anchor, k_max), -1, dtype=torch.int32)
    sets = []
    for b in range(B):
        sb = []
        for h in range(n_anchor):
            s = rs.permutation(rs.choice(lens[b], ks[b] - 3, replace=False))      # unordered
            row = np.concatenate([s[:5], [-1, lens[b], 2 ** 30], s[5:]])          # 3 entries to ignore
            idx[b, h, : ks[b]] = torch.from_numpy(row).int()
            sb.append(s)
        sets.append(sb)
    out = binding.kascade_decode_reuse(q.to(DEV), k.to(DEV), v.to(DEV), i32(lens), i32(ks), k_max, idx.to(DEV),
                                       head_map=i32(hm))
    torch.cuda.synchronize()
    ref = oracle_reuse(q, k, v, lens, sets, head_map=hm)
    assert max_abs(f64(out), ref) <= TOL_OUT[dtype]


def test_decode_reuse_token_major_cache_and_custom_scale():
    dtype, d, Hq, Hkv, B = torch.bfloat16, 128, 8, 2, 2
    lens, ks, k_max = [600, 300], [64, 33], 64
    q, k, v = random_case(5, B, Hq, Hkv, d, dtype, lens)
    k_blhd = k.permute(0, 2, 1, 3).contiguous()          # [B, L, Hkv, d]
    v_blhd = v.permute(0, 2, 1, 3).contiguous()
    rs = np.random.default_rng(6)
    idx = torch.full((B, Hkv, k_max), -1, dtype=torch.int32)
    sets = []
    for b in range(B):
        sets.append([np.sort(rs.choice(lens[b], ks[b], replace=False)) for _ in range(Hkv)])
        for h in range(Hkv):
            idx[b, h, : ks[b]] = torch.from_numpy(sets[b][h]).int()
    out = binding.kascade_decode_reuse(q.to(DEV), k_blhd.to(DEV), v_blhd.to(DEV), i32(lens), i32(ks), k_max,
                                       idx.to(DEV), softmax_scale=0.05, kv_layout="BLHD")
    torch.cuda.synchronize()
    ref = oracle_reuse(q, k, v, lens, sets, scale=0.05)
    assert max_abs(f64(out), ref) <= TOL_OUT[dtype]


def test_decode_reuse_many_chunks_and_empty_sequence():
    # k large enough for several workgroups per (sequence, head); one sequence has k = 0
    dtype, d, Hq, Hkv, B = torch.bfloat16, 128, 8, 2, 3
    lens, ks, k_max = [9000, 5000, 7777], [4100, 0, 1031], 4100
    q, k, v = random_case(7, B, Hq, Hkv, d, dtype, lens)
    rs = np.random.default_rng(8)
    idx = torch.full((B, Hkv, k_max), -1, dtype=torch.int32)
    sets = []
    for b in range(B):
        sets.append([np.sort(rs.choice(lens[b], ks[b], replace=False)) for _ in range(Hkv)])
        for h in range(Hkv):
            idx[b, h, : ks[b]] = torch.from_numpy(sets[b][h]).int()
    out = binding.kascade_decode_reuse(q.to(DEV), k.to(DEV), v.to(DEV), i32(lens), i32(ks), k_max, idx.to(DEV))
    torch.cuda.synchronize()
    o = f64(out)
    assert np.all(o[1] == 0.0)                          # empty set -> zero output by definition
    for b in (0, 2):
        ref = ko.sparse_decode(f64(q[b]), f64(k[b, :, :lens[b]]), f64(v[b, :, :lens[b]]), sets[b], ko.default_scale(d))
        assert max_abs(o[b], ref) <= TOL_OUT[dtype]
    # deterministic: a second call gives the same bits
    out2 = binding.kascade_decode_reuse(q.to(DEV), k.to(DEV), v.to(DEV), i32(lens), i32(ks), k_max, idx.to(DEV))
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


def test_decode_reuse_many_chunks_fp32_and_wide_groups():
    for dtype, d, Hq, Hkv in [(torch.float32, 64, 8, 1), (torch.float32, 128, 4, 2), (torch.bfloat16, 64, 16, 2)]:
        lens, ks = [6000, 2500], [5000, 700]
        q, k, v = random_case(90, 2, Hq, Hkv, d, dtype, lens)
        rs = np.random.default_rng(91)
        idx = torch.full((2, Hkv, 5000), -1, dtype=torch.int32)
        sets = []
        for b in range(2):
            sets.append([np.sort(rs.choice(lens[b], ks[b], replace=False)) for _ in range(Hkv)])
            for h in range(Hkv):
                idx[b, h, : ks[b]] = torch.from_numpy(sets[b][h]).int()
        print(f"case many chunks dtype={dtype} d={d} Hq={Hq} Hkv={Hkv}", flush=True)
        for _ in range(2):
            out = binding.kascade_decode_reuse(q.to(DEV), k.to(DEV), v.to(DEV), i32(lens), i32(ks), 5000, idx.to(DEV))
            torch.cuda.synchronize()
            assert max_abs(f64(out), oracle_reuse(q, k, v, lens, sets)) <= TOL_OUT[dtype]


# --------------------------------------------------------------------------- anchor

def run_anchor_case(q, k, v, lens, ks, W, out_mode, dtype, max_seqlen=None, where=""):
    B, Hq, d = q.shape
    Hkv = k.shape[1]
    k_max = max(ks)
    max_seqlen = max_seqlen or max(lens)
    idx, out = binding.kascade_decode_anchor(q.to(DEV), k.to(DEV), v.to(DEV), i32(lens), i32(ks), max_seqlen, k_max,
                                             recent_window=W, out_mode=out_mode)
    torch.cuda.synchronize()
    idx = idx.cpu().numpy()
    o = f64(out)
    scale = ko.default_scale(d)
    swaps = 0
    worst = 0.0
    for b in range(B):
        L, kb = lens[b], ks[b]
        qb, kb_, vb = f64(q[b]), f64(k[b, :, :L]), f64(v[b, :, :L])
        idx_ref, a = ko.decode_anchor_indices(qb, kb_, scale, kb, W)
        for h in range(Hkv):
            assert (idx[b, h, kb:] == -1).all(), f"{where} b{b} h{h}: padding"
            swaps += check_index_set(idx[b, h, :kb], idx_ref[h], a[h], n_forced=W, where=f"{where} b{b} h{h}")
        if out_mode == binding.KASCADE_OUT_DENSE:
            ref = ko.dense_decode(qb, kb_, vb, scale)
        else:
            # oracle attention over the GPU's own (already validated) sets
            ref = ko.sparse_decode(qb, kb_, vb, [idx[b, h, :kb] for h in range(Hkv)], scale)
        worst = max(worst, max_abs(o[b], ref))
    print(f"  {where}: swaps {swaps}, max-abs {worst:.3e}", flush=True)
    assert worst <= TOL_OUT[dtype]
    return idx, out


def test_decode_anchor_config1_then_reuse():
    """The small fp32 configuration end to end: anchor layer, then a reuse layer that
    consumes the anchor's indices with its own Q/K/V."""
    print("case anchor config1", flush=True)
    wl = workloads.config1()
    a, r = wl.layers
    idx, _ = run_anchor_case(a.q, a.k, a.v, wl.seqlens, wl.k_per_seq, 0, binding.KASCADE_OUT_SPARSE, wl.dtype,
                             where="cfg1 anchor")
    assert wl.k_per_seq == [205]
    out = binding.kascade_decode_reuse(r.q.to(DEV), r.k.to(DEV), r.v.to(DEV), i32(wl.seqlens), i32(wl.k_per_seq),
                                       wl.k_max, torch.from_numpy(idx).to(DEV))
    torch.cuda.synchronize()
    sets = [[idx[0, h, :205] for h in range(wl.Hkv)]]
    ref = oracle_reuse(r.q, r.k, r.v, wl.seqlens, sets)
    assert max_abs(f64(out), ref) <= TOL_OUT[wl.dtype]
    # planted hitters are over-represented in the Top-k (a 10 % set would hold 6.4 of the 64 by
    # chance; the literal boost of the configuration shifts their logits by only 3/sqrt(d))
    for h in range(wl.Hkv):
        hit = set(a.hitters[0][h].tolist())
        assert len(hit & set(idx[0, h, :205].tolist())) >= 13


@pytest.mark.parametrize("dtype,d,Hq,Hkv", [
    (torch.float32, 64, 8, 2), (torch.bfloat16, 128, 32, 8), (torch.bfloat16, 64, 4, 4),
    (torch.float32, 128, 16, 2), (torch.bfloat16, 128, 4, 2),
])
@pytest.mark.parametrize("out_mode", [0, 1])
def test_decode_anchor_ragged_batch_with_window(dtype, d, Hq, Hkv, out_mode):
    print(f"case anchor dtype={dtype} d={d} Hq={Hq} Hkv={Hkv} out_mode={out_mode}", flush=True)
    lens = [3000, 77, 1025, 2500]
    W = 16
    ks = [300, 77, 103, 16]         # 10 %, k = L, ragged, k = W (window only)
    q, k, v = random_case(11, 4, Hq, Hkv, d, dtype, lens)
    run_anchor_case(q, k, v, lens, ks, W, out_mode, dtype, where="ragged")


def test_decode_anchor_exact_ties_go_to_lower_index():
    """Duplicate key rows give bit-identical pooled scores; the lower position must win."""
    dtype, d, Hq, Hkv = torch.float32, 64, 4, 1
    L, kk = 512, 40
    q, k, v = random_case(13, 1, Hq, Hkv, d, dtype, [L])
    k[0, 0, 256:] = k[0, 0, :256]           # every key appears twice: j and j + 256
    idx, _ = binding.kascade_decode_anchor(q.to(DEV), k.to(DEV), v.to(DEV), i32([L]), i32([kk]), L, kk)
    torch.cuda.synchronize()
    got = idx[0, 0].cpu().numpy()
    ref, a = ko.decode_anchor_indices(f64(q[0]), f64(k[0]), ko.default_scale(d), kk)
    np.testing.assert_array_equal(got, ref[0])
    # with kk even and all scores paired, pairs (j, j+256) enter together: both members present
    s = set(got.tolist())
    assert all(((j + 256) in s) for j in got if j < 256)


def test_decode_anchor_padded_cache_and_larger_max_seqlen():
    # cache allocated for 4096 tokens, sequences shorter; max_seqlen is only an upper bound
    dtype, d, Hq, Hkv = torch.bfloat16, 128, 8, 2
    lens, ks = [1500, 2049], [150, 205]
    q, k, v = random_case(17, 2, Hq, Hkv, d, dtype, lens, Lmax=4096)
    run_anchor_case(q, k, v, lens, ks, 0, 1, dtype, max_seqlen=4096, where="padded")


def test_decode_config2_shape_reduced_batch():
    """Llama-3.1-8B attention shape at full context (32768, k = 3277), batch 2: every output
    and every index set against the oracle; anchor followed by a reuse layer."""
    print("case config2 B=2", flush=True)
    wl = workloads.config2(device="cpu", n_layers=2, B=2)
    a, r = wl.layers
    idx, _ = run_anchor_case(a.q, a.k, a.v, wl.seqlens, wl.k_per_seq, 0, 1, wl.dtype, where="cfg2 anchor")
    out = binding.kascade_decode_reuse(r.q.to(DEV), r.k.to(DEV), r.v.to(DEV), i32(wl.seqlens), i32(wl.k_per_seq),
                                       wl.k_max, torch.from_numpy(idx).to(DEV))
    torch.cuda.synchronize()
    kk = wl.k_per_seq[0]
    sets = [[idx[b, h, :kk] for h in range(wl.Hkv)] for b in range(wl.B)]
    ref = oracle_reuse(r.q, r.k, r.v, wl.seqlens, sets)
    err = max_abs(f64(out), ref)
    print(f"  cfg2 reuse max-abs {err:.3e}", flush=True)
    assert err <= TOL_OUT[wl.dtype]


# --------------------------------------------------------------------------- full-size configurations

def test_decode_config2_full_size():
    """The benchmark configuration itself (batch 8, 32768 tokens, k = 3277), generated on the GPU
    exactly as bench.py does, in bench.py's launch configuration: anchor (sparse output) then the
    three reuse layers.  Every sequence, every head, every index set against the oracle."""
    print("case config2 full size", flush=True)
    wl = workloads.config2(device=DEV)
    sl, kp = i32(wl.seqlens), i32(wl.k_per_seq)
    a = wl.layers[0]
    idx_d, out_a = binding.kascade_decode_anchor(a.q, a.k, a.v, sl, kp, wl.Lmax, wl.k_max)
    outs = [binding.kascade_decode_reuse(r.q, r.k, r.v, sl, kp, wl.k_max, idx_d) for r in wl.layers[1:]]
    torch.cuda.synchronize()
    idx = idx_d.cpu().numpy()
    scale = ko.default_scale(wl.d)
    kk = wl.k_per_seq[0]
    swaps, worst = 0, 0.0
    for b in range(wl.B):
        qb, kb, vb = f64(a.q[b]), f64(a.k[b]), f64(a.v[b])
        idx_ref, pooled = ko.decode_anchor_indices(qb, kb, scale, kk)
        for h in range(wl.Hkv):
            swaps += check_index_set(idx[b, h, :kk], idx_ref[h], pooled[h], where=f"cfg2 b{b} h{h}")
        sets = [idx[b, h, :kk] for h in range(wl.Hkv)]
        worst = max(worst, max_abs(f64(out_a[b]), ko.sparse_decode(qb, kb, vb, sets, scale)))
        for r, o in zip(wl.layers[1:], outs):
            worst = max(worst, max_abs(f64(o[b]), ko.sparse_decode(f64(r.q[b]), f64(r.k[b]), f64(r.v[b]), sets, scale)))
        print(f"  cfg2 full b{b}: swaps so far {swaps}, worst max-abs {worst:.3e}", flush=True)
    assert worst <= TOL_OUT[wl.dtype]


def test_decode_config3_full_size_sampled():
    """Bandwidth-stress configuration (batch 32, ragged 65536..131072 tokens, k = 5 %, 64 recent
    tokens forced), all four layers at full size: eight sequences spread over the length range - the
    shortest, the longest and six at even steps of the sorted lengths in between - are checked against
    the oracle in every layer (anchor sets and output, three reuse outputs, all heads); structural
    properties for every sequence."""
    print("case config3 full size", flush=True)
    wl = workloads.config3(device=DEV, n_layers=4)
    sl, kp = i32(wl.seqlens), i32(wl.k_per_seq)
    a = wl.layers[0]
    W = wl.recent_window
    idx_d, out_a = binding.kascade_decode_anchor(a.q, a.k, a.v, sl, kp, wl.Lmax, wl.k_max, recent_window=W)
    outs_r = [binding.kascade_decode_reuse(r.q, r.k, r.v, sl, kp, wl.k_max, idx_d) for r in wl.layers[1:]]
    torch.cuda.synchronize()
    idx = idx_d.cpu().numpy()
    # properties at any size: set size, order, range, forced window, padding
    for b in range(wl.B):
        L, kb = wl.seqlens[b], wl.k_per_seq[b]
        for h in range(wl.Hkv):
            row = idx[b, h]
            assert (np.diff(row[:kb]) > 0).all() and row[0] >= 0 and row[kb - 1] == L - 1
            assert (row[kb - W:kb] == np.arange(L - W, L)).all()
            assert (row[kb:] == -1).all()
    order = np.argsort(wl.seqlens)
    picks = sorted({int(order[round(i * (len(order) - 1) / 7)]) for i in range(8)}, key=lambda b: wl.seqlens[b])
    assert len(picks) == 8
    scale = ko.default_scale(wl.d)
    worst, swaps = 0.0, 0
    for b in picks:
        L, kb = wl.seqlens[b], wl.k_per_seq[b]
        qb, kc, vc = f64(a.q[b]), f64(a.k[b, :, :L]), f64(a.v[b, :, :L])
        idx_ref, pooled = ko.decode_anchor_indices(qb, kc, scale, kb, W)
        for h in range(wl.Hkv):
            swaps += check_index_set(idx[b, h, :kb], idx_ref[h], pooled[h], n_forced=W, where=f"cfg3 b{b} h{h}")
        sets = [idx[b, h, :kb] for h in range(wl.Hkv)]
        worst = max(worst, max_abs(f64(out_a[b]), ko.sparse_decode(qb, kc, vc, sets, scale)))
        del qb, kc, vc
        for r, o in zip(wl.layers[1:], outs_r):
            ref = ko.sparse_decode(f64(r.q[b]), f64(r.k[b, :, :L]), f64(r.v[b, :, :L]), sets, scale)
            worst = max(worst, max_abs(f64(o[b]), ref))
        print(f"  cfg3 b{b} L={L} k={kb}: swaps {swaps}, worst max-abs {worst:.3e}", flush=True)
    assert worst <= TOL_OUT[wl.dtype]


@pytest.mark.parametrize("seed", range(10))
def test_decode_anchor_random_shapes(seed):
    """Seeded random shapes: both dtypes and head dimensions, every group size, ragged lengths down to a
    single token, budgets from 1 to the whole sequence, with and without a recent window."""
    rs = np.random.default_rng(5000 + seed)
    dtype = [torch.bfloat16, torch.float32][seed % 2]
    d = [128, 64][(seed // 2) % 2]
    G = [4, 1, 8, 2, 4][seed % 5]
    Hkv = int(rs.integers(1, 4))
    Hq = Hkv * G
    B = int(rs.integers(1, 5))
    lens = [int(rs.choice([1, 2, 63, 64, 65, 257, 1000, 3000, 4097])) for _ in range(B)]
    W = int(rs.choice([0, 0, 1, 16]))
    ks = [int(min(L, max(W, rs.choice([1, 2, 31, 64, 100, 1500, L])))) for L in lens]
    print(f"case decode anchor random seed={seed}: {dtype} d={d} Hq={Hq} Hkv={Hkv} lens={lens} ks={ks} W={W}", flush=True)
    q, k, v = random_case(6000 + seed, B, Hq, Hkv, d, dtype, lens, Lmax=max(lens) + int(rs.integers(0, 70)))
    run_anchor_case(q, k, v, lens, ks, min(W, min(ks)), seed % 2, dtype, where=f"random {seed}")


@pytest.mark.parametrize("seed", range(8))
def test_decode_anchor_random_shapes_matrix_unit(seed):
    """The same for the kernels that run on the matrix unit, bf16 and fp16: any group size from 5 to 16, both
    head dimensions, lengths around the 32-row batch, the 8-logit store runs and the 1024-row chunk."""
    rs = np.random.default_rng(7000 + seed)
    dtype = [torch.bfloat16, torch.float16][(seed // 2) % 2]
    d = [128, 64][seed % 2]
    G = int(rs.integers(5, 17))
    Hkv = int(rs.integers(1, 3))
    B = int(rs.integers(1, 5))
    lens = [int(rs.choice([1, 7, 8, 9, 127, 128, 129, 1023, 1025, 2050, 5000])) for _ in range(B)]
    W = int(rs.choice([0, 0, 1, 16]))
    ks = [int(min(L, max(W, rs.choice([1, 2, 31, 64, 100, 1500, L])))) for L in lens]
    print(f"case decode anchor random matrix unit seed={seed}: {dtype} d={d} G={G} Hkv={Hkv} lens={lens} ks={ks} W={W}", flush=True)
    q, k, v = random_case(8000 + seed, B, G * Hkv, Hkv, d, dtype, lens, Lmax=max(lens) + int(rs.integers(0, 70)))
    run_anchor_case(q, k, v, lens, ks, min(W, min(ks)), seed % 2, dtype, where=f"random matrix unit {seed}")


# --------------------------------------------------------------------------- split selection
# Few long segments: the Top-k of a segment is computed by several workgroups (three launches).

@pytest.mark.parametrize("dtype,d,Hq,Hkv,W", [(torch.bfloat16, 128, 8, 2, 0), (torch.float32, 64, 4, 1, 64),
                                              (torch.bfloat16, 64, 8, 1, 5)])
@pytest.mark.parametrize("out_mode", [0, 1])
def test_decode_anchor_split_selection_long_sequences(dtype, d, Hq, Hkv, W, out_mode):
    print(f"case split selection {dtype} d={d} Hq={Hq} Hkv={Hkv} W={W} out_mode={out_mode}", flush=True)
    lens, ks = [70001, 33000], [7000, max(W, 1)]      # max length >= 65536: several workgroups per segment
    wl = workloads.make_decode_workload("split", 11, 1, 2, Hq, Hkv, d, dtype, lens, ks, 512, 0.8, recent_window=W)
    a = wl.layers[0]
    run_anchor_case(a.q, a.k, a.v, lens, ks, W, out_mode, dtype, where="split")


def test_decode_anchor_split_selection_ties_across_parts():
    """Every key row appears 40 times, spread over the whole sequence: exact ties cross the part
    boundaries and the cut falls inside a tie group; the lowest positions must win."""
    dtype, d, Hq, Hkv = torch.float32, 64, 4, 1
    L, period = 70000, 1000
    q, k, v = random_case(23, 1, Hq, Hkv, d, dtype, [L])
    k[0, 0] = k[0, 0, :period].repeat(L // period, 1)
    for kk in (1, 69, 70, 71, 4017, 69999):
        idx, _ = binding.kascade_decode_anchor(q.to(DEV), k.to(DEV), v.to(DEV), i32([L]), i32([kk]), L, kk)
        torch.cuda.synchronize()
        ref, _ = ko.decode_anchor_indices(f64(q[0]), f64(k[0]), ko.default_scale(d), kk)
        np.testing.assert_array_equal(idx[0, 0].cpu().numpy(), ref[0])


def test_decode_anchor_split_selection_falls_back_when_all_scores_are_equal():
    """Identical keys: every pooled score is 1/L, far more than the selection keeps on chip."""
    dtype, d, Hq, Hkv = torch.bfloat16, 128, 4, 2
    L, kk, W = 66000, 777, 10
    q, k, v = random_case(29, 1, Hq, Hkv, d, dtype, [L])
    k[0, :, :] = k[0, :, :1]
    idx, out = binding.kascade_decode_anchor(q.to(DEV), k.to(DEV), v.to(DEV), i32([L]), i32([kk]), L, kk,
                                             recent_window=W)
    torch.cuda.synchronize()
    want = np.concatenate([np.arange(kk - W), np.arange(L - W, L)])
    for h in range(Hkv):
        np.testing.assert_array_equal(idx[0, h].cpu().numpy(), want)
    ref = ko.sparse_decode(f64(q[0]), f64(k[0]), f64(v[0]), [want] * Hkv, ko.default_scale(d))
    assert max_abs(f64(out)[0], ref) <= TOL_OUT[dtype]


def test_decode_anchor_split_and_single_selection_agree(tuning):
    dtype, d, Hq, Hkv = torch.bfloat16, 128, 8, 2
    lens, ks = [45000, 36000, 66000], [4500, 3600, 1]
    wl = workloads.make_decode_workload("split-ab", 12, 1, 3, Hq, Hkv, d, dtype, lens, ks, 700, 0.8)
    a = wl.layers[0]
    args = (a.q.to(DEV), a.k.to(DEV), a.v.to(DEV), i32(lens), i32(ks), max(lens), max(ks))
    res = {}
    for parts in ("1", "7", "64"):
        tuning(binding.TUNE_TOPK_PARTS, int(parts))
        idx, out = binding.kascade_decode_anchor(*args)
        torch.cuda.synchronize()
        res[parts] = (idx.clone(), out.clone())
    for parts in ("7", "64"):
        assert torch.equal(res[parts][0], res["1"][0])
        assert torch.equal(res[parts][1], res["1"][1])


@pytest.mark.parametrize("dtype,d,Hq,Hkv", [(torch.bfloat16, 128, 8, 2), (torch.float32, 64, 4, 4)])
@pytest.mark.parametrize("variant", ["per_head", "shared", "presoftmax"])
def test_decode_anchor_degenerate_sequences(dtype, d, Hq, Hkv, variant):
    """Sequences of zero, one and a few keys, k = 0, k = 1, k = L and a window as large as k, next to an
    ordinary sequence in the same batch: empty sets give a zero output and an all -1 index row, the rest
    matches the oracle."""
    print(f"case degenerate decode dtype={dtype} d={d} Hq={Hq} Hkv={Hkv} variant={variant}", flush=True)
    lens = [0, 1, 5, 300, 64, 7]
    ks = [0, 1, 5, 30, 0, 3]
    storage = {torch.float32: "fp32", torch.bfloat16: "bf16"}[dtype]
    q, k, v = random_case(99, len(lens), Hq, Hkv, d, dtype, lens, Lmax=320)
    call = {"per_head": binding.kascade_decode_anchor, "shared": binding.kascade_decode_anchor_shared,
            "presoftmax": binding.kascade_decode_anchor_presoftmax}[variant]
    scale = ko.default_scale(d)
    for W in (0, 3):
        ks_w = ks       # where the window exceeds k the kernels shrink it to k, as the oracle call below does
        for mode in (binding.KASCADE_OUT_SPARSE, binding.KASCADE_OUT_DENSE):
            idx, out = call(q.to(DEV), k.to(DEV), v.to(DEV), i32(lens), i32(ks_w), 320, max(ks_w), recent_window=W,
                            out_mode=mode)
            torch.cuda.synchronize()
            idx_h, o = idx.cpu().numpy(), f64(out)
            n_sets = 1 if variant == "shared" else Hkv
            for b, (L, kb) in enumerate(zip(lens, ks_w)):
                assert (idx_h[b, :, kb:] == -1).all()
                if L == 0:
                    assert np.all(o[b] == 0.0)
                    continue
                qb, kb_, vb = f64(q[b]), f64(k[b, :, :L]), f64(v[b, :, :L])
                if kb > 0:
                    if variant == "per_head":
                        ref_idx, a = ko.decode_anchor_indices(qb, kb_, scale, kb, min(W, kb))
                    elif variant == "presoftmax":
                        ref_idx, a = ko.decode_presoftmax_indices(qb, kb_, scale, kb, storage, min(W, kb))
                    else:
                        ri, aa = ko.decode_shared_indices(qb, kb_, scale, kb, min(W, kb))
                        ref_idx, a = ri[None], aa[None]
                    for h in range(n_sets):
                        check_index_set(idx_h[b, h, :kb], ref_idx[h], a[h], n_forced=min(W, kb), where=f"b{b} h{h}")
                if mode == binding.KASCADE_OUT_DENSE:
                    want = ko.dense_decode(qb, kb_, vb, scale)
                elif kb == 0:
                    want = np.zeros_like(o[b])
                else:
                    sets = [idx_h[b, h, :kb] for h in range(n_sets)]
                    want = ko.sparse_decode(qb, kb_, vb, sets, scale, None if variant != "shared" else [0] * Hkv)
                assert max_abs(o[b], want) <= TOL_OUT[dtype], f"b{b} L{L} k{kb} mode{mode}"


@pytest.mark.parametrize("G,Hkv,d", [(1, 3, 128), (2, 2, 128), (4, 2, 128), (8, 2, 128), (8, 1, 128), (2, 2, 64), (8, 2, 64)])
def test_decode_reuse_matrix_unit_kernel_every_group_size(tuning, G, Hkv, d):
    """The gather kernel that runs q.k and P.V on the matrix unit (the default from eight heads per key
    head on), forced for every group size: ragged batch, one and many chunks, a head map, unordered
    lists with entries to ignore, an empty sequence; and the same bits as the unforced default where
    that is the same kernel."""
    print(f"case decode reuse on the matrix unit G={G} Hkv={Hkv} d={d}", flush=True)
    tuning(binding.TUNE_DECODE_FAMILY, binding.DECODE_FAMILY_MATRIX)
    dtype = torch.bfloat16
    Hq = G * Hkv
    lens, ks = [9000, 0, 777, 131, 40000], [4100, 0, 777, 5, 2000]
    B, k_max = len(lens), max(ks)
    q, k, v = random_case(40 + G, B, Hq, Hkv, d, dtype, lens)
    rs = np.random.default_rng(41 + G)
    n_anchor = max(1, Hkv - 1)
    hm = rs.integers(0, n_anchor, size=Hkv).tolist()
    idx = torch.full((B, n_anchor, k_max), -1, dtype=torch.int32)
    sets = []
    for b in range(B):
        sb = []
        for h in range(n_anchor):
            n_bad = min(ks[b], 2)
            good = rs.permutation(rs.choice(lens[b], ks[b] - n_bad, replace=False)) if ks[b] - n_bad > 0 else np.zeros(0, np.int64)
            row = rs.permutation(np.concatenate([good, [-1, lens[b] + 3][:n_bad]]).astype(np.int64))
            idx[b, h, : ks[b]] = torch.from_numpy(row).int()
            sb.append(np.asarray(good, dtype=np.int64))
        sets.append(sb)
    args = (q.to(DEV), k.to(DEV), v.to(DEV), i32(lens), i32(ks), k_max, idx.to(DEV))
    out = binding.kascade_decode_reuse(*args, head_map=i32(hm))
    torch.cuda.synchronize()
    o = f64(out)
    assert np.all(o[1] == 0.0)
    for b in range(B):
        if lens[b] == 0:
            continue
        L = lens[b]
        ref = ko.sparse_decode(f64(q[b]), f64(k[b, :, :L]), f64(v[b, :, :L]), sets[b], ko.default_scale(d), hm)
        assert max_abs(o[b], ref) <= TOL_OUT[dtype], f"sequence {b}"
    out2 = binding.kascade_decode_reuse(*args, head_map=i32(hm))
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    if G >= 8:
        tuning(binding.TUNE_DECODE_FAMILY, binding.DECODE_FAMILY_AUTO)
        out3 = binding.kascade_decode_reuse(*args, head_map=i32(hm))
        torch.cuda.synchronize()
        assert torch.equal(out, out3)


@pytest.mark.parametrize("G,Hkv,d", [(1, 2, 128), (2, 2, 128), (4, 2, 128), (8, 2, 128), (8, 1, 128), (4, 2, 64), (8, 1, 64)])
@pytest.mark.parametrize("out_mode", [0, 1])
def test_decode_anchor_matrix_unit_kernels_every_group_size(tuning, G, Hkv, d, out_mode):
    """The anchor's sweep over every key on the matrix unit (the default from eight heads per key head
    on), forced for every group size, with dense and sparse output: ragged lengths that end inside a
    pass, inside a run of eight logits and after a single key, an empty sequence, several chunks per
    sequence; and the same bits as the unforced default where that is the same kernel."""
    print(f"case decode anchor on the matrix unit G={G} Hkv={Hkv} d={d} out_mode={out_mode}", flush=True)
    tuning(binding.TUNE_DECODE_FAMILY, binding.DECODE_FAMILY_MATRIX)
    dtype = torch.bfloat16
    lens = [5000, 0, 1027, 1, 133, 2048]
    ks = [500, 0, 103, 1, 133, 64]
    W = 8
    ks = [max(k_, min(W, L)) for k_, L in zip(ks, lens)]
    q, k, v = random_case(60 + G, len(lens), G * Hkv, Hkv, d, dtype, lens)
    live = [b for b in range(len(lens)) if lens[b] > 0]
    # the oracle has no empty sequences: check those rows by hand, the others against it
    idx, out = binding.kascade_decode_anchor(q.to(DEV), k.to(DEV), v.to(DEV), i32(lens), i32(ks), max(lens), max(ks),
                                             recent_window=W, out_mode=out_mode)
    torch.cuda.synchronize()
    assert (idx[1] == -1).all() and (out[1] == 0).all()
    scale = ko.default_scale(d)
    swaps, worst = 0, 0.0
    idx_np, o = idx.cpu().numpy(), f64(out)
    for b in live:
        L, kb = lens[b], ks[b]
        qb, kb_, vb = f64(q[b]), f64(k[b, :, :L]), f64(v[b, :, :L])
        idx_ref, a = ko.decode_anchor_indices(qb, kb_, scale, kb, min(W, kb))
        for h in range(Hkv):
            assert (idx_np[b, h, kb:] == -1).all()
            swaps += check_index_set(idx_np[b, h, :kb], idx_ref[h], a[h], n_forced=min(W, kb), where=f"b{b} h{h}")
        ref = ko.dense_decode(qb, kb_, vb, scale) if out_mode == binding.KASCADE_OUT_DENSE else \
            ko.sparse_decode(qb, kb_, vb, [idx_np[b, h, :kb] for h in range(Hkv)], scale)
        worst = max(worst, max_abs(o[b], ref))
    print(f"  swaps {swaps}, max-abs {worst:.3e}", flush=True)
    assert worst <= TOL_OUT[dtype]
    if G >= 8:
        tuning(binding.TUNE_DECODE_FAMILY, binding.DECODE_FAMILY_AUTO)
        idx2, out2 = binding.kascade_decode_anchor(q.to(DEV), k.to(DEV), v.to(DEV), i32(lens), i32(ks), max(lens),
                                                   max(ks), recent_window=W, out_mode=out_mode)
        torch.cuda.synchronize()
        assert torch.equal(idx, idx2) and torch.equal(out, out2)


@pytest.mark.parametrize("G,Hkv,d", [(3, 2, 128), (5, 1, 128), (6, 2, 128), (7, 4, 128), (12, 1, 128), (16, 2, 128),
                                     (7, 2, 64), (16, 1, 64)])
def test_decode_group_sizes_that_are_not_powers_of_two(G, Hkv, d):
    """bf16 caches take any number of query heads per key head up to 16 (the matrix-unit
    kernels and the pooling kernel with a run-time group size): anchor layer with both output modes, the
    shared-set and Pre-Softmax variants, and a reuse layer with a head map, on a ragged batch with an empty
    sequence."""
    print(f"case decode G={G} Hkv={Hkv} d={d}", flush=True)
    dtype = torch.bfloat16
    lens, ks, W = [4100, 0, 700, 9], [410, 0, 70, 9], 4
    B, Hq = len(lens), G * Hkv
    q, k, v = random_case(70 + G, B, Hq, Hkv, d, dtype, lens)
    scale = ko.default_scale(d)
    args = (q.to(DEV), k.to(DEV), v.to(DEV), i32(lens), i32(ks), max(lens), max(ks))
    for variant in ("per_head", "shared", "presoftmax"):
        call = {"per_head": binding.kascade_decode_anchor, "shared": binding.kascade_decode_anchor_shared,
                "presoftmax": binding.kascade_decode_anchor_presoftmax}[variant]
        n_sets = 1 if variant == "shared" else Hkv
        for mode in (binding.KASCADE_OUT_SPARSE, binding.KASCADE_OUT_DENSE):
            idx, out = call(*args, recent_window=W, out_mode=mode)
            torch.cuda.synchronize()
            idx_h, o = idx.cpu().numpy(), f64(out)
            assert (idx_h[1] == -1).all() and np.all(o[1] == 0.0)
            swaps = 0
            for b, (L, kb) in enumerate(zip(lens, ks)):
                if L == 0:
                    continue
                qb, kb_, vb = f64(q[b]), f64(k[b, :, :L]), f64(v[b, :, :L])
                if variant == "per_head":
                    ref_idx, a = ko.decode_anchor_indices(qb, kb_, scale, kb, W)
                elif variant == "presoftmax":
                    ref_idx, a = ko.decode_presoftmax_indices(qb, kb_, scale, kb, "bf16", W)
                else:
                    ri, aa = ko.decode_shared_indices(qb, kb_, scale, kb, W)
                    ref_idx, a = ri[None], aa[None]
                for h in range(n_sets):
                    assert (idx_h[b, h, kb:] == -1).all()
                    swaps += check_index_set(idx_h[b, h, :kb], ref_idx[h], a[h], n_forced=W, where=f"{variant} b{b} h{h}")
                if mode == binding.KASCADE_OUT_DENSE:
                    want = ko.dense_decode(qb, kb_, vb, scale)
                else:
                    sets = [idx_h[b, h, :kb] for h in range(n_sets)]
                    want = ko.sparse_decode(qb, kb_, vb, sets, scale, None if variant != "shared" else [0] * Hkv)
                assert max_abs(o[b], want) <= TOL_OUT[dtype], f"{variant} b{b} mode{mode}"
            print(f"  {variant} mode {mode}: swaps {swaps}", flush=True)
    # a reuse layer over the per-head sets of another layer, heads mapped
    idx, _ = binding.kascade_decode_anchor(*args, recent_window=W, out_mode=binding.KASCADE_OUT_SPARSE)
    q2, k2, v2 = random_case(170 + G, B, Hq, Hkv, d, dtype, lens)
    hm = [(h + 1) % Hkv for h in range(Hkv)]
    out = binding.kascade_decode_reuse(q2.to(DEV), k2.to(DEV), v2.to(DEV), i32(lens), i32(ks), max(ks), idx, head_map=i32(hm))
    torch.cuda.synchronize()
    idx_h, o = idx.cpu().numpy(), f64(out)
    for b, (L, kb) in enumerate(zip(lens, ks)):
        if L == 0:
            assert np.all(o[b] == 0.0)
            continue
        sets = [idx_h[b, h, :kb] for h in range(Hkv)]
        want = ko.sparse_decode(f64(q2[b]), f64(k2[b, :, :L]), f64(v2[b, :, :L]), sets, scale, hm)
        assert max_abs(o[b], want) <= TOL_OUT[dtype], f"reuse b{b}"


@pytest.mark.parametrize("dtype,d,G", [(torch.bfloat16, 128, 4), (torch.bfloat16, 128, 8), (torch.float32, 64, 2)])
@pytest.mark.parametrize("variant", ["per_head", "shared", "presoftmax"])
def test_decode_anchor_holds_lengths_to_max_seqlen(dtype, d, G, variant):
    """max_seqlen sizes the grid and the workspace; a device-side length above it is processed as
    max_seqlen (same bits as the call with the lengths already cut), never written past the buffers."""
    print(f"case lengths above max_seqlen dtype={dtype} d={d} G={G} variant={variant}", flush=True)
    Hkv, max_seqlen = 2, 1500
    q, k, v = random_case(321, 3, G * Hkv, Hkv, d, dtype, [max_seqlen] * 3)
    call = {"per_head": binding.kascade_decode_anchor, "shared": binding.kascade_decode_anchor_shared,
            "presoftmax": binding.kascade_decode_anchor_presoftmax}[variant]
    ks = [150, 20, 150]
    for mode in (binding.KASCADE_OUT_SPARSE, binding.KASCADE_OUT_DENSE):
        res = []
        for lens in ([max_seqlen + 500, 77, max_seqlen + 1], [max_seqlen, 77, max_seqlen]):
            idx, out = call(q.to(DEV), k.to(DEV), v.to(DEV), i32(lens), i32(ks), max_seqlen, max(ks), recent_window=4,
                            out_mode=mode)
            torch.cuda.synchronize()
            res.append((idx.clone(), out.clone()))
        assert torch.equal(res[0][0], res[1][0]) and torch.equal(res[0][1], res[1][1])
        assert int(res[0][0].max()) < max_seqlen


@pytest.mark.parametrize("dtype,d,G", [(torch.bfloat16, 128, 4), (torch.bfloat16, 128, 8), (torch.bfloat16, 64, 2),
                                       (torch.float32, 64, 4)])
@pytest.mark.parametrize("out_mode", [0, 1])
def test_decode_anchor_token_major_cache(dtype, d, G, out_mode):
    """Anchor layer over a cache laid out [B, L, Hkv, d] (rows of a key head Hkv*d elements apart) with a
    custom softmax scale: the same bits as over the head-major copy of the cache."""
    print(f"case anchor token-major cache dtype={dtype} d={d} G={G} out_mode={out_mode}", flush=True)
    Hkv, lens, ks = 2, [1300, 257, 40], [130, 26, 40]
    q, k, v = random_case(55, 3, G * Hkv, Hkv, d, dtype, lens)
    a = (i32(lens), i32(ks), max(lens), max(ks))
    idx0, out0 = binding.kascade_decode_anchor(q.to(DEV), k.to(DEV), v.to(DEV), *a, recent_window=2, out_mode=out_mode,
                                               softmax_scale=0.11)
    k_t, v_t = k.permute(0, 2, 1, 3).contiguous(), v.permute(0, 2, 1, 3).contiguous()
    idx1, out1 = binding.kascade_decode_anchor(q.to(DEV), k_t.to(DEV), v_t.to(DEV), *a, recent_window=2, out_mode=out_mode,
                                               softmax_scale=0.11, kv_layout="BLHD")
    torch.cuda.synchronize()
    assert torch.equal(idx0, idx1) and torch.equal(out0, out1)
    # and the head-major result against the oracle
    idx_h, o = idx0.cpu().numpy(), f64(out0)
    for b, (L, kb) in enumerate(zip(lens, ks)):
        qb, kb_, vb = f64(q[b]), f64(k[b, :, :L]), f64(v[b, :, :L])
        ref_idx, aa = ko.decode_anchor_indices(qb, kb_, 0.11, kb, 2)
        for h in range(Hkv):
            check_index_set(idx_h[b, h, :kb], ref_idx[h], aa[h], n_forced=2, where=f"b{b} h{h}")
        want = ko.dense_decode(qb, kb_, vb, 0.11) if out_mode == binding.KASCADE_OUT_DENSE else \
            ko.sparse_decode(qb, kb_, vb, [idx_h[b, h, :kb] for h in range(Hkv)], 0.11)
        assert max_abs(o[b], want) <= TOL_OUT[dtype]


def test_decode_one_request_of_a_million_tokens():
    """Longest single sequence the sweeps are timed at (Table 3's 512K, doubled): 32/8 heads, d 128, bf16, one
    request of 1,048,576 tokens, k = 1 % with a 64-token recent window; anchor (sparse output) and a reuse
    layer on a second query.  Row offsets pass 2^28 bytes per key head and the selection runs split over many
    workgroups.  The oracle takes one key head at a time (a head's fp64 K and V are 2 GB)."""
    print("case one million tokens", flush=True)
    L, Hq, Hkv, d, W = 1 << 20, 32, 8, 128, 64
    G = Hq // Hkv
    kk = workloads.budget(L, 10)
    g = torch.Generator(device=DEV).manual_seed(4242)
    q = torch.randn(2, 1, Hq, d, generator=g, device=DEV).to(torch.bfloat16)
    k = torch.randn(1, Hkv, L, d, generator=g, device=DEV).to(torch.bfloat16)
    v = torch.randn(1, Hkv, L, d, generator=g, device=DEV).to(torch.bfloat16)
    # planted hitters so that the pooled scores are not flat: 4096 keys per head lean towards the head's queries
    for h in range(Hkv):
        u = torch.nn.functional.normalize(torch.randn(d, generator=g, device=DEV), dim=0)
        pos = torch.randperm(L, generator=g, device=DEV)[:4096]
        k[0, h, pos] = (k[0, h, pos].float() + 3.0 * u).to(torch.bfloat16)
        q[:, 0, h * G:(h + 1) * G] = (q[:, 0, h * G:(h + 1) * G].float() + u).to(torch.bfloat16)
    sl, kp = i32([L]), i32([kk])
    idx_d, o_anchor = binding.kascade_decode_anchor(q[0], k, v, sl, kp, L, kk, recent_window=W,
                                                    out_mode=binding.KASCADE_OUT_SPARSE)
    o_reuse = binding.kascade_decode_reuse(q[1], k, v, sl, kp, kk, idx_d)
    torch.cuda.synchronize()
    idx = idx_d.cpu().numpy()
    scale = ko.default_scale(d)
    swaps, worst = 0, 0.0
    for h in range(Hkv):
        kh, vh = f64(k[0, h:h + 1]), f64(v[0, h:h + 1])
        qa, qr = f64(q[0, 0, h * G:(h + 1) * G]), f64(q[1, 0, h * G:(h + 1) * G])
        idx_ref, pooled = ko.decode_anchor_indices(qa, kh, scale, kk, W)
        swaps += check_index_set(idx[0, h, :kk], idx_ref[0], pooled[0], n_forced=W, where=f"1M head {h}")
        sets = [idx[0, h, :kk]]
        worst = max(worst, max_abs(f64(o_anchor[0, h * G:(h + 1) * G]), ko.sparse_decode(qa, kh, vh, sets, scale)),
                    max_abs(f64(o_reuse[0, h * G:(h + 1) * G]), ko.sparse_decode(qr, kh, vh, sets, scale)))
        del kh, vh
    print(f"  1M tokens k={kk}: swaps {swaps}, max-abs {worst:.3e}", flush=True)
    assert worst <= TOL_OUT[torch.bfloat16]
