"""The reuse-layer entry point that allocates nothing (its partial results live in a fixed device array of
the library): same bits as kascade_decode_reuse, on two calls in a row, the second with a smaller input."""
import pytest
import torch

from paper_2512_16391_amd import binding, workloads

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def i32(x):
    return torch.tensor(x, dtype=torch.int32, device=DEV)


def one_case(seed, B, Hq, Hkv, d, dtype, lens, ks):
    wl = workloads.make_decode_workload("no-alloc", 30 + seed, 2, B, Hq, Hkv, d, dtype, lens, ks, 200, 0.8)
    a, r = wl.layers
    k_max = max(ks)
    idx, _ = binding.kascade_decode_anchor(a.q.to(DEV), a.k.to(DEV), a.v.to(DEV), i32(lens), i32(ks), max(lens), k_max)
    args = (r.q.to(DEV), r.k.to(DEV), r.v.to(DEV), i32(lens), i32(ks), k_max, idx)
    want = binding.kascade_decode_reuse(*args)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    out = torch.empty_like(want)
    got = binding.kascade_decode_reuse_static(*args, out=out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() - before == out.numel() * out.element_size()   # the caller's output only
    assert torch.equal(got, want), f"seed {seed}: outputs differ"
    return got


def test_zz_decode_reuse_static_matches_the_workspace_entry_point():
    print("case no-alloc reuse: large call, then a smaller one", flush=True)
    assert binding.kascade_decode_reuse_static_capacity() == 8 << 20
    # several chunks per (sequence, head): partial results go through the fixed array and the merge kernel
    one_case(0, 4, 32, 8, 128, torch.bfloat16, [20000, 9000, 16384, 777], [6000, 900, 1639, 78])
    # a smaller input right after it: one chunk per pair, then a few short ragged sequences
    one_case(1, 2, 8, 2, 128, torch.bfloat16, [3000, 1500], [300, 150])
    one_case(2, 3, 8, 2, 64, torch.float32, [2048, 5, 300], [205, 5, 30])


def test_zz_decode_reuse_static_refuses_what_does_not_fit():
    B, Hq, Hkv, d = 4096, 32, 8, 128          # 4096 x 32 heads x (2 + 128) floats = 68 MB of partial results
    q = torch.zeros(B, Hq, d, dtype=torch.bfloat16, device=DEV)
    kv = torch.zeros(1, Hkv, 64, d, dtype=torch.bfloat16, device=DEV).expand(B, Hkv, 64, d)
    idx = torch.zeros(B, Hkv, 8, dtype=torch.int32, device=DEV)
    lens = torch.full((B,), 64, dtype=torch.int32, device=DEV)
    ks = torch.full((B,), 8, dtype=torch.int32, device=DEV)
    with pytest.raises(binding.KascadeError) as err:
        binding.kascade_decode_reuse_static(q, kv, kv, lens, ks, 8, idx)
    assert err.value.status == -4
