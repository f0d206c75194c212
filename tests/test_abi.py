"""The C-ABI library loads, exports what include/kascade.h declares, and rejects bad
arguments before any launch (no GPU needed: none of these calls reaches a kernel)."""
import ctypes
import os
import re

import pytest

from paper_2512_16391_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return binding.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "kascade.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kascade_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(binding.EXPORTS) == set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings_and_version(lib):
    assert binding.status_string(0) == "ok"
    for st in range(-5, 0):
        assert binding.status_string(st) not in ("ok", "unknown status")
    assert binding.status_string(-99) == "unknown status"
    assert re.match(r"^\d+\.\d+$", binding.version())


def make_desc(**kw):
    d = binding.KascadeDesc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim, d.dtype = 2, 8, 2, 64, binding.KASCADE_F32
    d.softmax_scale = 0.0
    d.q_stride[:] = (8 * 64, 0, 64)
    d.kv_stride[:] = (2 * 100 * 64, 100 * 64, 64)
    d.o_stride[:] = (8 * 64, 0, 64)
    for k, v in kw.items():
        if isinstance(v, tuple):
            getattr(d, k)[:] = v
        else:
            setattr(d, k, v)
    return d


def call_reuse(lib, d, q=0x1000, k=0x2000, v=0x3000, sl=0x4000, kp=0x5000, kmax=10, idx=0x6000, nah=2, hm=0,
               out=0x7000, ws=0x8000, wsb=1 << 30):
    vp = ctypes.c_void_p
    return lib.kascade_decode_reuse(ctypes.byref(d), vp(q), vp(k), vp(v), vp(sl), vp(kp), kmax, vp(idx), nah, vp(hm),
                                    vp(out), vp(ws), wsb, vp(0))


def test_argument_checks_happen_before_any_launch(lib):
    # the pointers are fake: every call below must return from validation
    assert call_reuse(lib, make_desc(head_dim=96)) == -2
    assert call_reuse(lib, make_desc(dtype=7)) == -2
    assert call_reuse(lib, make_desc(dtype=3)) == -2
    assert call_reuse(lib, make_desc(n_q_heads=6, n_kv_heads=2)) == -2          # G = 3 in fp32 / head_dim 64: not built
    wide = dict(head_dim=128, dtype=binding.KASCADE_BF16, q_stride=(34 * 128, 0, 128), o_stride=(34 * 128, 0, 128),
                kv_stride=(2 * 100 * 128, 100 * 128, 128))
    assert call_reuse(lib, make_desc(n_q_heads=34, n_kv_heads=2, **wide)) == -2    # G = 17: beyond the matrix-unit kernels
    assert call_reuse(lib, make_desc(n_q_heads=7)) == -1
    assert call_reuse(lib, make_desc(batch=0)) == -1
    assert call_reuse(lib, make_desc(), q=0) == -1
    assert call_reuse(lib, make_desc(), kmax=0) == -1
    assert call_reuse(lib, make_desc(), nah=3) == -1                             # identity map needs Hkv rows
    assert call_reuse(lib, make_desc(), k=0x2004) == -3
    assert call_reuse(lib, make_desc(kv_stride=(12800, 6400, 66))) == -3
    assert call_reuse(lib, make_desc(kv_stride=(12800, 6400, 32))) == -1         # rows overlap
    assert call_reuse(lib, make_desc(), wsb=16) == -4
    assert call_reuse(lib, make_desc(), ws=0) == -4


def test_workspace_query(lib):
    d = make_desc()
    reuse = binding.kascade_workspace_bytes(binding.OP_DECODE_REUSE, d, 100, 10)
    anchor = binding.kascade_workspace_bytes(binding.OP_DECODE_ANCHOR, d, 100, 10)
    assert reuse > 0 and anchor > reuse
    assert anchor >= 2 * 8 * 100 * 4 + 2 * 2 * 100 * 4       # logits + pooled scores in fp32
    assert binding.kascade_workspace_bytes(99, d, 100, 10) == 0
    assert binding.kascade_workspace_bytes(binding.OP_DECODE_REUSE, make_desc(head_dim=96), 100, 10) == 0


def test_binding_refuses_cpu_tensors(lib):
    import torch
    q = torch.zeros(1, 8, 64)
    k = torch.zeros(1, 2, 16, 64)
    sl = torch.tensor([16], dtype=torch.int32)
    idx = torch.zeros(1, 2, 4, dtype=torch.int32)
    with pytest.raises(RuntimeError, match="GPU"):
        binding.kascade_decode_reuse(q, k, k, sl, sl, 4, idx)


def call_prefill_reuse(lib, d, S, T, q=0x1000, k=0x2000, v=0x3000, kpt=0x4000, off=0x5000, total=10, idx=0x6000,
                       out=0x7000):
    vp = ctypes.c_void_p
    return lib.kascade_prefill_reuse(ctypes.byref(d), vp(q), vp(k), vp(v), S, T, vp(kpt), vp(off), total, vp(idx),
                                     d.n_kv_heads, vp(0), vp(out), vp(0), 0, vp(0))


def test_prefill_argument_checks(lib):
    # fake pointers again: all of these return from validation
    bf = dict(batch=1, n_q_heads=32, n_kv_heads=8, head_dim=128, dtype=binding.KASCADE_BF16,
              q_stride=(0, 32 * 128, 128), kv_stride=(0, 4096 * 128, 128), o_stride=(0, 32 * 128, 128))
    assert call_prefill_reuse(lib, make_desc(**bf), 4096, 16) == -2                       # T * G = 64
    assert call_prefill_reuse(lib, make_desc(**bf), 4096, 48) == -2                       # T * G = 192
    assert call_prefill_reuse(lib, make_desc(**{**bf, "dtype": binding.KASCADE_F32}), 4096, 32) == -2
    assert call_prefill_reuse(lib, make_desc(**{**bf, "n_q_heads": 24, "q_stride": (0, 24 * 128, 128),
                                                "o_stride": (0, 24 * 128, 128)}), 4096, 128) == -2   # G = 3: decode only
    assert call_prefill_reuse(lib, make_desc(**{**bf, "batch": 2}), 4096, 32) == -1
    assert call_prefill_reuse(lib, make_desc(**bf), 0, 32) == -1
    assert call_prefill_reuse(lib, make_desc(**bf), 4096, 32, idx=0) == -1
    assert call_prefill_reuse(lib, make_desc(**bf), 4096, 32, k=0x2008) == -3
    # one key head's rows must stay below 4 GiB: 2^24 tokens of 256 bytes are exactly 4 GiB
    huge = {**bf, "kv_stride": (0, (1 << 24) * 128, 128)}
    assert call_prefill_reuse(lib, make_desc(**huge), 1 << 24, 32) == -2


def test_binding_fails_loudly_without_library_or_gpu(tmp_path):
    """There is no fallback path: a missing library and host tensors are errors, not detours."""
    import torch
    with pytest.raises(RuntimeError, match="not built"):
        binding.load_library(str(tmp_path / "libkascade_missing.so"))
    q = torch.zeros(1, 8, 64)
    k = torch.zeros(1, 2, 16, 64)
    lens = torch.tensor([16], dtype=torch.int32)
    with pytest.raises(RuntimeError, match="GPU"):
        binding.kascade_decode_anchor(q, k, k, lens, lens, 16, 16)
    with pytest.raises(RuntimeError, match="GPU"):
        binding.kascade_decode_reuse(q, k, k, lens, lens, 16, torch.zeros(1, 2, 16, dtype=torch.int32))
    with pytest.raises(RuntimeError, match="GPU"):
        binding.kascade_prefill_reuse(torch.zeros(32, 8, 64), torch.zeros(2, 32, 64), torch.zeros(2, 32, 64), 16,
                                      torch.zeros(2, dtype=torch.int32), torch.zeros(3, dtype=torch.int64), 0,
                                      torch.zeros(2, 1, dtype=torch.int32))
