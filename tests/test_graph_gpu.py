"""The entry points enqueue kernels only (no allocation, no synchronisation, no memset nodes), so a
sequence of calls can be captured into a HIP graph.  Every replay must reproduce the eager bits."""
import pytest
import torch

from paper_2512_16391_amd import binding, workloads

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def i32(x):
    return torch.tensor(x, dtype=torch.int32, device=DEV)


def replay_matches(run, outputs, n_replays=3):
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):       # warm-up on a side stream, as graph capture wants
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    run()
    torch.cuda.synchronize()
    eager = [o.clone() for o in outputs]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run()
    for _ in range(n_replays):
        for o in outputs:
            o.fill_(0)                  # eager work between replays; also proves the replay rewrites everything
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for e, o in zip(eager, outputs):
            assert torch.equal(e, o)


def test_decode_step_with_split_selection_in_a_graph():
    print("case graph decode (split selection)", flush=True)
    B, Hq, Hkv, d = 1, 8, 2, 128
    lens, ks = [70000], [7000]
    wl = workloads.make_decode_workload("graph", 13, 2, B, Hq, Hkv, d, torch.bfloat16, lens, ks, 256, 0.8, device=DEV)
    a, r = wl.layers
    sl, kp = i32(lens), i32(ks)
    L, k = lens[0], ks[0]
    idx = torch.empty(B, Hkv, k, dtype=torch.int32, device=DEV)
    out_a, out_r = torch.empty_like(a.q), torch.empty_like(r.q)
    desc = binding.decode_desc(a.q, a.k)
    ws = torch.empty(binding.kascade_workspace_bytes(binding.OP_DECODE_ANCHOR, desc, L, k), dtype=torch.uint8, device=DEV)

    def run():
        binding.kascade_decode_anchor(a.q, a.k, a.v, sl, kp, L, k, 0, binding.KASCADE_OUT_SPARSE, idx, out_a, ws)
        binding.kascade_decode_reuse(r.q, r.k, r.v, sl, kp, k, idx, None, out_r, ws)

    replay_matches(run, [idx, out_a, out_r])


def test_prefill_anchor_and_reuse_in_a_graph():
    print("case graph prefill", flush=True)
    wl = workloads.config4(device=DEV, n_layers=2, S=2048)
    a, r = wl.layers
    off = wl.idx_offsets
    kpt = i32(wl.k_per_tile)
    offs = torch.tensor(off, dtype=torch.int64, device=DEV)
    idx = torch.empty(wl.Hkv, off[-1], dtype=torch.int32, device=DEV)
    out_a, out_r = torch.empty_like(a.q), torch.empty_like(r.q)
    desc = binding.prefill_desc(a.q, a.k)
    ws = torch.empty(binding.kascade_workspace_bytes(binding.OP_PREFILL_ANCHOR, desc, wl.S, off[-1], wl.T),
                     dtype=torch.uint8, device=DEV)

    def run():
        binding.kascade_prefill_anchor(a.q, a.k, a.v, wl.T, kpt, offs, off[-1], binding.KASCADE_OUT_SPARSE, idx, out_a, ws)
        binding.kascade_prefill_reuse(r.q, r.k, r.v, wl.T, kpt, offs, off[-1], idx, None, None, out_r, ws)

    replay_matches(run, [idx, out_a, out_r])
