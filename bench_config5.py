#!/usr/bin/env python3
"""The 32-layer attention-only stack of the largest configuration, end to end on one MI355X:
32/8 heads, head dimension 128, bf16; causal prefill of 131072 tokens (tiles of 32 tokens x 4
heads, k_t = 10 % of the prefix), then 256 decode steps at batch 1 with fresh random q/k/v per
step and layer (k = 10 % of the context).  Anchor layers {0, 1, 4, 12, 20} (layer 0 returns
dense attention, Sec. 3.1); every other layer reuses the nearest preceding anchor's index sets
(Sec. 3.2).  Seeded synthetic inputs; planted heavy hitters drift 15 % per layer.

Timing only (parity of these shapes is covered by the GPU tests).  Prints one JSON line.
Not part of bench.py's contract.  Needs about 35 GB of HBM."""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--seqlen", type=int, default=131072)
    ap.add_argument("--decode-steps", type=int, default=256)
    ap.add_argument("--layers", type=int, default=32)
    args = ap.parse_args()
    import torch
    from paper_2512_16391_amd import binding, workloads
    if not torch.cuda.is_available():
        print("bench_config5.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    binding.load_library()
    dev = torch.device("cuda:0")
    S, T, steps, NL = args.seqlen, 32, args.decode_steps, args.layers
    Hq, Hkv, d = 32, 8, 128
    anchors = set(a for a in workloads.CONFIG5_ANCHORS if a < NL)

    # ---- prefill, layer by layer (a layer's q is dropped after use; K/V stay for the decode steps)
    kpt_h = workloads.prefill_budgets(S, T, 100, 0)
    off_h = [0]
    for kt in kpt_h:
        off_h.append(off_h[-1] + kt)
    total = off_h[-1]
    kpt = torch.tensor(kpt_h, dtype=torch.int32, device=dev)
    off = torch.tensor(off_h, dtype=torch.int64, device=dev)
    idx = torch.empty(Hkv, total, dtype=torch.int32, device=dev)
    out = torch.empty(S, Hq, d, dtype=torch.bfloat16, device=dev)
    ws = None
    caches, prefill_ms = [], []
    for layer, data in workloads.iter_config5_layers(dev, NL, S, steps):
        if ws is None:
            desc = binding.prefill_desc(data.q, data.k[:, :S])
            ws = torch.empty(binding.kascade_workspace_bytes(binding.OP_PREFILL_ANCHOR, desc, S, total, T),
                             dtype=torch.uint8, device=dev)
        k, v = data.k[:, :S], data.v[:, :S]
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        if layer in anchors:
            mode = binding.KASCADE_OUT_DENSE if layer == 0 else binding.KASCADE_OUT_SPARSE
            binding.kascade_prefill_anchor(data.q, k, v, T, kpt, off, total, mode, idx, out, ws)
        else:
            binding.kascade_prefill_reuse(data.q, k, v, T, kpt, off, total, idx, None, None, out, ws)
        e1.record()
        e1.synchronize()
        prefill_ms.append(e0.elapsed_time(e1))
        caches.append((data.k, data.v))
        print(f"prefill layer {layer:2d} ({'anchor' if layer in anchors else 'reuse '}): {prefill_ms[-1]:8.2f} ms", file=sys.stderr, flush=True)
        del data
    del ws, idx, out
    torch.cuda.empty_cache()

    # ---- decode: one token per step, every layer appends its k/v row and attends over L = S + step + 1
    gen = torch.Generator(device=dev)
    gen.manual_seed(workloads.layer_seed(workloads.BASE_SEED, 5, 1000))
    Lmax = S + steps
    kmax = workloads.budget(Lmax, 100)
    didx = torch.empty(1, Hkv, kmax, dtype=torch.int32, device=dev)
    dout = torch.empty(1, Hq, d, dtype=torch.bfloat16, device=dev)
    q0 = torch.empty(1, Hq, d, dtype=torch.bfloat16, device=dev)
    ddesc = binding.decode_desc(q0, caches[0][0].unsqueeze(0))
    dws = torch.empty(binding.kascade_workspace_bytes(binding.OP_DECODE_ANCHOR, ddesc, Lmax, kmax), dtype=torch.uint8, device=dev)
    # all of a step's random rows are drawn before the step is timed; lengths and budgets live in device
    # tensors, the host arguments (max_seqlen, k_max) are the same for every step - so the step's launches
    # can also be captured once into a HIP graph and replayed
    sl = torch.zeros(1, dtype=torch.int32, device=dev)
    kp = torch.zeros(1, dtype=torch.int32, device=dev)
    qs = torch.zeros(NL, 1, Hq, d, dtype=torch.bfloat16, device=dev)

    def decode_step():
        for layer, (kc, vc) in enumerate(caches):
            kb, vb = kc.unsqueeze(0), vc.unsqueeze(0)
            if layer in anchors:
                mode = binding.KASCADE_OUT_DENSE if layer == 0 else binding.KASCADE_OUT_SPARSE
                binding.kascade_decode_anchor(qs[layer], kb, vb, sl, kp, Lmax, kmax, 0, mode, didx, dout, dws)
            else:
                binding.kascade_decode_reuse(qs[layer], kb, vb, sl, kp, kmax, didx, None, dout, dws)

    def run_steps(launch):
        times = []
        for step in range(steps):
            L = S + step + 1
            sl.fill_(L)
            kp.fill_(workloads.budget(L, 100))
            qs.copy_(torch.randn(NL, 1, Hq, d, generator=gen, device=dev))
            rows = torch.randn(NL, 2, Hkv, d, generator=gen, device=dev).to(torch.bfloat16)
            for layer, (kc, vc) in enumerate(caches):
                kc[:, L - 1] = rows[layer, 0]
                vc[:, L - 1] = rows[layer, 1]
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            launch()
            e1.record()
            e1.synchronize()
            times.append(e0.elapsed_time(e1))
        return times

    step_ms = run_steps(decode_step)
    graph_ms = None
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            decode_step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            decode_step()
        graph_ms = sorted(run_steps(g.replay))
    except Exception as exc:
        print(f"bench_config5.py: graph replay skipped: {exc}", file=sys.stderr)
    step_sorted = sorted(step_ms)
    n_anchor = len(anchors)
    rec = {
        "workload": f"cfg5: {NL} attention layers, prefill {S} tokens then {steps} decode steps, batch 1, Top-k 10 %, anchors {sorted(anchors)}",
        "dtype": "bf16", "data": "synthetic",
        "prefill_s": round(sum(prefill_ms) / 1e3, 4),
        "prefill_tokens_per_s": round(S / (sum(prefill_ms) / 1e3), 1),
        "prefill_layer_ms": {"layer0_dense_anchor": round(prefill_ms[0], 2),
                             "anchor_mean": round(sum(prefill_ms[a] for a in anchors if a) / max(n_anchor - 1, 1), 2),
                             "reuse_mean": round(sum(m for i, m in enumerate(prefill_ms) if i not in anchors) / max(NL - n_anchor, 1), 2)},
        "decode_ms_per_step_p10_p50_p90": [round(step_sorted[int(f * (len(step_sorted) - 1))], 4) for f in (0.1, 0.5, 0.9)],
        "decode_tokens_per_s": round(1e3 / step_sorted[len(step_sorted) // 2], 1),
        "decode_us_per_layer": round(step_sorted[len(step_sorted) // 2] * 1e3 / NL, 2),
        "decode_step_as_hip_graph_ms_p50": round(graph_ms[len(graph_ms) // 2], 4) if graph_ms else None,
        "decode_tokens_per_s_hip_graph": round(1e3 / graph_ms[len(graph_ms) // 2], 1) if graph_ms else None,
    }
    print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
