#!/usr/bin/env python3
"""Attention-only sweep in the layout of the paper's Table 3 (Sec. 4.3), on one MI355X.

For every context length: time of the three layer kinds (anchor with dense output = layer 0,
anchor with sparse output, reuse), the paper's weighted per-layer average
(1 x anchor-0 + 4 x anchor + 27 x reuse) / 32, and this library's own dense pass as the
same-hardware denominator of the speed-up column (decode: the K/V streaming kernel of the
layer-0 anchor plus its merge; prefill: the causal flash sweep of the layer-0 anchor; both do
slightly MORE than a plain dense kernel - they also store logits / row statistics - so the
speed-ups printed here are upper-bounded by that).  Shapes follow the paper: Llama-3.1-8B
attention (32 query heads, 8 key heads, head dimension 128), decode batch 64 (32 at 524288),
prefill batch 1, Top-k 10 % (plus 20 % and 30 % at one length); bf16 (or fp16 with --dtype fp16, the
precision of the paper's own timings), seeded synthetic inputs.

Prints one JSON line per row and a text table at the end.  Not part of bench.py's contract.
"""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# the paper's H100 / fp16 numbers for the same rows (ms per layer: Kascade average, speed-up over FA3)
PAPER_DECODE = {(8192, 100): (0.24, 2.91), (32768, 100): (0.74, 3.97), (65536, 100): (1.43, 4.08),
                (131072, 100): (2.83, 4.12), (262144, 100): (5.34, 4.08), (524288, 100): (5.33, 4.10),
                (131072, 200): (4.01, 2.92), (131072, 300): (5.39, 2.17)}
PAPER_PREFILL = {(8192, 100): (0.62, 1.23), (32768, 100): (6.42, 1.91), (65536, 100): (24.63, 2.18),
                 (131072, 100): (98.55, 2.19), (32768, 200): (8.65, 1.42), (32768, 300): (10.70, 1.15)}


def timed(torch, fn, reps):
    fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / reps


def kernel_ms(binding, torch, fn, names, reps):
    """Summed device time of the named library kernels over one call of fn (event pairs)."""
    binding.kascade_profile_enable(True)
    binding.kascade_profile_reset()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    prof = binding.kascade_profile_read()
    binding.kascade_profile_enable(False)
    return sum(prof[n][0] for n in names if n in prof) / reps


def decode_row(torch, binding, workloads, dev, L, B, permille, reps, dtype):
    k = workloads.budget(L, permille)
    wl = workloads.make_decode_workload(f"table3-decode-L{L}-B{B}", 7, 1, B, 32, 8, 128, dtype, [L] * B,
                                        [k] * B, 1024, 0.85, device=dev, keep_hitters=False)
    a = wl.layers[0]
    seqlens = torch.full((B,), L, dtype=torch.int32, device=dev)
    kps = torch.full((B,), k, dtype=torch.int32, device=dev)
    idx = torch.empty(B, 8, k, dtype=torch.int32, device=dev)
    out = torch.empty_like(a.q)
    desc = binding.decode_desc(a.q, a.k)
    ws = torch.empty(binding.kascade_workspace_bytes(binding.OP_DECODE_ANCHOR, desc, L, k), dtype=torch.uint8, device=dev)
    anchor0 = lambda: binding.kascade_decode_anchor(a.q, a.k, a.v, seqlens, kps, L, k, 0, binding.KASCADE_OUT_DENSE, idx, out, ws)
    anchor = lambda: binding.kascade_decode_anchor(a.q, a.k, a.v, seqlens, kps, L, k, 0, binding.KASCADE_OUT_SPARSE, idx, out, ws)
    reuse = lambda: binding.kascade_decode_reuse(a.q, a.k, a.v, seqlens, kps, k, idx, None, out, ws)
    t_a0, t_a, t_r = timed(torch, anchor0, reps), timed(torch, anchor, reps), timed(torch, reuse, reps * 4)
    t_dense = kernel_ms(binding, torch, anchor0, ("decode_stream_v", "decode_merge"), reps)
    kv_bytes = 2.0 * B * 8 * L * 128 * 2
    return {"mode": "decode", "context": L, "batch": B, "topk_permille": permille, "k": k,
            "dense_ms": t_dense, "anchor0_ms": t_a0, "anchor_ms": t_a, "reuse_ms": t_r,
            "dense_GBps": kv_bytes / (t_dense * 1e-3) / 1e9,
            "reuse_GBps": kv_bytes * k / L / (t_r * 1e-3) / 1e9}


def prefill_row(torch, binding, workloads, dev, S, permille, reps, dtype, T=32):
    wl = workloads.make_prefill_workload(f"table3-prefill-S{S}", 8, 1, S, 32, 8, 128, dtype, T, permille, 256,
                                         64, 0.80, device=dev)
    a = wl.layers[0]
    off = wl.idx_offsets
    total = off[-1]
    kpt = torch.tensor(wl.k_per_tile, dtype=torch.int32, device=dev)
    offs = torch.tensor(off, dtype=torch.int64, device=dev)
    idx = torch.empty(8, total, dtype=torch.int32, device=dev)
    out = torch.empty_like(a.q)
    desc = binding.prefill_desc(a.q, a.k)
    ws = torch.empty(binding.kascade_workspace_bytes(binding.OP_PREFILL_ANCHOR, desc, S, total, T), dtype=torch.uint8,
                     device=dev)
    anchor0 = lambda: binding.kascade_prefill_anchor(a.q, a.k, a.v, T, kpt, offs, total, binding.KASCADE_OUT_DENSE, idx, out, ws)
    anchor = lambda: binding.kascade_prefill_anchor(a.q, a.k, a.v, T, kpt, offs, total, binding.KASCADE_OUT_SPARSE, idx, out, ws)
    reuse = lambda: binding.kascade_prefill_reuse(a.q, a.k, a.v, T, kpt, offs, total, idx, None, None, out, ws)
    t_a0, t_a, t_r = timed(torch, anchor0, reps), timed(torch, anchor, reps), timed(torch, reuse, reps * 2)
    t_dense = kernel_ms(binding, torch, anchor0, ("prefill_sweep1_v",), reps)
    dense_flop = 2.0 * S * S * 128 * 32      # causal QK^T + PV
    return {"mode": "prefill", "context": S, "batch": 1, "topk_permille": permille, "tile_tokens": T,
            "dense_ms": t_dense, "anchor0_ms": t_a0, "anchor_ms": t_a, "reuse_ms": t_r,
            "dense_TFLOPs": dense_flop / (t_dense * 1e-3) / 1e12}


def finish(row, paper):
    avg = (row["anchor0_ms"] + 4 * row["anchor_ms"] + 27 * row["reuse_ms"]) / 32
    row["kascade_avg_ms"] = avg
    row["speedup_vs_own_dense"] = row["dense_ms"] / avg
    ref = paper.get((row["context"], row["topk_permille"]))
    if ref:
        row["paper_h100_avg_ms"], row["paper_h100_speedup_vs_fa3"] = ref
    return {k: (round(v, 4) if isinstance(v, float) else v) for k, v in row.items()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--max-decode-context", type=int, default=524288)
    ap.add_argument("--max-prefill-context", type=int, default=131072)
    ap.add_argument("--quick", action="store_true", help="10 %% rows only")
    ap.add_argument("--dtype", choices=["bf16", "fp16"], default="bf16", help="storage type (the paper's own timings are fp16)")
    args = ap.parse_args()
    import torch
    from paper_2512_16391_amd import binding, workloads
    if not torch.cuda.is_available():
        print("bench_table3.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    binding.load_library()
    dev = torch.device("cuda:0")
    dtype = torch.float16 if args.dtype == "fp16" else torch.bfloat16
    rows = []
    decode_cases = [(L, 64 if L < 524288 else 32, 100) for L in (8192, 16384, 32768, 65536, 131072, 262144, 524288)
                    if L <= args.max_decode_context]
    if not args.quick and args.max_decode_context >= 131072:
        decode_cases += [(131072, 64, 200), (131072, 64, 300)]
    for L, B, pm in decode_cases:
        reps = 10 if L * B <= 1 << 22 else 4
        row = finish(decode_row(torch, binding, workloads, dev, L, B, pm, reps, dtype), PAPER_DECODE)
        rows.append(row)
        print(json.dumps(row), flush=True)
        torch.cuda.empty_cache()
    prefill_cases = [(S, 100) for S in (8192, 16384, 32768, 65536, 131072, 262144) if S <= args.max_prefill_context]
    if not args.quick and args.max_prefill_context >= 32768:
        prefill_cases += [(32768, 200), (32768, 300)]
    if not args.quick and args.max_prefill_context >= 32768:
        prefill_cases += [(32768, 100, 128)]      # tiles of 128 tokens x 4 heads = 512 rows (one index set per 512 rows)
    for case in prefill_cases:
        S, pm = case[0], case[1]
        T = case[2] if len(case) > 2 else 32
        reps = 5 if S <= 32768 else (2 if S <= 131072 else 1)
        row = finish(prefill_row(torch, binding, workloads, dev, S, pm, reps, dtype, T), PAPER_PREFILL if T == 32 else {})
        rows.append(row)
        print(json.dumps(row), flush=True)
        torch.cuda.empty_cache()
    print("prefill rows use tiles of 32 tokens x 4 heads = 128 rows unless tile_tokens says otherwise")
    hdr = f"{'mode':12s}{'context':>9s}{'batch':>6s}{'topk':>6s}{'dense':>10s}{'anchor0':>10s}{'anchor':>10s}{'reuse':>10s}" \
          f"{'avg':>10s}{'speedup':>9s}{'paper avg':>11s}{'paper x':>9s}"
    print(hdr)
    for r in rows:
        mode = r['mode'] if r.get('tile_tokens', 32) == 32 else f"{r['mode']}/T{r['tile_tokens']}"
        print(f"{mode:12s}{r['context']:9d}{r['batch']:6d}{r['topk_permille'] // 10:5d}%{r['dense_ms']:10.3f}"
              f"{r['anchor0_ms']:10.3f}{r['anchor_ms']:10.3f}{r['reuse_ms']:10.3f}{r['kascade_avg_ms']:10.3f}"
              f"{r['speedup_vs_own_dense']:8.2f}x{r.get('paper_h100_avg_ms', float('nan')):11.2f}"
              f"{r.get('paper_h100_speedup_vs_fa3', float('nan')):8.2f}x")


if __name__ == "__main__":
    main()
