#!/usr/bin/env python3
"""Decode layer times against the GQA group size, on one MI355X.

The paper's models have four query heads per key head; others have eight, or a group that is not
a power of two.  The decode row passes exist in two families - vector-ALU kernels whose arithmetic
grows with the group, and matrix-unit kernels whose cost does not depend on it - and this sweep
times both wherever both exist: per-kernel device times of an anchor layer (sparse and dense
output) and of a reuse layer, at 8 key heads, head dimension 128 (and 64 for two groups), context
32768, Top-k 10 %, batch 8 and 64; bf16, seeded synthetic inputs, every sequence at full length.

Prints one JSON line per row.  Not part of bench.py's contract.
"""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def kernel_us(binding, torch, fn, reps):
    """Device time of each library kernel per call of fn (event pairs minus the pair's own reading)."""
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    binding.kascade_profile_enable(True)
    binding.kascade_profile_reset()
    for _ in range(reps):
        fn()
    binding.kascade_profile_calibrate(30)
    torch.cuda.synchronize()
    prof = binding.kascade_profile_read()
    binding.kascade_profile_enable(False)
    base = prof.pop("empty_kernel")
    base = base[0] * 1e3 / base[1]
    return {n: round(v[0] * 1e3 / reps - base * v[1] / reps, 1) for n, v in prof.items()}


def wall_us(torch, fn, reps):
    for _ in range(3):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    e1.synchronize()
    return round(e0.elapsed_time(e1) * 1e3 / reps, 1)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--context", type=int, default=32768)
    args = ap.parse_args()
    import torch
    from paper_2512_16391_amd import binding
    if not torch.cuda.is_available():
        sys.exit("bench_groups.py needs an MI355X")
    dev = torch.device("cuda:0")
    L, Hkv = args.context, 8
    kk = (L + 9) // 10
    forced = os.environ.get("KASCADE_DECODE_MFMA")
    for d, groups in ((128, (1, 2, 4, 7, 8, 16)), (64, (4, 8))):
        for B in (8, 64):
            for G in groups:
                g = torch.Generator(device=dev).manual_seed(1000 * G + B)
                q = torch.randn(B, G * Hkv, d, device=dev, generator=g).bfloat16()
                k = torch.randn(B, Hkv, L, d, device=dev, generator=g).bfloat16()
                v = torch.randn(B, Hkv, L, d, device=dev, generator=g).bfloat16()
                lens = torch.full((B,), L, dtype=torch.int32, device=dev)
                ks = torch.full((B,), kk, dtype=torch.int32, device=dev)
                families = ("vector_alu", "matrix_unit") if G in (1, 2, 4, 8) else ("matrix_unit",)
                for fam in families:
                    os.environ["KASCADE_DECODE_MFMA"] = "1" if fam == "matrix_unit" else "0"
                    row = {"head_dim": d, "batch": B, "context": L, "k": kk, "group": G, "kernels": fam}
                    idx = None
                    for mode, name in ((binding.KASCADE_OUT_SPARSE, "anchor_sparse_out"), (binding.KASCADE_OUT_DENSE, "anchor_dense_out")):
                        fn = lambda: binding.kascade_decode_anchor(q, k, v, lens, ks, L, kk, recent_window=0, out_mode=mode)
                        row[name + "_us"] = wall_us(torch, fn, args.reps)
                        row[name + "_kernel_us"] = kernel_us(binding, torch, fn, args.reps)
                        if mode == binding.KASCADE_OUT_SPARSE:
                            idx = fn()[0]
                    fn = lambda: binding.kascade_decode_reuse(q, k, v, lens, ks, kk, idx)
                    row["reuse_us"] = wall_us(torch, fn, args.reps)
                    row["reuse_kernel_us"] = kernel_us(binding, torch, fn, args.reps)
                    kv_bytes = 2.0 * B * Hkv * kk * d * 2
                    row["reuse_gather_TBps"] = round(kv_bytes / (row["reuse_kernel_us"]["decode_gather"] * 1e-6) / 1e12, 2)
                    sweep_bytes = B * Hkv * L * (d * 2 + G * 4)
                    row["anchor_sweep_TBps"] = round(sweep_bytes / (row["anchor_sparse_out_kernel_us"]["decode_stream"] * 1e-6) / 1e12, 2)
                    print(json.dumps(row), flush=True)
                del q, k, v
                torch.cuda.empty_cache()
    if forced is None:
        os.environ.pop("KASCADE_DECODE_MFMA", None)
    else:
        os.environ["KASCADE_DECODE_MFMA"] = forced


if __name__ == "__main__":
    main()
