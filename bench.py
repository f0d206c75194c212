#!/usr/bin/env python3
"""Benchmark of the Kascade hot path on one MI355X.

One "step" = one pass of the hot path over one batch of seeded synthetic input:
  decode  - the Llama-3.1-8B-shaped configuration (32 query / 8 key heads, d 128, bf16,
            batch 8, 32768-token contiguous KV cache per sequence, k = 10 %): one anchor
            layer followed by three reuse layers, each layer with its own Q/K/V;
  prefill - batch 1, 32768 tokens causal, same heads, tiles of 32 tokens x 4 heads,
            k_t = 10 % of the prefix (min 256): one anchor layer followed by three reuse layers.
All inputs are resident in HBM before the timed region; nothing is allocated inside it.
A second leg, outside the step, runs the bandwidth-stress decode configuration (batch 32,
ragged 65536-131072 tokens, k = 5 %, 64-token recent window; one anchor + three reuse layers)
and reports its reuse layer against the HBM peak.

Prints ONE JSON line.  `value` is the decode attention time per layer (the headline metric's
first component); HBM GB/s of the reuse gather and prefill TFLOP/s ride along in extra keys.
Per-kernel durations are the begin-to-end device times of the library's own dispatches (a start and
a stop event bound to each dispatch, recorded by the library on the launch stream in a second timed
pass of the same K steps) - the figure a rocprofv3 kernel trace of this command reports; nothing is
subtracted from them.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prefill", action="store_true")
    ap.add_argument("--no-config3", action="store_true")
    ap.add_argument("--only-config3", action="store_true",
                    help="run the bandwidth-stress decode leg alone (profiling aid: its kernels then are the only ones of their names)")
    ap.add_argument("--cpu-sample-seqs", type=int, default=8)
    return ap.parse_args()


def hbm_roofline(kernel, nbytes, t_us, traffic=None, **extra):
    gbs = nbytes / t_us / 1e3
    r = {"kernel": kernel, "bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": traffic, "algorithmic_bytes": int(nbytes),
         "avg_kernel_us": round(t_us, 2)}
    r.update(extra)
    return r


def mfma_roofline(kernel, flop, t_us, traffic=None, **extra):
    tf = flop / (t_us * 1e-6) / 1e12
    r = {"kernel": kernel, "bound": "mfma", "achieved": round(tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
         "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": traffic, "algorithmic_flop": float(flop),
         "avg_kernel_us": round(t_us, 1)}
    r.update(extra)
    return r


def profiled(binding, fn, reps):
    """Runs fn() reps times with a start/stop event on every dispatch; returns {step name: average us per run of
    that step} (a step that needs several dispatches is their sum)."""
    import torch
    binding.kascade_profile_enable(True)
    binding.kascade_profile_reset()
    torch.cuda.synchronize()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    prof = binding.kascade_profile_read()
    binding.kascade_profile_enable(False)
    return {k: v[0] * 1e3 / v[1] for k, v in prof.items()}


def wall_us(fn, reps, warm=2):
    """Average wall time of fn() on the device, event pair around `reps` back-to-back calls."""
    import torch
    for _ in range(warm):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2512_16391_amd import binding, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    binding.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.only_config3:
        print(json.dumps({"config3": config3_leg(dev, load_traffic(), max(5, min(args.steps, 20)))}), flush=True)
        return

    # ---------------- decode workload (resident, preallocated) ----------------
    wl = workloads.config2(device=dev)
    B, Hq, Hkv, d = wl.B, wl.Hq, wl.Hkv, wl.d
    L, kmax = wl.Lmax, wl.k_max
    dec = DecodeLeg(dev, wl)

    # ---------------- prefill workload ----------------
    prefill = None if args.no_prefill else PrefillBench(dev)

    def step():
        dec.step()
        if prefill is not None:
            prefill.step()

    # one plain 1 GiB device copy: the yardstick that hardware-counter runs (FETCH_SIZE / WRITE_SIZE)
    # scale their readings by; it is outside every timed region
    cal_src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    copy_gbs = 2.0 * (1 << 30) / (wall_us(lambda: cal_dst.copy_(cal_src), 5, warm=0) * 1e-6) / 1e9
    del cal_src, cal_dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region 1: K whole steps, nothing but the library's own launches -------------------
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for e0, e1 in evs:
        e0.record()
        dec.step()
        e1.record()
        if prefill is not None:
            prefill.step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    dec_ms = sum(e0.elapsed_time(e1) for e0, e1 in evs)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    n_layers = len(wl.layers)
    dec_us_per_layer = dec_ms * 1e3 / args.steps / n_layers
    per_step = sorted(e0.elapsed_time(e1) * 1e3 / n_layers for e0, e1 in evs)
    pct = lambda f: round(per_step[min(len(per_step) - 1, int(f * len(per_step)))], 2)

    # ---- timed region 2: the same K steps, every dispatch carrying its own start/stop event --------
    kus = profiled(binding, step, args.steps)

    # ---- the decode step as one HIP graph (no launch gaps): replayed K times -----------------------
    graph_us_per_layer = None
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            dec.step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        ref_outs = [o.clone() for o in dec.outs]
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            dec.step()
        for _ in range(3):
            g.replay()
        torch.cuda.synchronize()
        same = all(torch.equal(a_, b_) for a_, b_ in zip(ref_outs, dec.outs))
        if same:
            graph_us_per_layer = wall_us(g.replay, max(args.steps, 20), warm=0) / n_layers
    except Exception as exc:   # graph capture is an extra, never the headline
        print(f"bench.py: graph replay skipped: {exc}", file=sys.stderr)

    traffic = load_traffic()
    layer_us = dec.layer_times()
    rec = {
        "metric": "sparse decode attn us/layer + HBM GB/s; prefill attn TFLOPS at 32K ctx",
        "value": round(dec_us_per_layer, 2), "unit": "us/layer (decode, mean of 1 anchor + 3 reuse layers)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name + " k=%d (10%%), 1 anchor + 3 reuse layers" % kmax
                   + ("; " + prefill.name if prefill is not None else ""),
                   "batch": B, "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": d, "context": L, "k": kmax},
        "decode_us_per_layer_p10_p50_p90": [pct(0.1), pct(0.5), pct(0.9)],
        "decode_tokens_per_s": round(B / (dec_us_per_layer * n_layers * 1e-6), 1),
        "decode_us_per_layer_hip_graph": round(graph_us_per_layer, 2) if graph_us_per_layer else None,
        "kernel_timing": "second timed pass of the same K steps; begin-to-end device time of each dispatch from a start "
                         "and a stop event bound to the dispatch itself (what a kernel trace reports), nothing subtracted",
        "device_copy_GBps_measured": round(copy_gbs, 1),
        "kernel_us": {k: round(v, 2) for k, v in kus.items()},
        "decode_layer_us": layer_us,
    }
    # ---- rooflines.  `roofline` is the kernel that takes the most device time in the step.
    dec_roof = dec.rooflines(kus, layer_us, traffic)
    if prefill is not None:
        pre = prefill.report(kus, traffic, binding)
        rec["roofline"] = pre.pop("roofline")
        rec.update(pre)
        rec["prefill_layer_ms"] = prefill.layer_times()
    else:
        rec["roofline"] = dec_roof["roofline_decode_stream"]
    rec.update(dec_roof)
    rec["decode_reuse_hbm_GBps"] = dec_roof["roofline_decode_gather"]["achieved"]

    del dec
    torch.cuda.empty_cache()
    if not args.no_config3:
        rec["config3"] = config3_leg(dev, traffic, max(5, min(args.steps, 20)))

    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(wl, args.cpu_sample_seqs)
        if prefill is not None:
            rec["cpu_baseline_prefill"] = cpu_baseline_prefill(prefill)
    print(json.dumps(rec), flush=True)


class DecodeLeg:
    """One anchor layer (sparse output) followed by the reuse layers of a decode workload, every buffer
    allocated up front."""

    def __init__(self, dev, wl):
        import torch
        from paper_2512_16391_amd import binding
        self.binding, self.wl = binding, wl
        self.seqlens = torch.tensor(wl.seqlens, dtype=torch.int32, device=dev)
        self.kps = torch.tensor(wl.k_per_seq, dtype=torch.int32, device=dev)
        self.idx = torch.empty(wl.B, wl.Hkv, wl.k_max, dtype=torch.int32, device=dev)
        self.outs = [torch.empty_like(l.q) for l in wl.layers]
        desc = binding.decode_desc(wl.layers[0].q, wl.layers[0].k)
        need = max(binding.kascade_workspace_bytes(binding.OP_DECODE_ANCHOR, desc, wl.Lmax, wl.k_max),
                   binding.kascade_workspace_bytes(binding.OP_DECODE_REUSE, desc, wl.Lmax, wl.k_max))
        self.ws = torch.empty(need, dtype=torch.uint8, device=dev)

    def anchor(self, out_mode=None):
        b, wl, a = self.binding, self.wl, self.wl.layers[0]
        mode = b.KASCADE_OUT_SPARSE if out_mode is None else out_mode
        b.kascade_decode_anchor(a.q, a.k, a.v, self.seqlens, self.kps, wl.Lmax, wl.k_max, wl.recent_window, mode,
                                self.idx, self.outs[0], self.ws)

    def reuse(self, i):
        b, wl, r = self.binding, self.wl, self.wl.layers[i]
        b.kascade_decode_reuse(r.q, r.k, r.v, self.seqlens, self.kps, wl.k_max, self.idx, None, self.outs[i], self.ws)

    def step(self):
        self.anchor()
        for i in range(1, len(self.wl.layers)):
            self.reuse(i)

    def layer_times(self):
        """Wall time per layer kind (event pair around back-to-back calls of that layer, launch gaps included);
        the reuse figure rotates over the reuse layers' own K/V so that the selected rows do not sit in the
        Infinity Cache from the previous call."""
        b = self.binding
        n = len(self.wl.layers)
        dense = wall_us(lambda: self.anchor(b.KASCADE_OUT_DENSE), 20, warm=3)
        sparse = wall_us(lambda: self.anchor(b.KASCADE_OUT_SPARSE), 20, warm=3)
        state = {"i": 0}

        def rotate():
            self.reuse(1 + state["i"] % (n - 1))
            state["i"] += 1
        reuse = wall_us(rotate, 7 * (n - 1), warm=n - 1)
        warm = wall_us(lambda: self.reuse(1), 21, warm=2)
        return {"anchor_dense_out": round(dense, 2), "anchor_sparse_out": round(sparse, 2), "reuse": round(reuse, 2),
                "reuse_same_layer_cache_warm": round(warm, 2),
                "paper_weighted_avg_32_layers_5_anchors": round((dense + 4 * sparse + 27 * reuse) / 32, 2)}

    def bytes(self):
        """Algorithmic bytes per launch: bf16 rows of d elements, int32 indices, fp32 logits, Q and O."""
        wl = self.wl
        row_pairs = sum(wl.k_per_seq) * wl.Hkv
        gather = row_pairs * (2 * wl.d * 2 + 4) + 2 * wl.B * wl.Hq * wl.d * 2
        stream = sum(wl.seqlens) * wl.Hkv * wl.d * 2 + sum(wl.seqlens) * wl.Hq * 4 + wl.B * wl.Hq * wl.d * 2
        return gather, stream

    def rooflines(self, kus, layer_us, traffic, suffix=""):
        gather_b, stream_b = self.bytes()
        t_layer_kernels = kus["decode_gather"] + kus.get("decode_merge", 0.0)
        return {
            "roofline_decode_stream" + suffix: hbm_roofline("decode_stream (anchor pass 1: K sweep + logits)", stream_b,
                                                            kus["decode_stream"], traffic.get("decode_stream" + suffix)),
            "roofline_decode_gather" + suffix: hbm_roofline("decode_gather (reuse layer / anchor pass 4, gather kernel alone)",
                                                            gather_b, kus["decode_gather"], traffic.get("decode_gather" + suffix)),
            "roofline_decode_reuse_layer" + suffix: hbm_roofline(
                "reuse layer = gather + merge", gather_b, layer_us["reuse"], None,
                kernels_only_us=round(t_layer_kernels, 2),
                frac_kernels_only=round(gather_b / t_layer_kernels / 1e3 / HBM_PEAK_GBS, 4),
                note="avg_kernel_us is the layer's wall time (dispatch gaps included), K/V rotating over the reuse layers"),
        }


def config3_leg(dev, traffic, reps):
    """Bandwidth-stress decode (batch 32, ragged 65536-131072 tokens, k = 5 % with a 64-token recent window):
    one anchor + three reuse layers, each with its own Q/K/V (69 GB resident)."""
    import torch
    from paper_2512_16391_amd import binding, workloads
    t0 = time.perf_counter()
    wl = workloads.config3(device=dev)
    torch.cuda.synchronize()
    gen_s = time.perf_counter() - t0
    leg = DecodeLeg(dev, wl)
    for _ in range(2):
        leg.step()
    step_us = wall_us(leg.step, reps, warm=0)
    kus = profiled(binding, leg.step, reps)
    layer_us = leg.layer_times()
    gather_b, stream_b = leg.bytes()
    out = {"workload": wl.name + " k=5% (64-token recent window inside k), 1 anchor + 3 reuse layers",
           "batch": wl.B, "sum_seqlens": sum(wl.seqlens), "sum_k": sum(wl.k_per_seq), "steps": reps,
           "us_per_layer": round(step_us / len(wl.layers), 2),
           "tokens_per_s": round(wl.B / (step_us * 1e-6), 1),
           "kernel_us": {k: round(v, 2) for k, v in kus.items()}, "decode_layer_us": layer_us,
           "input_generation_s": round(gen_s, 1)}
    roofs = leg.rooflines(kus, layer_us, traffic, suffix="_cfg3")
    out["roofline_reuse_cfg3"] = roofs.pop("roofline_decode_gather_cfg3")
    out["roofline_reuse_layer_cfg3"] = roofs.pop("roofline_decode_reuse_layer_cfg3")
    out["roofline_stream_cfg3"] = roofs.pop("roofline_decode_stream_cfg3")
    del leg, wl
    torch.cuda.empty_cache()
    return out


class PrefillBench:
    """Config 4: batch 1, 32768 tokens causal, 32/8 heads, d 128, bf16, tiles of 32 tokens x 4
    heads, k_t = 10 % of the prefix (min 256); one anchor layer (sparse output) + three reuse
    layers, each with its own Q/K/V."""

    def __init__(self, dev, S=32768, T=32):
        import torch
        from paper_2512_16391_amd import binding, workloads
        self.binding = binding
        wl = workloads.config4(device=dev, S=S, T=T)
        self.wl = wl
        self.name = wl.name + " k_t=10% (min 256), 1 anchor + 3 reuse layers"
        off = wl.idx_offsets
        self.idx_total = off[-1]
        self.kpt = torch.tensor(wl.k_per_tile, dtype=torch.int32, device=dev)
        self.off = torch.tensor(off, dtype=torch.int64, device=dev)
        self.idx = torch.empty(wl.Hkv, self.idx_total, dtype=torch.int32, device=dev)
        self.outs = [torch.empty_like(l.q) for l in wl.layers]
        desc = binding.prefill_desc(wl.layers[0].q, wl.layers[0].k)
        need = binding.kascade_workspace_bytes(binding.OP_PREFILL_ANCHOR, desc, S, self.idx_total, T)
        self.ws = torch.empty(need, dtype=torch.uint8, device=dev)
        # MFMA-class FLOP the method needs (each causal QK^T sweep = U)
        d, Hq = wl.d, wl.Hq
        self.U = float(S) * S * d * Hq
        self.sparse_flop = 4.0 * d * Hq * sum(min(T, S - t * T) * (kt + (min(T, S - t * T) + 1) / 2.0)
                                              for t, kt in enumerate(wl.k_per_tile))

    def anchor(self, out_mode):
        b, wl, a = self.binding, self.wl, self.wl.layers[0]
        b.kascade_prefill_anchor(a.q, a.k, a.v, wl.T, self.kpt, self.off, self.idx_total, out_mode, self.idx, self.outs[0], self.ws)

    def reuse(self, i):
        b, wl, r = self.binding, self.wl, self.wl.layers[i]
        b.kascade_prefill_reuse(r.q, r.k, r.v, wl.T, self.kpt, self.off, self.idx_total, self.idx, None, None, self.outs[i], self.ws)

    def step(self):
        self.anchor(self.binding.KASCADE_OUT_SPARSE)
        for i in range(1, len(self.wl.layers)):
            self.reuse(i)

    def layer_times(self):
        """Per-layer wall time of the three layer kinds, and the paper's weighting (Table 3 caption)."""
        b = self.binding
        dense = wall_us(lambda: self.anchor(b.KASCADE_OUT_DENSE), 5, warm=1) / 1e3
        sparse = wall_us(lambda: self.anchor(b.KASCADE_OUT_SPARSE), 5, warm=1) / 1e3
        reuse = wall_us(lambda: self.reuse(1), 5, warm=1) / 1e3
        avg = (dense + 4 * sparse + 27 * reuse) / 32
        return {"anchor_dense_out": round(dense, 3), "anchor_sparse_out": round(sparse, 3), "reuse": round(reuse, 3),
                "paper_weighted_avg_32_layers_5_anchors": round(avg, 3),
                "dense_attention_equivalent_tflops_at_weighted_avg_counting_skipped_work": round(2 * self.U / (avg * 1e-3) / 1e12, 1)}

    def report(self, kus, traffic, binding):
        # the per-head Top-k selection runs inside the pass-2 kernel; a separate selection kernel exists
        # only for the shared-set variant
        t1, t2, ts = kus["prefill_sweep1"], kus["prefill_sweep2"], kus["prefill_sparse"]
        tk = kus.get("prefill_topk", 0.0)
        anchor_us = t1 + t2 + tk + ts
        anchor_flop = 2 * self.U + self.sparse_flop
        # layer 0 (dense output): pass 1 carries P.V as well (2U); measured in a short pass of its own
        kd = profiled(binding, lambda: self.anchor(binding.KASCADE_OUT_DENSE), 3)
        t1v, t2d = kd["prefill_sweep1_v"], kd["prefill_sweep2"]
        tf = lambda flop, t_us: flop / (t_us * 1e-6) / 1e12
        return {
            "prefill_anchor_ms": round(anchor_us / 1e3, 3), "prefill_reuse_ms": round(ts / 1e3, 3),
            "prefill_anchor_tflops": round(tf(anchor_flop, anchor_us), 1),
            "prefill_reuse_tflops": round(tf(self.sparse_flop, ts), 1),
            "prefill_tokens_per_s": round(self.wl.S / ((anchor_us + 3 * ts) * 1e-6), 1),
            "roofline": mfma_roofline("prefill_sweep2 (prefill_pool_kernel: anchor pass 2, tile pooling and the per-tile Top-k)",
                                      self.U, t2, traffic.get("prefill_sweep2")),
            "roofline_prefill_sweep1": mfma_roofline("prefill_sweep1 (anchor pass 1, row statistics only)", self.U, t1,
                                                     traffic.get("prefill_sweep1")),
            "roofline_prefill_sweep1_dense_out": mfma_roofline("prefill_sweep1_v (layer 0: pass 1 with P.V, dense output)",
                                                               2 * self.U, t1v, traffic.get("prefill_sweep1_v")),
            "roofline_prefill_sparse": mfma_roofline("prefill_sparse (reuse layer / anchor pass 4)", self.sparse_flop, ts,
                                                     traffic.get("prefill_sparse")),
            "roofline_prefill_anchor": mfma_roofline("anchor layer, sparse output: sweep 1 + sweep 2 + sparse attention",
                                                     anchor_flop, anchor_us, None, out_mode="sparse"),
            "roofline_prefill_anchor_dense_out": mfma_roofline("anchor layer 0, dense output: sweep 1 with P.V + sweep 2",
                                                               3 * self.U, t1v + t2d, None, out_mode="dense"),
        }


def load_traffic():
    """HBM bytes per launch measured offline with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on this same
    command (scaled by the 1 GiB copy above): the table in profiles/bench_hbm_traffic.txt
    (columns: kernel, read MB, write MB, total MB)."""
    path = os.path.join(ROOT, "profiles", "bench_hbm_traffic.txt")
    out = {}
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 4 and not line.startswith("#") and parts[0] != "kernel":
                    out[parts[0]] = float(parts[3]) * 1e6
    except (OSError, ValueError):
        return {}
    return out


def _cpu_threads():
    """Threads numpy's BLAS (the oracle's matrix products) runs with, and the cores the box reports."""
    blas = 1
    try:
        from threadpoolctl import threadpool_info
        n = [i.get("num_threads", 1) for i in threadpool_info() if i.get("user_api") == "blas"]
        blas = int(max(n)) if n else 1
    except Exception:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    return blas, os.cpu_count() or 1, usable


def cpu_baseline(wl, n_seqs):
    """The fp64 oracle, as it stands, on a bounded sample of the decode workload: the first
    `n_seqs` sequences of the batch through the same four layers.  Scaled to the full batch."""
    import torch
    from oracle import kascade_oracle as ko

    n_seqs = min(n_seqs, wl.B)
    f = lambda t: t.to("cpu").to(torch.float32).to(torch.float64).numpy()
    scale = ko.default_scale(wl.d)
    dt = 0.0
    for b in range(n_seqs):
        Lb, kb = wl.seqlens[b], wl.k_per_seq[b]
        # widening the device bits to fp64 is input plumbing, not oracle work: not timed
        host = [(f(l.q[b]), f(l.k[b, :, :Lb]), f(l.v[b, :, :Lb])) for l in wl.layers]
        t0 = time.perf_counter()
        q, k, v = host[0]
        idx, _ = ko.decode_anchor_indices(q, k, scale, kb, wl.recent_window)
        ko.sparse_decode(q, k, v, idx, scale)
        for q, k, v in host[1:]:
            ko.sparse_decode(q, k, v, idx, scale)
        dt += time.perf_counter() - t0
        del host
    us_per_layer = dt * 1e6 / len(wl.layers) * (wl.B / n_seqs)
    blas, cores, usable = _cpu_threads()
    return {"value": round(us_per_layer, 1), "unit": "us/layer (decode, scaled to the full batch)",
            "cores": blas, "host_cores_reported": cores, "host_cores_usable": usable, "kind": "oracle",
            "threads_note": "matrix products run on `cores` BLAS threads; the oracle's own loops are one Python thread",
            "sample": f"{n_seqs} of {wl.B} sequences, all heads, 1 anchor + 3 reuse layers, {dt:.2f} s measured"}


def cpu_baseline_prefill(pb, n_random=16):
    """The fp64 oracle on a sample of query tiles of the prefill anchor layer (the first tiles, the tiles
    where 10 % of the prefix passes the minimum budget, the last one, and seeded random ones): pooled scores,
    Top-k and sparse attention per tile.  A tile's work grows with the keys before it, so the sample
    is extrapolated to the whole layer by (prefix + half a tile) and reported as such."""
    import numpy as np
    import torch
    from oracle import kascade_oracle as ko

    wl = pb.wl
    a = wl.layers[0]
    f = lambda t: t.to("cpu").to(torch.float32).to(torch.float64).numpy()
    Q, Kp, Vp = f(a.q), f(a.k), f(a.v)
    scale = ko.default_scale(wl.d)
    rs = np.random.default_rng(4)
    tiles = sorted(set([0, 1, 80, 81, wl.n_tiles - 1] + rs.integers(2, wl.n_tiles, n_random).tolist()))
    tiles = [t for t in tiles if t < wl.n_tiles]
    weight = lambda t: t * wl.T + 0.5 * wl.T
    t0 = time.perf_counter()
    for t in tiles:
        kt = wl.k_per_tile[t]
        idx, _ = ko.prefill_anchor_indices_tile(Q, Kp, t, wl.T, scale, kt)
        ko.prefill_sparse_tile(Q, Kp, Vp, t, wl.T, idx, scale)
    dt = time.perf_counter() - t0
    full_s = dt * sum(weight(t) for t in range(wl.n_tiles)) / sum(weight(t) for t in tiles)
    flop = 2.0 * pb.U + pb.sparse_flop
    blas, cores, usable = _cpu_threads()
    return {"value": round(flop / full_s / 1e12, 5), "unit": "TFLOP/s (prefill anchor layer, sparse output, extrapolated)",
            "cores": blas, "host_cores_reported": cores, "host_cores_usable": usable, "kind": "oracle",
            "sample": f"{len(tiles)} tiles of {wl.n_tiles} (first, budget boundary, last, {n_random} seeded random), all heads, "
                      f"{dt:.2f} s measured, {full_s:.0f} s extrapolated by keys per tile",
            "anchor_layer_s_extrapolated": round(full_s, 1)}


if __name__ == "__main__":
    main()
