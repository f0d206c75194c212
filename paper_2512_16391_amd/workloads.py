"""Seeded synthetic inputs shaped like the paper's attention micro-benchmarks
(Sec. 4.3 / Table 3: Llama-3.1-8B attention shape, 32 query heads, 8 key
heads, head dimension 128) and the smaller parity cases.

This module holds no arithmetic of the method itself: it only draws Q, K, V,
plants heavy-hitter keys, and lists sequence lengths and Top-k budgets.  It is
the one module that both the CPU oracle's tests and the HIP path's callers
use, so that both sides see the same bits.

Recipe (per layer and (sequence, key head)): Q, K, V ~ N(0, 1); a unit vector
u and a set of hitter positions; K[j] += boost * u for hitters, q += q_boost *
u for the G query heads of that key head, so post-softmax mass concentrates on
the hitters.  From one layer to the next a fraction `overlap` of the hitter
positions is kept and the rest is redrawn, which gives neighbouring layers the
similar-but-not-equal Top-k sets that Sec. 3.2 of the paper describes.
Everything is rounded to the storage dtype before anyone sees it.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import torch


def layer_seed(base_seed: int, config_id: int, layer: int) -> int:
    return int(base_seed) + 1000 * int(config_id) + int(layer)


BASE_SEED = 20251216


def ceil_fraction(L: int, permille: int) -> int:
    """ceil(L * permille / 1000) in integers."""
    return -((-int(permille) * int(L)) // 1000)


def budget(L: int, permille: int, k_min: int = 0) -> int:
    """Top-k budget the caller passes in: fraction of L, at least k_min, at most L."""
    return int(min(max(ceil_fraction(L, permille), k_min), L))


@dataclass
class DecodeLayer:
    q: torch.Tensor          # [B, Hq, d]
    k: torch.Tensor          # [B, Hkv, Lmax, d]
    v: torch.Tensor          # [B, Hkv, Lmax, d]
    hitters: Optional[list] = None   # [B][Hkv] LongTensor of planted positions (cpu)


@dataclass
class DecodeWorkload:
    name: str
    B: int
    Hq: int
    Hkv: int
    d: int
    dtype: torch.dtype
    Lmax: int
    seqlens: List[int]
    k_per_seq: List[int]
    recent_window: int
    layers: List[DecodeLayer] = field(default_factory=list)

    @property
    def k_max(self) -> int:
        return max(self.k_per_seq)


def _unit(gen, d, device):
    u = torch.randn(d, generator=gen, device=device, dtype=torch.float32)
    return u / u.norm()


def _next_hitters(gen, prev, L, n, overlap, device):
    """Keep round(overlap * n) of prev's positions, redraw the rest in [0, L)."""
    n = min(n, L)
    if prev is None:
        return torch.randperm(L, generator=gen, device=device)[:n]
    n_keep = int(round(overlap * n))
    keep = prev[torch.randperm(prev.numel(), generator=gen, device=device)[:n_keep]]
    mask = torch.ones(L, dtype=torch.bool, device=device)
    mask[keep] = False
    free = mask.nonzero().flatten()
    fresh = free[torch.randperm(free.numel(), generator=gen, device=device)[: n - n_keep]]
    return torch.cat([keep, fresh])


def make_decode_workload(name, config_id, n_layers, B, Hq, Hkv, d, dtype, seqlens,
                         k_per_seq, n_hitters, overlap, recent_window=0, Lmax=None,
                         boost=3.0, q_boost=1.0, device="cpu", base_seed=BASE_SEED,
                         keep_hitters=True):
    """n_layers independent (q, K, V) triples over one batch of sequences, with
    hitter positions drifting from layer to layer.  `overlap` is one fraction or a
    per-layer list (entry l: fraction of layer l-1's hitters that layer l keeps)."""
    device = torch.device(device)
    Lmax = int(Lmax if Lmax is not None else max(seqlens))
    G = Hq // Hkv
    wl = DecodeWorkload(name, B, Hq, Hkv, d, dtype, Lmax, list(map(int, seqlens)),
                        list(map(int, k_per_seq)), int(recent_window))
    prev = [[None] * Hkv for _ in range(B)]
    for layer in range(n_layers):
        gen = torch.Generator(device=device)
        gen.manual_seed(layer_seed(base_seed, config_id, layer))
        q = torch.randn(B, Hq, d, generator=gen, device=device, dtype=torch.float32)
        k = torch.empty(B, Hkv, Lmax, d, device=device, dtype=dtype)
        v = torch.empty(B, Hkv, Lmax, d, device=device, dtype=dtype)
        hit_all = []
        for b in range(B):
            L = wl.seqlens[b]
            kb = torch.randn(Hkv, Lmax, d, generator=gen, device=device, dtype=torch.float32)
            vb = torch.randn(Hkv, Lmax, d, generator=gen, device=device, dtype=torch.float32)
            hit_b = []
            for hk in range(Hkv):
                u = _unit(gen, d, device)
                ov = overlap[layer] if isinstance(overlap, (list, tuple)) else overlap
                pos = _next_hitters(gen, prev[b][hk], L, n_hitters, ov, device)
                prev[b][hk] = pos
                kb[hk, pos] += boost * u
                q[b, hk * G:(hk + 1) * G] += q_boost * u
                hit_b.append(pos.cpu() if keep_hitters else None)
            k[b] = kb.to(dtype)
            v[b] = vb.to(dtype)
            hit_all.append(hit_b)
            del kb, vb
        wl.layers.append(DecodeLayer(q.to(dtype), k, v, hit_all if keep_hitters else None))
    return wl


@dataclass
class PrefillLayer:
    q: torch.Tensor          # [S, Hq, d]
    k: torch.Tensor          # [Hkv, S, d]
    v: torch.Tensor          # [Hkv, S, d]


@dataclass
class PrefillWorkload:
    name: str
    S: int
    Hq: int
    Hkv: int
    d: int
    dtype: torch.dtype
    T: int                       # query-tile size in tokens (tile rows = T * G)
    k_per_tile: List[int]
    layers: List[PrefillLayer] = field(default_factory=list)

    @property
    def n_tiles(self) -> int:
        return (self.S + self.T - 1) // self.T

    @property
    def idx_offsets(self) -> List[int]:
        off = [0]
        for kt in self.k_per_tile:
            off.append(off[-1] + kt)
        return off


def prefill_budgets(S, T, permille, k_min):
    """k_t for every tile: fraction of the tile's prefix t*T, at least k_min,
    never more than the prefix (tile 0 has none)."""
    n_tiles = (S + T - 1) // T
    return [budget(t * T, permille, k_min) for t in range(n_tiles)]


def make_prefill_workload(name, config_id, n_layers, S, Hq, Hkv, d, dtype, T, permille,
                          k_min, n_hitters, overlap, boost=3.0, q_boost=1.0,
                          device="cpu", base_seed=BASE_SEED):
    device = torch.device(device)
    G = Hq // Hkv
    wl = PrefillWorkload(name, S, Hq, Hkv, d, dtype, T, prefill_budgets(S, T, permille, k_min))
    prev = [None] * Hkv
    for layer in range(n_layers):
        gen = torch.Generator(device=device)
        gen.manual_seed(layer_seed(base_seed, config_id, layer))
        q = torch.randn(S, Hq, d, generator=gen, device=device, dtype=torch.float32)
        k = torch.randn(Hkv, S, d, generator=gen, device=device, dtype=torch.float32)
        v = torch.randn(Hkv, S, d, generator=gen, device=device, dtype=torch.float32)
        for hk in range(Hkv):
            u = _unit(gen, d, device)
            pos = _next_hitters(gen, prev[hk], S, n_hitters, overlap, device)
            prev[hk] = pos
            k[hk, pos] += boost * u
            q[:, hk * G:(hk + 1) * G] += q_boost * u
        wl.layers.append(PrefillLayer(q.to(dtype), k.to(dtype), v.to(dtype)))
    return wl


# ----------------------------------------------------------------------------
# The named configurations
# ----------------------------------------------------------------------------

def config1(device="cpu"):
    """Small fp32 decode: B1, 8/2 heads, d64, L2048, k = 10 % = 205; one anchor
    layer then one reuse layer, 64 hitters per key head, 80 % shared."""
    L = 2048
    return make_decode_workload("cfg1-decode-fp32-L2048", 1, 2, 1, 8, 2, 64, torch.float32,
                                [L], [budget(L, 100)], 64, 0.80, device=device)


def config2(device="cuda", n_layers=4, B=8, L=32768):
    """Llama-3.1-8B-shaped decode: 32/8 heads, d128, bf16, batch 8, 32768 tokens
    per sequence, k = 10 %; one anchor then three reuse layers; 1024 hitters per
    head, 85 % shared between adjacent layers."""
    return make_decode_workload(f"cfg2-decode-bf16-B{B}-L{L}", 2, n_layers, B, 32, 8, 128,
                                torch.bfloat16, [L] * B, [budget(L, 100)] * B, 1024, 0.85,
                                device=device, keep_hitters=False)


def config3_lengths(B=32, lo=65536, hi=131072, seed=BASE_SEED + 3000):
    g = torch.Generator()
    g.manual_seed(seed)
    return torch.randint(lo, hi + 1, (B,), generator=g).tolist()


def config3(device="cuda", n_layers=4, B=32):
    """Bandwidth-stress decode: batch 32, ragged lengths uniform in
    [65536, 131072], k = 5 % of each length with the 64 most recent tokens
    always kept (inside k)."""
    lens = config3_lengths(B)
    return make_decode_workload(f"cfg3-decode-bf16-B{B}-ragged", 3, n_layers, B, 32, 8, 128,
                                torch.bfloat16, lens, [budget(L, 50) for L in lens], 1024, 0.85,
                                recent_window=64, Lmax=131072, device=device, keep_hitters=False)


def config4(device="cuda", n_layers=4, S=32768, T=32):
    """Prefill: B1, S32768 causal, 32/8 heads, d128, bf16; tiles of T tokens x
    G heads = 128 rows share one index set per key head; k_t = 10 % of the
    prefix, at least 256."""
    return make_prefill_workload(f"cfg4-prefill-bf16-S{S}-T{T}", 4, n_layers, S, 32, 8, 128,
                                 torch.bfloat16, T, 100, 256, 64, 0.80, device=device)


CONFIG5_ANCHORS = (0, 1, 4, 12, 20)


def config5_layer_kind(layer: int):
    """("anchor" | "reuse", index of the anchor layer whose sets the layer uses)."""
    src = max(a for a in CONFIG5_ANCHORS if a <= layer)
    return ("anchor" if layer in CONFIG5_ANCHORS else "reuse"), src


def iter_config5_layers(device="cuda", n_layers=32, S=131072, decode_steps=256, keep=None):
    """Yields (layer index, PrefillLayer or None) for layers 0..n_layers-1 of the config-5 stack, one at a
    time (a 131072-token layer is 1.6 GB): hitters drift 15 % per layer; None for layers not in `keep`
    (their random draws are still consumed, so a layer's tensors do not depend on which others are kept).
    K/V have room for `decode_steps` more tokens."""
    device = torch.device(device)
    Hq, Hkv, d = 32, 8, 128
    G = Hq // Hkv
    prev = [None] * Hkv
    for layer in range(n_layers):
        gen = torch.Generator(device=device)
        gen.manual_seed(layer_seed(BASE_SEED, 5, layer))
        pos_all = []
        us = []
        for hk in range(Hkv):
            us.append(_unit(gen, d, device))
            prev[hk] = _next_hitters(gen, prev[hk], S, 64, 0.85, device)
            pos_all.append(prev[hk])
        if keep is not None and layer not in keep:
            yield layer, None
            continue
        q = torch.randn(S, Hq, d, generator=gen, device=device, dtype=torch.float32)
        k = torch.zeros(Hkv, S + decode_steps, d, device=device, dtype=torch.bfloat16)
        v = torch.zeros(Hkv, S + decode_steps, d, device=device, dtype=torch.bfloat16)
        for hk in range(Hkv):
            kh = torch.randn(S, d, generator=gen, device=device, dtype=torch.float32)
            kh[pos_all[hk]] += 3.0 * us[hk]
            k[hk, :S] = kh.to(torch.bfloat16)
            v[hk, :S] = torch.randn(S, d, generator=gen, device=device, dtype=torch.float32).to(torch.bfloat16)
            q[:, hk * G:(hk + 1) * G] += us[hk]
        yield layer, PrefillLayer(q.to(torch.bfloat16), k, v)


def config5_prefill(device="cuda", layers=(0, 1, 2, 3), S=131072, T=32, decode_steps=256):
    """Attention-only stack, 32/8 heads, d128, bf16: causal prefill of S tokens, k_t = 10 % of the prefix,
    anchors {0, 1, 4, 12, 20}, hitters drifting 15 % per layer.  Returns a PrefillWorkload holding only
    the requested layers (layer 0 is the dense-output anchor); K/V are allocated with room for
    `decode_steps` more tokens so that decode steps can append to the same cache."""
    wl = PrefillWorkload(f"cfg5-prefill-bf16-S{S}-T{T}", S, 32, 8, 128, torch.bfloat16, T, prefill_budgets(S, T, 100, 0))
    for _, layer in iter_config5_layers(device, max(layers) + 1, S, decode_steps, keep=set(layers)):
        if layer is not None:
            wl.layers.append(layer)
    return wl


def layer_stack(device="cpu", n_layers=8, block_starts=(0, 3, 5), B=2, Hq=8, Hkv=2, d=64, dtype=torch.float32,
                seqlens=(3000, 2500), k=96, n_hitters=32, within=0.95):
    """Calibration-shaped stack (Sec. 3.3): consecutive layers inside a block keep nearly all
    heavy-hitter positions, a new block redraws them, so the similarity matrix is block
    structured and the best anchors are the block starts."""
    overlap = [0.0 if l in block_starts else within for l in range(n_layers)]
    return make_decode_workload(f"stack-{n_layers}-layers", 6, n_layers, B, Hq, Hkv, d, dtype, list(seqlens),
                                [k] * B, n_hitters, overlap, 0, boost=12.0, q_boost=3.0, device=device)


def permuted_head_layer(layer, perm, Hq, noise=0.05, seed=BASE_SEED + 6500):
    """A second layer whose key head h (with its query group) is a noisy copy of key head
    perm[h] of `layer`: the planted head correspondence of Sec. 3.5."""
    g = torch.Generator().manual_seed(seed)
    Hkv = layer.k.shape[1]
    G = Hq // Hkv
    dtype = layer.q.dtype
    qh = [h2 * G + i for h2 in perm for i in range(G)]
    q = layer.q.float().cpu()[:, qh]
    k = layer.k.float().cpu()[:, list(perm)]
    v = layer.v.float().cpu()[:, list(perm)]
    q = q + noise * torch.randn(q.shape, generator=g)
    k = k + noise * torch.randn(k.shape, generator=g)
    return DecodeLayer(q.to(dtype), k.to(dtype), v.to(dtype), None)
