"""Plain CPU statement of what the Kascade hot path computes (fp64, numpy).

THIS IS TEST INFRASTRUCTURE.  Only the tests, the smoke check and the
benchmark's CPU-baseline leg may import it; the product (HIP kernels + C ABI +
binding) never does, and this file imports nothing from the product.

Everything here is "the definition written out": no blocking, no online
softmax, no fused passes.  Each function names the passage of the paper
(Kascade, arXiv 2512.16391) it follows.  All floating point is float64; the
caller widens the exact device bits (bf16 or fp32) before calling.

Shapes (paper notation: N keys of dimension d per key head; H key heads):
    q      [Hq, d]              one decode query token, all query heads
    K, V   [Hkv, L, d]          the first L rows of one sequence's KV cache
    Q      [S, Hq, d]           prefill queries (token major)
    Kp, Vp [Hkv, S, d]          prefill keys / values
Query head h reads key head h // G with G = Hq // Hkv (consecutive grouping;
the paper leaves the assignment open, Sec. 2.2).

Readings of the paper taken where it is silent or unclear:
  * the sparse softmax is renormalised over the selected keys (Sec. 3.1: Eq. 2
    evaluated only over k keys; Sec. 3.6: the reuse kernel is a flash
    attention over the gathered keys, which has no dense denominator);
  * "pooling" of post-softmax distributions is the arithmetic mean (Sec. 3.2
    defines the layer distribution as the average over heads);
  * ties in Top-k go to the lower key index, index sets are emitted ascending;
  * an optional recent window W forces the last W positions into the set and
    they count against k;
  * prefill: the candidates of tile t are the keys strictly before the tile
    (Sec. 4.1: each tile attends to a fraction of the previous tokens), the
    tile's own diagonal block is always attended, causally, on top of k_t;
    row normalisers used for pooling include the diagonal keys;
  * Pre-Softmax pooling (Sec. 3.4, evaluated and rejected by the paper): the
    pooled query is stored in the tensors' own type, and its distribution is
    normalised over the tile's candidates (the keys before the tile) - the
    ranking, which is all the method uses, does not depend on that choice.

parity unpinned: none of the functions below - each has a pin in
tests/test_oracle_pins.py that does not come from this file.  What stays
unpinned is the numerical value of attention on the paper's real model
activations (no worked example is printed, datasets and weights are absent).
"""
import numpy as np


# ----------------------------------------------------------------------------
# Eq. 1 / Eq. 2: scaled dot-product attention, with GQA (Sec. 2.1, 2.2)
# ----------------------------------------------------------------------------

def softmax_lastdim(s):
    """softmax along the last axis (Eq. 1), max-subtracted for range only."""
    s = np.asarray(s, dtype=np.float64)
    e = np.exp(s - np.max(s, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def default_scale(d):
    """1/sqrt(d) of Eq. 1."""
    return 1.0 / np.sqrt(float(d))


def decode_logits(q, K, scale):
    """s[h, j] = scale * <q[h], K[h // G, j]>   (argument of softmax in Eq. 1)."""
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    Hq, d = q.shape
    Hkv, L, _ = K.shape
    G = Hq // Hkv
    s = np.empty((Hq, L), dtype=np.float64)
    for h in range(Hq):
        s[h] = scale * (K[h // G] @ q[h])
    return s


def decode_probabilities(q, K, scale):
    """p[h, :] of Eq. 1 for every query head; returns [Hq, L]."""
    return softmax_lastdim(decode_logits(q, K, scale))


def dense_decode(q, K, V, scale):
    """y[h] = p[h] . V[h // G]   (Eq. 2); the anchor output in layer 0 (Sec. 3.1)."""
    V = np.asarray(V, dtype=np.float64)
    p = decode_probabilities(q, K, scale)
    Hq = p.shape[0]
    G = Hq // V.shape[0]
    return np.stack([p[h] @ V[h // G] for h in range(Hq)])


# ----------------------------------------------------------------------------
# Sec. 3.4: post-softmax pooling over the GQA group (decode)
# ----------------------------------------------------------------------------

def pool_gqa(p, n_kv_heads):
    """a[hk, j] = mean over the G query heads of key head hk of p[h, j]."""
    p = np.asarray(p, dtype=np.float64)
    Hq, L = p.shape
    G = Hq // n_kv_heads
    return p.reshape(n_kv_heads, G, L).mean(axis=1)


# ----------------------------------------------------------------------------
# Sec. 3.1 / 3.5 / 3.6 pass 3: exact Top-k per key head
# ----------------------------------------------------------------------------

def select_topk(a, k, recent_window=0):
    """Index set of the k largest entries of the 1-D score vector a.

    Order of preference: larger score first, lower index first among equal
    scores.  The last `recent_window` positions are members unconditionally
    and use up part of k.  Returned ascending, dtype int64, length k.
    """
    a = np.asarray(a, dtype=np.float64)
    L = a.shape[0]
    W = int(recent_window)
    if not (0 <= k <= L) or not (0 <= W <= k):
        raise ValueError("need 0 <= recent_window <= k <= L")
    n_cand = L - W
    n_pick = k - W
    # stable sort of the negated candidate scores = (score desc, index asc)
    order = np.argsort(-a[:n_cand], kind="stable")
    chosen = order[:n_pick]
    forced = np.arange(n_cand, L, dtype=np.int64)
    return np.sort(np.concatenate([chosen.astype(np.int64), forced]))


def decode_anchor_indices(q, K, scale, k, recent_window=0):
    """Pass 1-3 of an anchor layer in decode (Sec. 3.6): Eq. 1 per query head,
    mean over each GQA group (Sec. 3.4), Top-k per key head (Sec. 3.5).
    Returns (idx [Hkv, k] ascending, pooled a [Hkv, L])."""
    Hkv = np.asarray(K).shape[0]
    a = pool_gqa(decode_probabilities(q, K, scale), Hkv)
    idx = np.stack([select_topk(a[hk], k, recent_window) for hk in range(Hkv)])
    return idx, a


# ----------------------------------------------------------------------------
# Sec. 3.1 (Oracle Top-k attention) / Sec. 3.6 (reuse layers, head map)
# ----------------------------------------------------------------------------

def sparse_decode(q, K, V, idx_sets, scale, head_map=None):
    """Eq. 1-2 restricted to the keys idx_sets[head_map[h // G]].

    idx_sets: sequence of Hkv_anchor 1-D integer arrays (any order, unique).
    head_map[hk] = key head of the anchor layer whose set key head hk of this
    layer uses (Sec. 3.5, many-to-one allowed); None = identity.
    """
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    Hq, d = q.shape
    Hkv = K.shape[0]
    G = Hq // Hkv
    y = np.empty((Hq, d), dtype=np.float64)
    for h in range(Hq):
        hk = h // G
        src = hk if head_map is None else int(head_map[hk])
        I = np.asarray(idx_sets[src], dtype=np.int64)
        p = softmax_lastdim(scale * (K[hk, I] @ q[h]))
        y[h] = p @ V[hk, I]
    return y


# ----------------------------------------------------------------------------
# Prefill, tile granular (Sec. 3.4: one index set per query tile and key head;
# Sec. 3.6: pass 1 row normalisers, pass 2 pooled weights, pass 3 Top-k,
# pass 4 sparse attention; Sec. 4.1: rolling Top-k over previous tokens)
# ----------------------------------------------------------------------------

def tile_bounds(t, T, S):
    """Token range [lo, hi) of query tile t of T tokens in a prompt of S."""
    lo = t * T
    return lo, min(lo + T, S)


def prefill_tile_probabilities(Q, Kp, t, T, scale):
    """Causal Eq. 1 for the rows of tile t.

    Returns P [n_tok, Hq, hi]: P[r, h, j] is the post-softmax weight of key j
    for token lo + r and head h, zero for j > lo + r (causal mask)."""
    Q = np.asarray(Q, dtype=np.float64)
    Kp = np.asarray(Kp, dtype=np.float64)
    S, Hq, d = Q.shape
    Hkv = Kp.shape[0]
    G = Hq // Hkv
    lo, hi = tile_bounds(t, T, S)
    P = np.zeros((hi - lo, Hq, hi), dtype=np.float64)
    for r in range(hi - lo):
        i = lo + r
        for h in range(Hq):
            s = scale * (Kp[h // G, : i + 1] @ Q[i, h])
            P[r, h, : i + 1] = softmax_lastdim(s)
    return P


def prefill_dense_tile(Q, Kp, Vp, t, T, scale):
    """Plain causal attention (Eq. 1-2) for the rows of tile t: [n_tok, Hq, d].
    This is what an anchor layer returns in layer 0 (Sec. 3.1, 3.6)."""
    Vp = np.asarray(Vp, dtype=np.float64)
    P = prefill_tile_probabilities(Q, Kp, t, T, scale)
    n_tok, Hq, hi = P.shape
    G = Hq // Vp.shape[0]
    y = np.empty((n_tok, Hq, Vp.shape[2]), dtype=np.float64)
    for h in range(Hq):
        y[:, h, :] = P[:, h, :] @ Vp[h // G, :hi]
    return y


def prefill_pooled_tile(Q, Kp, t, T, scale):
    """a[hk, j], j < t*T: mean over the tile's (token, head-in-group) rows of
    the causal post-softmax weight of prefix key j (Sec. 3.4, pooling over a
    full query tile including the GQA grouping).  Returns [Hkv, t*T]."""
    Hkv = np.asarray(Kp).shape[0]
    P = prefill_tile_probabilities(Q, Kp, t, T, scale)
    n_tok, Hq, hi = P.shape
    G = Hq // Hkv
    prefix = t * T
    # rows of the tile for key head hk: all n_tok tokens x its G query heads
    a = P[:, :, :prefix].reshape(n_tok, Hkv, G, prefix).mean(axis=(0, 2))
    return a


def prefill_anchor_indices_tile(Q, Kp, t, T, scale, k_t):
    """Top-k_t of the pooled prefix scores of tile t, per key head.
    Returns (idx [Hkv, k_t] ascending, pooled a [Hkv, t*T])."""
    a = prefill_pooled_tile(Q, Kp, t, T, scale)
    idx = np.stack([select_topk(a[hk], k_t, 0) for hk in range(a.shape[0])])
    return idx, a


def prefill_sparse_tile(Q, Kp, Vp, t, T, idx_sets, scale, head_map=None):
    """Sparse attention of tile t: every row (token i, head h) attends to the
    prefix keys idx_sets[head_map[h // G]] (all < t*T, unmasked) and to the
    diagonal keys t*T .. i, one softmax over the union (Sec. 3.6 pass 4 /
    reuse layers; Sec. 4.1).  Returns [n_tok, Hq, d]."""
    Q = np.asarray(Q, dtype=np.float64)
    Kp = np.asarray(Kp, dtype=np.float64)
    Vp = np.asarray(Vp, dtype=np.float64)
    S, Hq, d = Q.shape
    Hkv = Kp.shape[0]
    G = Hq // Hkv
    lo, hi = tile_bounds(t, T, S)
    y = np.empty((hi - lo, Hq, Vp.shape[2]), dtype=np.float64)
    for r in range(hi - lo):
        i = lo + r
        for h in range(Hq):
            hk = h // G
            src = hk if head_map is None else int(head_map[hk])
            I = np.asarray(idx_sets[src], dtype=np.int64)
            if I.size and I.max() >= lo:
                raise ValueError("prefill index beyond the tile's prefix")
            keys = np.concatenate([I, np.arange(lo, i + 1, dtype=np.int64)])
            p = softmax_lastdim(scale * (Kp[hk, keys] @ Q[i, h]))
            y[r, h] = p @ Vp[hk, keys]
    return y


# ----------------------------------------------------------------------------
# Sec. 3.2, Eq. 3: how much of layer b's Top-k mass layer a's Top-k recovers
# (used here only as a quality figure on synthetic inputs)
# ----------------------------------------------------------------------------

def topk_similarity(p_b, idx_a, idx_b):
    """sim(a, b) of Eq. 3 for one distribution p_b and two index sets."""
    p_b = np.asarray(p_b, dtype=np.float64)
    return float(p_b[np.asarray(idx_a)].sum() / p_b[np.asarray(idx_b)].sum())


# ----------------------------------------------------------------------------
# Sec. 4.1: the k rule;  Table 3 caption: per-layer average time
# ----------------------------------------------------------------------------

def topk_budget(L, fraction, k_min=0):
    """k = min(max(ceil(fraction * L), k_min), L).  The paper prints
    min(max(0.1 L, 128), L) without a rounding rule; the ceiling is what
    turns 0.1 * 2048 into 205."""
    # exact integer ceiling of fraction*L for fractions given in per-mille
    permille = int(round(fraction * 1000))
    k = -((-permille * int(L)) // 1000)
    return int(min(max(k, int(k_min)), int(L)))


def kascade_layer_average(t_anchor0, t_anchor, t_reuse, n_layers=32, n_anchors=5):
    """Weighted per-layer time of Table 3's caption: one dense-output anchor
    (layer 0), n_anchors-1 other anchors, the rest reuse layers."""
    return (t_anchor0 + (n_anchors - 1) * t_anchor
            + (n_layers - n_anchors) * t_reuse) / n_layers


# ----------------------------------------------------------------------------
# Sec. 3.3, Algorithm 1: anchor-layer selection by dynamic programming
# ----------------------------------------------------------------------------

def segment_score(S, anchors):
    """Objective the selection maximises: every layer l is served by the last anchor i <= l and
    contributes S[i][l] (0-based layers; anchors ascending, anchors[0] == 0)."""
    S = np.asarray(S, dtype=np.float64)
    L = S.shape[0]
    bounds = list(anchors) + [L]
    return float(sum(S[i, l] for i, nxt in zip(bounds[:-1], bounds[1:]) for l in range(i, nxt)))


def select_anchor_layers(S, n_anchors):
    """Algorithm 1 in the paper's 1-based notation: dp[m][j] = best total similarity when the m-th
    anchor sits at layer j (j = L+1 is the end sentinel) and the (m-1)-th anchor at some i < j serves
    layers i..j-1.  Layer 1 is always the first anchor.  Ties keep the lowest i.
    Returns the anchors as ascending 0-based layer numbers."""
    S = np.asarray(S, dtype=np.float64)
    L, M = S.shape[0], int(n_anchors)
    if not (1 <= M <= L):
        raise ValueError("need 1 <= n_anchors <= n_layers")
    s1 = np.zeros((L + 2, L + 2))
    s1[1:L + 1, 1:L + 1] = S
    dp = np.full((M + 2, L + 2), -np.inf)
    path = np.zeros((M + 2, L + 2), dtype=np.int64)
    dp[1][1] = s1[1][1]
    for m in range(2, M + 2):
        for j in range(m, L + 2):
            best, arg = -np.inf, 0
            for i in range(m - 1, j):
                val = dp[m - 1][i] + sum(s1[i][l] for l in range(i, j))
                if val > best:
                    best, arg = val, i
            dp[m][j], path[m][j] = best, arg
    anchors, j = [], L + 1
    for m in range(M + 1, 1, -1):
        j = int(path[m][j])
        anchors.append(j - 1)
    return anchors[::-1]


def similarity_from_layers(pooled, index_sets):
    """S[a][b] for a <= b from per-layer pooled distributions and Top-k sets of ONE query position:
    pooled[l] is [n_seg, N] (one row per (sequence, key head)), index_sets[l] is [n_seg, k].
    Eq. 3 per segment; Sec. 3.3 takes the minimum over the samples (here: over the segments).
    Entries with a > b are 0 (an anchor only serves later layers)."""
    n = len(pooled)
    S = np.zeros((n, n))
    for a in range(n):
        for b in range(a, n):
            sims = [topk_similarity(pooled[b][g], index_sets[a][g], index_sets[b][g]) for g in range(len(pooled[b]))]
            S[a, b] = min(sims)
    return S


def weight_similarity(S, w):
    """Sec. 3.3, layer importance: entry (i, j) is scaled by the weight of the SERVED layer j."""
    return np.asarray(S, dtype=np.float64) * np.asarray(w, dtype=np.float64)[None, :]


def layer_importance(x, y):
    """Sec. 3.3: 1 - cosine similarity between the input x and the output y of a layer's
    attention block, one value per row (token)."""
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    cos = (x * y).sum(-1) / (np.sqrt((x * x).sum(-1)) * np.sqrt((y * y).sum(-1)))
    return 1.0 - cos


# ----------------------------------------------------------------------------
# Sec. 3.5: head map from head-level similarity
# ----------------------------------------------------------------------------

def head_similarity(pooled_b, sets_a, sets_b):
    """Eq. 3 at head level for ONE sample: pooled_b [H, N] of the reuse layer, sets_a [Ha, k] of
    the anchor layer, sets_b [H, k] of the reuse layer.  Entry (h, h') = similarity of anchor head
    h' used for reuse head h."""
    H, Ha = len(pooled_b), len(sets_a)
    return np.array([[topk_similarity(pooled_b[h], sets_a[g], sets_b[h]) for g in range(Ha)] for h in range(H)])


def head_map_from_similarity(sims):
    """sims [n_samples, H, Ha].  Each reuse head takes the anchor head with the largest mean
    similarity over the samples (many-to-one allowed); ties go to the lower anchor head.
    Reading: the paper aggregates over its development set without naming the statistic."""
    mean = np.asarray(sims, dtype=np.float64).mean(axis=0)
    return np.argmax(mean, axis=1).astype(np.int64), mean


# ----------------------------------------------------------------------------
# Sec. 3.5, first strategy: one Top-k set shared by all heads of a layer
# ----------------------------------------------------------------------------

def decode_shared_indices(q, K, scale, k, recent_window=0):
    """Post-softmax distributions of ALL query heads averaged into one layer distribution
    (the variant the paper reports as "all heads pooled"), then Top-k.
    Returns (idx [k] ascending, pooled a [L])."""
    a = decode_probabilities(q, K, scale).mean(axis=0)
    return select_topk(a, k, recent_window), a


def prefill_shared_indices_tile(Q, Kp, t, T, scale, k_t):
    """The same for a prefill tile: mean over the tile's tokens and all query heads of the causal
    post-softmax weight of each prefix key, then Top-k_t.  Returns (idx [k_t], pooled a [t*T])."""
    P = prefill_tile_probabilities(Q, Kp, t, T, scale)
    a = P[:, :, : t * T].mean(axis=(0, 1))
    return select_topk(a, k_t, 0), a


# ----------------------------------------------------------------------------
# Sec. 3.4, the alternative the paper evaluates and rejects: Pre-Softmax pooling
# (average the tile's query vectors, run attention once with the pooled query)
# ----------------------------------------------------------------------------

def round_to_bf16(x):
    """Nearest bfloat16 (ties to even) of float32 values, returned as float32.
    bfloat16 is the upper half of the float32 pattern: add half of the dropped
    part, plus the kept part's last bit on an exact tie, then cut."""
    bits = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    keep_lsb = (bits >> np.uint64(16)) & np.uint64(1)
    rounded = (bits + np.uint64(0x7FFF) + keep_lsb) & np.uint64(0xFFFF0000)
    return rounded.astype(np.uint32).view(np.float32)


def round_nearest_even(x, sig_bits, min_exp):
    """Nearest value of a binary floating-point format to each float64 in x, ties to the
    even neighbour, in ONE rounding.  The format has `sig_bits` significant bits (hidden
    bit included) and smallest normal value 2**min_exp; below that the step stays that of
    the smallest normals (subnormals).  bfloat16: (8, -126); binary16: (11, -14);
    binary32: (24, -126).  Overflow to infinity is not modelled (not reachable from
    averages of finite inputs of the same format).  Returns float64."""
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)                       # x = m * 2**e with 0.5 <= |m| < 1, so |x| < 2**e
    step_exp = np.maximum(e - 1, min_exp) - (sig_bits - 1)
    # x / step is exact (a power of two), rint rounds half to even, the product is exact
    return np.ldexp(np.rint(np.ldexp(x, -step_exp)), step_exp)


STORAGE_FORMATS = {"bf16": (8, -126), "fp16": (11, -14), "fp32": (24, -126)}


def pool_query_vectors(rows, storage):
    """Pooled query of Pre-Softmax pooling (Sec. 3.4): the average of the given query
    vectors [n, d].  The average is itself a query that the attention kernels consume, so
    it exists in the tensors' storage type: the mean is taken exactly (float64; the inputs
    are 16- or 32-bit values) and rounded ONCE to `storage` ("fp32", "bf16", "fp16";
    nearest, ties to even).  Returns float64 [d]."""
    if storage not in STORAGE_FORMATS:
        raise ValueError("storage is 'fp32', 'bf16' or 'fp16'")
    rows = np.asarray(rows, dtype=np.float64)
    mean = rows.sum(axis=0) / rows.shape[0]
    return round_nearest_even(mean, *STORAGE_FORMATS[storage])


def decode_presoftmax_indices(q, K, scale, k, storage, recent_window=0):
    """Anchor passes 1-3 with Pre-Softmax pooling, decode: per key head the G
    query heads of its group are averaged into one query, Eq. 1 is evaluated
    once with it, Top-k of that distribution.
    Returns (idx [Hkv, k] ascending, a [Hkv, L])."""
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    Hq, d = q.shape
    Hkv, L, _ = K.shape
    G = Hq // Hkv
    a = np.empty((Hkv, L), dtype=np.float64)
    for hk in range(Hkv):
        qbar = pool_query_vectors(q[hk * G:(hk + 1) * G], storage)
        a[hk] = softmax_lastdim(scale * (K[hk] @ qbar))
    idx = np.stack([select_topk(a[hk], k, recent_window) for hk in range(Hkv)])
    return idx, a


def prefill_presoftmax_indices_tile(Q, Kp, t, T, scale, k_t, storage):
    """The same for prefill tile t: the tile's (token, head-in-group) query
    vectors - tokens ascending, heads ascending inside a token - are averaged
    per key head, Eq. 1 is evaluated once with the pooled query over the keys
    strictly before the tile (the tile's Top-k candidates), Top-k_t of that.
    Returns (idx [Hkv, k_t] ascending, a [Hkv, t*T])."""
    Q = np.asarray(Q, dtype=np.float64)
    Kp = np.asarray(Kp, dtype=np.float64)
    S, Hq, d = Q.shape
    Hkv = Kp.shape[0]
    G = Hq // Hkv
    lo, hi = tile_bounds(t, T, S)
    a = np.empty((Hkv, lo), dtype=np.float64)
    for hk in range(Hkv):
        rows = Q[lo:hi, hk * G:(hk + 1) * G, :].reshape(-1, d)
        qbar = pool_query_vectors(rows, storage)
        a[hk] = softmax_lastdim(scale * (Kp[hk, :lo] @ qbar)) if lo > 0 else np.zeros(0)
    idx = np.stack([select_topk(a[hk], k_t, 0) for hk in range(Hkv)])
    return idx, a
