"""CPU oracle for the Task-KV hot path -- TEST INFRASTRUCTURE, not the product.

A plain, slow, fp64 numpy statement of what the path computes, written from the
paper (Task-KV, arXiv 2501.15113).  It shares no code with the HIP library and
never imports it; only the tests, the smoke check and the benchmark's CPU
baseline leg may import this module.  Every function takes ONE layer and ONE
batch element (batch elements and layers are independent in the method).

Inputs are converted exactly to float64 (fp32 and bf16 values are both exactly
representable); all arithmetic is IEEE fp64; nothing is blocked, fused or
re-ordered beyond what the cited equation states.

Notation (paper Sec. 3.1, 4.1, 4.2): N context length, d head dim, L observation
window, t top-t count, n heads, s1 sink tokens, s2 recent tokens, k middle
activations.  H_q query heads share H_kv key/value heads in groups of
G = H_q / H_kv (Sec. 5.3 names grouped-query attention but gives no mechanics).

Readings taken where the paper is silent (each is repeated at the function):
  * grouped-query attention: one separator decision per KV head; the column
    mean of Eq. 13 runs over the G*L window rows of the group   [parity unpinned]
  * middle activations are ranked by the same window score C (pooled if a
    pooling width > 1 is given)                                   [parity unpinned]
  * pooling = stride-1 mean with zero padding and fixed divisor   [parity unpinned]
  * compression happens once, after prefill; every head then appends every
    decoded token                                                 [parity unpinned]
  * ties (equal scores / equal distances) go to the lower index
  * the centre of Eq. 8 is taken over all KV heads of the layer; distance is
    the L2 norm of Sec. 3.3
"""
from __future__ import annotations

import math

import numpy as np

__all__ = [
    "window_scores", "pool_scores", "top_indices", "semantic_vectors",
    "centre_and_distances", "hetero_mask", "kept_tokens", "pack_cache",
    "decode_attention", "separate", "compress", "full_semantic_vector",
    "hetero_head_count", "middle_budget", "merge_partials",
    "kept_tokens_no_cache", "compressed_cache", "round_to_storage",
]


def _f64(x):
    return np.asarray(x, dtype=np.float64)


# --------------------------------------------------------------------------- #
# Semantic separator (Sec. 4.1)
# --------------------------------------------------------------------------- #
def window_scores(q_win, k, scale=None):
    """Eq. 12 and Eq. 13: local weight matrix A' and its column mean C.

    q_win [H_q, L, d]  last L query rows of the prompt (window row i sits at
                       absolute position N-L+i)
    k     [H_kv, N, d] key states
    ->    C [H_kv, N]

    A'[q,i,:] = softmax_j(scale * q_win[q,i] . k[h(q),j] + M'), h(q) = q // G,
    where the causal mask M' removes keys j > N-L+i (it only bites inside the
    trailing L x L block).  C[h] = sum over the group's G*L rows of A' divided
    by G*L -- for G = 1 exactly Eq. 13; always the fixed divisor, also for
    columns that only some rows can see.
    """
    q_win, k = _f64(q_win), _f64(k)
    hq, L, d = q_win.shape
    hkv, N, _ = k.shape
    assert hq % hkv == 0 and L <= N
    G = hq // hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    i = np.arange(L)[:, None]
    j = np.arange(N)[None, :]
    hidden = j > (N - L + i)
    C = np.zeros((hkv, N))
    for q in range(hq):
        h = q // G
        s = scale * (q_win[q] @ k[h].T)                 # [L, N]
        s = np.where(hidden, -np.inf, s)
        a = np.exp(s - s.max(axis=1, keepdims=True))
        a = a / a.sum(axis=1, keepdims=True)            # rows of A'
        C[h] += a.sum(axis=0)
    return C / float(G * L)


def pool_scores(C, width):
    """Average pooling of the selection scores (Sec. 5.4 sets the kernel to 7).

    Stride 1, zero padding, fixed divisor `width` (odd).  width 1 = identity.
    """
    C = _f64(C)
    if width == 1:
        return C.copy()
    assert width % 2 == 1 and width >= 1
    r = (width - 1) // 2
    N = C.shape[-1]
    P = np.zeros_like(C)
    for u in range(-r, r + 1):
        lo, hi = max(0, -u), min(N, N - u)
        P[..., lo:hi] += C[..., lo + u:hi + u]
    return P / float(width)


def top_indices(score, count):
    """Eq. 14: indices of the `count` largest entries, ordered by
    (score descending, index ascending) -- ties go to the lower index."""
    score = _f64(score)
    count = min(int(count), score.shape[0])
    order = np.lexsort((np.arange(score.shape[0]), -score))
    return order[:count]


def semantic_vectors(C, v, t):
    """Eq. 14-15: v'[h] = sum_{j in I[h]} C[h,j] * V[h,j,:], I[h] = Top(C[h], t).

    The garbled `C[I,:]` of Eq. 15 is read as the 1 x t row C[I]; no
    renormalisation by the captured mass.
    """
    C, v = _f64(C), _f64(v)
    hkv, N, d = v.shape
    out = np.zeros((hkv, d))
    picks = []
    for h in range(hkv):
        I = top_indices(C[h], t)
        picks.append(I)
        out[h] = C[h, I] @ v[h, I, :]
    return out, picks


def centre_and_distances(sem):
    """Eq. 7-8 with the L2 norm of Sec. 3.3: centre = mean over heads,
    dist[h] = || sem[h] - centre ||_2."""
    sem = _f64(sem)
    centre = sem.sum(axis=0) / sem.shape[0]
    delta = sem - centre[None, :]
    return centre, np.sqrt((delta * delta).sum(axis=1))


def hetero_mask(dist, n_hetero, add_centre_head=False):
    """Sec. 4.1, head ranking: the n_hetero heads farthest from the centre are
    heterogeneous; optionally the remaining head closest to the centre joins
    them.  Ties -> lower head index."""
    dist = _f64(dist)
    n = dist.shape[0]
    heads = np.arange(n)
    mask = np.zeros(n, dtype=np.uint8)
    far = np.lexsort((heads, -dist))[:max(0, min(int(n_hetero), n))]
    mask[far] = 1
    if add_centre_head and (mask == 0).any():
        rest = heads[mask == 0]
        near = rest[np.lexsort((rest, dist[rest]))[0]]
        mask[near] = 1
    return mask


# --------------------------------------------------------------------------- #
# KV cache allocation (Sec. 4.2)
# --------------------------------------------------------------------------- #
def kept_tokens(P_row, is_hetero, n_sink, n_recent, n_middle):
    """Sec. 4.2: heterogeneous heads keep every token; the others keep the s1
    sinks, the s2 most recent tokens and the k middle tokens with the highest
    score.  Returned ascending by position.  If sinks and recent window
    already cover the context, everything is kept; k is clipped to the size of
    the middle."""
    P_row = _f64(P_row)
    N = P_row.shape[0]
    if is_hetero or n_sink + n_recent >= N:
        return np.arange(N, dtype=np.int64)
    lo, hi = n_sink, N - n_recent
    mid = lo + top_indices(P_row[lo:hi], min(n_middle, hi - lo))
    kept = np.concatenate([np.arange(0, lo), mid, np.arange(hi, N)])
    return np.sort(kept).astype(np.int64)


def pack_cache(k, v, kept):
    """Sec. 4.2: the retained KV states of one head, copied bit-for-bit in the
    storage dtype, ascending by original position."""
    k, v = np.asarray(k), np.asarray(v)
    return k[kept].copy(), v[kept].copy()


# --------------------------------------------------------------------------- #
# Alternative compensation methods of the ablation (Sec. 6.2, Fig. 8):
# "No Cache" and "Compressed Cache"; "Selective Cache" is kept_tokens above.
# --------------------------------------------------------------------------- #
def kept_tokens_no_cache(N, is_hetero, n_sink, n_recent, n_extra):
    """No Cache: only sinks and recent tokens; the cache size that the other
    methods spend on the middle is added to the recent window."""
    if is_hetero or n_sink + n_recent + n_extra >= N:
        return np.arange(N, dtype=np.int64)
    return np.concatenate([np.arange(0, n_sink), np.arange(N - n_recent - n_extra, N)]).astype(np.int64)


def round_to_storage(x, dtype):
    """fp64 -> storage dtype, round to nearest, ties to even.  "f32": IEEE
    conversion.  "bf16": written out as the choice between the two bf16
    neighbours of each value (bf16 = 8 significant bits, so the neighbours of
    a = m * 2^E, 0.5 <= m < 1, are the multiples of 2^(E-8) around it); returned
    as float32 holding bf16-representable values (normal range assumed; the
    means of cached values are)."""
    x = _f64(x)
    if dtype == "f32":
        return x.astype(np.float32)
    a = np.abs(x)
    _, E = np.frexp(a)                               # a = m * 2^E
    ulp = np.ldexp(1.0, E - 8)                       # spacing of bf16 values in [2^(E-1), 2^E)
    steps = np.floor(a / ulp)                        # exact: a / ulp < 2^8 and ulp is a power of two
    below, above = steps * ulp, (steps + 1.0) * ulp
    d_below, d_above = a - below, above - a          # exact differences
    take_above = (d_above < d_below) | ((d_above == d_below) & (np.mod(steps, 2.0) == 1.0))
    nearest = np.where(take_above, above, below)
    nearest = np.where(a == 0.0, 0.0, nearest)
    return np.copysign(nearest, x).astype(np.float32)


def compressed_cache(k, v, is_hetero, n_sink, n_recent, n_groups, dtype):
    """Compressed Cache: the middle [s1, N-s2) is cut into n_groups contiguous
    groups of near-equal size (group g covers middle offsets
    [g*M/n, (g+1)*M/n), integer division) and each group is replaced by one
    compensation token, the arithmetic mean of its K rows and of its V rows,
    rounded once to the storage dtype.  The paper gives only "divides the
    intermediate tokens into groups, one compensation token per group"
    (reading: contiguous groups, plain mean) -- parity unpinned.
    Returns (k_cache, v_cache, first_positions): rows = sinks, compensation
    tokens, recent tokens; first_positions lists the original position of each
    row (first position of its group for a compensation token)."""
    k, v = np.asarray(k), np.asarray(v)
    N = k.shape[0]
    if is_hetero or n_sink + n_recent >= N:
        return k.copy(), v.copy(), np.arange(N, dtype=np.int64)
    lo, hi = n_sink, N - n_recent
    M = hi - lo
    n = min(n_groups, M)
    kk, vv, pos = [k[:lo]], [v[:lo]], list(range(lo))
    for g in range(n):
        a, b = lo + (g * M) // n, lo + ((g + 1) * M) // n
        km = _f64(k[a:b]).sum(axis=0) / float(b - a)
        vm = _f64(v[a:b]).sum(axis=0) / float(b - a)
        kk.append(round_to_storage(km, dtype)[None].astype(k.dtype))
        vv.append(round_to_storage(vm, dtype)[None].astype(v.dtype))
        pos.append(a)
    kk.append(k[hi:])
    vv.append(v[hi:])
    pos.extend(range(hi, N))
    return np.concatenate(kk), np.concatenate(vv), np.asarray(pos, dtype=np.int64)


# --------------------------------------------------------------------------- #
# Decode attention over the ragged cache (Sec. 3.1 Eq. 1 restricted to one
# query row and to the retained keys; Sec. 5.5.3 is where the paper times it)
# --------------------------------------------------------------------------- #
def decode_attention(q, k_cache, v_cache, scale=None):
    """q [H_q, d]; k_cache / v_cache: per-KV-head lists of [len_h, d] arrays.
    o[q] = softmax_p(scale * q[q] . K_c[h,p]) @ V_c[h], h = q // G.  No mask:
    the query is newer than everything cached."""
    q = _f64(q)
    hq, d = q.shape
    hkv = len(k_cache)
    G = hq // hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.zeros((hq, d))
    for qi in range(hq):
        h = qi // G
        K, V = _f64(k_cache[h]), _f64(v_cache[h])
        s = scale * (K @ q[qi])
        p = np.exp(s - s.max())
        p = p / p.sum()
        out[qi] = p @ V
    return out


def merge_partials(parts):
    """Exact recombination of softmax partials (m, l, o) of disjoint key sets:
    the property the GPU's split-K combine relies on.  o is unnormalised
    (sum of exp(s-m) * v).  Returns the normalised output."""
    M = max(m for m, _, _ in parts)
    Lsum = sum(l * math.exp(m - M) for m, l, _ in parts)
    O = sum(_f64(o) * math.exp(m - M) for m, _, o in parts)
    return O / Lsum


# --------------------------------------------------------------------------- #
# Whole steps, one batch element
# --------------------------------------------------------------------------- #
def separate(q_win, k, v, top_t, n_hetero, add_centre_head=False, scale=None):
    """Semantic separator for one layer, one batch element.
    Returns dict(scores C [H_kv,N], sem_vec [H_kv,d], dist [H_kv], mask uint8
    [H_kv], picks list of index arrays)."""
    C = window_scores(q_win, k, scale)
    sem, picks = semantic_vectors(C, v, top_t)
    _, dist = centre_and_distances(sem)
    mask = hetero_mask(dist, n_hetero, add_centre_head)
    return dict(scores=C, sem_vec=sem, dist=dist, mask=mask, picks=picks)


def compress(k, v, scores, mask, n_sink, n_recent, n_middle, pool_kernel=1, pack_mode=0, dtype="f32"):
    """Cache allocation for one layer, one batch element.
    pack_mode 0: selective cache (the method); 1: No Cache; 2: Compressed
    Cache (dtype names the storage type its means are rounded to).
    Returns (kept list of int64 arrays, k_cache list, v_cache list)."""
    P = pool_scores(scores, pool_kernel)
    kept, kc, vc = [], [], []
    for h in range(len(mask)):
        if pack_mode == 2:
            kk, vv, idx = compressed_cache(k[h], v[h], bool(mask[h]), n_sink, n_recent, n_middle, dtype)
            kept.append(idx)
            kc.append(kk)
            vc.append(vv)
            continue
        if pack_mode == 1:
            idx = kept_tokens_no_cache(P.shape[1], bool(mask[h]), n_sink, n_recent, n_middle)
        else:
            idx = kept_tokens(P[h], bool(mask[h]), n_sink, n_recent, n_middle)
        kk, vv = pack_cache(k[h], v[h], idx)
        kept.append(idx)
        kc.append(kk)
        vc.append(vv)
    return kept, kc, vc


# --------------------------------------------------------------------------- #
# The un-approximated definition, used as a pin (Sec. 3.1, Eq. 1-2)
# --------------------------------------------------------------------------- #
def full_semantic_vector(q, k, v, scale=None):
    """Eq. 1-2 for one head: A = softmax(Q K^T / sqrt(d) + causal mask),
    v = (sum_i A[i,:] / N) . V."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    N, d = q.shape
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    s = scale * (q @ k.T)
    s = np.where(np.arange(N)[None, :] > np.arange(N)[:, None], -np.inf, s)
    a = np.exp(s - s.max(axis=1, keepdims=True))
    a = a / a.sum(axis=1, keepdims=True)
    return (a.sum(axis=0) / N) @ v


# --------------------------------------------------------------------------- #
# Host-side budget arithmetic (Sec. 4.1 Eq. 16, Sec. 4.2 Eq. 17)
# --------------------------------------------------------------------------- #
def hetero_head_count(n_heads, beta, m_top, layer, n_layers):
    """Eq. 16: f(r) = n*beta - (n*beta - m)/(R-1) * r, r = 0..R-1; rounded half
    up and clipped to [0, n] (the paper leaves rounding open)."""
    f = n_heads * beta
    if n_layers > 1:
        f -= (n_heads * beta - m_top) / (n_layers - 1) * layer
    return int(min(max(math.floor(f + 0.5), 0), n_heads))


def layer_plan(n_heads, beta, m_top, n_layers, budget_frac, ctx_len, n_sink, n_recent):
    """Sec. 4.1-4.2 put together for a stack of R layers under one budget: every
    layer gets B = budget_frac * n * N tokens (the "KV cache budget" of Sec. 5.4,
    a share of the full cache, floored to whole tokens); layer r marks f(r)
    heads by Eq. 16 and gives each other head k(r) middle activations by Eq. 17.
    Returns [(f(r), k(r)) for r in 0..R-1]."""
    budget = int(math.floor(budget_frac * n_heads * ctx_len))
    plan = []
    for r in range(n_layers):
        f = hetero_head_count(n_heads, beta, m_top, r, n_layers)
        plan.append((f, middle_budget(budget, ctx_len, n_heads, f, n_sink, n_recent)))
    return plan


def middle_budget(layer_budget_tokens, ctx_len, n_heads, n_hetero, n_sink, n_recent):
    """Eq. 17: k = (B - N f(r)) / (n - f(r)) - s1 - s2, floored, clipped at 0."""
    if n_heads == n_hetero:
        return 0
    k = (layer_budget_tokens - ctx_len * n_hetero) // (n_heads - n_hetero) - n_sink - n_recent
    return int(max(k, 0))
