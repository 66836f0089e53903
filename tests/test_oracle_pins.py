"""Pins for the CPU oracle: each test checks it against something the paper or
the mathematics fixes independently of the oracle's own formulas -- closed
forms, invariants, library routines on special cases, brute force.  No GPU."""
import itertools
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import taskkv_oracle as orc

RNG = np.random.default_rng(20250115)


def rand(*shape):
    return RNG.standard_normal(shape)


# ----------------------------------------------------------------- Eq. 12-13
def test_scores_rows_sum_to_one():
    q, k = rand(6, 8, 16), rand(3, 50, 16)
    C = orc.window_scores(q, k)
    assert C.shape == (3, 50)
    np.testing.assert_allclose(C.sum(axis=1), 1.0, rtol=0, atol=1e-14)
    assert (C >= 0).all()


def test_scores_zero_keys_closed_form():
    """K == 0: every visible key of window row i gets weight 1/(N-L+i+1), so
    C[j] = (1/L) * sum_{i >= max(0, j-(N-L))} 1/(N-L+i+1)  (catches an
    off-by-one or reversed causal mask and a wrong divisor)."""
    N, L, d = 37, 5, 8
    C = orc.window_scores(rand(1, L, d), np.zeros((1, N, d)))[0]
    expect = np.zeros(N)
    for j in range(N):
        for i in range(L):
            if j <= N - L + i:
                expect[j] += 1.0 / (N - L + i + 1)
    expect /= L
    np.testing.assert_allclose(C, expect, rtol=1e-14)
    assert np.all(C[:N - L + 1] == C[0])        # flat before the window
    assert np.all(np.diff(C[N - L:]) < 0)       # strictly decreasing inside it


def test_full_window_equals_eq_1_2_via_library_sdpa():
    """L = N, t = N, G = 1: the reduced vector of Eq. 15 is Eq. 2's vector,
    which is the row-mean of ordinary causal attention output.  Checked
    against torch's scaled_dot_product_attention in fp64 (default scale
    1/sqrt(d), is_causal)."""
    N, d, H = 24, 16, 3
    q, k, v = rand(H, N, d), rand(H, N, d), rand(H, N, d)
    ref = F.scaled_dot_product_attention(torch.tensor(q), torch.tensor(k), torch.tensor(v),
                                         is_causal=True).numpy().mean(axis=1)
    C = orc.window_scores(q, k)
    sem, picks = orc.semantic_vectors(C, v, N)
    np.testing.assert_allclose(sem, ref, rtol=1e-12, atol=1e-14)
    for h in range(H):
        np.testing.assert_allclose(orc.full_semantic_vector(q[h], k[h], v[h]), ref[h],
                                   rtol=1e-12, atol=1e-14)
        assert sorted(picks[h].tolist()) == list(range(N))


def test_window_is_last_rows_of_full_attention():
    """A' is rows N-L.. of the full causal attention matrix: C equals the
    column-mean of those rows of a library softmax."""
    N, L, d = 40, 7, 8
    q, k = rand(1, N, d), rand(1, N, d)
    s = torch.tensor(q[0] @ k[0].T / math.sqrt(d))
    s = s.masked_fill(torch.triu(torch.ones(N, N, dtype=torch.bool), 1), float("-inf"))
    A = torch.softmax(s, dim=1).numpy()
    C = orc.window_scores(q[:, N - L:, :], k)[0]
    np.testing.assert_allclose(C, A[N - L:].mean(axis=0), rtol=1e-12, atol=1e-16)


def test_gqa_group_mapping_and_mean():
    """Query head q reads KV head q // G; the group score is the mean of the
    per-query-head scores (computed here through G = 1 calls)."""
    Hkv, G, L, N, d = 3, 4, 6, 30, 8
    q, k = rand(Hkv * G, L, d), rand(Hkv, N, d)
    C = orc.window_scores(q, k)
    for h in range(Hkv):
        per = [orc.window_scores(q[h * G + g][None], k[h][None])[0] for g in range(G)]
        np.testing.assert_allclose(C[h], np.mean(per, axis=0), rtol=1e-13)
    q_dup = np.repeat(q[::G], G, axis=0)            # identical heads inside a group
    np.testing.assert_allclose(orc.window_scores(q_dup, k), orc.window_scores(q[::G], k), rtol=1e-13)


def test_custom_scale_is_applied_to_logits():
    q, k = rand(2, 4, 8), rand(2, 20, 8)
    np.testing.assert_allclose(orc.window_scores(q, k, scale=0.5),
                               orc.window_scores(q * 0.5 * math.sqrt(8), k), rtol=1e-12)


# ----------------------------------------------------------------- pooling
@pytest.mark.parametrize("w", [1, 3, 7])
def test_pool_matches_library_avg_pool(w):
    C = np.abs(rand(3, 41))
    ref = F.avg_pool1d(torch.tensor(C)[None], w, stride=1, padding=(w - 1) // 2,
                       count_include_pad=True)[0].numpy()
    np.testing.assert_allclose(orc.pool_scores(C, w), ref, rtol=1e-14)


# ----------------------------------------------------------------- Eq. 14-15
def test_top_indices_order_and_ties():
    s = np.array([0.3, 0.9, 0.3, 0.1, 0.9, 0.3])
    assert orc.top_indices(s, 4).tolist() == [1, 4, 0, 2]
    assert orc.top_indices(s, 10).tolist() == [1, 4, 0, 2, 5, 3]
    x = RNG.permutation(200).astype(float)
    assert orc.top_indices(x, 17).tolist() == np.argsort(-x)[:17].tolist()


def test_semantic_vector_constant_values():
    """V rows all equal to c: v' = (sum of picked weights) * c; with t = N
    that is c itself because the weights sum to one."""
    Hkv, N, d, L = 2, 33, 8, 4
    q, k = rand(Hkv, L, d), rand(Hkv, N, d)
    c = rand(Hkv, d)
    v = np.broadcast_to(c[:, None, :], (Hkv, N, d))
    C = orc.window_scores(q, k)
    full, _ = orc.semantic_vectors(C, v, N)
    np.testing.assert_allclose(full, c, rtol=1e-13)
    t = 5
    part, picks = orc.semantic_vectors(C, v, t)
    for h in range(Hkv):
        mass = np.sort(C[h])[::-1][:t].sum()
        np.testing.assert_allclose(part[h], mass * c[h], rtol=1e-13)
        assert len(picks[h]) == t


def test_semantic_vector_is_weighted_sum_of_picked_rows():
    """One-hot V (V[j] = e_j) turns v' into the picked weights themselves:
    entry j is C[j] if j was picked, else 0 -- catches a transposed operand or
    weights taken from the wrong positions."""
    N, L = 12, 3
    q, k = rand(1, L, N), rand(1, N, N)
    v = np.eye(N)[None]
    C = orc.window_scores(q, k)
    sem, picks = orc.semantic_vectors(C, v, 4)
    expect = np.zeros(N)
    top4 = np.argsort(-C[0])[:4]
    expect[top4] = C[0, top4]
    np.testing.assert_allclose(sem[0], expect, rtol=1e-14)


# ----------------------------------------------------------------- Eq. 7-8, ranking
def test_centre_and_distances_hand_case():
    sem = np.zeros((4, 5))
    sem[3, 0] = 4.0
    centre, dist = orc.centre_and_distances(sem)
    np.testing.assert_allclose(centre, [1, 0, 0, 0, 0])
    np.testing.assert_allclose(dist, [1, 1, 1, 3])
    assert orc.hetero_mask(dist, 1).tolist() == [0, 0, 0, 1]
    # ties among the three near heads go to the lower index
    assert orc.hetero_mask(dist, 2).tolist() == [1, 0, 0, 1]
    assert orc.hetero_mask(dist, 1, add_centre_head=True).tolist() == [1, 0, 0, 1]
    assert orc.hetero_mask(dist, 0).tolist() == [0, 0, 0, 0]
    assert orc.hetero_mask(dist, 9).tolist() == [1, 1, 1, 1]
    # a 3-4-5 triangle: two heads at (0,0) and (6,8) are both 5 from their mean (the L1 distance would be 7)
    centre, dist = orc.centre_and_distances(np.array([[0.0, 0.0], [6.0, 8.0]]))
    np.testing.assert_allclose(centre, [3, 4])
    np.testing.assert_allclose(dist, [5, 5], rtol=1e-15)


def test_add_centre_head_picks_closest_remaining():
    dist = np.array([5.0, 1.0, 3.0, 0.5, 4.0])
    assert orc.hetero_mask(dist, 2).tolist() == [1, 0, 0, 0, 1]
    assert orc.hetero_mask(dist, 2, add_centre_head=True).tolist() == [1, 0, 0, 1, 1]
    assert orc.hetero_mask(dist, 5, add_centre_head=True).tolist() == [1, 1, 1, 1, 1]


def test_distance_permutation_and_translation_invariance():
    Hkv, N, d, L = 5, 28, 8, 4
    q, k, v = rand(Hkv, L, d), rand(Hkv, N, d), rand(Hkv, N, d)
    v[2] += 3.0
    a = orc.separate(q, k, v, top_t=9, n_hetero=2)
    perm = RNG.permutation(Hkv)
    b = orc.separate(q[perm], k[perm], v[perm], top_t=9, n_hetero=2)
    np.testing.assert_allclose(b["dist"], a["dist"][perm], rtol=1e-12)
    assert b["mask"].tolist() == a["mask"][perm].tolist()
    # with t = N the weights sum to one, so shifting every V row by one vector
    # shifts every head vector and the centre alike
    c = orc.separate(q, k, v, top_t=N, n_hetero=2)
    e = orc.separate(q, k, v + rand(d)[None, None, :], top_t=N, n_hetero=2)
    np.testing.assert_allclose(e["dist"], c["dist"], rtol=1e-10)


# ----------------------------------------------------------------- Sec. 4.2
def test_middle_pick_brute_force():
    """On tiny inputs with distinct scores the picked middle set is the
    k-subset of the middle with the largest total score (all subsets
    enumerated), sinks and recent tokens are always present, the result is
    sorted and duplicate-free."""
    for trial in range(20):
        N = int(RNG.integers(8, 13))
        s1, s2 = int(RNG.integers(0, 3)), int(RNG.integers(0, 4))
        k = int(RNG.integers(0, 4))
        P = RNG.random(N)
        kept = orc.kept_tokens(P, False, s1, s2, k)
        mid = list(range(s1, N - s2))
        k_eff = min(k, len(mid))
        best = max(itertools.combinations(mid, k_eff), key=lambda c: P[list(c)].sum())
        expect = sorted(set(range(s1)) | set(best) | set(range(N - s2, N)))
        assert kept.tolist() == expect
        assert len(kept) == s1 + k_eff + s2


def test_middle_pick_nested_and_tie_rule():
    N, s1, s2 = 60, 3, 5
    P = RNG.random(N)
    prev = set(orc.kept_tokens(P, False, s1, s2, 0).tolist())
    assert prev == set(range(s1)) | set(range(N - s2, N))
    for k in range(1, 12):
        cur = set(orc.kept_tokens(P, False, s1, s2, k).tolist())
        assert prev < cur and len(cur - prev) == 1
        assert (cur - prev).pop() in range(s1, N - s2)
        prev = cur
    flat = np.full(N, 0.25)                       # all equal -> lowest middle positions win
    assert orc.kept_tokens(flat, False, s1, s2, 4).tolist() == \
        list(range(s1)) + list(range(s1, s1 + 4)) + list(range(N - s2, N))


def test_keep_all_cases():
    P = RNG.random(20)
    full = list(range(20))
    assert orc.kept_tokens(P, True, 2, 3, 1).tolist() == full          # heterogeneous
    assert orc.kept_tokens(P, False, 12, 8, 1).tolist() == full         # sinks+recent cover N
    assert orc.kept_tokens(P, False, 2, 3, 99).tolist() == full         # k clipped to the middle
    assert orc.kept_tokens(P, False, 2, 3, 15).tolist() == full


def test_pack_is_byte_copy():
    k = rand(9, 4).astype(np.float32)
    v = rand(9, 4).astype(np.float32)
    kept = np.array([0, 3, 4, 8])
    kc, vc = orc.pack_cache(k, v, kept)
    assert kc.dtype == np.float32 and kc.tobytes() == k[kept].tobytes()
    assert vc.tobytes() == v[kept].tobytes()


# ----------------------------------------------------------------- decode
def _sdpa(q, k, v):
    return F.scaled_dot_product_attention(torch.tensor(q)[:, None, :], torch.tensor(k),
                                          torch.tensor(v)).numpy()[:, 0, :]


def test_decode_full_budget_equals_dense_attention():
    """All heads heterogeneous, or a middle budget covering the context: the
    decode output equals dense softmax attention over every token (library
    SDPA, fp64)."""
    Hkv, G, N, d, L = 3, 2, 45, 16, 5
    qw, k, v = rand(Hkv * G, L, d), rand(Hkv, N, d), rand(Hkv, N, d)
    q = rand(Hkv * G, d)
    ref = _sdpa(q, np.repeat(k, G, axis=0), np.repeat(v, G, axis=0))
    sep = orc.separate(qw, k, v, top_t=8, n_hetero=Hkv)
    _, kc, vc = orc.compress(k, v, sep["scores"], sep["mask"], 2, 4, 3)
    np.testing.assert_allclose(orc.decode_attention(q, kc, vc), ref, rtol=1e-12, atol=1e-14)
    sep = orc.separate(qw, k, v, top_t=8, n_hetero=0)
    _, kc, vc = orc.compress(k, v, sep["scores"], sep["mask"], 2, 4, N)
    np.testing.assert_allclose(orc.decode_attention(q, kc, vc), ref, rtol=1e-12, atol=1e-14)


def test_decode_restricted_equals_sdpa_on_kept_rows():
    Hkv, G, N, d = 2, 4, 50, 8
    k, v, q = rand(Hkv, N, d), rand(Hkv, N, d), rand(Hkv * G, d)
    kept = [np.array([0, 1, 7, 30, 49]), np.arange(N)]
    kc = [k[h][kept[h]] for h in range(Hkv)]
    vc = [v[h][kept[h]] for h in range(Hkv)]
    out = orc.decode_attention(q, kc, vc)
    for h in range(Hkv):
        ref = _sdpa(q[h * G:(h + 1) * G], np.repeat(kc[h][None], G, 0), np.repeat(vc[h][None], G, 0))
        np.testing.assert_allclose(out[h * G:(h + 1) * G], ref, rtol=1e-12, atol=1e-14)


def test_decode_degenerate_cases():
    d = 8
    k1, v1 = rand(1, d), rand(1, d)
    q = rand(2, d)
    out = orc.decode_attention(q, [k1], [v1])            # one cached token -> its value
    np.testing.assert_allclose(out, np.repeat(v1, 2, 0), rtol=1e-15)
    k, v = rand(2, 13, d), rand(2, 13, d)
    qd = np.repeat(rand(2, d), 3, axis=0)                # duplicated heads inside a group
    o = orc.decode_attention(qd, list(k), list(v))
    np.testing.assert_array_equal(o[0], o[1])
    np.testing.assert_array_equal(o[3], o[5])


def test_split_and_merge_equals_unsplit():
    N, d = 57, 8
    k, v, q = rand(N, d), rand(N, d), rand(d)
    ref = orc.decode_attention(q[None], [k], [v])[0]
    parts = []
    for lo, hi in [(0, 10), (10, 11), (11, 40), (40, 57)]:
        s = (k[lo:hi] @ q) / math.sqrt(d)
        m = s.max()
        p = np.exp(s - m)
        parts.append((m, p.sum(), p @ v[lo:hi]))
    np.testing.assert_allclose(orc.merge_partials(parts), ref, rtol=1e-13)


def test_compress_ranks_the_middle_by_pooled_scores():
    """One spike against a plateau: alone the spike is the best middle token,
    averaged over three neighbours the centre of the plateau is."""
    N, d = 11, 2
    scores = np.zeros((1, N))
    scores[0, 3] = 10.0
    scores[0, 6:9] = 6.0
    k, v = rand(1, N, d), rand(1, N, d)
    mask = np.zeros(1, dtype=np.uint8)
    kept, kc, vc = orc.compress(k, v, scores, mask, 1, 1, 1, pool_kernel=1)
    assert kept[0].tolist() == [0, 3, 10]
    kept, kc, vc = orc.compress(k, v, scores, mask, 1, 1, 1, pool_kernel=3)
    assert kept[0].tolist() == [0, 7, 10]
    assert kc[0].tobytes() == k[0, [0, 7, 10]].tobytes() and vc[0].tobytes() == v[0, [0, 7, 10]].tobytes()


# ----------------------------------------------------------------- Eq. 16-17
def test_layer_schedule_golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "layer_schedule.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert rows
    for n, beta, m, R, r, f in rows:
        assert orc.hetero_head_count(int(n), float(beta), int(m), int(r), int(R)) == int(f)
    fs = [orc.hetero_head_count(32, 0.25, 4, r, 32) for r in range(32)]
    assert fs[0] == 8 and fs[-1] == 4 and all(a >= b for a, b in zip(fs, fs[1:]))
    assert orc.hetero_head_count(8, 0.3, 1, 0, 1) == 2      # single layer: no interpolation term
    # Eq. 16 is the straight line from n*beta at r = 0 to m at r = R-1: from 16 to 0 over 17 layers it
    # passes through every integer, no rounding involved
    assert [orc.hetero_head_count(32, 0.5, 0, r, 17) for r in range(17)] == list(range(16, -1, -1))
    # fractional values go to the nearest integer, halves upwards: 2 -> 1 over 5 layers is 2, 1.75, 1.5, 1.25, 1
    assert [orc.hetero_head_count(8, 0.25, 1, r, 5) for r in range(5)] == [2, 2, 2, 1, 1]


def test_middle_budget_identity():
    """Eq. 17 rearranged: f*N + (n-f)*(s1+s2+k) = B up to the flooring."""
    for n, f, N, s1, s2, frac in [(32, 8, 8192, 16, 256, 0.4), (8, 2, 32768, 4, 128, 0.4),
                                  (8, 1, 32768, 4, 128, 0.4), (8, 3, 32768, 4, 128, 0.4)]:
        B = int(frac * n * N)
        k = orc.middle_budget(B, N, n, f, s1, s2)
        used = f * N + (n - f) * (s1 + s2 + k)
        assert 0 <= B - used < (n - f)
    assert orc.middle_budget(100, 50, 4, 4, 1, 1) == 0
    assert orc.middle_budget(10, 50, 4, 1, 1, 1) == 0        # budget too small -> clipped


# ----------------------------------------------------------------- Sec. 6.2 ablation modes
def test_round_to_storage_matches_library_conversion():
    """Values that are exactly float32: direct fp64 -> bf16 rounding must equal
    torch's float32 -> bfloat16 conversion (ties to even included)."""
    x32 = np.concatenate([rand(4000).astype(np.float32) * np.float32(3.0),
                          np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 0.0, 3.0e-5, 255.5, 256.5],
                                   dtype=np.float32)])
    ref = torch.tensor(x32).to(torch.bfloat16).float().numpy()
    got = orc.round_to_storage(x32.astype(np.float64), "bf16")
    assert got.dtype == np.float32 and got.tobytes() == ref.tobytes()
    x = rand(100)
    assert orc.round_to_storage(x, "f32").tobytes() == x.astype(np.float32).tobytes()
    # a double just above a bf16 tie must round up although float32 rounding first would land on the tie
    y = np.array([1.00390625 + 1e-12])
    assert orc.round_to_storage(y, "bf16")[0] == np.float32(1.0078125)


def test_no_cache_mode_keeps_sinks_and_longer_recent_window():
    assert orc.kept_tokens_no_cache(20, False, 2, 3, 4).tolist() == [0, 1] + list(range(13, 20))
    assert orc.kept_tokens_no_cache(20, True, 2, 3, 4).tolist() == list(range(20))
    assert orc.kept_tokens_no_cache(8, False, 2, 3, 4).tolist() == list(range(8))


def test_compressed_cache_groups_and_means():
    N, d, s1, s2, n = 23, 4, 2, 3, 5
    k = torch.tensor(rand(N, d)).to(torch.bfloat16).float().numpy()
    v = torch.tensor(rand(N, d)).to(torch.bfloat16).float().numpy()
    kc, vc, pos = orc.compressed_cache(k, v, False, s1, s2, n, "bf16")
    assert kc.shape == (s1 + n + s2, d) and pos[:s1].tolist() == [0, 1] and pos[-s2:].tolist() == [20, 21, 22]
    assert kc[:s1].tobytes() == k[:s1].tobytes() and kc[-s2:].tobytes() == k[-s2:].tobytes()
    bounds = pos[s1:s1 + n].tolist() + [N - s2]
    sizes = np.diff(bounds)
    assert bounds[0] == s1 and sizes.sum() == N - s1 - s2 and sizes.max() - sizes.min() <= 1
    for g in range(n):                       # each token is the (rounded) mean of its group
        ref = torch.tensor(k[bounds[g]:bounds[g + 1]].astype(np.float64).mean(axis=0)).to(torch.bfloat16)
        np.testing.assert_allclose(kc[s1 + g], ref.float().numpy(), rtol=2 ** -7)
        assert torch.tensor(kc[s1 + g]).to(torch.bfloat16).float().numpy().tobytes() == kc[s1 + g].tobytes()
        ref_v = torch.tensor(v[bounds[g]:bounds[g + 1]].astype(np.float64).mean(axis=0)).to(torch.bfloat16)
        np.testing.assert_allclose(vc[s1 + g], ref_v.float().numpy(), rtol=2 ** -7)
    assert vc[:s1].tobytes() == v[:s1].tobytes() and vc[-s2:].tobytes() == v[-s2:].tobytes()
    # constant rows compress to themselves; one group per token is the identity
    const = np.tile(k[5], (N, 1))
    cc, _, _ = orc.compressed_cache(const, const, False, s1, s2, 4, "bf16")
    assert (cc == k[5]).all()
    ident, _, p2 = orc.compressed_cache(k, v, False, s1, s2, 99, "bf16")
    assert ident.tobytes() == k.tobytes() and p2.tolist() == list(range(N))
    full, _, _ = orc.compressed_cache(k, v, True, s1, s2, 3, "bf16")
    assert full.tobytes() == k.tobytes()
    # fp32 storage: total mass of the middle is preserved by the means
    k32 = rand(N, d).astype(np.float32)
    c32, _, p3 = orc.compressed_cache(k32, k32, False, s1, s2, n, "f32")
    b3 = p3[s1:s1 + n].tolist() + [N - s2]
    np.testing.assert_allclose((c32[s1:s1 + n].astype(np.float64) * np.diff(b3)[:, None]).sum(axis=0),
                               k32[s1:N - s2].astype(np.float64).sum(axis=0), rtol=1e-6, atol=1e-6)


def test_layer_plan_spends_the_budget_in_every_layer():
    """Eq. 16 and Eq. 17 together: with f(r) full heads and k(r) middle tokens
    for each other head a layer holds f N + (n - f)(s1 + s2 + k) tokens, which
    is the layer budget up to the flooring of Eq. 17 (less than one token per
    compressed head) -- for the two settings of Sec. 5.4 at both budgets of
    Table 1, and the head counts run from n*beta down to m."""
    for n, beta, m in ((32, 0.25, 4), (8, 0.3, 1)):
        for frac in (0.4, 0.6):
            N, s1, s2, R = 30000, 16, 256, 32
            plan = orc.layer_plan(n, beta, m, R, frac, N, s1, s2)
            assert len(plan) == R
            assert plan[0][0] == math.floor(n * beta + 0.5) and plan[-1][0] == m
            assert all(a[0] >= b[0] for a, b in zip(plan, plan[1:]))          # fewer marked heads with depth
            for f, k in plan:
                held = f * N + (n - f) * (s1 + s2 + k)
                assert k > 0 and frac * n * N - (n - f) - 1 < held <= frac * n * N
    # a budget that the marked heads alone exhaust leaves no middle tokens
    assert all(k == 0 for _, k in orc.layer_plan(8, 0.5, 4, 4, 0.4, 1000, 4, 8))
