"""Shared by the GPU parity tests: run one layer through the HIP library and
compare every output with the CPU oracle on the same seeded inputs."""
from __future__ import annotations

import numpy as np
import torch

from oracle import taskkv_oracle as orc
from taskkv_synth import to_numpy

F32_REL_TOL = 1e-5      # max|o - ref| / max|ref| per (batch, query head) vector
BF16_ABS_TOL = 1e-2     # max|o - ref| for bf16 inputs with fp32 accumulation
SCORE_RTOL = 1e-9       # fp64 on both sides; differences are summation order and exp ulps
SCREEN_RTOL = 5e-3      # columns left at their fp32 screening value (bound: see score_screen.hip)
MIN_MARGIN = 1e-9       # a decision closer than this is not a well-posed test


def oracle_layer(ld, b, cfg):
    """Oracle results for batch element b, plus the relative margin of every
    discrete decision (top-t boundary, middle boundary, head ranking)."""
    q, k, v = to_numpy(ld.q_win[b]), to_numpy(ld.k[b]), to_numpy(ld.v[b])
    scale = cfg.softmax_scale if cfg.softmax_scale > 0 else None
    sep = orc.separate(q, k, v, cfg.top_t, cfg.n_hetero, bool(cfg.add_centre_head), scale)
    kept, kc, vc = orc.compress(k, v, sep["scores"], sep["mask"], cfg.n_sink, cfg.n_recent,
                                cfg.n_middle, cfg.pool_kernel, cfg.pack_mode,
                                "f32" if cfg.dtype == 0 else "bf16")
    margins = []
    C = sep["scores"]
    N = C.shape[1]
    P = orc.pool_scores(C, cfg.pool_kernel)
    for h in range(C.shape[0]):
        srt = np.sort(C[h])[::-1]
        t = min(cfg.top_t, N)
        if t < N and srt[t - 1] != srt[t]:
            margins.append((srt[t - 1] - srt[t]) / srt[t - 1])
        lo, hi = cfg.n_sink, N - cfg.n_recent
        if cfg.pack_mode == 0 and not sep["mask"][h] and hi - lo > cfg.n_middle > 0:
            ms = np.sort(P[h, lo:hi])[::-1]
            if ms[cfg.n_middle - 1] != ms[cfg.n_middle]:
                margins.append((ms[cfg.n_middle - 1] - ms[cfg.n_middle]) / ms[cfg.n_middle - 1])
    # head ranking: only the two comparisons that can change the mask, the cut
    # after the n_hetero farthest heads and the choice of the closest remaining
    # head.  Equal distances are a tie for both sides (index rule) only when the
    # two heads' vectors are identical bit for bit, so that both sides compute
    # the same value twice; an equality that holds in exact arithmetic only (two
    # KV heads are always equally far from their mean) is decided by rounding
    # and counts as margin 0.
    d, vec = sep["dist"], sep["sem_vec"]
    H = len(d)
    order = sorted(range(H), key=lambda h: (-d[h], h))
    nh = min(cfg.n_hetero, H)
    pairs = []
    if cfg.add_centre_head and H - nh <= 1:
        pass                                   # every head ends up marked, whatever the order
    else:
        if 0 < nh < H:
            pairs.append((order[nh - 1], order[nh]))
        if cfg.add_centre_head:
            pairs.append((order[-2], order[-1]))
    for a, c in pairs:
        if not np.array_equal(vec[a], vec[c]):
            margins.append(abs(d[a] - d[c]) / max(d.max(), 1e-300))
    sep.update(kept=kept, k_cache=kc, v_cache=vc, margin=min(margins) if margins else 1.0)
    return sep


def check_compression(ld, cfg, bufs, k_rows, v_rows, b, ref):
    """Scores, vectors, distances, mask, kept indices, lengths, packed rows."""
    Hkv, N = cfg.n_kv_heads, cfg.ctx_len
    scores = bufs.scores[b].cpu().numpy()
    # (with pooling, only contexts long enough for the band kernels that list a pooled column's neighbours)
    screened = (cfg.dtype == 1 and (cfg.pool_kernel == 1 or cfg.ctx_len >= 12288) and
                (cfg.n_q_heads // cfg.n_kv_heads) * cfg.obs_window <= 512 and getattr(bufs, "screening", True))
    if screened:
        # fp32-accurate everywhere, fp64-exact on every column that can decide something
        np.testing.assert_allclose(scores, ref["scores"], rtol=SCREEN_RTOL, atol=1e-30)
        for h in range(Hkv):
            idx = ref["picks"][h]
            np.testing.assert_allclose(scores[h, idx], ref["scores"][h, idx], rtol=SCORE_RTOL, atol=1e-300)
    else:
        np.testing.assert_allclose(scores, ref["scores"], rtol=SCORE_RTOL, atol=1e-300)
    np.testing.assert_allclose(bufs.sem_vec[b].cpu().numpy(), ref["sem_vec"], rtol=1e-8, atol=1e-12)
    np.testing.assert_allclose(bufs.dist[b].cpu().numpy(), ref["dist"], rtol=1e-8, atol=1e-12)
    assert bufs.mask[b].cpu().numpy().tolist() == ref["mask"].tolist(), "hetero mask differs"
    lens = bufs.lens.cpu().numpy().reshape(cfg.batch, Hkv)[b]
    offs = bufs.offsets.cpu().numpy()
    kept_gpu = bufs.kept_idx.cpu().numpy().reshape(cfg.batch, Hkv, -1)[b]
    k_src, v_src = ld.k[b], ld.v[b]
    for h in range(Hkv):
        kept = ref["kept"][h]
        assert lens[h] == len(kept), f"len differs for head {h}"
        keeps_all = bool(ref["mask"][h]) or len(kept) == N and (
            cfg.n_sink + cfg.n_recent >= N or (cfg.pack_mode == 1 and cfg.n_sink + cfg.n_recent + cfg.n_middle >= N))
        if bufs.row == 0:
            pass                                   # no kept_idx rows exist
        elif keeps_all:
            assert (kept_gpu[h] == -1).all()
        else:
            assert kept_gpu[h, :len(kept)].tolist() == kept.tolist(), f"kept indices differ, head {h}"
            assert (kept_gpu[h, len(kept):] == -1).all()
        u = b * Hkv + h
        assert offs[u] % 512 == 0 and offs[u + 1] - offs[u] >= lens[h]
        rows = slice(int(offs[u]), int(offs[u]) + len(kept))
        pad = slice(int(offs[u]) + len(kept), int(offs[u + 1]))
        assert not k_rows[pad].view(torch.uint8).any() and not v_rows[pad].view(torch.uint8).any()
        if len(kept) == 0:
            continue
        want_k = torch.as_tensor(np.ascontiguousarray(ref["k_cache"][h]), device=k_src.device).to(k_src.dtype)
        want_v = torch.as_tensor(np.ascontiguousarray(ref["v_cache"][h]), device=k_src.device).to(k_src.dtype)
        if cfg.pack_mode == 2 and cfg.dtype == 0 and not ref["mask"][h]:
            # fp32 group means: the fp64 sums may differ in the last bit with summation order
            torch.testing.assert_close(k_rows[rows], want_k, rtol=3e-7, atol=1e-12)
            torch.testing.assert_close(v_rows[rows], want_v, rtol=3e-7, atol=1e-12)
        else:
            assert torch.equal(k_rows[rows].view(torch.uint8), want_k.view(torch.uint8)), \
                f"packed K rows differ, head {h}"
            assert torch.equal(v_rows[rows].view(torch.uint8), want_v.view(torch.uint8)), \
                f"packed V rows differ, head {h}"
        if cfg.pack_mode != 2:      # selective / no-cache rows are bit copies of source rows
            sel = torch.as_tensor(kept, device=k_src.device)
            assert torch.equal(k_rows[rows].view(torch.uint8), k_src[h][sel].contiguous().view(torch.uint8))


def check_output(out_b, ref_out, dtype, what=""):
    """Attention output of one batch element against the oracle."""
    out_b = out_b.astype(np.float64)
    err = np.abs(out_b - ref_out).max(axis=1)
    if dtype == "f32":
        rel = err / np.maximum(np.abs(ref_out).max(axis=1), 1e-30)
        assert rel.max() <= F32_REL_TOL, f"{what}: fp32 relative error {rel.max():.3e}"
        return rel.max()
    assert err.max() <= BF16_ABS_TOL, f"{what}: bf16 max-abs error {err.max():.3e}"
    return err.max()


class OracleCache:
    """The oracle's per-head cache of one batch element, growing with decode."""

    def __init__(self, ref):
        self.k = [np.asarray(x, dtype=np.float64) for x in ref["k_cache"]]
        self.v = [np.asarray(x, dtype=np.float64) for x in ref["v_cache"]]
        self.new_k = [[] for _ in self.k]
        self.new_v = [[] for _ in self.v]

    def append(self, k_new_b, v_new_b):
        for h in range(len(self.k)):
            self.new_k[h].append(np.asarray(k_new_b[h], dtype=np.float64)[None])
            self.new_v[h].append(np.asarray(v_new_b[h], dtype=np.float64)[None])

    def attend(self, q_b, scale=None):
        ks = [np.concatenate([a] + n) if n else a for a, n in zip(self.k, self.new_k)]
        vs = [np.concatenate([a] + n) if n else a for a, n in zip(self.v, self.new_v)]
        return orc.decode_attention(q_b, ks, vs, scale)
