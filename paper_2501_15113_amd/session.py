"""Device-buffer plumbing around the C ABI: one layer's buffers allocated with
torch and handed to the library.  No arithmetic happens here."""
from __future__ import annotations

import torch

from . import binding as tk


def cfg_from_workload(wl, n_hetero=None, n_middle=None, **override) -> tk.LayerCfg:
    """LayerCfg of a taskkv_synth.Workload (per-layer counts may be overridden)."""
    kw = dict(batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim,
              ctx_len=wl.ctx_len, obs_window=wl.obs_window, top_t=wl.top_t, n_sink=wl.n_sink,
              n_recent=wl.n_recent, n_middle=wl.n_middle if n_middle is None else n_middle,
              n_hetero=wl.n_hetero if n_hetero is None else n_hetero,
              add_centre_head=wl.add_centre_head, pool_kernel=wl.pool_kernel,
              dtype=tk.F32 if wl.dtype == "f32" else tk.BF16, softmax_scale=0.0)
    kw.update(override)
    return tk.LayerCfg(**kw)


class Context:
    """Owns a taskkv_ctx sized for the given cfgs."""

    def __init__(self, cfgs, reserve: int, device: int = 0, screening: int = 1):
        self.bytes = max(tk.taskkv_workspace_bytes(c, reserve) for c in cfgs)
        self.handle = tk.taskkv_create(device, self.bytes)
        self.screening = screening
        tk.taskkv_set_screening(self.handle, screening)

    def close(self):
        if self.handle is not None:
            tk.taskkv_destroy(self.handle)
            self.handle = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()


class LayerBuffers:
    """All device buffers one layer needs for separate -> compress -> decode."""

    def __init__(self, cfg: tk.LayerCfg, reserve: int, device="cuda:0", cache=None, offsets=None):
        """cache = (k_cache, v_cache, lens) views, offsets = a [B*Hkv+1] int64 view, to use
        instead of fresh allocations."""
        self.cfg, self.reserve = cfg, reserve
        B, Hkv, Hq, d, N = cfg.batch, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, cfg.ctx_len
        dev = torch.device(device)
        self.elem = torch.float32 if cfg.dtype == tk.F32 else torch.bfloat16
        self.scores = torch.empty(B, Hkv, N, dtype=torch.float64, device=dev)
        self.sem_vec = torch.empty(B, Hkv, d, dtype=torch.float64, device=dev)
        self.dist = torch.empty(B, Hkv, dtype=torch.float64, device=dev)
        self.mask = torch.empty(B, Hkv, dtype=torch.uint8, device=dev)
        self.capacity = tk.taskkv_cache_tokens(cfg, reserve)
        if cache is None:
            self.k_cache = torch.empty(self.capacity * d, dtype=self.elem, device=dev)
            self.v_cache = torch.empty(self.capacity * d, dtype=self.elem, device=dev)
            self.lens = torch.empty(B * Hkv, dtype=torch.int32, device=dev)
        else:
            self.k_cache, self.v_cache, self.lens = cache
        self.offsets = torch.empty(B * Hkv + 1, dtype=torch.int64, device=dev) if offsets is None else offsets
        self.row = cfg.n_sink + cfg.n_middle + cfg.n_recent
        self.kept_idx = torch.empty(B * Hkv, max(self.row, 1), dtype=torch.int32, device=dev)
        self.out = torch.empty(B, Hq, d, dtype=torch.float32, device=dev)

    def separate(self, ctx: Context, q_win, k, v):
        tk.taskkv_separate(ctx.handle, self.cfg, q_win, k, v, self.scores, self.sem_vec, self.dist, self.mask)

    def compress(self, ctx: Context, k, v):
        tk.taskkv_compress(ctx.handle, self.cfg, k, v, self.scores, self.mask, self.k_cache, self.v_cache,
                           self.capacity, self.reserve, self.offsets, self.lens,
                           self.kept_idx if self.row > 0 else None)

    def decode(self, ctx: Context, q, k_new=None, v_new=None):
        tk.taskkv_decode_attn(ctx.handle, self.cfg, q, k_new, v_new, self.k_cache, self.v_cache,
                              self.capacity, self.offsets, self.lens, self.out)
        return self.out

    def export(self, ctx: Context):
        """Plain-row copies of the cache: (k_rows, v_rows), each [capacity, d]."""
        d = self.cfg.head_dim
        k_rows = torch.empty(self.capacity, d, dtype=self.elem, device=self.k_cache.device)
        v_rows = torch.empty_like(k_rows)
        tk.taskkv_cache_export(ctx.handle, self.cfg, self.k_cache, self.v_cache, self.capacity,
                               self.offsets, k_rows, v_rows)
        return k_rows, v_rows


class LayerStack:
    """The ragged caches of several layers in one allocation, so that a single
    taskkv_decode_attn_layers call serves one decode step of all of them.  Each
    layer is compressed into its own slice through its LayerBuffers;
    rebase() then has the library write the stack's offsets array
    (taskkv_stack_rebase).  Only buffer views are made here."""

    def __init__(self, cfgs, reserve: int, device="cuda:0"):
        c0 = cfgs[0]
        for c in cfgs:
            assert (c.batch, c.n_q_heads, c.n_kv_heads, c.head_dim, c.dtype, c.softmax_scale) == \
                   (c0.batch, c0.n_q_heads, c0.n_kv_heads, c0.head_dim, c0.dtype, c0.softmax_scale)
        dev = torch.device(device)
        d, U, R = c0.head_dim, c0.batch * c0.n_kv_heads, len(cfgs)
        self.elem = torch.float32 if c0.dtype == tk.F32 else torch.bfloat16
        self.caps = [tk.taskkv_cache_tokens(c, reserve) for c in cfgs]
        bases = [sum(self.caps[:r]) for r in range(R)]
        self.capacity = sum(self.caps)
        self.k_cache = torch.empty(self.capacity * d, dtype=self.elem, device=dev)
        self.v_cache = torch.empty(self.capacity * d, dtype=self.elem, device=dev)
        self.lens = torch.empty(R * U, dtype=torch.int32, device=dev)
        self.layer_offsets = torch.empty(R, U + 1, dtype=torch.int64, device=dev)
        self.offsets = torch.empty(R * U + 1, dtype=torch.int64, device=dev)
        self.layers = [
            LayerBuffers(c, reserve, device,
                         cache=(self.k_cache[b * d:(b + cap) * d], self.v_cache[b * d:(b + cap) * d],
                                self.lens[r * U:(r + 1) * U]), offsets=self.layer_offsets[r])
            for r, (c, b, cap) in enumerate(zip(cfgs, bases, self.caps))]
        self.cfg0, self.n_layers, self._U = c0, R, U
        # for sizing the ctx workspace: what the decode call resolves its cfg to
        self.cfg = tk.LayerCfg(batch=c0.batch * R, n_q_heads=c0.n_q_heads, n_kv_heads=c0.n_kv_heads,
                               head_dim=d, ctx_len=c0.ctx_len, obs_window=c0.obs_window, top_t=c0.top_t,
                               n_sink=c0.n_sink, n_recent=c0.n_recent,
                               n_middle=max(c.n_middle for c in cfgs), n_hetero=max(c.n_hetero for c in cfgs),
                               add_centre_head=c0.add_centre_head, pool_kernel=c0.pool_kernel,
                               pack_mode=c0.pack_mode, dtype=c0.dtype, softmax_scale=c0.softmax_scale)
        self.out = torch.empty(self.cfg.batch, c0.n_q_heads, d, dtype=torch.float32, device=dev)

    def rebase(self, ctx: Context):
        """Call after every layer has been compressed."""
        tk.taskkv_stack_rebase(ctx.handle, self.n_layers, self._U, self.layer_offsets, self.caps, self.offsets)

    def decode(self, ctx: Context, q, k_new=None, v_new=None):
        """q [layers*B,Hq,d], k_new / v_new [layers*B,Hkv,d], layer-major."""
        tk.taskkv_decode_attn_layers(ctx.handle, self.cfg0, self.n_layers, q, k_new, v_new, self.k_cache,
                                     self.v_cache, self.capacity, self.offsets, self.lens, self.out)
        return self.out
