"""The decode entry point that allocates nothing (taskkv_decode_attn_static),
called through the C ABI and checked against taskkv_decode_attn on the same
inputs: two calls in a row, the second on a smaller layer, so that whatever the
first call left in the library's fixed scratch array is in the way of the
second."""
import pytest
import torch

from taskkv_synth import make_layer, small_workload

pytestmark = pytest.mark.gpu


def _layer(wl, steps):
    """One compressed layer: (cfg, buffers, decode inputs of every step)."""
    from paper_2501_15113_amd import session as ses
    ld = make_layer(wl, 0, "cuda:0")
    cfg = ses.cfg_from_workload(wl, ld.n_hetero, ld.n_middle)
    bufs = ses.LayerBuffers(cfg, steps)
    with ses.Context([cfg], steps) as ctx:
        bufs.separate(ctx, ld.q_win, ld.k, ld.v)
        bufs.compress(ctx, ld.k, ld.v)
        torch.cuda.synchronize()
    return cfg, bufs, [ld.decode_inputs(s) for s in range(steps)]


def _both_ways(cfg, bufs, inputs):
    """The same decode steps (append included) through the ctx entry point and
    through the static one, each on its own copy of the cache."""
    import paper_2501_15113_amd as tk
    from paper_2501_15113_amd import session as ses
    steps = len(inputs)
    kc, vc, lens = bufs.k_cache.clone(), bufs.v_cache.clone(), bufs.lens.clone()
    out_ctx, out_static = [], []
    with ses.Context([cfg], steps) as ctx:
        for q, kn, vn in inputs:
            out_ctx.append(bufs.decode(ctx, q, kn, vn).clone())
        assert tk.taskkv_last_async_error(ctx.handle) == 0
    flag = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    out = torch.empty_like(bufs.out)
    for q, kn, vn in inputs:
        tk.taskkv_decode_attn_static(cfg, q, kn, vn, kc, vc, bufs.capacity, bufs.offsets, lens, out, flag)
        out_static.append(out.clone())
    torch.cuda.synchronize()
    assert flag.item() == 0
    for a, b in zip(out_ctx, out_static):
        # the same kernels on the same split points: the tolerance of the parity tests holds with room to spare
        assert torch.isfinite(b).all()
        assert (a - b).abs().max().item() <= (1e-2 if cfg.dtype == tk.BF16 else 1e-5 * a.abs().max().item())
        assert torch.equal(a, b)
    assert torch.equal(lens, bufs.lens)
    assert torch.equal(kc.view(torch.int16), bufs.k_cache.view(torch.int16))
    assert torch.equal(vc.view(torch.int16), bufs.v_cache.view(torch.int16))


def test_static_entry_point_matches_the_ctx_one_twice_in_a_row():
    big = small_workload(name="static-a", wid=270, batch=2, n_q_heads=16, n_kv_heads=4, ctx_len=9000,
                         n_middle=300, n_recent=200, n_hetero=1, decode_steps=3)
    small = small_workload(name="static-b", wid=271, batch=1, n_q_heads=4, n_kv_heads=2, ctx_len=700,
                           n_middle=40, n_recent=20, n_hetero=2, decode_steps=2)
    first = _layer(big, 3)
    second = _layer(small, 2)
    _both_ways(*first)
    _both_ways(*second)


def test_static_entry_point_fp32_and_error_paths():
    import paper_2501_15113_amd as tk
    wl = small_workload(name="static-f32", wid=272, dtype="f32", head_dim=64, n_q_heads=4, n_kv_heads=4,
                        ctx_len=800, recipe="gauss", offset=3.0, decode_steps=2)
    cfg, bufs, inputs = _layer(wl, 2)
    _both_ways(cfg, bufs, inputs)
    # a step that needs more scratch than the fixed array holds is refused before anything runs
    huge = tk.LayerCfg(batch=64, n_q_heads=64 * 64, n_kv_heads=64, head_dim=128, ctx_len=4096, n_sink=4,
                       n_recent=32, n_middle=64, n_hetero=0, dtype=tk.F32)
    need = tk.taskkv_workspace_bytes(huge, 0)
    assert need > (24 << 20)
    q, kn, vn = inputs[0]
    with pytest.raises(tk.TaskKVError, match="workspace too small"):
        tk.taskkv_decode_attn_static(huge, q, None, None, bufs.k_cache, bufs.v_cache, 64 * 64 * 512, bufs.offsets,
                                     bufs.lens, bufs.out)
    # a full unit: the token is dropped and bit 1 lands in the caller's flag
    full = small_workload(name="static-full", wid=273, ctx_len=512, n_hetero=4, batch=1, decode_steps=1)
    cfg, bufs, inputs = _layer(full, 0)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    q, kn, vn = inputs[0] if inputs else make_layer(full, 0, "cuda:0").decode_inputs(0)
    tk.taskkv_decode_attn_static(cfg, q, kn, vn, bufs.k_cache, bufs.v_cache, bufs.capacity, bufs.offsets,
                                 bufs.lens, bufs.out, flag)
    torch.cuda.synchronize()
    assert flag.item() == 1 and bufs.lens.cpu().tolist() == [512] * 4
