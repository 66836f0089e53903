"""GPU parity at the full sizes of the named workloads, in the launch
configuration the benchmark times.  The oracle checks sampled batch elements
(all heads of each) and sampled decode steps."""
import pytest

from taskkv_synth import WORKLOADS
from tests.test_gpu_parity import run_layer

pytestmark = pytest.mark.gpu


def test_cfg4_mistral_shaped_zipf():
    run_layer(WORKLOADS["cfg4"], check_steps={0, 1, 64, 127})


def test_cfg5_load_imbalance_stress():
    # automatic screening, as the benchmark runs it (it is on at this size)
    run_layer(WORKLOADS["cfg5"], check_batches=(3, 6), check_steps={0, 63}, screening=1)


@pytest.mark.parametrize("layer", [0, 5])
def test_cfg3_stack_layers(layer):
    run_layer(WORKLOADS["cfg3"], layer=layer, check_batches=(1,), steps=4, check_steps={0, 3}, reserve=256)


def test_cfg3_whole_stack_in_one_call():
    """All 32 layers' caches in one allocation and a decode step of the whole
    stack as one call (1024 units, 6.9 GB), the configuration `bench.py
    --layer-batched` times.  Sampled layers are checked against the oracle, and
    every layer's lengths against the budget."""
    import numpy as np
    import torch

    from paper_2501_15113_amd import session as ses, taskkv_last_async_error
    from taskkv_synth import layer_params, make_layer, to_numpy
    from tests._harness import MIN_MARGIN, OracleCache, check_output, oracle_layer

    wl = WORKLOADS["cfg3"]
    sampled, b_sels, steps = (0, 5, 17), (1, 3), 2
    cfgs = [ses.cfg_from_workload(wl, *layer_params(wl, r)) for r in range(wl.n_layers)]
    stack = ses.LayerStack(cfgs, steps)
    B = wl.batch
    with ses.Context(cfgs + [stack.cfg], steps) as ctx:
        refs, inputs = {}, []
        for r in range(wl.n_layers):
            ld = make_layer(wl, r, "cuda:0")
            stack.layers[r].separate(ctx, ld.q_win, ld.k, ld.v)
            stack.layers[r].compress(ctx, ld.k, ld.v)
            if r in sampled:
                for b_sel in b_sels:
                    refs[r, b_sel] = oracle_layer(ld, b_sel, cfgs[r])
                    assert refs[r, b_sel]["margin"] >= MIN_MARGIN
            inputs.append([ld.decode_inputs(s) for s in range(steps)])
            del ld
        stack.rebase(ctx)
        caches = {key: OracleCache(ref) for key, ref in refs.items()}
        for s in range(steps):
            q, kn, vn = (torch.cat([inputs[r][s][j] for r in range(wl.n_layers)]) for j in range(3))
            out = stack.decode(ctx, q, kn, vn)
            for (r, b_sel), cache in caches.items():
                cache.append(to_numpy(kn[r * B + b_sel]), to_numpy(vn[r * B + b_sel]))
                ref = cache.attend(to_numpy(q[r * B + b_sel]))
                check_output(out[r * B + b_sel].cpu().numpy(), ref, wl.dtype, f"stack layer {r} step {s}")
        assert taskkv_last_async_error(ctx.handle) == 0
        lens = stack.lens.cpu().numpy().reshape(wl.n_layers, B, wl.n_kv_heads)
        for (r, b_sel), ref in refs.items():
            assert lens[r, b_sel].tolist() == [len(x) + steps for x in ref["kept"]]
        # every layer holds the budget of Eq. 17: about 40 % of its full cache
        per_layer = lens.reshape(wl.n_layers, -1).sum(axis=1) - steps * B * wl.n_kv_heads
        assert np.all(np.abs(per_layer / (B * wl.n_kv_heads * wl.ctx_len) - 0.4) < 0.002)


def _stack_layer_with(n_hetero):
    """First layer of the 32-layer workload that marks this many heads."""
    from taskkv_synth import layer_params
    wl = WORKLOADS["cfg3"]
    return next(r for r in range(wl.n_layers) if layer_params(wl, r)[0] == n_hetero)


@pytest.mark.parametrize("name,n_het", [("cfg5", None), ("cfg4", None), ("cfg3", 1), ("cfg3", 2), ("cfg3", 3)])
def test_outputs_are_consistent_for_every_unit(name, n_het):
    """Properties that hold at any size, checked for every unit of the full
    workload with library routines (the oracle above checks sampled batch
    elements value by value): the mask marks exactly the farthest heads of the
    distances recomputed from the semantic vectors, which are the weighted sums
    of the t best-scored value rows; every compressed unit keeps the sinks, the
    recent window and a middle set no unkept token of which scores higher
    (equal scores: lower positions kept); packed rows are bit copies of the
    source rows; and the decode output is dense softmax attention over the
    unit's own cache."""
    import torch

    from paper_2501_15113_amd import session as ses, taskkv_last_async_error
    from taskkv_synth import make_layer

    wl = WORKLOADS[name]
    ld = make_layer(wl, 0 if n_het is None else _stack_layer_with(n_het), "cuda:0")
    assert n_het is None or ld.n_hetero == n_het
    cfg = ses.cfg_from_workload(wl, ld.n_hetero, ld.n_middle)
    B, H, G, N, d = wl.batch, wl.n_kv_heads, wl.group, wl.ctx_len, wl.head_dim
    s1, s2, k_mid, t = wl.n_sink, wl.n_recent, ld.n_middle, min(wl.top_t, N)
    bufs = ses.LayerBuffers(cfg, 1)
    with ses.Context([cfg], 1, screening=1) as ctx:
        bufs.separate(ctx, ld.q_win, ld.k, ld.v)
        bufs.compress(ctx, ld.k, ld.v)
        k_rows, v_rows = bufs.export(ctx)
        q, kn, vn = ld.decode_inputs(0)
        out = bufs.decode(ctx, q, kn, vn).clone()
        torch.cuda.synchronize()
        assert taskkv_last_async_error(ctx.handle) == 0
    sc, mask = bufs.scores, bufs.mask.bool()
    assert (sc >= 0).all() and torch.allclose(sc.sum(dim=2), torch.ones(B, H, dtype=sc.dtype, device=sc.device),
                                              rtol=1e-4)
    # separator: v' from the t best columns, distances from v', mask from the distances
    top = torch.topk(sc, t, dim=2)
    picked_v = torch.gather(ld.v, 2, top.indices[..., None].expand(B, H, t, d)).double()
    sem = (top.values[..., None] * picked_v).sum(dim=2)
    torch.testing.assert_close(bufs.sem_vec, sem, rtol=1e-9, atol=1e-12)
    dist = (sem - sem.mean(dim=1, keepdim=True)).norm(dim=2)
    torch.testing.assert_close(bufs.dist, dist, rtol=1e-9, atol=1e-12)
    far = torch.topk(bufs.dist, ld.n_hetero, dim=1).indices
    want = torch.zeros_like(mask)
    want.scatter_(1, far, True)
    assert torch.equal(mask, want)
    assert mask.sum(dim=1).tolist() == [ld.n_hetero] * B
    # cache allocation
    lens = bufs.lens.cpu().view(B, H)
    offs = bufs.offsets.cpu()
    kept = bufs.kept_idx.view(B, H, -1)
    sinks = torch.arange(s1, device=kept.device, dtype=kept.dtype)
    recent = torch.arange(N - s2, N, device=kept.device, dtype=kept.dtype)
    for b in range(B):
        for h in range(H):
            u = b * H + h
            rows = slice(int(offs[u]), int(offs[u]) + int(lens[b, h]) - 1)       # before the appended token
            if mask[b, h]:
                assert lens[b, h] == N + 1 and (kept[b, h] == -1).all()
                idx = None
                assert torch.equal(k_rows[rows].view(torch.int16), ld.k[b, h].view(torch.int16))
                assert torch.equal(v_rows[rows].view(torch.int16), ld.v[b, h].view(torch.int16))
            else:
                assert lens[b, h] == s1 + k_mid + s2 + 1
                idx = kept[b, h].long()
                assert (idx[1:] > idx[:-1]).all()
                assert torch.equal(kept[b, h, :s1], sinks) and torch.equal(kept[b, h, s1 + k_mid:], recent)
                mid = sc[b, h, s1:N - s2]
                chosen = torch.zeros(N - s1 - s2, dtype=torch.bool, device=mid.device)
                chosen[idx[s1:s1 + k_mid] - s1] = True
                lo, hi = mid[chosen].min(), mid[~chosen].max()
                assert lo >= hi
                if lo == hi:
                    where = torch.arange(N - s1 - s2, device=mid.device)
                    assert where[chosen & (mid == lo)].max() < where[~chosen & (mid == lo)].min()
                assert torch.equal(k_rows[rows].view(torch.int16), ld.k[b, h][idx].view(torch.int16))
                assert torch.equal(v_rows[rows].view(torch.int16), ld.v[b, h][idx].view(torch.int16))
            # decode over the unit's own rows plus the appended token
            kk = torch.cat([ld.k[b, h] if idx is None else ld.k[b, h][idx], kn[b, h][None]]).double()
            vv = torch.cat([ld.v[b, h] if idx is None else ld.v[b, h][idx], vn[b, h][None]]).double()
            qq = q[b, h * G:(h + 1) * G].double()
            ref = torch.softmax(qq @ kk.T / d ** 0.5, dim=1) @ vv
            err = (out[b, h * G:(h + 1) * G].double() - ref).abs().max().item()
            assert err <= 1e-2, f"unit ({b},{h}): max-abs error {err:.3e}"


def test_context_of_a_million_tokens():
    """Far beyond the named workloads: one batch element, three KV heads of
    2^20 + 77 tokens, a middle budget of 30000 and 2000 top-t tokens on
    Zipf-weighted keys; every index and length fits the library's 32-bit page
    arithmetic with room to spare."""
    from taskkv_synth import small_workload
    wl = small_workload(name="million", wid=801, batch=1, n_kv_heads=3, n_q_heads=6, n_hetero=1,
                        ctx_len=(1 << 20) + 77, obs_window=32, top_t=2000, n_middle=30000, n_recent=5000,
                        decode_steps=2, recipe="zipf")
    run_layer(wl, screening=1)
