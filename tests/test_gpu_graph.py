"""The three hot calls enqueue kernels only, so a caller can record them into a
HIP graph.  One graph holding separate -> compress -> several decode steps is
replayed on changing inputs, with eager work and synchronisations between the
replays, and every replay must give bit for bit what the eager calls give on
the same inputs (the kernels are deterministic); one replay is also checked
against the oracle."""
import numpy as np
import pytest
import torch

from taskkv_synth import make_layer, small_workload, to_numpy
from tests._harness import MIN_MARGIN, OracleCache, check_output, oracle_layer

pytestmark = pytest.mark.gpu

STEPS = 3


def _eager(ses, ctx, cfg, ld):
    bufs = ses.LayerBuffers(cfg, STEPS)
    bufs.separate(ctx, ld.q_win, ld.k, ld.v)
    bufs.compress(ctx, ld.k, ld.v)
    outs = [bufs.decode(ctx, *ld.decode_inputs(s)).clone() for s in range(STEPS)]
    torch.cuda.synchronize()
    return bufs, outs


@pytest.mark.parametrize("dtype,ctx_len", [("bf16", 3000), ("f32", 700)])
def test_graph_replays_match_eager_calls(dtype, ctx_len):
    from paper_2501_15113_amd import session as ses, taskkv_last_async_error
    wl = small_workload(name=f"graph-{dtype}", wid=230, dtype=dtype, ctx_len=ctx_len, n_middle=100,
                        decode_steps=STEPS)
    draws = [make_layer(wl, layer, "cuda:0") for layer in (0, 1)]
    cfg = ses.cfg_from_workload(wl)
    ref = oracle_layer(draws[1], 0, cfg)
    assert ref["margin"] >= MIN_MARGIN

    # static buffers the graph reads; each replay's inputs are copied into them
    first = draws[0]
    q_win, k, v = (torch.empty_like(x) for x in (first.q_win, first.k, first.v))
    steps_in = [tuple(torch.empty_like(x) for x in first.decode_inputs(0)) for _ in range(STEPS)]
    bufs = ses.LayerBuffers(cfg, STEPS)
    outs = [torch.empty_like(bufs.out) for _ in range(STEPS)]

    def load(ld):
        q_win.copy_(ld.q_win), k.copy_(ld.k), v.copy_(ld.v)
        for s in range(STEPS):
            for dst, src in zip(steps_in[s], ld.decode_inputs(s)):
                dst.copy_(src)

    def record():
        bufs.separate(ctx, q_win, k, v)
        bufs.compress(ctx, k, v)
        for s in range(STEPS):
            outs[s].copy_(bufs.decode(ctx, *steps_in[s]))

    with ses.Context([cfg], STEPS) as ctx:
        load(first)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            record()                               # warm-up outside the capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            record()
        for rep, which in enumerate((0, 1, 0, 1)):
            ld = draws[which]
            want, want_outs = _eager(ses, ctx, cfg, ld)      # eager work between the replays
            load(ld)
            for o in outs:
                o.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            what = f"replay {rep}"
            assert torch.equal(bufs.mask, want.mask), what
            assert torch.equal(bufs.kept_idx, want.kept_idx), what
            assert torch.equal(bufs.lens, want.lens), what
            assert torch.equal(bufs.offsets, want.offsets), what
            for s in range(STEPS):
                assert torch.equal(outs[s], want_outs[s]), f"{what}, step {s}"
            if which == 1:
                assert bufs.mask[0].cpu().numpy().tolist() == ref["mask"].tolist()
                cache = OracleCache(ref)
                for s in range(STEPS):
                    qs, kn, vn = ld.decode_inputs(s)
                    cache.append(to_numpy(kn[0]), to_numpy(vn[0]))
                    check_output(outs[s][0].cpu().numpy(), cache.attend(to_numpy(qs[0])), wl.dtype,
                                 f"{what}, step {s}")
        assert taskkv_last_async_error(ctx.handle) == 0
        assert np.isfinite(outs[-1].cpu().numpy()).all()


@pytest.mark.parametrize("pool", [1, 7])
@pytest.mark.parametrize("whole", [True, False])
def test_graph_of_a_long_screened_layer(whole, pool):
    """On a long screened layer the compressor takes its middle threshold from
    column lists that the separator leaves in the workspace, and whether they
    are still there is bookkeeping on the host.  A graph is replayed without
    that bookkeeping: recorded together, separator and compressor may share the
    lists; a compressor recorded alone must not count on them, whatever ran
    before the recording -- here the separator of another layer leaves its own
    lists in the workspace before every replay."""
    from paper_2501_15113_amd import session as ses
    wl = small_workload(name="graph-long", wid=231, batch=1, ctx_len=34000, n_middle=1200, top_t=256,
                        decode_steps=STEPS, pool_kernel=pool)
    ld, other_ld = make_layer(wl, 0, "cuda:0"), make_layer(wl, 1, "cuda:0")
    cfg = ses.cfg_from_workload(wl)
    with ses.Context([cfg], STEPS, screening=2) as ctx:
        want, _ = _eager(ses, ctx, cfg, ld)
        bufs, other = ses.LayerBuffers(cfg, STEPS), ses.LayerBuffers(cfg, STEPS)

        def record():
            if whole:
                bufs.separate(ctx, ld.q_win, ld.k, ld.v)
            bufs.compress(ctx, ld.k, ld.v)

        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            bufs.separate(ctx, ld.q_win, ld.k, ld.v)
            bufs.compress(ctx, ld.k, ld.v)             # warm-up outside the capture
            bufs.separate(ctx, ld.q_win, ld.k, ld.v)   # the lists are in the workspace when the recording starts
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            record()
        for rep in range(3):
            other.separate(ctx, other_ld.q_win, other_ld.k, other_ld.v)   # another layer's lists, valid ones
            bufs.kept_idx.fill_(-7)
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(bufs.kept_idx, want.kept_idx), f"replay {rep}"
            assert torch.equal(bufs.mask, want.mask), f"replay {rep}"
