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
    run_layer(WORKLOADS["cfg5"], check_batches=(3,), check_steps={0, 63}, screening=1)


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
    sampled, b_sel, steps = (0, 5), 1, 2
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
                refs[r] = oracle_layer(ld, b_sel, cfgs[r])
                assert refs[r]["margin"] >= MIN_MARGIN
            inputs.append([ld.decode_inputs(s) for s in range(steps)])
            del ld
        stack.rebase()
        caches = {r: OracleCache(refs[r]) for r in sampled}
        for s in range(steps):
            q, kn, vn = (torch.cat([inputs[r][s][j] for r in range(wl.n_layers)]) for j in range(3))
            out = stack.decode(ctx, q, kn, vn)
            for r in sampled:
                caches[r].append(to_numpy(kn[r * B + b_sel]), to_numpy(vn[r * B + b_sel]))
                ref = caches[r].attend(to_numpy(q[r * B + b_sel]))
                check_output(out[r * B + b_sel].cpu().numpy(), ref, wl.dtype, f"stack layer {r} step {s}")
        assert taskkv_last_async_error(ctx.handle) == 0
        lens = stack.lens.cpu().numpy().reshape(wl.n_layers, B, wl.n_kv_heads)
        for r in sampled:
            assert lens[r, b_sel].tolist() == [len(x) + steps for x in refs[r]["kept"]]
        # every layer holds the budget of Eq. 17: about 40 % of its full cache
        per_layer = lens.reshape(wl.n_layers, -1).sum(axis=1) - steps * B * wl.n_kv_heads
        assert np.all(np.abs(per_layer / (B * wl.n_kv_heads * wl.ctx_len) - 0.4) < 0.002)
