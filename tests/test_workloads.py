"""Generator self-checks (CPU): the synthetic recipes produce the structure the
workloads name -- intended heterogeneous heads are the ones the oracle finds,
budget literals match the oracle's Eq. 17 helper."""
import numpy as np
import pytest

from oracle import taskkv_oracle as orc
from taskkv_synth import WORKLOADS, layer_params, make_layer, small_workload, to_numpy
from taskkv_synth.workloads import STACK_MIDDLE


def _oracle_mask(ld, b):
    wl = ld.wl
    sep = orc.separate(to_numpy(ld.q_win[b]), to_numpy(ld.k[b]), to_numpy(ld.v[b]),
                       wl.top_t, ld.n_hetero, bool(wl.add_centre_head))
    return sep


@pytest.mark.parametrize("name", ["cfg1", "cfg2"])
def test_intended_hetero_heads_are_found(name):
    wl = WORKLOADS[name]
    ld = make_layer(wl, 0, "cpu")
    assert ld.k.shape == (wl.batch, wl.n_kv_heads, wl.ctx_len, wl.head_dim)
    assert ld.k.dtype == wl.torch_dtype
    for b in range(wl.batch):
        sep = _oracle_mask(ld, b)
        assert np.flatnonzero(sep["mask"]).tolist() == ld.hetero_heads[b]
        d = np.sort(sep["dist"])[::-1]
        assert d[ld.n_hetero - 1] > 2.0 * d[ld.n_hetero]      # a clear gap, not luck


def test_small_zipf_profile_shapes_scores():
    wl = small_workload(recipe="zipf", ctx_len=600, batch=1, n_hetero=1)
    ld = make_layer(wl, 0, "cpu")
    C = orc.window_scores(to_numpy(ld.q_win[0]), to_numpy(ld.k[0]))
    body = np.sort(C[0][: wl.ctx_len - wl.obs_window])[::-1]
    assert body[0] > 20 * np.median(body)                   # heavy head, long tail


def test_generators_are_seeded():
    wl = small_workload()
    a, b = make_layer(wl, 0, "cpu"), make_layer(wl, 0, "cpu")
    assert a.k.equal(b.k) and a.v.equal(b.v) and a.q_win.equal(b.q_win)
    c = make_layer(wl, 0, "cpu", seed_bump=1)
    assert not a.k.equal(c.k)
    q0, k0, v0 = a.decode_inputs(0)
    q1, _, _ = a.decode_inputs(1)
    assert q0.equal(b.decode_inputs(0)[0]) and not q0.equal(q1)
    assert q0.shape == (wl.batch, wl.n_q_heads, wl.head_dim)


def test_stack_budget_literals_match_eq_17():
    wl = WORKLOADS["cfg3"]
    layer_budget = int(0.4 * wl.n_kv_heads * wl.ctx_len)
    seen = set()
    for layer in range(wl.n_layers):
        f, k = layer_params(wl, layer)
        seen.add(f)
        assert k == STACK_MIDDLE[f] == orc.middle_budget(layer_budget, wl.ctx_len, wl.n_kv_heads, f,
                                                         wl.n_sink, wl.n_recent)
        tokens = f * wl.ctx_len + (wl.n_kv_heads - f) * (wl.n_sink + wl.n_recent + k)
        assert 0.399 < tokens / (wl.n_kv_heads * wl.ctx_len) <= 0.4
    assert seen == {1, 2, 3}
