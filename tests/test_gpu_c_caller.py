"""The library called from a plain C program (tests/c_caller/taskkv_c_caller.c,
compiled with gcc by the build step): no Python binding, no torch between the
caller and the C ABI.  The test hands it seeded inputs as raw files and checks
what it writes back against the oracle."""
import os
import subprocess

import numpy as np
import pytest
import torch

from taskkv_synth import make_layer, small_workload, to_numpy
from tests._harness import MIN_MARGIN, OracleCache, check_output, oracle_layer

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))
CALLER = os.path.join(HERE, "c_caller", "taskkv_c_caller")


def _raw(t: torch.Tensor) -> bytes:
    t = t.contiguous().cpu()
    return (t.view(torch.int16) if t.dtype == torch.bfloat16 else t).numpy().tobytes()


@pytest.mark.parametrize("dtype,ctx_len", [("bf16", 2500), ("f32", 800)])
def test_c_program_gets_the_oracles_results(dtype, ctx_len, tmp_path):
    assert os.path.exists(CALLER), "tests/c_caller/taskkv_c_caller is not built (run __graft_entry__.build())"
    from paper_2501_15113_amd import session as ses
    wl = small_workload(name=f"c-{dtype}", wid=250, dtype=dtype, ctx_len=ctx_len, n_middle=90, n_hetero=1)
    ld = make_layer(wl, 0, "cuda:0")
    cfg = ses.cfg_from_workload(wl)
    refs = [oracle_layer(ld, b, cfg) for b in range(wl.batch)]
    assert min(r["margin"] for r in refs) >= MIN_MARGIN
    q, kn, vn = ld.decode_inputs(0)
    for name, t in (("q_win", ld.q_win), ("k", ld.k), ("v", ld.v), ("q", q), ("k_new", kn), ("v_new", vn)):
        (tmp_path / f"{name}.bin").write_bytes(_raw(t))
    fields = [getattr(cfg, f) for f, _ in type(cfg)._fields_]
    reserve = 4
    (tmp_path / "cfg.txt").write_text(" ".join(repr(float(x)) if isinstance(x, float) else str(x) for x in fields)
                                      + f" {reserve}\n")
    run = subprocess.run([CALLER, str(tmp_path)], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    B, H, Hq, d = wl.batch, wl.n_kv_heads, wl.n_q_heads, wl.head_dim
    row = cfg.n_sink + cfg.n_middle + cfg.n_recent
    mask = np.fromfile(tmp_path / "mask.bin", dtype=np.uint8).reshape(B, H)
    lens = np.fromfile(tmp_path / "lens.bin", dtype=np.int32).reshape(B, H)
    kept = np.fromfile(tmp_path / "kept_idx.bin", dtype=np.int32).reshape(B, H, row)
    dist = np.fromfile(tmp_path / "dist.bin", dtype=np.float64).reshape(B, H)
    out = np.fromfile(tmp_path / "out.bin", dtype=np.float32).reshape(B, Hq, d)
    for b, ref in enumerate(refs):
        assert mask[b].tolist() == ref["mask"].tolist()
        np.testing.assert_allclose(dist[b], ref["dist"], rtol=1e-8, atol=1e-12)
        for h in range(H):
            want = ref["kept"][h]
            assert lens[b, h] == len(want) + 1                      # one token appended by the decode step
            if not ref["mask"][h]:
                assert kept[b, h, :len(want)].tolist() == want.tolist()
        cache = OracleCache(ref)
        cache.append(to_numpy(kn[b]), to_numpy(vn[b]))
        check_output(out[b], cache.attend(to_numpy(q[b])), wl.dtype, f"C caller, batch element {b}")


def test_c_program_runs_a_stack_of_two_layers_in_one_decode_call(tmp_path):
    """`taskkv_c_caller DIR stack`: two layers (the second with half the middle
    budget) compressed into one allocation, offsets written by
    taskkv_stack_rebase, one taskkv_decode_attn_layers step; both layers'
    outputs are checked against the oracle."""
    assert os.path.exists(CALLER), "tests/c_caller/taskkv_c_caller is not built (run __graft_entry__.build())"
    from paper_2501_15113_amd import session as ses
    wl = small_workload(name="c-stack", wid=251, ctx_len=2100, n_middle=120, n_hetero=1)
    ld = make_layer(wl, 0, "cuda:0")
    cfgs = [ses.cfg_from_workload(wl), ses.cfg_from_workload(wl, n_middle=60)]
    refs = [[oracle_layer(ld, b, c) for b in range(wl.batch)] for c in cfgs]
    assert min(r["margin"] for rr in refs for r in rr) >= MIN_MARGIN
    q, kn, vn = ld.decode_inputs(0)
    for name, t in (("q_win", ld.q_win), ("k", ld.k), ("v", ld.v), ("q", q), ("k_new", kn), ("v_new", vn)):
        (tmp_path / f"{name}.bin").write_bytes(_raw(t))
    fields = [getattr(cfgs[0], f) for f, _ in type(cfgs[0])._fields_]
    (tmp_path / "cfg.txt").write_text(" ".join(repr(float(x)) if isinstance(x, float) else str(x) for x in fields)
                                      + " 4\n")
    run = subprocess.run([CALLER, str(tmp_path), "stack"], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    B, H, Hq, d = wl.batch, wl.n_kv_heads, wl.n_q_heads, wl.head_dim
    out = np.fromfile(tmp_path / "out_stack.bin", dtype=np.float32).reshape(2, B, Hq, d)
    lens = np.fromfile(tmp_path / "lens_stack.bin", dtype=np.int32).reshape(2, B, H)
    for r in range(2):
        for b, ref in enumerate(refs[r]):
            assert lens[r, b].tolist() == [len(x) + 1 for x in ref["kept"]]
            cache = OracleCache(ref)
            cache.append(to_numpy(kn[b]), to_numpy(vn[b]))
            check_output(out[r, b], cache.attend(to_numpy(q[b])), wl.dtype, f"C caller, layer {r}, batch element {b}")
