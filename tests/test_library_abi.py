"""CPU-side checks of the C ABI: the library loads, exports every symbol the
header declares, and its host-only helpers agree with the oracle."""
import os
import re

import pytest

import paper_2501_15113_amd as tk
from oracle import taskkv_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "taskkv.h")).read()
    declared = set(re.findall(r"\b(taskkv_[a-z_0-9]+)\s*\(", header))
    assert declared and declared == set(tk.EXPORTED_SYMBOLS)
    lib = tk.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    assert int(re.search(r"#define TASKKV_CHUNK_TOKENS (\d+)", header).group(1)) == tk.CHUNK_TOKENS


def test_cfg_struct_matches_header_field_order():
    header = open(os.path.join(ROOT, "include", "taskkv.h")).read()
    body = header[header.index("typedef struct taskkv_layer_cfg {"):header.index("} taskkv_layer_cfg;")]
    fields = re.findall(r"^\s*(?:int32_t|float)\s+(\w+);", body, flags=re.M)
    assert fields == [f for f, _ in tk.LayerCfg._fields_]


def test_strerror():
    assert tk.taskkv_strerror(0) == "ok"
    assert tk.taskkv_strerror(-2) == "cache buffer too small"


def test_budget_helpers_match_oracle():
    for layer in range(32):
        assert tk.taskkv_hetero_head_count(32, 0.25, 4, layer, 32) == orc.hetero_head_count(32, 0.25, 4, layer, 32)
        assert tk.taskkv_hetero_head_count(8, 0.3, 1, layer, 32) == orc.hetero_head_count(8, 0.3, 1, layer, 32)
    assert tk.taskkv_hetero_head_count(8, 0.3, 1, 0, 1) == orc.hetero_head_count(8, 0.3, 1, 0, 1)
    for n, beta, m, R in [(32, 0.5, 0, 17), (8, 0.25, 1, 5), (8, 0.25, 1, 3), (40, 0.9, 50, 7), (8, 0.0, 0, 4)]:
        for layer in range(R):
            assert tk.taskkv_hetero_head_count(n, beta, m, layer, R) == orc.hetero_head_count(n, beta, m, layer, R)
    for args in [(104857, 32768, 8, 1, 4, 128), (104857, 32768, 8, 3, 4, 128), (100, 50, 4, 4, 1, 1),
                 (10, 50, 4, 1, 1, 1), (1000, 64, 8, 2, 4, 4)]:
        assert tk.taskkv_middle_budget(*args) == orc.middle_budget(*args)


def test_layer_plan_matches_oracle():
    for n, beta, m, R, frac, N, s1, s2 in [(32, 0.25, 4, 32, 0.4, 30000, 16, 256), (8, 0.3, 1, 32, 0.6, 32768, 16, 256),
                                           (8, 0.3, 1, 32, 0.4, 16384, 4, 128), (8, 0.5, 4, 4, 0.4, 1000, 4, 8),
                                           (4, 0.5, 0, 1, 1.0, 77, 0, 0), (8, 0.3, 1, 7, 0.123, 5001, 3, 9)]:
        assert tk.taskkv_layer_plan(n, beta, m, R, frac, N, s1, s2) == orc.layer_plan(n, beta, m, R, frac, N, s1, s2)
    with pytest.raises(tk.TaskKVError):
        tk.taskkv_layer_plan(8, 0.3, 1, 32, 1.5, 1000, 4, 8)


def _cfg(**kw):
    base = dict(batch=2, n_q_heads=8, n_kv_heads=4, head_dim=128, ctx_len=5000, n_sink=4, n_recent=32,
                n_middle=64, n_hetero=1, dtype=tk.BF16)
    base.update(kw)
    return tk.LayerCfg(**base)


def test_cache_tokens_counts_regions():
    c = 512
    up = lambda n: (n + c - 1) // c * c
    assert tk.taskkv_cache_tokens(_cfg(), 10) == 2 * (up(5010) + 3 * up(110))
    assert tk.taskkv_cache_tokens(_cfg(add_centre_head=1), 0) == 2 * (2 * up(5000) + 2 * up(100))
    assert tk.taskkv_cache_tokens(_cfg(n_hetero=9), 0) == 2 * 4 * up(5000)
    assert tk.taskkv_cache_tokens(_cfg(n_sink=3000, n_recent=2000), 0) == 2 * 4 * up(5000)   # covers N
    assert tk.taskkv_cache_tokens(_cfg(n_middle=10 ** 6, n_hetero=0), 0) == 2 * 4 * up(5000)  # k clipped
    assert tk.taskkv_workspace_bytes(_cfg(), 10) > 0


@pytest.mark.parametrize("bad", [dict(head_dim=96), dict(n_q_heads=6), dict(obs_window=6000),
                                 dict(pool_kernel=4), dict(dtype=3), dict(ctx_len=0), dict(top_t=0),
                                 dict(n_sink=-1), dict(n_q_heads=4 * 80)])
def test_invalid_cfg_is_rejected_on_the_host(bad):
    with pytest.raises(tk.TaskKVError):
        tk.taskkv_cache_tokens(_cfg(**bad), 0)
    with pytest.raises(tk.TaskKVError):
        tk.taskkv_workspace_bytes(_cfg(**bad), 0)


def _imports_of(path):
    import ast
    names = set()
    for node in ast.walk(ast.parse(open(path).read())):
        if isinstance(node, ast.Import):
            names.update(a.name.split(".")[0] for a in node.names)
        elif isinstance(node, ast.ImportFrom) and node.level == 0 and node.module:
            names.add(node.module.split(".")[0])
    return names


def test_product_and_oracle_do_not_import_each_other():
    """The oracle is test infrastructure: nothing in the package or in the input
    generators imports it, and it imports neither of them."""
    import glob
    for path in glob.glob(os.path.join(ROOT, "paper_2501_15113_amd", "*.py")) + \
            glob.glob(os.path.join(ROOT, "taskkv_synth", "*.py")):
        assert "oracle" not in _imports_of(path), path
    for path in glob.glob(os.path.join(ROOT, "oracle", "*.py")):
        assert not {"paper_2501_15113_amd", "taskkv_synth", "torch", "ctypes"} & _imports_of(path), path
    for src in glob.glob(os.path.join(ROOT, "paper_2501_15113_amd", "csrc", "*")):
        assert "oracle" not in open(src).read(), src


def test_missing_library_is_an_error_not_a_fallback(monkeypatch, tmp_path):
    from paper_2501_15113_amd import binding
    monkeypatch.setenv("TASKKV_LIBRARY", str(tmp_path / "nothing_here.so"))
    monkeypatch.setattr(binding, "_LIB", None, raising=False)
    with pytest.raises(tk.TaskKVError):
        binding.load_library()


def test_header_is_plain_c(tmp_path):
    """include/taskkv.h compiles as C99 on its own: no C++, no HIP or torch types in the signatures."""
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text('#include "taskkv.h"\nint main(void) { taskkv_layer_cfg c; (void)c; return TASKKV_OK; }\n')
    r = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-I",
                        os.path.join(ROOT, "include"), str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
