"""Do the oracle's pins bite?  Each case plants one plausible mistake in a copy
of the oracle's source (a dropped term, a wrong sign or index, an off-by-one,
a swapped operand), on the CPU, and the pins of tests/test_oracle_pins.py are
run against the mistaken copy: at least one of them has to fail.  The
untouched copy has to pass all of them under the same runner."""
import inspect
import os
import types

import numpy as np
import pytest

import tests.test_oracle_pins as pins

SOURCE = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "taskkv_oracle.py")

# (what is planted, text in the oracle, replacement); the text must occur once
MISTAKES = [
    ("layer plan budgets the whole cache instead of the stated share",
     "budget = int(math.floor(budget_frac * n_heads * ctx_len))", "budget = int(math.floor(n_heads * ctx_len))"),
    ("layer plan takes the budget per head",
     "budget = int(math.floor(budget_frac * n_heads * ctx_len))", "budget = int(math.floor(budget_frac * ctx_len))"),
    ("layer plan gives every layer the first layer's head count",
     "f = hetero_head_count(n_heads, beta, m_top, r, n_layers)\n        plan.append",
     "f = hetero_head_count(n_heads, beta, m_top, 0, n_layers)\n        plan.append"),
    ("causal mask of the window hides the diagonal too",
     "hidden = j > (N - L + i)", "hidden = j >= (N - L + i)"),
    ("query head mapped to its KV head by modulo",
     "        h = q // G\n        s = scale", "        h = q % hkv\n        s = scale"),
    ("column mean forgets the group size",
     "return C / float(G * L)", "return C / float(L)"),
    ("window logits not scaled",
     "s = scale * (q_win[q] @ k[h].T)", "s = (q_win[q] @ k[h].T)"),
    ("softmax normalised over the window rows instead of the keys",
     "a = a / a.sum(axis=1, keepdims=True)            # rows of A'", "a = a / a.sum(axis=0, keepdims=True)"),
    ("pooling radius off by one",
     "r = (width - 1) // 2", "r = (width + 1) // 2"),
    ("pooling divides by the number of valid neighbours",
     "return P / float(width)",
     "return P / np.minimum(np.minimum(np.arange(N) + r + 1, N - np.arange(N) + r), width)"),
    ("equal scores go to the higher index",
     "order = np.lexsort((np.arange(score.shape[0]), -score))",
     "order = np.lexsort((-np.arange(score.shape[0]), -score))"),
    ("top-t takes the smallest scores",
     "order = np.lexsort((np.arange(score.shape[0]), -score))",
     "order = np.lexsort((np.arange(score.shape[0]), score))"),
    ("semantic vector renormalised by the captured mass",
     "out[h] = C[h, I] @ v[h, I, :]", "out[h] = (C[h, I] / C[h, I].sum()) @ v[h, I, :]"),
    ("semantic vector sums the picked rows without weights",
     "out[h] = C[h, I] @ v[h, I, :]", "out[h] = np.ones(len(I)) @ v[h, I, :]"),
    ("semantic vector weights taken at the wrong positions",
     "out[h] = C[h, I] @ v[h, I, :]", "out[h] = C[h, :len(I)] @ v[h, I, :]"),
    ("centre divided by the vector length instead of the head count",
     "centre = sem.sum(axis=0) / sem.shape[0]", "centre = sem.sum(axis=0) / sem.shape[1]"),
    ("L1 distance",
     "np.sqrt((delta * delta).sum(axis=1))", "np.abs(delta).sum(axis=1)"),
    ("squared distance",
     "np.sqrt((delta * delta).sum(axis=1))", "(delta * delta).sum(axis=1)"),
    ("closest heads marked heterogeneous",
     "far = np.lexsort((heads, -dist))", "far = np.lexsort((heads, dist))"),
    ("head ties go to the higher index",
     "far = np.lexsort((heads, -dist))", "far = np.lexsort((-heads, -dist))"),
    ("added centre head is the farthest remaining one",
     "near = rest[np.lexsort((rest, dist[rest]))[0]]", "near = rest[np.lexsort((rest, -dist[rest]))[0]]"),
    ("recent window one token short",
     "    lo, hi = n_sink, N - n_recent\n    mid =", "    lo, hi = n_sink, N - n_recent + 1\n    mid ="),
    ("middle indices not shifted by the sinks",
     "mid = lo + top_indices(P_row[lo:hi], min(n_middle, hi - lo))",
     "mid = top_indices(P_row[lo:hi], min(n_middle, hi - lo))"),
    ("middle pick ranks the whole context",
     "mid = lo + top_indices(P_row[lo:hi], min(n_middle, hi - lo))",
     "mid = top_indices(P_row, min(n_middle, hi - lo))"),
    ("heterogeneous heads compressed like the others",
     "if is_hetero or n_sink + n_recent >= N:\n        return np.arange(N, dtype=np.int64)\n    lo, hi = n_sink, N - n_recent\n    mid",
     "if n_sink + n_recent >= N:\n        return np.arange(N, dtype=np.int64)\n    lo, hi = n_sink, N - n_recent\n    mid"),
    ("packed V rows copied from K",
     "return k[kept].copy(), v[kept].copy()", "return k[kept].copy(), k[kept].copy()"),
    ("No Cache forgets the transferred budget",
     "np.arange(N - n_recent - n_extra, N)", "np.arange(N - n_recent, N)"),
    ("compensation token divided by the nominal group size",
     "km = _f64(k[a:b]).sum(axis=0) / float(b - a)", "km = _f64(k[a:b]).sum(axis=0) / float(max(M // n, 1))"),
    ("compensation token of V taken from K",
     "vm = _f64(v[a:b]).sum(axis=0) / float(b - a)", "vm = _f64(k[a:b]).sum(axis=0) / float(b - a)"),
    ("groups start one token late",
     "a, b = lo + (g * M) // n, lo + ((g + 1) * M) // n", "a, b = lo + (g * M) // n + (g > 0), lo + ((g + 1) * M) // n"),
    ("bf16 rounding breaks ties upwards",
     "take_above = (d_above < d_below) | ((d_above == d_below) & (np.mod(steps, 2.0) == 1.0))",
     "take_above = d_above <= d_below"),
    ("bf16 conversion truncates",
     "take_above = (d_above < d_below) | ((d_above == d_below) & (np.mod(steps, 2.0) == 1.0))",
     "take_above = np.zeros(a.shape, dtype=bool)"),
    ("bf16 spacing of the next binade",
     "ulp = np.ldexp(1.0, E - 8)", "ulp = np.ldexp(1.0, E - 7)"),
    ("decode maps query heads by modulo",
     "        h = qi // G\n", "        h = qi % hkv\n"),
    ("decode logits not scaled",
     "s = scale * (K @ q[qi])", "s = (K @ q[qi])"),
    ("decode weights applied to K",
     "out[qi] = p @ V", "out[qi] = p @ K"),
    ("decode output not normalised",
     "        p = p / p.sum()\n", ""),
    ("partials rescaled with the wrong sign",
     "Lsum = sum(l * math.exp(m - M) for m, l, _ in parts)", "Lsum = sum(l * math.exp(M - m) for m, l, _ in parts)"),
    ("partial outputs not rescaled",
     "O = sum(_f64(o) * math.exp(m - M) for m, _, o in parts)", "O = sum(_f64(o) for m, _, o in parts)"),
    ("exact vector forgets the division by N",
     "return (a.sum(axis=0) / N) @ v", "return a.sum(axis=0) @ v"),
    ("exact vector hides the diagonal",
     "np.arange(N)[None, :] > np.arange(N)[:, None]", "np.arange(N)[None, :] >= np.arange(N)[:, None]"),
    ("layer schedule divides by R",
     "/ (n_layers - 1) * layer", "/ n_layers * layer"),
    ("layer schedule truncates",
     "math.floor(f + 0.5)", "math.floor(f)"),
    ("layer schedule rises with depth",
     "f -= (n_heads * beta - m_top)", "f += (n_heads * beta - m_top)"),
    ("middle budget forgets the recent window",
     "// (n_heads - n_hetero) - n_sink - n_recent", "// (n_heads - n_hetero) - n_sink"),
    ("middle budget charges one full head only",
     "(layer_budget_tokens - ctx_len * n_hetero)", "(layer_budget_tokens - ctx_len)"),
    ("middle budget shared among all heads",
     "// (n_heads - n_hetero) - n_sink", "// n_heads - n_sink"),
    ("compress ignores the pooling width",
     "P = pool_scores(scores, pool_kernel)", "P = pool_scores(scores, 1)"),
    ("separator ranks heads by the raw vector norm",
     "_, dist = centre_and_distances(sem)", "dist = np.sqrt((sem * sem).sum(axis=1))"),
]


def _load(text):
    mod = types.ModuleType("taskkv_oracle_copy")
    mod.__file__ = SOURCE
    exec(compile(text, SOURCE, "exec"), mod.__dict__)
    return mod


def _cases():
    """(name, callable) for every pin, parametrised ones expanded."""
    out = []
    for name, fn in sorted(vars(pins).items()):
        if not name.startswith("test_") or not inspect.isfunction(fn):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            out.append((name, fn))
            continue
        assert len(marks) == 1 and "," not in marks[0].args[0]
        arg = marks[0].args[0]
        for val in marks[0].args[1]:
            out.append((f"{name}[{val}]", lambda fn=fn, arg=arg, val=val: fn(**{arg: val})))
    return out


def _first_failure(oracle_module, monkeypatch):
    monkeypatch.setattr(pins, "orc", oracle_module)
    monkeypatch.setattr(pins, "RNG", np.random.default_rng(20250115))
    for name, fn in _cases():
        try:
            fn()
        except Exception as exc:      # an assertion, or a crash the mistake causes
            return f"{name}: {type(exc).__name__}"
    return None


def test_untouched_copy_passes_every_pin(monkeypatch):
    assert len(_cases()) >= 25
    assert _first_failure(_load(open(SOURCE).read()), monkeypatch) is None


@pytest.mark.parametrize("what,old,new", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_planted_mistake_fails_a_pin(what, old, new, monkeypatch):
    text = open(SOURCE).read()
    assert text.count(old) == 1, f"cannot plant '{what}': the oracle's text has changed"
    caught = _first_failure(_load(text.replace(old, new)), monkeypatch)
    assert caught is not None, f"no pin notices: {what}"
    print(f"{what}: caught by {caught}")
