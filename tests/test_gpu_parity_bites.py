"""Does the GPU parity check bite?  The comparison of tests/test_gpu_parity.py
is run with a mistake planted in a copy of the oracle (on the CPU; the HIP
library is untouched): it must then report a difference.  Mistakes that touch
the path from window scores to attention output are taken from the list in
tests/test_oracle_mutations.py."""
import pytest

import tests._harness as harness
from taskkv_synth import small_workload
import tests.test_gpu_parity as parity
from tests.test_oracle_mutations import MISTAKES, SOURCE, _load

pytestmark = pytest.mark.gpu


def _dup_keys(ld):
    ld.k[:, :, 200:400] = ld.k[:, :, 0:200]


# mistake -> (workload overrides, input mutation) of the layer that shows it
ON_PATH = {
    "causal mask of the window hides the diagonal too": (dict(), None),
    "query head mapped to its KV head by modulo": (dict(), None),
    "column mean forgets the group size": (dict(), None),
    "window logits not scaled": (dict(), None),
    "softmax normalised over the window rows instead of the keys": (dict(), None),
    "pooling radius off by one": (dict(pool_kernel=7, ctx_len=1300), None),
    "pooling divides by the number of valid neighbours": ("edges", None),
    "compress ignores the pooling width": (dict(pool_kernel=7, ctx_len=1300), None),
    "equal scores go to the higher index": (dict(ctx_len=1000, n_middle=120), _dup_keys),
    "top-t takes the smallest scores": (dict(), None),
    "semantic vector renormalised by the captured mass": (dict(), None),
    "semantic vector sums the picked rows without weights": (dict(), None),
    "semantic vector weights taken at the wrong positions": (dict(), None),
    "centre divided by the vector length instead of the head count": (dict(), None),
    "L1 distance": (dict(), None),
    "squared distance": (dict(), None),
    "closest heads marked heterogeneous": (dict(), None),
    "added centre head is the farthest remaining one": (dict(add_centre_head=1, ctx_len=800), None),
    "recent window one token short": (dict(), None),
    "middle indices not shifted by the sinks": (dict(), None),
    "middle pick ranks the whole context": (dict(), None),
    "heterogeneous heads compressed like the others": (dict(), None),
    "packed V rows copied from K": (dict(), None),
    "decode maps query heads by modulo": (dict(), None),
    "decode logits not scaled": (dict(), None),
    "decode weights applied to K": (dict(), None),
    "decode output not normalised": (dict(), None),
}


def test_the_list_names_known_mistakes():
    assert set(ON_PATH) <= {m[0] for m in MISTAKES}


@pytest.mark.parametrize("what", sorted(ON_PATH))
def test_parity_check_reports_a_planted_oracle_mistake(what, monkeypatch):
    (old, new), = [(o, n) for w, o, n in MISTAKES if w == what]
    text = open(SOURCE).read()
    assert text.count(old) == 1
    kw, mutate = ON_PATH[what]
    if kw == "edges":       # only the ends of the context tell the two divisors apart
        check = parity.test_pooled_scores_keep_the_full_divisor_at_the_edges
    else:
        wl = small_workload(name="bites", wid=231, **kw)
        check = lambda: parity.run_layer(wl, mutate=mutate)
    check()                                            # the honest oracle agrees
    monkeypatch.setattr(harness, "orc", _load(text.replace(old, new)))
    with pytest.raises(AssertionError) as info:
        check()
    msg = str(info.value)
    assert msg and "MIN_MARGIN" not in msg, "failed on the decision margin, not on a difference"
    print(f"{what}: {msg.strip().splitlines()[0][:100]}")
