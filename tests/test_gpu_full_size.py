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
