"""Why the bf16 parity bar is applied to compute error and not to storage rounding: rounding the
oracle's own exact output to bf16 already exceeds 2e-2 * RMS(O) on the measured workloads, because
O has elements ~20x its RMS (early queries whose only visible softmax key returns one value row)."""
import numpy as np

from nats_inputs import CONFIGS, make_config_inputs, round_to_bf16
from oracle import c_oracle

from gpu_util import rel_err


def test_bf16_storage_rounding_alone_exceeds_the_raw_bar():
    x = make_config_inputs(CONFIGS["cfg1_bf16"])
    O = c_oracle.fwd(**x, want=())["O"]
    O_stored = round_to_bf16(O.astype(np.float32)).astype(np.float64)
    assert rel_err(O_stored, O) > 2e-2                  # an exact computation would "fail" the raw metric
    assert rel_err(O_stored, O, stored="bf16") < 1e-6   # ... and has no compute error under the adjusted one
    # the adjustment never hides an error larger than half a bf16 ulp of the element itself
    bad = O_stored * (1 + 2.0 ** -7)
    assert rel_err(bad, O, stored="bf16") > 2e-2
