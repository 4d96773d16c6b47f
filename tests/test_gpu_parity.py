"""GPU parity: the HIP path against the CPU oracle, element by element, on the
same seeded inputs.  Everything goes through the C ABI."""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode", ["lcn", "nystrom", "sparse", "dense"])
def test_config1(mode):
    from parity import compare
    p = workloads.config1()
    out = compare(p, mode)
    print("C1", mode, out, flush=True)
