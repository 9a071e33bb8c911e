"""The CPU oracle against what the paper and mathematics fix (no GPU needed)."""
import numpy as np
import pytest

import oracle
from oracle_pins import ALL_PINS, _close
from paper_2406_07368_amd import workloads


@pytest.mark.parametrize("pin", ALL_PINS, ids=lambda f: f.__name__)
def test_pin(pin):
    pin(None)


def test_config1_recurrent_equals_quadratic_in_full():
    """The whole fp32 workload (B1 H4 L256 d64, Kc 3): both forms, every output."""
    wl = workloads.CONFIGS["cfg1_fp32_tiny"]
    q, k, v, w = workloads.prefill_inputs(wl)
    a = oracle.prefill_quadratic(q, k, v, w)
    b = oracle.prefill_recurrent(q, k, v, w)
    for x, y, n in zip(a, b, ("out", "S", "z", "hist")):
        _close(x, y, 1e-11, n)
    assert np.all(np.isfinite(a[0]))


def test_oracle_thread_count_is_reported():
    assert oracle.num_threads() >= 1
