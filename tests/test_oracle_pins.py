"""The float64 oracle against its pins (see tests/oracle_pins.py for what each one fixes)."""
import numpy as np
import pytest

import oracle
from oracle_pins import ALL_PINS
from workloads import CONFIG_NAMES, make_workload, weight_count


@pytest.mark.parametrize("pin", ALL_PINS, ids=lambda p: p.__name__)
def test_pin(pin, oracle_lib):
    pin(oracle_lib)


def test_weight_count_matches_interface():
    for D, H, L, g in [(2, 8, 2, 1), (4, 32, 2, 1), (8, 128, 2, 1), (3, 5, 1, 0), (4, 64, 3, 0)]:
        assert oracle.weight_count(D, H, L, g) == weight_count(D, H, L, bool(g))


def test_bf16_rounding_is_nearest_even():
    # 1 + 2^-8 is exactly half-way between bf16 neighbours 1 and 1 + 2^-7: ties go to even
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20,
                  -(1.0 + 2.0 ** -9), 3.0], dtype=np.float32)
    want = np.array([1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -1.0, 3.0], dtype=np.float32)
    np.testing.assert_array_equal(oracle.round_to_bf16(x), want)
    import torch
    r = np.random.default_rng(0).normal(0, 0.1, 4096).astype(np.float32)
    np.testing.assert_array_equal(oracle.round_to_bf16(r),
                                  torch.tensor(r).to(torch.bfloat16).to(torch.float32).numpy())


@pytest.mark.parametrize("name", CONFIG_NAMES)
def test_finite_at_scale(name):
    """Sanity on the five workload shapes: every embedding and logit stays finite."""
    w = make_workload(name, B=2)
    r = oracle.forward_workload(w, n_threads=2)
    assert np.isfinite(r["emb"]).all() and np.isfinite(r["logits"]).all()
    assert np.all(np.abs(r["probs"].sum(axis=1) - 1.0) < 1e-12)
