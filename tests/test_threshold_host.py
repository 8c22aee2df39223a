"""The library's host-side threshold arithmetic (section 4.3, equation 2) against the oracle.
No GPU work is involved: these run wherever the library loads."""

import math
import os

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2508_18736_amd", "libsiso.so")


@pytest.fixture(scope="module")
def siso():
    if not os.path.exists(LIB):
        from paper_2508_18736_amd import build
        build.build(verbose=False)
    from paper_2508_18736_amd import siso as binding
    return binding


def test_md1_wait_matches_oracle(siso, oracle):
    rng = np.random.Generator(np.random.Philox(key=5))
    for _ in range(2000):
        L, lam, h = rng.uniform(0.1, 10.0), rng.uniform(0.0, 2.0), rng.uniform(0.0, 1.0)
        want, got = oracle.md1_wait(L, lam, h), siso.md1_wait(L, lam, h)
        if math.isinf(want):
            assert math.isinf(got) and got > 0
        else:
            assert got == pytest.approx(want, rel=1e-13, abs=0)  # same formula, other order of operations
    assert siso.md1_wait(1.0, 1.0, 0.0) == math.inf
    assert siso.md1_wait(3.0, 0.0, 0.25) == 2.25


def test_pick_threshold_matches_oracle(siso, oracle):
    rng = np.random.Generator(np.random.Philox(key=6))
    thetas = np.round(np.arange(0.98, 0.599, -0.02), 2).astype(np.float32)
    seen = set()
    for _ in range(500):
        h = np.sort(rng.uniform(0.0, 1.0, thetas.shape[0]))
        order = rng.permutation(thetas.shape[0])
        L, lam, slo = rng.uniform(0.5, 5.0), rng.uniform(0.0, 1.5), rng.uniform(0.1, 6.0)
        want = oracle.pick_threshold(thetas[order], h[order], L, lam, slo)
        assert siso.pick_threshold(thetas[order], h[order], L, lam, slo) == want
        seen.add(want >= 0)
    assert seen == {True, False}  # both outcomes were exercised
    assert siso.pick_threshold(np.zeros(0, np.float32), np.zeros(0), 1.0, 0.1, 1.0) == -1


def test_adjust_threshold_matches_oracle(siso, oracle):
    rng = np.random.Generator(np.random.Philox(key=7))
    for _ in range(500):
        m = int(rng.integers(1, 12))
        thetas = rng.permutation(np.round(np.linspace(0.6, 0.98, m), 3)).astype(np.float32)
        index = int(rng.integers(-1, m + 1))
        w_est = rng.uniform(0.1, 3.0)
        w_act = w_est * rng.choice([0.5, 0.89, 0.9, 0.95, 1.0, 1.05, 1.1, 1.11, 2.0])
        assert siso.adjust_threshold(thetas, index, w_est, w_act) == oracle.adjust_threshold(thetas, index, w_est, w_act)
